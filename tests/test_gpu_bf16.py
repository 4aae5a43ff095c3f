"""GPU parity, bf16: the tuned HIP path (MFMA GEMMs with fused epilogues, flash-style prefill
attention, split-K decode attention) against the CPU oracle, on small shapes that span several
tiles, ragged tails and every kernel-selection branch, and at the full Mid PT sizes."""
import dataclasses

import numpy as np
import pytest

from oracle import pt_oracle as O
from paper_2602_07306_amd import inputs as I
from tests.helpers import (BF16_TOL, GEMM_CLASSES, PATH_CLASSES, argmax_agrees, assert_close, oracle_prefill,
                           path_counts, rel_err, small_bf16_config)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def run_case(cfg, seed, B, S, steps, paths):
    from paper_2602_07306_amd import binding as PB
    W = I.make_weights(cfg, seed)
    tokens = I.make_tokens(seed, B, S, cfg.vocab)
    ref, st = oracle_prefill(cfg, W, tokens)
    nxt = np.argmax(ref["logits"][:, -1], -1).astype(np.int32)
    refs = []
    for _ in range(steps):
        r = O.pt_decode_step(cfg, W, st, tokens=nxt)
        refs.append((nxt.copy(), r))
        nxt = r["argmax"]
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    outs, counts = {}, {}
    for path in paths:
        model.pt_set_kernel_path(path)
        model.pt_reset()
        model.pt_profile_reset()
        taps, _ = model.pt_set_taps(B * S)
        lg, hid = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL,
                                   want_hidden=True)
        torch.cuda.synchronize()
        L = lg.cpu().numpy().reshape(B, S, -1)
        assert_close(L, ref["logits"], BF16_TOL, "prefill logits")
        assert_close(hid.cpu().numpy(), ref["hidden"], BF16_TOL, "prefill hidden")
        for b in range(B):
            for k in range(cfg.n_merges):
                got = taps[k].cpu().numpy().reshape(B, S, -1)[b]
                assert_close(got, ref["taps"][b][k], BF16_TOL, "tap %d of sequence %d" % (k, b))
            assert argmax_agrees(L[b], ref["logits"][b], BF16_TOL)
        model.pt_clear_taps()
        pre_counts = path_counts(model)
        model.pt_profile_reset()
        for i, (tok, r) in enumerate(refs):
            lg, _, am = model.pt_decode_step(torch.from_numpy(tok).cuda(), want_argmax=True)
            torch.cuda.synchronize()
            assert_close(lg.cpu().numpy(), r["logits"], BF16_TOL, "decode step %d" % i)
            assert argmax_agrees(lg.cpu().numpy(), r["logits"], BF16_TOL)
            assert np.array_equal(am.cpu().numpy(), np.argmax(lg.cpu().numpy(), -1))
        assert model.pt_seq_len() == S + steps
        model.pt_sync_status()
        outs[path] = L
        counts[path] = (pre_counts, path_counts(model))
    model.close()
    return outs, counts


def check_kernel_families(cfg, S, steps, counts):
    """Which kernels served the two legs.  The forced leg must have launched shape-generic kernels only.  The
    automatic leg must not have fallen back to them, except for the one documented reason among these cases:
    prefill attention needs a prompt length that is a multiple of 32 (a one-token prompt runs the decode kernel)."""
    from paper_2602_07306_amd import binding as PB
    L = cfg.n_layers
    pre, dec = counts[PB.PT_PATH_GENERIC]
    for leg, n_layers_calls in ((pre, 1), (dec, steps)):
        for c in PATH_CLASSES:
            assert sum(leg[c][1:]) == 0, (c, leg[c])
    assert pre["gemm_qkv"][0] == L and dec["gemm_qkv"][0] == L * steps
    pre, dec = counts[PB.PT_PATH_AUTO]
    attn_generic = S != 1 and (S % 32 != 0 or S < 32)
    for c in GEMM_CLASSES:
        assert pre[c][0] == 0 and dec[c][0] == 0, ("fell back to the generic GEMM", c, pre[c], dec[c])
        expect = 1 if c == "gemm_head" else L
        assert sum(pre[c]) == expect and sum(dec[c]) == expect * steps, (c, pre[c], dec[c])
    pre_attn = pre["attn_decode"] if S == 1 else pre["attn_prefill"]
    assert pre_attn[0] == (L if attn_generic else 0) and sum(pre_attn) == L, pre_attn
    assert dec["attn_decode"][0] == 0 and sum(dec["attn_decode"]) == L * steps, dec["attn_decode"]
    return pre, dec


CASES = {
    # name: (config overrides, B, S, decode steps)
    "hd64_tiles": (dict(), 2, 128, 2),
    "hd128": (dict(head_dim=128, n_heads=2, n_kv_heads=2), 2, 128, 2),
    "gqa_hd64": (dict(n_kv_heads=2), 2, 96, 2),
    "gqa_1kv_hd128": (dict(head_dim=128, n_heads=4, n_kv_heads=1, d_model=512), 1, 160, 2),
    "ragged_rows": (dict(), 2, 100, 2),                  # S not a multiple of any tile: M tail, generic attention
    "three_tracks": (dict(n_tracks=3, n_layers=3, block_depth=1, merge_scale=1.0 / 3), 1, 64, 1),
    "split_decode": (dict(max_batch=1, max_seq=1024), 1, 704, 3),   # decode context split in two, ragged tail
    "one_token_prompt": (dict(), 2, 1, 3),
    # grouped-query decode with a split, ragged context; 16 query heads on one KV head
    "gqa_split_decode": (dict(n_kv_heads=1, max_batch=2, max_seq=1024), 2, 701, 3),
    "gqa_16_per_group": (dict(n_heads=16, n_kv_heads=1, head_dim=64, max_seq=512), 1, 333, 2),
    # 24 query heads per KV head (matrix-core decode kernel, more than 16 columns) and 40 (vector decode kernel)
    "gqa_24_per_group": (dict(n_heads=24, n_kv_heads=1, head_dim=64, max_seq=512), 1, 200, 2),
    "gqa_40_per_group": (dict(n_heads=40, n_kv_heads=1, head_dim=64, max_seq=512), 1, 200, 2),
    # decode GEMM planner: odd row counts, three tracks, K = 3 x 512 (three K slices), uneven tile dealing
    "decode_5_rows_3_tracks": (dict(n_tracks=3, n_layers=2, block_depth=1, d_model=512, n_heads=8, n_kv_heads=2,
                                    head_dim=64, d_ffn=1536, max_batch=5, max_seq=128, merge_scale=1.0 / 3), 5, 70, 3),
    "decode_33_rows": (dict(n_layers=2, block_depth=2, d_model=512, n_heads=8, n_kv_heads=8, head_dim=64,
                            d_ffn=1024, max_batch=33, max_seq=64), 33, 8, 2),
    # long prompts: many key tiles per query block in prefill, split decode over a long cache
    "long_prompt_hd64": (dict(max_batch=1, max_seq=2112), 1, 2048, 2),
    "long_prompt_hd128_gqa": (dict(head_dim=128, n_heads=4, n_kv_heads=2, d_model=512, n_layers=2, block_depth=2,
                                   max_batch=1, max_seq=1600), 1, 1536, 2),
    # matrix-vector decode kernel: two and three rows
    "gemv_2_rows": (dict(n_tracks=4, n_layers=2, block_depth=2, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64,
                         d_ffn=1024, max_batch=2, max_seq=128), 2, 40, 3),
    "gemv_3_rows": (dict(n_tracks=4, n_layers=2, block_depth=1, d_model=512, n_heads=4, n_kv_heads=4, head_dim=128,
                         d_ffn=1536, max_batch=3, max_seq=128), 3, 33, 3),
    # one track that merges after every layer (the dense twin of a PT model): the merge is the identity and is
    # skipped over several blocks once no tap is requested (the decode steps here)
    "dense_one_track_three_blocks": (dict(n_tracks=1, n_layers=3, block_depth=1), 2, 64, 3),
    # the largest track count the library takes; decoding up to the last row of the KV cache (max_seq is not a
    # multiple of the cache's 64-row granularity)
    "sixteen_tracks": (dict(n_tracks=16, n_layers=2, block_depth=1, merge_scale=1.0 / 16), 1, 64, 2),
    "cache_filled_to_the_last_row": (dict(max_batch=2, max_seq=99), 2, 96, 3),
    # per-track shape of the paper's 30B model (Table 1: 8 tracks, 8 query heads and 1 KV head per track), batch 1
    "paper30b_track_shape": (dict(n_tracks=8, n_layers=2, block_depth=2, d_model=512, n_heads=8, n_kv_heads=1,
                                  head_dim=128, d_ffn=1024, max_batch=1, max_seq=512), 1, 192, 3),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_small_bf16_models_match_the_oracle(name):
    from paper_2602_07306_amd import binding as PB
    over, B, S, steps = CASES[name]
    cfg = small_bf16_config(**over)
    outs, counts = run_case(cfg, 7 + len(name), B, S, steps, (PB.PT_PATH_AUTO, PB.PT_PATH_GENERIC))
    # the tuned and the shape-generic kernels agree with each other as well
    assert rel_err(outs[PB.PT_PATH_AUTO], outs[PB.PT_PATH_GENERIC]) <= BF16_TOL
    pre, dec = check_kernel_families(cfg, S, steps, counts)
    # cases built for one kernel must have reached it (families: 1 MFMA tile GEMM / first attention kernel,
    # 2 weight-streaming GEMM / second attention kernel, 3 matrix-vector GEMM)
    L = cfg.n_layers
    if name in ("decode_5_rows_3_tracks", "decode_33_rows"):
        for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down"):
            assert dec[c][2] == L * steps, (c, dec[c])
    if name == "gemv_2_rows":
        assert dec["gemm_gateup"][3] == L * steps
    if name in ("gemv_3_rows", "paper30b_track_shape"):
        assert dec["gemm_qkv"][3] == L * steps and dec["gemm_gateup"][3] == L * steps
    if name == "gqa_40_per_group":
        assert dec["attn_decode"][2] == L * steps
    if name in ("gqa_24_per_group", "gqa_16_per_group", "split_decode", "gqa_split_decode"):
        assert dec["attn_decode"][1] == L * steps
    if name == "gqa_hd64":
        assert pre["attn_prefill"][2] == L          # 96 tokens: the register-operand flash kernel
    if name in ("hd64_tiles", "hd128", "long_prompt_hd64", "long_prompt_hd128_gqa"):
        assert pre["attn_prefill"][1] == L          # the LDS-tiled flash kernel


def test_results_are_reproducible_run_to_run():
    """Two runs of the same forward give bit-identical logits (no races in LDS staging)."""
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config()
    model = PB.PTModel(cfg)
    model.pt_init_weights(3)
    tokens = torch.from_numpy(I.make_tokens(3, 2, 256, cfg.vocab)).cuda()
    a, _ = model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_ALL)
    a = a.clone()
    b, _ = model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_ALL)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    model.close()


def test_causal_prefix_and_batch_independence_on_the_gpu():
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config(max_batch=3)
    model = PB.PTModel(cfg)
    model.pt_init_weights(5)
    tok = I.make_tokens(5, 3, 128, cfg.vocab)
    full, _ = model.pt_prefill(torch.from_numpy(tok).cuda(), logits_mode=PB.PT_LOGITS_ALL)
    full = full.cpu().numpy().reshape(3, 128, -1)
    # appended tokens do not change earlier positions; batch-mates do not change a sequence
    part, _ = model.pt_prefill(torch.from_numpy(np.ascontiguousarray(tok[1:2, :64])).cuda(),
                               logits_mode=PB.PT_LOGITS_ALL)
    part = part.cpu().numpy().reshape(1, 64, -1)
    assert rel_err(part[0], full[1, :64]) <= 1e-2     # different tile shapes, same mathematics
    model.close()


def test_mid_prefill_full_size_matches_the_oracle_on_sampled_sequences():
    """Mid PT prefill at the benchmark's sizes and launch configuration (T=4, L=16, D=4, d=1024,
    16 heads x 64, FFN 4096, vocab 32000, batch 4 x 1024).  The oracle evaluates two of the four
    sequences (sequences are independent) at every position."""
    from paper_2602_07306_amd import binding as PB
    cfg = I.config_mid(max_batch=4, max_seq=1024)
    B, S = 4, 1024
    W = I.make_weights(cfg, 1)
    tokens = I.make_tokens(1, B, S, cfg.vocab)
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    got_w = model.pt_get_weight("wd", 3, 15, W["wd"][3, 15].shape)
    assert np.array_equal(got_w, W["wd"][3, 15])
    taps, _ = model.pt_set_taps(B * S)
    lg, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL)
    torch.cuda.synchronize()
    assert model.pt_merge_count() == 4
    counts = path_counts(model)      # the benchmark's launch configuration: no shape-generic kernel anywhere
    for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down"):
        assert counts[c] == [0, 16, 0, 0], (c, counts[c])
    assert counts["attn_prefill"] == [0, 16, 0, 0] and counts["gemm_head"] == [0, 1, 0, 0]
    L = lg.cpu().numpy().reshape(B, S, -1)
    last, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_LAST)
    torch.cuda.synchronize()
    # last-row logits come from the weight-streaming GEMM (M = 4 rows), all-row logits from the
    # tiled one: same inputs, different summation order
    np.testing.assert_allclose(last.cpu().numpy(), L[:, -1], rtol=0, atol=1e-5 * np.max(np.abs(L[:, -1])))
    for b in (0, 3):
        st = O.PTState(cfg, 1, S)
        ref = O.pt_prefill(cfg, W, st, tokens=tokens[b:b + 1], collect_taps=True)
        assert_close(L[b], ref["logits"][0], BF16_TOL, "logits of sequence %d" % b)
        for k in range(4):
            got = taps[k].cpu().numpy().reshape(B, S, -1)[b]
            assert_close(got, ref["taps"][0][k], BF16_TOL, "tap %d of sequence %d" % (k, b))
        assert argmax_agrees(L[b], ref["logits"][0], BF16_TOL)
    model.close()


def test_mid_decode_full_context_matches_the_oracle_on_a_sampled_sequence():
    """Mid PT decode shape: batch 32, 2048-token prompts (seed 2), then KV-cached steps.  The
    oracle follows one of the 32 sequences (prefill + the same decode tokens)."""
    from paper_2602_07306_amd import binding as PB
    B, prompt, steps, pick = 32, 2048, 3, 17
    cfg = I.config_mid(max_batch=B, max_seq=prompt + 64)
    W = I.make_weights(cfg, 1)
    tokens = I.make_tokens(2, B, prompt, cfg.vocab)
    feed = I.make_tokens(12, steps, B, cfg.vocab)            # decode inputs, [step, B]
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    lg, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_LAST)
    torch.cuda.synchronize()
    st = O.PTState(cfg, 1, prompt + 64)
    ref = O.pt_prefill(cfg, W, st, tokens=tokens[pick:pick + 1])
    assert rel_err(lg.cpu().numpy()[pick], ref["logits"][0, -1]) <= BF16_TOL
    model.pt_profile_reset()
    for i in range(steps):
        r = O.pt_decode_step(cfg, W, st, tokens=feed[i, pick:pick + 1])
        g, _, _ = model.pt_decode_step(torch.from_numpy(np.ascontiguousarray(feed[i])).cuda())
        torch.cuda.synchronize()
        assert rel_err(g.cpu().numpy()[pick], r["logits"][0]) <= BF16_TOL, i
    assert model.pt_seq_len() == prompt + steps
    counts = path_counts(model)
    for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down"):
        assert counts[c] == [0, 0, cfg.n_layers * steps, 0], (c, counts[c])
    assert counts["attn_decode"] == [0, cfg.n_layers * steps, 0, 0]
    model.close()


def test_block_end_merge_at_the_one_gpu_share_shape():
    """The block-end merge of one GPU's share of a wide 8-track model: own hidden state plus the
    other 7 tracks' hidden states as seeded N(0,1) bf16 tensors [8192 tokens, 8192]."""
    from paper_2602_07306_amd import binding as PB
    tokens, d, n = 8192, 8192, 8
    hs = [I.make_hidden(4, i, tokens, d) for i in range(n)]
    dev = [torch.from_numpy(h).cuda().to(torch.bfloat16) for h in hs]
    out = PB.pt_track_merge(dev, 1.0)
    torch.cuda.synchronize()
    got = out.float().cpu().numpy()
    rows = np.random.default_rng(0).choice(tokens, 64, replace=False)
    ref = O.track_merge([h[rows] for h in hs], 1.0)
    assert rel_err(got[rows], ref) <= 2.0 ** -8
    acc = hs[0][rows].copy()
    for h in hs[1:]:
        acc = acc + h[rows]
    assert np.array_equal(got[rows], I.round_to_dtype(acc, I.PT_BF16))
    # every element, against a property that holds at any size: |out| <= sum |h_i| (+ rounding)
    bound = np.zeros((tokens, d), np.float32)
    for h in hs:
        bound += np.abs(h)
    assert np.all(np.abs(got) <= bound * (1 + 2.0 ** -7) + 1e-6)


def _reduced_depth_case(cfg, seed, B, S):
    """Full layer widths of a large configuration, reduced depth and token count (the oracle cost
    of the full configuration is hours): logits / hidden and every block tap against the oracle."""
    from paper_2602_07306_amd import binding as PB
    W = I.make_weights(cfg, seed)
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    if cfg.vocab:
        tokens = I.make_tokens(seed, B, S, cfg.vocab)
        ref, st = oracle_prefill(cfg, W, tokens)
        taps, _ = model.pt_set_taps(B * S)
        lg, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL)
        torch.cuda.synchronize()
        assert rel_err(lg.cpu().numpy().reshape(B, S, -1), ref["logits"]) <= BF16_TOL
        tap_np = taps.cpu().numpy().copy()
        model.pt_clear_taps()
        nxt = np.argmax(ref["logits"][:, -1], -1).astype(np.int32)
        r = O.pt_decode_step(cfg, W, st, tokens=nxt)
        g, _, _ = model.pt_decode_step(torch.from_numpy(nxt).cuda())
        torch.cuda.synchronize()
        assert rel_err(g.cpu().numpy(), r["logits"]) <= BF16_TOL
    else:
        x = np.stack([I.make_hidden(seed, 0, S, cfg.d_model) for _ in range(B)])       # [B, S, d], bf16 values
        ref, st = oracle_prefill(cfg, W, hidden_in=x.astype(np.float64))
        taps, _ = model.pt_set_taps(B * S)
        _, hid = model.pt_prefill(hidden_in=torch.from_numpy(x).cuda(), logits_mode=PB.PT_LOGITS_NONE,
                                  want_hidden=True)
        torch.cuda.synchronize()
        assert rel_err(hid.cpu().numpy(), ref["hidden"]) <= BF16_TOL
        tap_np = taps.cpu().numpy().copy()
        model.pt_clear_taps()
        xn = I.make_hidden(seed, 9, B, cfg.d_model)                                     # [B, d]
        r = O.pt_decode_step(cfg, W, st, hidden_in=xn.astype(np.float64))
        _, g, _ = model.pt_decode_step(hidden_in=torch.from_numpy(xn).cuda(), want_logits=False,
                                       want_hidden=True)
        torch.cuda.synchronize()
        assert rel_err(g.cpu().numpy(), r["hidden"]) <= BF16_TOL
    for b in range(B):
        for k in range(cfg.n_merges):
            got = tap_np[k].reshape(B, S, -1)[b]
            assert rel_err(got, ref["taps"][b][k]) <= BF16_TOL, (b, k)
    model.close()


def test_large_config_widths_at_reduced_depth():
    """Large PT layer shape (T=8, d=2048, 16 heads x 128, FFN 8192, vocab 32000), 2 layers with a
    merge after each, 1 x 256 tokens."""
    cfg = dataclasses.replace(I.config_large(max_batch=1, max_seq=320), n_layers=2, block_depth=1)
    _reduced_depth_case(cfg, 3, 1, 256)


def test_share_config_widths_at_reduced_depth():
    """One GPU's share of the wide model (single track, d=8192, 64 heads x 128, FFN 28672,
    hidden-state in / out), 2 layers, 1 x 128 tokens."""
    cfg = dataclasses.replace(I.config_share(max_batch=1, max_seq=192), n_layers=2, block_depth=2)
    _reduced_depth_case(cfg, 4, 1, 128)


def test_single_track_prefill_without_taps_skips_the_identity_merge():
    """T = 1 with a merge after every layer and the literal sum: the all-reduce of one track is the identity, so
    the library runs no merge kernel (the track continues from its own residual stream) yet counts the merges.
    Prefill logits and hidden state against the oracle, three blocks deep."""
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config(n_tracks=1, n_layers=3, block_depth=1, max_batch=2, max_seq=128)
    W = I.make_weights(cfg, 21)
    tokens = I.make_tokens(21, 2, 96, cfg.vocab)
    ref, _ = oracle_prefill(cfg, W, tokens, taps=False)
    model = PB.PTModel(cfg)
    model.pt_init_weights(21)
    model.pt_profile_enable(["merge"])
    lg, hid = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL, want_hidden=True)
    torch.cuda.synchronize()
    assert model.pt_profile_read("merge")[1] == 0          # no merge kernel was launched ...
    assert model.pt_merge_count() == 3                       # ... for the three merges of Algorithm 1
    assert_close(lg.cpu().numpy().reshape(2, 96, -1), ref["logits"], BF16_TOL, "logits")
    assert_close(hid.cpu().numpy(), ref["hidden"], BF16_TOL, "hidden")
    model.close()


def _decode_at_batch_64(cfg, seed, S, picks, steps=2):
    """Full layer widths of a large configuration, one layer, decode at batch 64 (the benchmark's batch: two
    32-row blocks per weight tile, K slices for the residual GEMMs).  The GPU runs all 64 sequences; the oracle
    follows the sampled ones (sequences are independent)."""
    from paper_2602_07306_amd import binding as PB
    B = 64
    print("decode at batch 64: generating weights", flush=True)
    W32 = I.make_weights(cfg, seed)
    W = {k: v.astype(np.float64) for k, v in W32.items()}    # converted once: the oracle then takes views
    del W32
    print("decode at batch 64: GPU leg", flush=True)
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    if cfg.vocab:
        tokens = I.make_tokens(seed, B, S, cfg.vocab)
        feed = I.make_tokens(seed + 100, steps, B, cfg.vocab)
        model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_NONE)
    else:
        x = np.stack([I.make_hidden(seed, b, S, cfg.d_model) for b in range(B)])             # [B, S, d]
        feed = np.stack([I.make_hidden(seed + 100, i, B, cfg.d_model) for i in range(steps)])  # [steps, B, d]
        model.pt_prefill(hidden_in=torch.from_numpy(x).cuda(), logits_mode=PB.PT_LOGITS_NONE)
    model.pt_profile_reset()
    got = []
    for i in range(steps):
        if cfg.vocab:
            lg, _, _ = model.pt_decode_step(torch.from_numpy(np.ascontiguousarray(feed[i])).cuda())
            got.append(lg.cpu().numpy())
        else:
            _, hid, _ = model.pt_decode_step(hidden_in=torch.from_numpy(feed[i]).cuda(), want_logits=False,
                                             want_hidden=True)
            got.append(hid.cpu().numpy())
    torch.cuda.synchronize()
    counts = path_counts(model)
    for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down"):
        # every decode GEMM went to the weight-streaming kernel
        assert counts[c] == [0, 0, cfg.n_layers * steps, 0], (c, counts[c])
    assert counts["attn_decode"] == [0, cfg.n_layers * steps, 0, 0]
    model.close()
    key = "logits" if cfg.vocab else "hidden"
    for b in picks:
        print("decode at batch 64: oracle follows sequence %d" % b, flush=True)
        st = O.PTState(cfg, 1, cfg.max_seq)
        if cfg.vocab:
            O.pt_prefill(cfg, W, st, tokens=tokens[b:b + 1])
        else:
            O.pt_prefill(cfg, W, st, hidden_in=x[b:b + 1].astype(np.float64))
        for i in range(steps):
            if cfg.vocab:
                r = O.pt_decode_step(cfg, W, st, tokens=feed[i, b:b + 1])
            else:
                r = O.pt_decode_step(cfg, W, st, hidden_in=feed[i, b:b + 1].astype(np.float64))
            assert_close(got[i][b], r[key][0], BF16_TOL, "sequence %d step %d" % (b, i))


def test_share_config_widths_decode_at_batch_64():
    """One GPU's share of the wide model (d = 8192, 64 heads x 128, FFN 28672), one layer, 32-token prompts,
    decode at batch 64: the decode GEMMs at K = 8192 and 28672 with 64 rows."""
    cfg = dataclasses.replace(I.config_share(max_batch=64, max_seq=64), n_layers=1, block_depth=1)
    _decode_at_batch_64(cfg, 4, 32, (0, 31, 32, 63))


def test_large_config_widths_two_kv_heads_decode_at_batch_64():
    """Large PT layer shape with 2 KV heads per track (the decode benchmark's deviation from MHA), all 8 tracks,
    one layer and one merge, 32-token prompts, decode at batch 64."""
    cfg = dataclasses.replace(I.config_large(max_batch=64, max_seq=64, n_kv_heads=2), n_layers=1, block_depth=1)
    _decode_at_batch_64(cfg, 3, 32, (0, 33, 63))


def test_long_context_decode_with_32_splits():
    """Batch 1, a 16320-token prompt: the first decode step sees 16321 keys, which the split-K decode attention
    cuts into the maximum of 32 ranges; prefill walks 255 key tiles per late query block."""
    from paper_2602_07306_amd import binding as PB
    S, steps = 16320, 2
    cfg = small_bf16_config(n_tracks=2, n_layers=1, block_depth=1, d_model=512, n_heads=2, n_kv_heads=1,
                            head_dim=128, d_ffn=512, max_batch=1, max_seq=16384)
    W = I.make_weights(cfg, 31)
    tokens = I.make_tokens(31, 1, S, cfg.vocab)
    feed = I.make_tokens(32, steps, 1, cfg.vocab)
    model = PB.PTModel(cfg)
    model.pt_init_weights(31)
    lg, _ = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL)
    got = [lg.cpu().numpy()]
    model.pt_profile_reset()
    for i in range(steps):
        g, _, _ = model.pt_decode_step(torch.from_numpy(np.ascontiguousarray(feed[i])).cuda())
        got.append(g.cpu().numpy())
    torch.cuda.synchronize()
    assert model.pt_profile_paths("attn_decode") == [0, steps, 0, 0]
    model.close()
    st = O.PTState(cfg, 1, cfg.max_seq)
    ref = O.pt_prefill(cfg, W, st, tokens=tokens)
    # every 97th position and the last 64: early, middle and late query blocks
    rows = np.unique(np.concatenate([np.arange(0, S, 97), np.arange(S - 64, S)]))
    assert_close(got[0][rows], ref["logits"][0][rows], BF16_TOL, "prefill logits")
    for i in range(steps):
        r = O.pt_decode_step(cfg, W, st, tokens=feed[i])
        assert_close(got[1 + i], r["logits"], BF16_TOL, "decode step %d" % i)


@pytest.mark.parametrize("over,B,S", [
    (dict(max_batch=2, max_seq=640), 2, 576),                                              # head_dim 64, 9 key tiles
    (dict(head_dim=128, n_heads=4, n_kv_heads=2, d_model=512, max_batch=1, max_seq=1100), 1, 1088),
])
def test_software_pipelined_prefill_attention_matches_the_oracle(over, B, S):
    """The alternative flash prefill kernel behind PT_TUNE_ATTN_PREFILL (8 wavefronts per workgroup, four
    direct-to-LDS stages, softmax slices between the MFMAs): slower than the default, kept selectable, and held to
    the same parity bar."""
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config(n_layers=2, block_depth=2, **over)
    PB.pt_set_tuning(PB.PT_TUNE_ATTN_PREFILL, 1)
    try:
        outs, counts = run_case(cfg, 77, B, S, 1, (PB.PT_PATH_AUTO,))
        assert counts[PB.PT_PATH_AUTO][0]["attn_prefill"] == [0, cfg.n_layers, 0, 0]
    finally:
        PB.pt_set_tuning(PB.PT_TUNE_ATTN_PREFILL, 0)
