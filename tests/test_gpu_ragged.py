"""GPU parity of ragged batches (sequences of different lengths in one prefill, each continuing at its own
position in decode: the throughput mode of Section 3.3) against the CPU oracle."""
import dataclasses

import numpy as np
import pytest

from oracle import pt_oracle as O
from paper_2602_07306_amd import inputs as I
from tests.helpers import (BF16_TOL, FP32_TOL, argmax_agrees, assert_close, path_counts, small_bf16_config)

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def packed(arr, lens):
    """Rows [b, :lens[b]] of a padded [B, S, ...] array, sequence after sequence."""
    return np.concatenate([arr[b, :n] for b, n in enumerate(lens)], axis=0)


def ragged_case(cfg, seed, lens, steps, tol, path=None, hidden_tracks=0):
    """Ragged prefill (all logits, hidden, taps) and teacher-forced decode steps against the oracle."""
    from paper_2602_07306_amd import binding as PB
    B, S = len(lens), max(lens)
    W = I.make_weights(cfg, seed)
    st = O.PTState(cfg, B, cfg.max_seq)
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    if path is not None:
        model.pt_set_kernel_path(path)
    n = int(sum(lens))
    taps, _ = model.pt_set_taps(n)
    if hidden_tracks == 0:
        tokens = I.make_tokens(seed, B, S, cfg.vocab)
        ref = O.pt_prefill(cfg, W, st, tokens=tokens, lengths=np.array(lens), collect_taps=True)
        lg, hid = model.pt_prefill_ragged(lens, tokens=torch.from_numpy(packed(tokens, lens)).cuda(),
                                          logits_mode=PB.PT_LOGITS_ALL, want_hidden=True)
    else:
        T = cfg.n_tracks
        x = np.stack([np.stack([I.make_hidden(seed, 10 * i + b, S, cfg.d_model) for b in range(B)]) for i in range(hidden_tracks)])
        xin = x if hidden_tracks == T else x[0]                      # [T, B, S, d] or [B, S, d]
        ref = O.pt_prefill(cfg, W, st, hidden_in=xin.astype(np.float64), lengths=np.array(lens), collect_taps=True)
        pk = np.stack([packed(x[i], lens) for i in range(hidden_tracks)])
        lg, hid = model.pt_prefill_ragged(lens, hidden_in=torch.from_numpy(pk if hidden_tracks == T else pk[0]).cuda(),
                                          logits_mode=PB.PT_LOGITS_ALL if cfg.vocab else PB.PT_LOGITS_NONE, want_hidden=True)
    torch.cuda.synchronize()
    model.pt_sync_status()
    assert model.pt_seq_lens()[:B] == list(lens) and model.pt_seq_len() == S
    assert_close(hid.cpu().numpy(), packed(ref["hidden"], lens), tol, "hidden")
    if cfg.vocab:
        L = lg.cpu().numpy()
        assert_close(L, packed(ref["logits"], lens), tol, "logits")
        off = 0
        for b, nb in enumerate(lens):
            assert argmax_agrees(L[off:off + nb], ref["logits"][b, :nb], tol)
            off += nb
    for k in range(cfg.n_merges):
        want = np.concatenate([ref["taps"][b][k] for b in range(B)], axis=0)
        assert_close(taps[k].cpu().numpy(), want, tol, "tap %d" % k)
    model.pt_clear_taps()
    pre = path_counts(model)
    model.pt_profile_reset()
    if cfg.vocab:
        nxt = np.array([np.argmax(ref["logits"][b, nb - 1]) for b, nb in enumerate(lens)], dtype=np.int32)
        # last-token logits of every sequence, gathered by the library
        last, _ = model.pt_prefill_ragged(lens, tokens=torch.from_numpy(packed(tokens, lens)).cuda(),
                                          logits_mode=PB.PT_LOGITS_LAST) if hidden_tracks == 0 else (None, None)
        if last is not None:
            ends = np.cumsum(lens) - 1
            np.testing.assert_allclose(last.cpu().numpy(), L[ends], rtol=0, atol=2e-5 * np.max(np.abs(L[ends])))
            model.pt_profile_reset()
    for i in range(steps):
        if cfg.vocab:
            r = O.pt_decode_step(cfg, W, st, tokens=nxt)
            g, _, am = model.pt_decode_step(torch.from_numpy(nxt).cuda(), want_argmax=True)
            torch.cuda.synchronize()
            assert_close(g.cpu().numpy(), r["logits"], tol, "decode step %d" % i)
            assert argmax_agrees(g.cpu().numpy(), r["logits"], tol)
            nxt = r["argmax"]
        else:
            xn = I.make_hidden(seed + 50, i, B, cfg.d_model)
            r = O.pt_decode_step(cfg, W, st, hidden_in=xn.astype(np.float64))
            _, g, _ = model.pt_decode_step(hidden_in=torch.from_numpy(xn).cuda(), want_logits=False, want_hidden=True)
            torch.cuda.synchronize()
            assert_close(g.cpu().numpy(), r["hidden"], tol, "decode step %d" % i)
    assert model.pt_seq_lens()[:B] == [nb + steps for nb in lens] == list(st.length)
    dec = path_counts(model)
    model.close()
    return pre, dec


def test_tiny_fp32_ragged_batch():
    cfg = dataclasses.replace(I.config_tiny(), max_batch=4, max_seq=80)
    ragged_case(cfg, 0, [32, 7, 19, 1], 4, FP32_TOL)


@pytest.mark.parametrize("name,over,lens", [
    ("hd64", dict(max_batch=5, max_seq=320), [128, 70, 1, 200, 64]),
    ("hd128_gqa", dict(head_dim=128, n_heads=4, n_kv_heads=2, d_model=512, max_batch=3, max_seq=300), [257, 30, 129]),
    ("three_tracks_mean", dict(n_tracks=3, n_layers=3, block_depth=1, merge_scale=1.0 / 3, max_batch=2, max_seq=200), [100, 191]),
])
def test_bf16_ragged_batches(name, over, lens):
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config(**over)
    pre, dec = ragged_case(cfg, 17 + len(name), lens, 3, BF16_TOL)
    L = cfg.n_layers
    # padded lengths are multiples of 64: the LDS-tiled flash kernel and the matrix-core decode kernel serve them
    assert pre["attn_prefill"] == [0, L, 0, 0], pre["attn_prefill"]
    assert dec["attn_decode"] == [0, 3 * L, 0, 0], dec["attn_decode"]
    for c in ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down", "gemm_head"):
        assert pre[c][0] == 0 and dec[c][0] == 0, (c, pre[c], dec[c])
    ragged_case(cfg, 17 + len(name), lens, 2, BF16_TOL, path=PB.PT_PATH_GENERIC)


def test_bf16_ragged_hidden_state_inputs():
    """The hidden-in / hidden-out form (no vocabulary), one input for all tracks and one per track."""
    cfg = small_bf16_config(vocab=0, max_batch=3, max_seq=200)
    ragged_case(cfg, 29, [90, 1, 160], 2, BF16_TOL, hidden_tracks=1)
    ragged_case(cfg, 30, [65, 130], 2, BF16_TOL, hidden_tracks=cfg.n_tracks)


def test_throughput_mode_batch_256_mixed_lengths():
    """The shape of the paper's throughput experiments (Tables 5 and 8: maximum batch 256, inputs of mixed
    lengths) on a narrow model: 256 sequences of 1 to 512 tokens in one prefill, then decode steps at batch 256.
    The oracle follows sampled sequences (sequences are independent)."""
    from paper_2602_07306_amd import binding as PB
    B, steps = 256, 2
    cfg = small_bf16_config(n_tracks=2, n_layers=2, block_depth=1, d_model=512, n_heads=8, n_kv_heads=2, head_dim=64,
                            d_ffn=1024, max_batch=B, max_seq=520)
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(1, 513, B)]
    lens[0], lens[1], lens[255] = 512, 1, 333
    W = I.make_weights(cfg, 33)
    tokens = I.make_tokens(33, B, 512, cfg.vocab)
    feed = I.make_tokens(34, steps, B, cfg.vocab)
    model = PB.PTModel(cfg)
    model.pt_init_weights(33)
    last, _ = model.pt_prefill_ragged(lens, tokens=torch.from_numpy(packed(tokens, lens)).cuda(), logits_mode=PB.PT_LOGITS_LAST)
    got = [last.cpu().numpy()]
    for i in range(steps):
        g, _, _ = model.pt_decode_step(torch.from_numpy(np.ascontiguousarray(feed[i])).cuda())
        got.append(g.cpu().numpy())
    torch.cuda.synchronize()
    model.pt_sync_status()
    assert model.pt_seq_lens() == [n + steps for n in lens]
    model.close()
    for b in (0, 1, 100, 255, int(np.argmin(lens)), int(np.argmax(lens))):
        st = O.PTState(cfg, 1, cfg.max_seq)
        ref = O.pt_prefill(cfg, W, st, tokens=tokens[b:b + 1, :lens[b]])
        assert_close(got[0][b], ref["logits"][0, -1], BF16_TOL, "prefill, sequence %d" % b)
        for i in range(steps):
            r = O.pt_decode_step(cfg, W, st, tokens=feed[i, b:b + 1])
            assert_close(got[1 + i][b], r["logits"][0], BF16_TOL, "step %d, sequence %d" % (i, b))


def test_ragged_lengths_are_validated():
    from paper_2602_07306_amd import binding as PB
    cfg = small_bf16_config(max_batch=2, max_seq=128)
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    tok = torch.zeros(300, dtype=torch.int32, device="cuda")
    for lens, code in (([0, 5], PB.PT_ERR_INVALID_ARGUMENT), ([129, 5], PB.PT_ERR_CAPACITY), ([5, 5, 5], PB.PT_ERR_CAPACITY)):
        with pytest.raises(PB.PTError) as e:
            model.pt_prefill_ragged(lens, tokens=tok[:sum(lens)])
        assert e.value.code == code
    model.close()
