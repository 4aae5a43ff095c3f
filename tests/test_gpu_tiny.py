"""GPU parity, fp32: the Tiny PT configuration (T=2, L=4, D=2, d=128, 4 heads x 32, FFN 512,
vocab 512; batch 1, prefill 32, 8 KV-cached greedy decode steps) against the CPU oracle, plus
the invariants of Algorithm 1 on the HIP path."""
import dataclasses

import numpy as np
import pytest

from oracle import pt_oracle as O
from paper_2602_07306_amd import inputs as I
from tests.helpers import FP32_TOL, argmax_agrees, oracle_prefill, rel_err

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tiny():
    from paper_2602_07306_amd import binding as PB
    cfg = I.config_tiny()
    W = I.make_weights(cfg, 0)
    model = PB.PTModel(cfg)
    model.pt_init_weights(0)
    torch.cuda.synchronize()
    return PB, cfg, W, model


def test_device_weight_generator_matches_the_host_generator(tiny):
    PB, cfg, W, model = tiny
    for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2"):
        for i in range(cfg.n_tracks):
            for l in range(cfg.n_layers):
                got = model.pt_get_weight(name, i, l, W[name][i, l].shape)
                assert np.array_equal(got, W[name][i, l]), (name, i, l)
    assert np.array_equal(model.pt_get_weight("embed", 0, 0, W["embed"].shape), W["embed"])
    assert np.array_equal(model.pt_get_weight("head", 0, 0, W["head"].shape), W["head"])
    assert np.array_equal(model.pt_get_weight("gf", 0, 0, W["gf"].shape), W["gf"])


def test_device_weight_generator_bf16_rounding():
    from paper_2602_07306_amd import binding as PB
    cfg = dataclasses.replace(I.config_tiny(), dtype=I.PT_BF16, n_layers=2, d_ffn=96)
    W = I.make_weights(cfg, 11)
    model = PB.PTModel(cfg)
    model.pt_init_weights(11)
    for name in ("wq", "wg", "wu", "wd", "wo"):
        got = model.pt_get_weight(name, 1, 1, W[name][1, 1].shape)
        assert np.array_equal(got, W[name][1, 1]), name
    assert np.array_equal(model.pt_get_weight("head", 0, 0, W["head"].shape), W["head"])
    model.close()


def test_set_weight_roundtrip(tiny):
    PB, cfg, W, model = tiny
    x = np.random.default_rng(0).normal(size=W["wg"][0, 0].shape).astype(np.float32)
    model.pt_set_weight("wg", 1, 2, x)
    assert np.array_equal(model.pt_get_weight("wg", 1, 2, x.shape), x)
    assert np.array_equal(model.pt_get_weight("wu", 1, 2, x.shape), W["wu"][1, 2])   # neighbour intact
    model.pt_set_weight("wg", 1, 2, W["wg"][1, 2])


def test_tiny_prefill_and_greedy_decode_match_the_oracle(tiny):
    PB, cfg, W, model = tiny
    tokens = I.make_tokens(0, 1, 32, cfg.vocab)
    ref, st = oracle_prefill(cfg, W, tokens)
    model.pt_reset()
    taps, ttaps = model.pt_set_taps(32, track_taps=True)
    m0 = model.pt_merge_count()
    logits, hidden = model.pt_prefill(torch.from_numpy(tokens).cuda(), logits_mode=PB.PT_LOGITS_ALL,
                                      want_hidden=True)
    torch.cuda.synchronize()
    assert model.pt_merge_count() - m0 == cfg.n_layers // cfg.block_depth == 2
    assert model.pt_seq_len() == 32
    assert rel_err(logits.cpu().numpy(), ref["logits"][0]) <= FP32_TOL
    assert rel_err(hidden.cpu().numpy()[0], ref["hidden"][0]) <= FP32_TOL
    for k in range(2):
        assert rel_err(taps[k].cpu().numpy(), ref["taps"][0][k]) <= FP32_TOL
        for i in range(cfg.n_tracks):
            assert rel_err(ttaps[k, i].cpu().numpy(), ref["track_taps"][0][k][i]) <= FP32_TOL
    assert argmax_agrees(logits.cpu().numpy(), ref["logits"][0], FP32_TOL)
    model.pt_clear_taps()
    # 8 greedy steps, teacher-forced with the oracle's ids
    nxt = np.argmax(ref["logits"][:, -1], axis=-1).astype(np.int32)
    for step in range(8):
        r = O.pt_decode_step(cfg, W, st, tokens=nxt)
        lg, _, am = model.pt_decode_step(torch.from_numpy(nxt).cuda(), want_argmax=True)
        torch.cuda.synchronize()
        assert rel_err(lg.cpu().numpy(), r["logits"]) <= FP32_TOL, step
        assert argmax_agrees(lg.cpu().numpy(), r["logits"], FP32_TOL)
        assert np.array_equal(am.cpu().numpy(), np.argmax(lg.cpu().numpy(), -1))
        nxt = r["argmax"]
    assert model.pt_seq_len() == 40 == st.length[0]


def test_last_row_logits_equal_all_row_logits(tiny):
    PB, cfg, W, model = tiny
    tokens = torch.from_numpy(I.make_tokens(5, 1, 17, cfg.vocab)).cuda()
    model.pt_reset()
    all_l, _ = model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_ALL)
    last_l, _ = model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST)
    torch.cuda.synchronize()
    assert torch.equal(all_l[-1:], last_l)


def test_track_isolation_and_fanout_on_the_gpu(tiny):
    PB, cfg, W, model = tiny
    rng = np.random.default_rng(3)
    x = rng.normal(size=(cfg.n_tracks, 1, 9, cfg.d_model)).astype(np.float32)
    x2 = x.copy()
    x2[1] += 0.25
    outs = []
    for inp in (x, x2):
        model.pt_reset()
        taps, ttaps = model.pt_set_taps(9, track_taps=True)
        model.pt_prefill(hidden_in=torch.from_numpy(inp).cuda(), logits_mode=PB.PT_LOGITS_NONE)
        torch.cuda.synchronize()
        outs.append((taps.cpu().numpy().copy(), ttaps.cpu().numpy().copy()))
        model.pt_clear_taps()
    (ta, tta), (tb, ttb) = outs
    assert np.array_equal(tta[0, 0], ttb[0, 0])          # untouched track: bit-identical
    assert not np.array_equal(tta[0, 1], ttb[0, 1])
    assert not np.array_equal(tta[1, 0], ttb[1, 0])      # after the merge every track differs
    ref, _ = oracle_prefill(cfg, W, hidden_in=x.astype(np.float64))
    assert rel_err(ta[1], ref["taps"][0][1]) <= FP32_TOL


def test_merge_closed_form_on_the_gpu():
    from paper_2602_07306_amd import binding as PB
    cfg = dataclasses.replace(I.config_tiny(), n_tracks=4, n_layers=6, block_depth=2, vocab=0)
    model = PB.PTModel(cfg)
    model.pt_init_weights(2)
    zeros_o = np.zeros((cfg.n_heads * cfg.head_dim, cfg.d_model), np.float32)
    zeros_d = np.zeros((cfg.d_ffn, cfg.d_model), np.float32)
    for i in range(cfg.n_tracks):
        for l in range(cfg.n_layers):
            model.pt_set_weight("wo", i, l, zeros_o)
            model.pt_set_weight("wd", i, l, zeros_d)
    x = np.random.default_rng(4).normal(size=(1, 5, cfg.d_model)).astype(np.float32)
    _, hidden = model.pt_prefill(hidden_in=torch.from_numpy(x).cuda(), logits_mode=PB.PT_LOGITS_NONE,
                                 want_hidden=True)
    torch.cuda.synchronize()
    assert np.array_equal(hidden.cpu().numpy(), (4.0 ** 3) * x)      # (scale*T)^(L/D) x, exact
    assert model.pt_merge_count() == 3
    model.close()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n,tokens,d", [(2, 7, 128), (8, 33, 256), (1, 3, 8), (16, 5, 64)])
def test_track_merge_matches_the_oracle(dtype, n, tokens, d):
    from paper_2602_07306_amd import binding as PB
    rng = np.random.default_rng(n * 1000 + tokens)
    hs = [rng.normal(size=(tokens, d)).astype(np.float32) for _ in range(n)]
    if dtype == "bf16":
        hs = [I.round_to_dtype(h, I.PT_BF16) for h in hs]
        dev = [torch.from_numpy(h).cuda().to(torch.bfloat16) for h in hs]
    else:
        dev = [torch.from_numpy(h).cuda() for h in hs]
    out = PB.pt_track_merge(dev, 0.5)
    torch.cuda.synchronize()
    ref = O.track_merge(hs, 0.5)
    if dtype == "bf16":
        # fp32 accumulation in track order, one final rounding to bf16
        acc = hs[0].astype(np.float32).copy()
        for h in hs[1:]:
            acc = acc + h
        exact = I.round_to_dtype(acc * np.float32(0.5), I.PT_BF16)
        assert np.array_equal(out.float().cpu().numpy(), exact)
        assert rel_err(out.float().cpu().numpy(), ref) <= 2.0 ** -8
    else:
        assert rel_err(out.cpu().numpy(), ref) <= 1e-6
    # in place on the first track
    PB.pt_track_merge(dev, 0.5, out=dev[0])
    torch.cuda.synchronize()
    assert torch.equal(dev[0], out)


def test_out_of_range_token_ids_are_reported_at_the_next_status_check(tiny):
    """Forward calls are asynchronous and cannot return an error for data that lives on the device: a token id
    outside the vocabulary raises a device flag that pt_sync_status turns into PT_ERR_INVALID_ARGUMENT, once."""
    PB, cfg, W, model = tiny
    model.pt_reset()
    good = I.make_tokens(0, 1, 16, cfg.vocab)
    model.pt_prefill(torch.from_numpy(good).cuda())
    model.pt_sync_status()
    for bad_id in (cfg.vocab, -1, 2 ** 31 - 1):
        bad = good.copy()
        bad[0, 5] = bad_id
        model.pt_prefill(torch.from_numpy(bad).cuda())
        with pytest.raises(PB.PTError) as e:
            model.pt_sync_status()
        assert e.value.code == PB.PT_ERR_INVALID_ARGUMENT
        model.pt_sync_status()          # the flag was cleared
    model.pt_prefill(torch.from_numpy(good).cuda())
    model.pt_decode_step(torch.from_numpy(np.array([cfg.vocab + 3], np.int32)).cuda())
    with pytest.raises(PB.PTError):
        model.pt_sync_status()
