"""Pins for the CPU oracle: every check here compares oracle/pt_oracle.py with something
other than itself - a torch CPU library composition, closed forms, invariants of
Algorithm 1, or numbers the paper prints (tests/golden/)."""
import copy
import math
import os
import types

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def cfg_of(**kw):
    base = dict(n_tracks=3, n_layers=4, block_depth=2, d_model=16, n_heads=4, n_kv_heads=2,
                head_dim=4, d_ffn=24, vocab=50, merge_scale=1.0, rms_eps=1e-5, rope_theta=10000.0)
    base.update(kw)
    return types.SimpleNamespace(**base)


def rand_weights(cfg, seed=0, std=0.3):
    """Test-local random weights (numpy Generator; not the product's generator)."""
    rng = np.random.default_rng(seed)
    T, L, d = cfg.n_tracks, cfg.n_layers, cfg.d_model
    hq, hk, f = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.d_ffn
    W = {
        "wq": rng.normal(0, std, (T, L, d, hq)), "wk": rng.normal(0, std, (T, L, d, hk)),
        "wv": rng.normal(0, std, (T, L, d, hk)), "wo": rng.normal(0, std, (T, L, hq, d)),
        "wg": rng.normal(0, std, (T, L, d, f)), "wu": rng.normal(0, std, (T, L, d, f)),
        "wd": rng.normal(0, std, (T, L, f, d)),
        "g1": 1 + 0.1 * rng.normal(size=(T, L, d)), "g2": 1 + 0.1 * rng.normal(size=(T, L, d)),
        "gf": 1 + 0.1 * rng.normal(size=(d,)),
    }
    if cfg.vocab:
        W["embed"] = rng.normal(0, 1.0, (cfg.vocab, d))
        W["head"] = rng.normal(0, std, (d, cfg.vocab))
    return W


def prefill(cfg, W, tokens=None, hidden_in=None, taps=False, max_seq=None):
    if tokens is not None:
        B, S = np.asarray(tokens).shape
    else:
        B, S = np.asarray(hidden_in).shape[-3:-1]
    st = O.PTState(cfg, B, max_seq or S + 8)
    return O.pt_prefill(cfg, W, st, tokens=tokens, hidden_in=hidden_in, collect_taps=taps), st


# ---------------------------------------------------------------- P1: T=1, D=1 vs torch library ops
def torch_decoder(cfg, W, tokens):
    """A standard decoder-only transformer from torch CPU library routines, float64.
    RoPE is written a second way: pairs (u_j, u_{j+hd/2}) as complex numbers times e^{i p w_j}."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    H, Hkv, hd, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_model
    tok = torch.from_numpy(np.asarray(tokens)).long()
    B, S = tok.shape
    h = F.embedding(tok, t(W["embed"]))
    inv = 1.0 / (cfg.rope_theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    rot = torch.polar(torch.ones(S, hd // 2, dtype=torch.float64),
                      torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :])

    def rope(u):  # u [B, S, nh, hd]
        z = torch.complex(u[..., : hd // 2], u[..., hd // 2:]) * rot[None, :, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(cfg.n_layers):
        a = F.rms_norm(h, (d,), t(W["g1"][0, l]), cfg.rms_eps)
        q = rope(torch.matmul(a, t(W["wq"][0, l])).view(B, S, H, hd))
        k = rope(torch.matmul(a, t(W["wk"][0, l])).view(B, S, Hkv, hd))
        v = torch.matmul(a, t(W["wv"][0, l])).view(B, S, Hkv, hd)
        k = k.repeat_interleave(H // Hkv, dim=2)
        v = v.repeat_interleave(H // Hkv, dim=2)
        o = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                           is_causal=True)
        h = h + torch.matmul(o.transpose(1, 2).reshape(B, S, H * hd), t(W["wo"][0, l]))
        a = F.rms_norm(h, (d,), t(W["g2"][0, l]), cfg.rms_eps)
        m = F.silu(torch.matmul(a, t(W["wg"][0, l]))) * torch.matmul(a, t(W["wu"][0, l]))
        h = h + torch.matmul(m, t(W["wd"][0, l]))
    logits = torch.matmul(F.rms_norm(h, (d,), t(W["gf"]), cfg.rms_eps), t(W["head"]))
    return h.numpy(), logits.numpy()


@pytest.mark.parametrize("hkv", [1, 2, 4])
def test_single_track_every_layer_merge_is_a_standard_transformer(hkv):
    cfg = cfg_of(n_tracks=1, block_depth=1, n_layers=3, n_kv_heads=hkv)
    W = rand_weights(cfg, seed=hkv)
    tokens = np.random.default_rng(5).integers(0, cfg.vocab, (2, 9))
    out, _ = prefill(cfg, W, tokens)
    h_ref, logits_ref = torch_decoder(cfg, W, tokens)
    np.testing.assert_allclose(out["hidden"], h_ref, rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(out["logits"], logits_ref, rtol=1e-10, atol=1e-10)


# ---------------------------------------------------------------- P2/P3: isolation and fan-out
def test_track_isolation_until_next_merge():
    cfg = cfg_of(vocab=0)
    W = rand_weights(cfg)
    rng = np.random.default_rng(1)
    x = rng.normal(size=(cfg.n_tracks, 1, 6, cfg.d_model))
    x2 = x.copy()
    x2[1] += 0.5                                    # perturb track 1's input only
    a, _ = prefill(cfg, W, hidden_in=x, taps=True)
    b, _ = prefill(cfg, W, hidden_in=x2, taps=True)
    ta, tb = a["track_taps"][0], b["track_taps"][0]
    # before the first merge: other tracks bit-identical, track 1 differs
    assert np.array_equal(ta[0][0], tb[0][0]) and np.array_equal(ta[0][2], tb[0][2])
    assert not np.array_equal(ta[0][1], tb[0][1])
    # after the first merge every track has seen the perturbation
    for i in range(cfg.n_tracks):
        assert not np.array_equal(ta[1][i], tb[1][i])
    assert not np.array_equal(a["taps"][0][0], b["taps"][0][0])


def test_every_track_receives_the_same_input_after_a_merge():
    # If all tracks hold identical weights, identical post-merge inputs give identical
    # per-track activations before the next merge - even though the first block's inputs differ.
    cfg = cfg_of(vocab=0)
    W = rand_weights(cfg)
    for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2"):
        W[k][:] = W[k][0:1]
    x = np.random.default_rng(2).normal(size=(cfg.n_tracks, 1, 5, cfg.d_model))
    out, _ = prefill(cfg, W, hidden_in=x, taps=True)
    first, second = out["track_taps"][0]
    assert not np.array_equal(first[0], first[1])
    assert np.array_equal(second[0], second[1]) and np.array_equal(second[0], second[2])


# ---------------------------------------------------------------- P4: merge closed form and count
@pytest.mark.parametrize("T,scale", [(2, 1.0), (4, 1.0), (8, 1.0), (4, 0.25), (2, 0.5)])
def test_merge_closed_form_with_zero_output_projections(T, scale):
    cfg = cfg_of(n_tracks=T, n_layers=6, block_depth=2, merge_scale=scale, vocab=0)
    W = rand_weights(cfg)
    W["wo"][:] = 0.0
    W["wd"][:] = 0.0
    x = np.random.default_rng(3).normal(size=(1, 4, cfg.d_model))
    out, st = prefill(cfg, W, hidden_in=x)
    np.testing.assert_allclose(out["hidden"], (scale * T) ** 3 * x, rtol=1e-14, atol=0)
    if T == 2:                                                       # x + x is exact
        assert np.array_equal(out["hidden"], (scale * T) ** 3 * x)
    assert st.merge_count == 3 == O.sync_points_track_parallel(6, 2)


def test_merge_is_a_sum_in_track_order():
    hs = [np.full((2, 3), 1e16), np.full((2, 3), 1.0), np.full((2, 3), -1e16)]
    # (1e16 + 1) - 1e16 in float64 = 0 (track order), not 1
    assert np.array_equal(O.track_merge(hs, 1.0), np.zeros((2, 3)))
    assert np.array_equal(O.track_merge([np.ones(4), 2 * np.ones(4), 3 * np.ones(4)], 0.5),
                          3.0 * np.ones(4))


def test_sync_point_counts_match_the_paper():
    for line in open(os.path.join(GOLDEN, "sync_points.txt")):
        if line.startswith("#") or not line.strip():
            continue
        D, pct, factor = line.split()
        D, pct, factor = int(D), float(pct), float(factor)
        for L in (32, 40, 48):
            tp = O.sync_points_tensor_parallel(L)
            pt = O.sync_points_track_parallel(L, D)
            assert 100.0 * (1 - pt / tp) == pct
            assert tp / pt == factor


def test_table1_heads_split_evenly_over_tracks():
    for line in open(os.path.join(GOLDEN, "table1_heads.txt")):
        if line.startswith("#") or not line.strip():
            continue
        _, layers, heads, hpt, kv, kvpt = line.split()
        assert int(heads) == 8 * int(hpt) and int(kv) == 8 * int(kvpt)
        # such a track is a valid oracle configuration (grouped-query attention)
        cfg = cfg_of(n_tracks=2, n_layers=2, block_depth=2, n_heads=int(hpt), n_kv_heads=int(kvpt),
                     d_model=8, head_dim=4, d_ffn=8, vocab=0)
        out, _ = prefill(cfg, rand_weights(cfg), hidden_in=np.ones((1, 3, 8)))
        assert np.all(np.isfinite(out["hidden"]))


# ---------------------------------------------------------------- P5/P6: linearity and symmetry
def test_replicated_tracks_with_mean_merge_equal_the_single_track_model():
    cfg1 = cfg_of(n_tracks=1)
    W1 = rand_weights(cfg1)
    cfg4 = cfg_of(n_tracks=4, merge_scale=0.25)
    W4 = {k: (np.repeat(v, 4, axis=0) if v.ndim >= 3 else v) for k, v in W1.items()}
    tokens = np.random.default_rng(4).integers(0, cfg1.vocab, (1, 7))
    a, _ = prefill(cfg1, W1, tokens)
    b, _ = prefill(cfg4, W4, tokens)
    np.testing.assert_allclose(b["logits"], a["logits"], rtol=1e-12, atol=1e-12)


def test_track_permutation_leaves_the_output_unchanged():
    cfg = cfg_of()
    W = rand_weights(cfg)
    perm = [2, 0, 1]
    Wp = {k: (v[perm] if v.ndim >= 3 else v) for k, v in W.items()}
    tokens = np.random.default_rng(6).integers(0, cfg.vocab, (1, 6))
    a, _ = prefill(cfg, W, tokens)
    b, _ = prefill(cfg, Wp, tokens)
    np.testing.assert_allclose(b["logits"], a["logits"], rtol=1e-11, atol=1e-11)


# ---------------------------------------------------------------- P7/P8/P9: causality, cache, batch
def test_causal_prefix_is_invariant_to_appended_tokens():
    cfg = cfg_of()
    W = rand_weights(cfg)
    tokens = np.random.default_rng(7).integers(0, cfg.vocab, (1, 12))
    full, _ = prefill(cfg, W, tokens)
    part, _ = prefill(cfg, W, tokens[:, :7])
    np.testing.assert_allclose(full["logits"][:, :7], part["logits"], rtol=1e-12, atol=1e-13)
    other = tokens.copy()
    other[0, 7:] = (other[0, 7:] + 1) % cfg.vocab
    alt, _ = prefill(cfg, W, other)
    np.testing.assert_allclose(alt["logits"][:, :7], full["logits"][:, :7], rtol=1e-12, atol=1e-13)
    assert not np.allclose(alt["logits"][:, 7:], full["logits"][:, 7:])


def test_cached_decode_equals_full_recompute():
    cfg = cfg_of()
    W = rand_weights(cfg)
    tokens = np.random.default_rng(8).integers(0, cfg.vocab, (2, 10))
    full, _ = prefill(cfg, W, tokens)
    out, st = prefill(cfg, W, tokens[:, :6], max_seq=16)
    for p in range(6, 10):
        step = O.pt_decode_step(cfg, W, st, tokens=tokens[:, p])
        np.testing.assert_allclose(step["logits"], full["logits"][:, p], rtol=1e-10, atol=1e-11)
        assert np.array_equal(step["argmax"], np.argmax(full["logits"][:, p], axis=-1))
    assert list(st.length) == [10, 10]
    assert st.merge_count == 5 * (cfg.n_layers // cfg.block_depth)


@pytest.mark.parametrize("per_track", [False, True])
def test_cached_decode_from_hidden_states_equals_full_recompute(per_track):
    """The hidden-state entry of the decode step ([B, d]: the same input for every track, and
    [T, B, d]: one input per track) against a prefill of the sequence extended by those rows."""
    cfg = cfg_of(vocab=0)
    W = rand_weights(cfg)
    rng = np.random.default_rng(18)
    T, B, S, d = cfg.n_tracks, 2, 9, cfg.d_model
    x = rng.normal(size=(T, B, S, d)) if per_track else rng.normal(size=(B, S, d))
    full, _ = prefill(cfg, W, hidden_in=x)
    _, st = prefill(cfg, W, hidden_in=x[..., :5, :], max_seq=16)
    for p in range(5, S):
        step = O.pt_decode_step(cfg, W, st, hidden_in=x[..., p, :])
        np.testing.assert_allclose(step["hidden"], full["hidden"][:, p], rtol=1e-10, atol=1e-11)
        assert "logits" not in step
    assert list(st.length) == [S, S]
    # the two forms agree when every track is handed the same rows
    if not per_track:
        _, st1 = prefill(cfg, W, hidden_in=x[:, :5], max_seq=16)
        _, st2 = prefill(cfg, W, hidden_in=np.broadcast_to(x[:, :5], (T,) + x[:, :5].shape), max_seq=16)
        a = O.pt_decode_step(cfg, W, st1, hidden_in=x[:, 5])
        b = O.pt_decode_step(cfg, W, st2, hidden_in=np.broadcast_to(x[:, 5], (T, B, d)))
        assert np.array_equal(a["hidden"], b["hidden"])
    else:
        # a per-track input must reach its own track: swapping two tracks' rows changes the result
        _, st3 = prefill(cfg, W, hidden_in=x[..., :5, :], max_seq=16)
        swapped = x[[1, 0, 2], :, 5, :]
        c = O.pt_decode_step(cfg, W, st3, hidden_in=swapped)
        assert not np.allclose(c["hidden"], full["hidden"][:, 5])


def test_ragged_batch_equals_each_sequence_alone():
    """A batch of mixed lengths (the paper's throughput mode batches such inputs): every sequence of the ragged
    batch equals the same sequence run alone, in prefill and in the cached decode steps that follow, each at its
    own position; rows beyond a sequence's length do not exist."""
    cfg = cfg_of()
    W = rand_weights(cfg)
    rng = np.random.default_rng(21)
    lens = [7, 3, 10, 1]
    tokens = rng.integers(0, cfg.vocab, (4, 10))
    nxt = rng.integers(0, cfg.vocab, (2, 4))
    st = O.PTState(cfg, 4, 16)
    rag = O.pt_prefill(cfg, W, st, tokens=tokens, lengths=np.array(lens), collect_taps=True)
    assert list(st.length) == lens
    steps = [O.pt_decode_step(cfg, W, st, tokens=nxt[i]) for i in range(2)]
    assert list(st.length) == [n + 2 for n in lens]
    for b, n in enumerate(lens):
        one, st1 = prefill(cfg, W, tokens[b:b + 1, :n], taps=True, max_seq=16)
        # the head is one library product over the whole batch: equal up to its blocking, not bit for bit
        np.testing.assert_allclose(rag["logits"][b, :n], one["logits"][0], rtol=1e-12, atol=1e-13)
        assert np.array_equal(rag["hidden"][b, :n], one["hidden"][0])
        assert np.all(np.isnan(rag["logits"][b, n:]))
        for k in range(cfg.n_layers // cfg.block_depth):
            assert rag["taps"][b][k].shape == (n, cfg.d_model)
            assert np.array_equal(rag["taps"][b][k], one["taps"][0][k])
        for i in range(2):
            s1 = O.pt_decode_step(cfg, W, st1, tokens=nxt[i, b:b + 1])
            assert np.array_equal(steps[i]["hidden"][b], s1["hidden"][0])
            np.testing.assert_allclose(steps[i]["logits"][b], s1["logits"][0], rtol=1e-12, atol=1e-13)
        # and the decode steps continue the sequence: they equal a prefill of the extended sequence
        ext = np.concatenate([tokens[b, :n], nxt[:, b]])[None]
        full, _ = prefill(cfg, W, ext)
        np.testing.assert_allclose(steps[1]["logits"][b], full["logits"][0, n + 1], rtol=1e-10, atol=1e-11)


def test_batch_independence():
    cfg = cfg_of()
    W = rand_weights(cfg)
    tokens = np.random.default_rng(9).integers(0, cfg.vocab, (3, 5))
    both, _ = prefill(cfg, W, tokens)
    for b in range(3):
        one, _ = prefill(cfg, W, tokens[b:b + 1])
        assert np.array_equal(one["logits"][0], both["logits"][b])


# ---------------------------------------------------------------- P10: textbook special cases
def test_rmsnorm_special_cases():
    a = O.rmsnorm(np.array([[3.0, 4.0]]), np.ones(2), 0.0)
    np.testing.assert_allclose(a, np.array([[3.0, 4.0]]) / math.sqrt(12.5), rtol=1e-15)
    x = np.random.default_rng(0).normal(size=(5, 32))
    np.testing.assert_allclose(np.sqrt(np.mean(O.rmsnorm(x, np.ones(32), 0.0) ** 2, -1)), 1.0,
                               rtol=1e-14)
    g = np.arange(1, 33, dtype=float)
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), O.rmsnorm(x, np.ones(32), 1e-5) * g, rtol=1e-15)
    # eps sits inside the square root, added to the mean square
    np.testing.assert_allclose(O.rmsnorm(np.zeros((1, 4)) + 2.0, np.ones(4), 5.0), 2.0 / 3.0)


def test_rope_special_cases():
    u = np.random.default_rng(1).normal(size=(4, 2, 8))
    # position 0 is the identity
    np.testing.assert_array_equal(O.rope(u[:1], np.array([0]), 10000.0), u[:1])
    # a rotation preserves each pair's norm and relative angles depend on p - r only
    r = O.rope(u, np.arange(4), 10000.0)
    np.testing.assert_allclose(r[..., :4] ** 2 + r[..., 4:] ** 2, u[..., :4] ** 2 + u[..., 4:] ** 2,
                               rtol=1e-13)
    q = np.random.default_rng(2).normal(size=(1, 1, 8))
    k = np.random.default_rng(3).normal(size=(1, 1, 8))
    d1 = np.sum(O.rope(q, [5], 100.0) * O.rope(k, [2], 100.0))
    d2 = np.sum(O.rope(q, [9], 100.0) * O.rope(k, [6], 100.0))
    np.testing.assert_allclose(d1, d2, rtol=1e-12)
    # pair j=0 turns by exactly p radians (frequency theta^0 = 1): quarter turn at p = pi/2,
    # and the direction is counter-clockwise: (1, 0) -> (cos p, sin p)
    e = np.zeros((1, 1, 8))
    e[0, 0, 0] = 1.0
    t = O.rope(e, [math.pi / 2], 10000.0)
    np.testing.assert_allclose(t[0, 0, 0], 0.0, atol=1e-15)
    np.testing.assert_allclose(t[0, 0, 4], 1.0, rtol=1e-15)
    # pair j turns by p * theta^(-2j/hd)
    e = np.zeros((1, 1, 8))
    e[0, 0, 2] = 1.0
    t = O.rope(e, [3.0], 16.0)               # 16^(-2*2/8) = 1/4
    np.testing.assert_allclose([t[0, 0, 2], t[0, 0, 6]], [math.cos(0.75), math.sin(0.75)], rtol=1e-14)


def test_attention_special_cases():
    rng = np.random.default_rng(4)
    v = rng.normal(size=(6, 2, 4))
    k = rng.normal(size=(6, 2, 4))
    # zero queries: uniform weights over the visible prefix -> running mean of v
    o = O.causal_attention(np.zeros((6, 4, 4)), k, v, np.arange(6))
    for p in range(6):
        for c in range(4):
            np.testing.assert_allclose(o[p, c], v[: p + 1, c // 2].mean(0), rtol=1e-13)
    # a single visible key returns its value exactly
    o = O.causal_attention(rng.normal(size=(1, 4, 4)), k[:1], v[:1], np.array([0]))
    for c in range(4):
        np.testing.assert_array_equal(o[0, c], v[0, c // 2])
    # softmax rows sum to one; scale is 1/sqrt(hd): two keys, scores (hd, 0)/sqrt(hd)
    hd = 4
    q = np.ones((1, 1, hd))
    kk = np.stack([np.ones((1, hd)), np.zeros((1, hd))])
    vv = np.stack([np.ones((1, hd)), np.zeros((1, hd))])
    o = O.causal_attention(q, kk, vv, np.array([1]))
    w0 = math.exp(hd / math.sqrt(hd)) / (math.exp(hd / math.sqrt(hd)) + 1.0)
    np.testing.assert_allclose(o[0, 0], w0, rtol=1e-14)
    # decode-style call: one query at position 3 sees keys 0..3 only
    q1 = rng.normal(size=(1, 4, 4))
    o_a = O.causal_attention(q1, k[:4], v[:4], np.array([3]))
    k2, v2 = k.copy(), v.copy()
    k2[4:] += 10.0
    o_b = O.causal_attention(q1, k2, v2, np.array([3]))
    np.testing.assert_allclose(o_a, o_b, rtol=1e-14)


def test_silu_and_ffn_closed_form():
    np.testing.assert_allclose(O.silu(np.array([0.0, 1.0, -1.0])),
                               [0.0, 1 / (1 + math.exp(-1)), -1 / (1 + math.exp(1))], rtol=1e-15)
    # one layer, attention switched off (wo = 0), identity-like FFN weights: closed form
    cfg = cfg_of(n_tracks=1, n_layers=1, block_depth=1, d_model=4, n_heads=1, n_kv_heads=1,
                 head_dim=4, d_ffn=4, vocab=0, rms_eps=0.0)
    W = rand_weights(cfg)
    W["wo"][:] = 0
    W["g1"][:] = 1
    W["g2"][:] = 1
    W["wg"][0, 0] = np.eye(4)
    W["wu"][0, 0] = 2 * np.eye(4)
    W["wd"][0, 0] = 3 * np.eye(4)
    x = np.array([[[1.0, -2.0, 0.5, 3.0]]])
    out, _ = prefill(cfg, W, hidden_in=x)
    a = x / math.sqrt(np.mean(x ** 2))
    expect = x + 3 * (a / (1 + np.exp(-a))) * (2 * a)
    np.testing.assert_allclose(out["hidden"], expect, rtol=1e-14)


def test_hand_computed_two_track_example():
    """tests/golden/tiny_two_track.txt: a two-track, one-layer, one-merge model small enough
    to evaluate by hand (values derived in the fixture's header)."""
    vals = [float(x) for line in open(os.path.join(GOLDEN, "tiny_two_track.txt"))
            if not line.startswith("#") for x in line.split()]
    cfg = cfg_of(n_tracks=2, n_layers=1, block_depth=1, d_model=2, n_heads=1, n_kv_heads=1,
                 head_dim=2, d_ffn=2, vocab=0, rms_eps=0.0)
    z = lambda *s: np.zeros(s)
    W = {"wq": z(2, 1, 2, 2), "wk": z(2, 1, 2, 2), "wv": z(2, 1, 2, 2), "wo": z(2, 1, 2, 2),
         "wg": z(2, 1, 2, 2), "wu": z(2, 1, 2, 2), "wd": z(2, 1, 2, 2),
         "g1": np.ones((2, 1, 2)), "g2": np.ones((2, 1, 2)), "gf": np.ones(2)}
    # track 0: attention only (v = a, wo = I); track 1: FFN only (gate = up = a, wd = I)
    W["wv"][0, 0] = np.eye(2)
    W["wo"][0, 0] = np.eye(2)
    W["wg"][1, 0] = np.eye(2)
    W["wu"][1, 0] = np.eye(2)
    W["wd"][1, 0] = np.eye(2)
    x = np.array([[[1.0, 1.0], [1.0, -1.0]]])
    out, _ = prefill(cfg, W, hidden_in=x)
    np.testing.assert_allclose(out["hidden"].reshape(-1), vals, rtol=1e-12)
