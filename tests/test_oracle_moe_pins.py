"""Pins for the PT-MoE part of the CPU oracle (routed mixture of SwiGLU experts inside every track): special
cases that reduce to the dense model, a torch CPU composition that evaluates every expert densely, closed
forms for the gates and the tie rule."""
import math
import types

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import pt_oracle as O
from tests.test_oracle_pins import cfg_of, prefill, rand_weights


def moe_weights(cfg, seed=0, std=0.3):
    """Dense test weights plus E experts per (track, layer) and a router (numpy Generator, test-local)."""
    dense = types.SimpleNamespace(**{**vars(cfg), "n_experts": 0})
    W = rand_weights(dense, seed, std)
    rng = np.random.default_rng(seed + 1000)
    T, L, d, f, E = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn, cfg.n_experts
    W["wg"] = rng.normal(0, std, (T, L, E, d, f))
    W["wu"] = rng.normal(0, std, (T, L, E, d, f))
    W["wd"] = rng.normal(0, std, (T, L, E, f, d))
    W["wr"] = rng.normal(0, 1.0, (T, L, d, E))
    return W


def test_one_expert_is_the_dense_model():
    cfg = cfg_of(n_experts=1, top_k=1)
    W = moe_weights(cfg, 3)
    dense = cfg_of()
    Wd = dict(W)
    Wd["wg"], Wd["wu"], Wd["wd"] = W["wg"][:, :, 0], W["wu"][:, :, 0], W["wd"][:, :, 0]
    tokens = np.random.default_rng(1).integers(0, cfg.vocab, (2, 7))
    a, _ = prefill(cfg, W, tokens)
    b, _ = prefill(dense, Wd, tokens)
    np.testing.assert_allclose(a["hidden"], b["hidden"], rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(a["logits"], b["logits"], rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("k", [1, 2, 4])
def test_identical_experts_are_the_dense_model(k):
    """The gates of a token sum to one, so E copies of one expert give that expert's output whatever is routed."""
    cfg = cfg_of(n_experts=4, top_k=k)
    W = moe_weights(cfg, 4)
    for name in ("wg", "wu", "wd"):
        W[name][:] = W[name][:, :, :1]
    dense = cfg_of()
    Wd = dict(W)
    Wd["wg"], Wd["wu"], Wd["wd"] = W["wg"][:, :, 0], W["wu"][:, :, 0], W["wd"][:, :, 0]
    tokens = np.random.default_rng(2).integers(0, cfg.vocab, (1, 9))
    a, _ = prefill(cfg, W, tokens)
    b, _ = prefill(dense, Wd, tokens)
    np.testing.assert_allclose(a["hidden"], b["hidden"], rtol=1e-12, atol=1e-12)


def torch_moe_decoder(cfg, W, tokens):
    """Single-track decoder whose feed-forward network evaluates every expert on every token and weights the
    results with a dense [S, E] gate matrix built by torch.topk / softmax / scatter."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    H, Hkv, hd, d = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim, cfg.d_model
    tok = torch.from_numpy(np.asarray(tokens)).long()
    B, S = tok.shape
    h = F.embedding(tok, t(W["embed"]))
    inv = 1.0 / (cfg.rope_theta ** (torch.arange(0, hd, 2, dtype=torch.float64) / hd))
    ang = torch.arange(S, dtype=torch.float64)[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]

    def rope(u):
        x1, x2 = u[..., : hd // 2], u[..., hd // 2:]
        return torch.cat([x1 * cos - x2 * sin, x2 * cos + x1 * sin], dim=-1)

    for l in range(cfg.n_layers):
        a = F.rms_norm(h, (d,), t(W["g1"][0, l]), cfg.rms_eps)
        q = rope((a @ t(W["wq"][0, l])).view(B, S, H, hd))
        k = rope((a @ t(W["wk"][0, l])).view(B, S, Hkv, hd)).repeat_interleave(H // Hkv, dim=2)
        v = (a @ t(W["wv"][0, l])).view(B, S, Hkv, hd).repeat_interleave(H // Hkv, dim=2)
        o = F.scaled_dot_product_attention(q.transpose(1, 2), k.transpose(1, 2), v.transpose(1, 2),
                                           is_causal=True)
        h = h + o.transpose(1, 2).reshape(B, S, H * hd) @ t(W["wo"][0, l])
        a = F.rms_norm(h, (d,), t(W["g2"][0, l]), cfg.rms_eps)
        r = a @ t(W["wr"][0, l])                                    # [B, S, E]
        top, idx = torch.topk(r, cfg.top_k, dim=-1)
        gates = torch.zeros_like(r).scatter(-1, idx, F.softmax(top, dim=-1))
        every = torch.stack([(F.silu(a @ t(W["wg"][0, l, e])) * (a @ t(W["wu"][0, l, e]))) @ t(W["wd"][0, l, e])
                             for e in range(cfg.n_experts)], dim=-1)  # [B, S, d, E]
        h = h + torch.einsum("bsde,bse->bsd", every, gates)
    return h.numpy()


@pytest.mark.parametrize("E,k", [(4, 1), (4, 2), (6, 3), (3, 3)])
def test_single_track_moe_against_a_dense_gate_matrix_in_torch(E, k):
    cfg = cfg_of(n_tracks=1, block_depth=1, n_layers=2, n_experts=E, top_k=k)
    W = moe_weights(cfg, 10 + E)
    tokens = np.random.default_rng(E).integers(0, cfg.vocab, (2, 8))
    out, _ = prefill(cfg, W, tokens)
    np.testing.assert_allclose(out["hidden"], torch_moe_decoder(cfg, W, tokens), rtol=1e-10, atol=1e-10)


def test_routing_by_hand():
    """Top-2 of four logits, the tie rule, and the gate values written out."""
    r = np.array([[0.0, 2.0, 1.0, -1.0],      # experts 1, 2
                  [3.0, 3.0, 3.0, 3.0],       # all equal: the two lowest indices, equal gates
                  [-5.0, 0.5, 0.5, 7.0]])     # expert 3, then the lower index of the tied pair
    ids, gates = O.top_k_route(r, 2)
    assert ids.tolist() == [[1, 2], [0, 1], [3, 1]]
    e = math.e
    np.testing.assert_allclose(gates[0], [e / (e + 1), 1 / (e + 1)], rtol=1e-15)
    np.testing.assert_allclose(gates[1], [0.5, 0.5], rtol=1e-15)
    np.testing.assert_allclose(gates[2], [1 / (1 + math.exp(-6.5)), 1 / (1 + math.exp(6.5))], rtol=1e-14)
    ids1, gates1 = O.top_k_route(r, 1)
    assert ids1[:, 0].tolist() == [1, 0, 3] and np.all(gates1 == 1.0)


def test_moe_layer_closed_form_with_diagonal_experts():
    """One layer, attention off, expert e multiplies SwiGLU's product by (e + 1): out = x + sum gate_e (e+1) s(a)."""
    cfg = cfg_of(n_tracks=1, n_layers=1, block_depth=1, d_model=4, n_heads=1, n_kv_heads=1, head_dim=4,
                 d_ffn=4, vocab=0, rms_eps=0.0, n_experts=3, top_k=2)
    W = moe_weights(cfg)
    W["wo"][:] = 0
    W["g1"][:] = 1
    W["g2"][:] = 1
    for e in range(3):
        W["wg"][0, 0, e] = np.eye(4)
        W["wu"][0, 0, e] = np.eye(4)
        W["wd"][0, 0, e] = (e + 1) * np.eye(4)
    W["wr"][0, 0] = np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 0, 1.0], [0, 0, 0]])
    x = np.array([[[2.0, 1.0, -1.0, 0.5], [-1.0, 0.0, 3.0, 1.0]]])
    out, _ = prefill(cfg, W, hidden_in=x)
    expect = np.empty_like(x)
    for s in range(2):
        a = x[0, s] / math.sqrt(np.mean(x[0, s] ** 2))
        order = sorted(range(3), key=lambda e: (-a[e], e))[:2]     # logits are a[0..2]
        w = np.exp([a[e] for e in order])
        w /= w.sum()
        base = a / (1 + np.exp(-a)) * a
        expect[0, s] = x[0, s] + sum(w[j] * (order[j] + 1) for j in range(2)) * base
    np.testing.assert_allclose(out["hidden"], expect, rtol=1e-14)
    assert out["routes"][0][0, 0].tolist() == [[0, 1], [2, 1]]


def test_expert_permutation_leaves_the_output_unchanged():
    cfg = cfg_of(n_experts=5, top_k=2)
    W = moe_weights(cfg, 8)
    perm = np.array([3, 0, 4, 1, 2])
    Wp = dict(W)
    for name in ("wg", "wu", "wd"):
        Wp[name] = W[name][:, :, perm]
    Wp["wr"] = W["wr"][..., perm]
    tokens = np.random.default_rng(3).integers(0, cfg.vocab, (1, 6))
    a, _ = prefill(cfg, W, tokens)
    b, _ = prefill(cfg, Wp, tokens)
    np.testing.assert_allclose(a["hidden"], b["hidden"], rtol=1e-12, atol=1e-12)
    assert np.array_equal(perm[b["routes"][0]], a["routes"][0])


def test_forced_routes_and_cached_decode():
    cfg = cfg_of(n_experts=4, top_k=2)
    W = moe_weights(cfg, 9)
    tokens = np.random.default_rng(4).integers(0, cfg.vocab, (2, 6))
    full, _ = prefill(cfg, W, tokens)
    # forcing the selection the oracle made itself changes nothing
    st = O.PTState(cfg, 2, 16)
    same = O.pt_prefill(cfg, W, st, tokens=tokens, forced_routes=full["routes"])
    assert np.array_equal(same["hidden"], full["hidden"])
    # cached decode of the last token equals the full pass, routes included
    st = O.PTState(cfg, 2, 16)
    O.pt_prefill(cfg, W, st, tokens=tokens[:, :5])
    step = O.pt_decode_step(cfg, W, st, tokens=tokens[:, 5])
    np.testing.assert_allclose(step["hidden"], full["hidden"][:, 5], rtol=1e-11, atol=1e-11)
    for b in range(2):
        assert np.array_equal(step["routes"][:, :, b], full["routes"][b][:, :, 5])
    # forcing another selection moves the output
    other = [(r + 1) % cfg.n_experts for r in full["routes"]]
    st = O.PTState(cfg, 2, 16)
    moved = O.pt_prefill(cfg, W, st, tokens=tokens, forced_routes=other)
    assert np.abs(moved["hidden"] - full["hidden"]).max() > 1e-3
