"""CPU oracle for the Parallel Track (PT) transformer forward pass.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library computes; it is imported by the tests, by the smoke check and by
the benchmark's ``cpu_baseline`` leg, never by the product path.  It shares no
code with the HIP path and imports nothing from the package.

What it follows
---------------
* Algorithm 1 of the paper ("Track Parallelism for PT Transformer"): every
  track starts from the same embedding input, the layers of all tracks run
  independently, and after every D-th layer the per-track activations are
  all-reduced and every track continues from the reduced activation
  (Section 2.2).  The assignment "h_i = h" is taken to belong to the branch
  that performs the all-reduce (the comment printed next to it says "after all
  reduce"; outside the branch it would overwrite every track after every layer).
* The paper leaves the "standard transformer layer" unspecified (Section 2.2,
  Figure 1 caption) apart from grouped-query attention (Section 3.1, Table 1).
  The layer used here is the common pre-norm decoder layer: RMSNorm, rotary
  position embedding with rotate-half pairing, causal softmax attention with
  grouped KV heads, a SwiGLU feed-forward network, no biases.
* PT-MoE (Section 2.2, "Contrast with MoE / expert parallelism", and the Conclusion): MoE sparsity is applied
  within tracks, i.e. the dense feed-forward network of a layer is replaced by a routed mixture of experts while
  tracks and merges stay as they are.  The paper gives no formula; the routing used here is the sparsely-gated
  form of the work it cites: router logits r = a W_r, the k largest logits select the experts (lowest index on
  exact ties), the gates are the softmax over those k logits, every expert is a SwiGLU network, no shared expert,
  no capacity limit.  A model is a PT-MoE model when cfg.n_experts > 0 (cfg.top_k experts per token).
* All arithmetic is float64 on numpy arrays.  Matrix products use ``@`` as a
  library step; attention materialises the full score matrix and uses a
  two-pass softmax, so it is also the brute force that flash-style and split-K
  kernels are compared against.  There is no blocking, fusion or reordering.

Weights are passed in as a dict of arrays in the logical ``x @ W`` layouts
``wq [T,L,d,H*hd]``, ``wk, wv [T,L,d,Hkv*hd]``, ``wo [T,L,H*hd,d]``,
``wg, wu [T,L,d,f]``, ``wd [T,L,f,d]`` (PT-MoE: ``wg, wu [T,L,E,d,f]``, ``wd [T,L,E,f,d]`` and the
router ``wr [T,L,d,E]``), ``g1, g2 [T,L,d]``, ``gf [d]``,
``embed [V,d]``, ``head [d,V]``.  ``cfg`` is any object with the attributes
n_tracks, n_layers, block_depth, d_model, n_heads, n_kv_heads, head_dim, d_ffn,
vocab, merge_scale, rms_eps, rope_theta.

Pins (tests/test_oracle_pins.py): T=1, D=1 against an independent composition of
torch CPU library routines; track isolation and post-merge equality; the merge
closed form with zeroed output projections; replicated tracks against the
one-track model; track permutation; causal prefix invariance; cached decode
against full recompute; batch independence; softmax / RoPE / RMSNorm special
cases; hand-computed tiny values under tests/golden/.
"""
from __future__ import annotations

from typing import Dict, List, Optional

import numpy as np

F64 = np.float64


def _f64(w: np.ndarray) -> np.ndarray:
    """The array as float64 (the same values; no copy when the caller already holds float64)."""
    return np.asarray(w, dtype=F64)


def rmsnorm(h: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """a = h * g / sqrt(mean_d(h^2) + eps) over the last axis."""
    h = np.asarray(h, dtype=F64)
    ms = np.mean(h * h, axis=-1, keepdims=True)
    return h / np.sqrt(ms + eps) * np.asarray(g, dtype=F64)


def rope(u: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing.  u [S, heads, hd]; positions [S].

    For j < hd/2 with angle p * theta^(-2j/hd):
      out[j]        = u[j] cos - u[j+hd/2] sin
      out[j+hd/2]   = u[j+hd/2] cos + u[j] sin
    """
    u = np.asarray(u, dtype=F64)
    hd = u.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=F64)
    inv_freq = np.power(F64(theta), -2.0 * j / hd)
    ang = np.asarray(positions, dtype=F64)[:, None] * inv_freq[None, :]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = u[..., :half], u[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    """Two-pass softmax over the last axis (-inf entries get probability 0)."""
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def causal_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """q [Sq, H, hd]; k, v [Sk, Hkv, hd] holding positions 0..Sk-1; q_pos [Sq] absolute
    positions.  Query at position p sees keys r <= p.  Query head c uses KV head
    c // (H / Hkv).  Returns [Sq, H, hd]."""
    Sq, H, hd = q.shape
    Sk, Hkv, _ = k.shape
    group = H // Hkv
    out = np.empty((Sq, H, hd), dtype=F64)
    r = np.arange(Sk)
    visible = r[None, :] <= np.asarray(q_pos)[:, None]
    for c in range(H):
        kv = c // group
        s = (q[:, c, :] @ k[:, kv, :].T) / np.sqrt(F64(hd))
        s = np.where(visible, s, -np.inf)
        out[:, c, :] = softmax_rows(s) @ v[:, kv, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def top_k_route(r: np.ndarray, k: int):
    """Sparse gating over router logits r [S, E]: the indices of the k largest logits of every row in decreasing
    order of logit (lowest index first on exact ties) and the softmax over just those k logits."""
    S, E = r.shape
    ids = np.empty((S, k), dtype=np.int64)
    for s in range(S):
        ids[s] = sorted(range(E), key=lambda e: (-r[s, e], e))[:k]
    sel = np.take_along_axis(r, ids, axis=1)
    return ids, softmax_rows(sel)


def moe_ffn(cfg, W, i: int, l: int, a: np.ndarray, routes: Optional[list], forced: Optional[np.ndarray]) -> np.ndarray:
    """Routed mixture of SwiGLU experts on the normalised rows a [S, d] of track i, layer l.  `forced` [S, k]
    replaces the selection (the gates are still the softmax of the router's logits at the forced experts);
    `routes`, when given, receives the selection that was used."""
    r = a @ _f64(W["wr"][i, l])
    ids, gates = top_k_route(r, cfg.top_k)
    if forced is not None:
        ids = np.asarray(forced, dtype=np.int64)
        gates = softmax_rows(np.take_along_axis(r, ids, axis=1))
    if routes is not None:
        # also how decided the (unforced) selection was: the gap between the last logit taken and the first one
        # left out, relative to the largest |logit| of the row (infinite when every expert is taken)
        srt = -np.sort(-r, axis=1)
        gap = (srt[:, cfg.top_k - 1] - srt[:, cfg.top_k] if cfg.top_k < cfg.n_experts
               else np.full(r.shape[0], np.inf))
        routes.append((ids.copy(), gap / np.maximum(np.max(np.abs(r), axis=1), 1e-300)))
    out = np.zeros_like(a)
    for e in range(cfg.n_experts):
        rows, slot = np.nonzero(ids == e)
        if rows.size == 0:
            continue
        x = a[rows]
        y = (silu(x @ _f64(W["wg"][i, l, e])) * (x @ _f64(W["wu"][i, l, e]))) @ _f64(W["wd"][i, l, e])
        out[rows] += gates[rows, slot][:, None] * y
    return out


def track_merge(hs: List[np.ndarray], scale: float) -> np.ndarray:
    """The all-reduce of Algorithm 1 on one device: scale * (h_1 + ... + h_n), summed in
    track order."""
    acc = np.array(hs[0], dtype=F64, copy=True)
    for h in hs[1:]:
        acc = acc + np.asarray(h, dtype=F64)
    return F64(scale) * acc


class PTState:
    """KV cache and per-sequence lengths carried from prefill to decode."""

    def __init__(self, cfg, batch: int, max_seq: int):
        T, L = cfg.n_tracks, cfg.n_layers
        shp = (T, L, batch, max_seq, cfg.n_kv_heads, cfg.head_dim)
        self.k = np.zeros(shp, dtype=F64)
        self.v = np.zeros(shp, dtype=F64)
        self.length = np.zeros(batch, dtype=np.int64)
        self.merge_count = 0


def _layer(cfg, W: Dict[str, np.ndarray], i: int, l: int, h: np.ndarray, pos: np.ndarray,
           state: PTState, b: int, routes: Optional[list] = None, forced: Optional[np.ndarray] = None) -> np.ndarray:
    """One transformer layer of track i on the rows ``h [S, d]`` of sequence b, which sit
    at absolute positions ``pos``.  Appends this layer's keys and values to the cache."""
    H, Hkv, hd = cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    S = h.shape[0]
    a = rmsnorm(h, W["g1"][i, l], cfg.rms_eps)
    q = (a @ _f64(W["wq"][i, l])).reshape(S, H, hd)
    k = (a @ _f64(W["wk"][i, l])).reshape(S, Hkv, hd)
    v = (a @ _f64(W["wv"][i, l])).reshape(S, Hkv, hd)
    q = rope(q, pos, cfg.rope_theta)
    k = rope(k, pos, cfg.rope_theta)
    state.k[i, l, b, pos] = k
    state.v[i, l, b, pos] = v
    ctx = int(pos[-1]) + 1
    o = causal_attention(q, state.k[i, l, b, :ctx], state.v[i, l, b, :ctx], pos)
    h = h + o.reshape(S, H * hd) @ _f64(W["wo"][i, l])
    a2 = rmsnorm(h, W["g2"][i, l], cfg.rms_eps)
    if getattr(cfg, "n_experts", 0) > 0:
        return h + moe_ffn(cfg, W, i, l, a2, routes, forced)
    gate = a2 @ _f64(W["wg"][i, l])
    up = a2 @ _f64(W["wu"][i, l])
    h = h + (silu(gate) * up) @ _f64(W["wd"][i, l])
    return h


def _run_rows(cfg, W, state: PTState, x_tracks: List[np.ndarray], b: int, pos: np.ndarray,
              taps: Optional[list], track_taps: Optional[list], routes: Optional[list] = None,
              forced: Optional[np.ndarray] = None):
    """Algorithm 1 on the rows of one sequence.  x_tracks: per-track input [S, d].  PT-MoE: `routes` collects the
    expert selection of every (layer, track) in that order; `forced` [L, T, S, k] prescribes it."""
    T, L, D = cfg.n_tracks, cfg.n_layers, cfg.block_depth
    hs = [np.array(x, dtype=F64, copy=True) for x in x_tracks]
    h = None
    for l in range(L):
        for i in range(T):
            hs[i] = _layer(cfg, W, i, l, hs[i], pos, state, b, routes, None if forced is None else forced[l][i])
        if (l + 1) % D == 0:
            if track_taps is not None:
                track_taps.append([t.copy() for t in hs])
            h = track_merge(hs, cfg.merge_scale)
            hs = [h.copy() for _ in range(T)]
            if taps is not None:
                taps.append(h.copy())
    return h


def logits_from_hidden(cfg, W, h: np.ndarray) -> np.ndarray:
    """Final RMSNorm and the (untied) output head on merged hidden rows [.., d]."""
    return rmsnorm(h, W["gf"], cfg.rms_eps) @ _f64(W["head"])


def pt_prefill(cfg, W, state: PTState, tokens: Optional[np.ndarray] = None,
               hidden_in: Optional[np.ndarray] = None, collect_taps: bool = False,
               lengths: Optional[np.ndarray] = None, forced_routes: Optional[list] = None):
    """Prefill a batch from position 0.

    tokens [B, S] int, or hidden_in [B, S, d] (same input for every track) or
    [T, B, S, d] (per-track input).  Returns a dict with ``hidden`` [B, S, d] (the output
    activation of Algorithm 1), ``logits`` [B, S, V] when the model has a vocabulary, and,
    if requested, ``taps``: per sequence, the merged activation after every block, and
    ``track_taps``: per sequence, the per-track activations right before every merge.

    ``lengths`` [B] (optional) makes the batch ragged: sequence b consists of the first
    lengths[b] of its S rows only (the throughput mode of Section 3.3 batches inputs of mixed
    lengths); Algorithm 1 runs on exactly those rows, the rest of ``hidden`` / ``logits`` is
    NaN, taps hold lengths[b] rows, and decoding continues at position lengths[b].

    PT-MoE models also return ``routes``: per sequence an int array [L, T, S, k] with the experts every token
    was sent to, and ``route_margins`` [L, T, S]: the relative gap between the last logit taken and the first left
    out; ``forced_routes`` (same shape as routes, per sequence) prescribes the selection instead.
    """
    T, d = cfg.n_tracks, cfg.d_model
    if tokens is not None:
        tokens = np.asarray(tokens)
        B, S = tokens.shape
    else:
        hidden_in = np.asarray(hidden_in, dtype=F64)
        B, S = hidden_in.shape[-3], hidden_in.shape[-2]
    hidden = np.full((B, S, d), np.nan, dtype=F64)
    all_taps, all_track_taps, all_routes, all_margins = [], [], [], []
    for b in range(B):
        n = S if lengths is None else int(lengths[b])
        pos = np.arange(n)
        if tokens is not None:
            x = _f64(W["embed"][tokens[b, :n]])
            xs = [x] * T
        elif hidden_in.ndim == 3:
            xs = [hidden_in[b, :n]] * T
        else:
            xs = [hidden_in[i, b, :n] for i in range(T)]
        taps = [] if collect_taps else None
        ttaps = [] if collect_taps else None
        moe = getattr(cfg, "n_experts", 0) > 0
        routes = [] if moe else None
        hidden[b, :n] = _run_rows(cfg, W, state, xs, b, pos, taps, ttaps, routes,
                                  None if forced_routes is None else forced_routes[b])
        state.length[b] = n
        all_taps.append(taps)
        all_track_taps.append(ttaps)
        if moe:
            all_routes.append(np.stack([ids for ids, _ in routes]).reshape(cfg.n_layers, T, n, cfg.top_k))
            all_margins.append(np.stack([m for _, m in routes]).reshape(cfg.n_layers, T, n))
    state.merge_count += cfg.n_layers // cfg.block_depth
    out = {"hidden": hidden}
    if cfg.vocab > 0:
        out["logits"] = logits_from_hidden(cfg, W, hidden)
    if collect_taps:
        out["taps"] = all_taps
        out["track_taps"] = all_track_taps
    if all_routes:
        out["routes"] = all_routes
        out["route_margins"] = all_margins
    return out


def pt_decode_step(cfg, W, state: PTState, tokens: Optional[np.ndarray] = None,
                   hidden_in: Optional[np.ndarray] = None, forced_routes: Optional[np.ndarray] = None):
    """One KV-cached decode step: one new row per sequence at position length[b].

    tokens [B] int, or hidden_in [B, d] / [T, B, d].  Returns ``hidden`` [B, d], and with a
    vocabulary ``logits`` [B, V] and ``argmax`` [B] (lowest id on exact ties).  PT-MoE: ``routes`` [L, T, B, k];
    ``forced_routes`` (same shape) prescribes the expert selection."""
    T, d = cfg.n_tracks, cfg.d_model
    B = len(tokens) if tokens is not None else np.asarray(hidden_in).shape[-2]
    hidden = np.empty((B, d), dtype=F64)
    moe = getattr(cfg, "n_experts", 0) > 0
    all_routes = []
    for b in range(B):
        pos = np.array([state.length[b]])
        if tokens is not None:
            x = _f64(W["embed"][np.asarray(tokens)[b]])[None, :]
            xs = [x] * T
        else:
            hin = np.asarray(hidden_in, dtype=F64)
            xs = [hin[b][None, :]] * T if hin.ndim == 2 else [hin[i, b][None, :] for i in range(T)]
        routes = [] if moe else None
        forced = None if forced_routes is None else np.asarray(forced_routes)[:, :, b:b + 1]
        hidden[b] = _run_rows(cfg, W, state, xs, b, pos, None, None, routes, forced)[0]
        state.length[b] += 1
        if moe:
            all_routes.append(np.stack([ids for ids, _ in routes]).reshape(cfg.n_layers, T, 1, cfg.top_k))
    state.merge_count += cfg.n_layers // cfg.block_depth
    out = {"hidden": hidden}
    if cfg.vocab > 0:
        out["logits"] = logits_from_hidden(cfg, W, hidden)
        out["argmax"] = np.argmax(out["logits"], axis=-1).astype(np.int32)
    if moe:
        out["routes"] = np.concatenate(all_routes, axis=2)
    return out


def sync_points_tensor_parallel(n_layers: int) -> int:
    """Synchronisation points of tensor parallelism: one after attention and one after the
    FFN of every layer (Section 2.1)."""
    return 2 * n_layers


def sync_points_track_parallel(n_layers: int, block_depth: int) -> int:
    """Synchronisation points of track parallelism: one per track block (Section 2.2)."""
    return n_layers // block_depth
