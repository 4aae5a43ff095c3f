"""Seeded synthetic inputs for the Parallel Track (PT) transformer forward pass.

This module holds *only* input generation: a counter-based pseudo-random
generator and the recipes that turn it into weights, token ids and hidden-state
tensors.  It contains none of the method's arithmetic (no norm, attention, FFN
or merge) and imports neither the CPU oracle nor the HIP binding; both of those
are fed from here so that they see identical inputs.

Generator (fixed by this repository; the paper gives only "N(0, 0.02)" style
recipes through the benchmark configurations):

* a stream is named by ``(seed, kind, track, layer)`` and hashed to a 64-bit key;
* counter ``c`` of a stream yields 64 bits ``mix64(key + (c + 1) * GAMMA)``
  (the splitmix64 finaliser);
* the high and low 32-bit halves give ``u1 in (0, 1]`` and ``u2 in [0, 1)``;
  a Box-Muller transform turns them into two standard normals; element ``e`` of
  a tensor takes normal ``e & 1`` of counter ``e >> 1``;
* the logarithm and the sine/cosine are evaluated with short fixed polynomials
  that use only ``+ - * /`` and ``sqrt`` in double precision, one rounding per
  operation, so that any IEEE-754 implementation that evaluates the same
  expression tree without fused multiply-add reproduces every bit.  The HIP
  library's ``pt_init_weights`` is such a second implementation.

Tensors are indexed in their *logical* row-major layout ``[in, out]`` (weights),
``[vocab, d]`` (embedding) or ``[tokens, d]`` (hidden states); a consumer that
stores a different physical layout must map back to the logical index.
"""
from __future__ import annotations

import dataclasses
import os
from concurrent.futures import ThreadPoolExecutor
from typing import Dict, Optional

import numpy as np

MASK64 = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15

# stream kinds
KIND_EMBED = 1
KIND_HEAD = 2
KIND_WQ = 3
KIND_WK = 4
KIND_WV = 5
KIND_WO = 6
KIND_WG = 7
KIND_WU = 8
KIND_WD = 9
KIND_WR = 13
KIND_TOKENS = 16
KIND_HIDDEN = 17

PT_F32 = 0
PT_BF16 = 1


@dataclasses.dataclass(frozen=True)
class PTConfig:
    """Shape of a PT model (Algorithm 1's n, L, D plus the per-track layer shape)."""

    n_tracks: int
    n_layers: int
    block_depth: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    max_batch: int
    max_seq: int
    dtype: int = PT_BF16
    merge_scale: float = 1.0
    rms_eps: float = 1e-5
    rope_theta: float = 10000.0
    init_std: float = 0.02
    n_experts: int = 0      # PT-MoE: experts per (track, layer); 0 = dense feed-forward network
    top_k: int = 0          # PT-MoE: experts every token is routed to

    @property
    def n_merges(self) -> int:
        return self.n_layers // self.block_depth


def _mix64_int(z: int) -> int:
    z &= MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
    return z ^ (z >> 31)


def expert_layer(layer: int, expert: int) -> int:
    """The `layer` field of the stream of expert `expert`'s tensors in layer `layer` (layer < 4096)."""
    return layer | ((expert + 1) << 12)


def stream_key(seed: int, kind: int, track: int = 0, layer: int = 0) -> int:
    """64-bit key of the stream ``(seed, kind, track, layer)``."""
    tag = ((kind & 0xFFFF) << 40) | ((track & 0xFFFFF) << 20) | (layer & 0xFFFFF)
    return _mix64_int(_mix64_int((seed + GAMMA) & MASK64) ^ tag)


def _mix64(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def raw_bits(key: int, counters: np.ndarray) -> np.ndarray:
    """64 random bits for each counter of the stream ``key`` (uint64 in, uint64 out)."""
    with np.errstate(over="ignore"):
        c = counters.astype(np.uint64)
        return _mix64(np.uint64(key) + (c + np.uint64(1)) * np.uint64(GAMMA))


_LN2 = 0.6931471805599453
_HALF_PI = 1.5707963267948966
_SQRT_HALF = 0.7071067811865476


def _log_poly(u: np.ndarray) -> np.ndarray:
    """ln(u) for u in (0, 1]: frexp, then the atanh series in s = (m-1)/(m+1)."""
    m, e = np.frexp(u)
    small = m < _SQRT_HALF
    m = np.where(small, m * 2.0, m)
    e = np.where(small, e - 1, e).astype(np.float64)
    s = (m - 1.0) / (m + 1.0)
    s2 = s * s
    p = np.full_like(s, 1.0 / 19.0)
    for k in (17.0, 15.0, 13.0, 11.0, 9.0, 7.0, 5.0, 3.0, 1.0):
        p = p * s2 + (1.0 / k)
    return (2.0 * s) * p + e * _LN2


def _sincos_poly(a: np.ndarray):
    """(cos a, sin a) for |a| <= pi/4 by Taylor polynomials in Horner form."""
    a2 = a * a
    sp = np.full_like(a, -1.0 / 1307674368000.0)          # -1/15!
    for f in (6227020800.0, -39916800.0, 362880.0, -5040.0, 120.0, -6.0, 1.0):
        sp = sp * a2 + (1.0 / f)
    sn = a * sp
    cp = np.full_like(a, 1.0 / 20922789888000.0)           # 1/16!
    for f in (-87178291200.0, 479001600.0, -3628800.0, 40320.0, -720.0, 24.0, -2.0, 1.0):
        cp = cp * a2 + (1.0 / f)
    return cp, sn


def standard_normals(key: int, start: int, count: int) -> np.ndarray:
    """Elements ``start .. start+count-1`` of the N(0,1) stream ``key`` (float64)."""
    if count <= 0:
        return np.zeros(0, dtype=np.float64)
    first_pair = start >> 1
    last_pair = (start + count - 1) >> 1
    ctr = np.arange(first_pair, last_pair + 1, dtype=np.uint64)
    z = raw_bits(key, ctr)
    hi = (z >> np.uint64(32)).astype(np.float64)
    lo = (z & np.uint64(0xFFFFFFFF)).astype(np.float64)
    u1 = (hi + 1.0) * (1.0 / 4294967296.0)
    u2 = lo * (1.0 / 4294967296.0)
    r = np.sqrt(-2.0 * _log_poly(u1))
    t = u2 * 4.0
    q = np.floor(t)
    a = ((t - q) - 0.5) * _HALF_PI
    c0, s0 = _sincos_poly(a)
    qi = q.astype(np.int64)
    c = np.where(qi == 0, c0, np.where(qi == 1, -s0, np.where(qi == 2, -c0, s0)))
    s = np.where(qi == 0, s0, np.where(qi == 1, c0, np.where(qi == 2, -s0, -c0)))
    out = np.empty((ctr.size, 2), dtype=np.float64)
    out[:, 0] = r * c
    out[:, 1] = r * s
    flat = out.reshape(-1)
    off = start - (first_pair << 1)
    return flat[off:off + count]


def normal_tensor(key: int, shape, std: float, chunk: int = 1 << 17,
                  workers: Optional[int] = None) -> np.ndarray:
    """float32 tensor of ``shape`` filled, in row-major order, with
    ``float32(double(n_e) * double(float32(std)))``.  Chunks are independent
    (counter-based), so they are filled by a small thread pool."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32)
    sd = float(np.float32(std))

    def fill(s: int) -> None:
        c = min(chunk, n - s)
        out[s:s + c] = (standard_normals(key, s, c) * sd).astype(np.float32)

    starts = range(0, n, chunk)
    if workers is None:
        workers = min(16, os.cpu_count() or 1)
    if len(starts) <= 1 or workers <= 1:
        for s in starts:
            fill(s)
    else:
        with ThreadPoolExecutor(max_workers=workers) as ex:
            list(ex.map(fill, starts))
    return out.reshape(shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns the uint16 bit patterns."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_dtype(x: np.ndarray, dtype: int) -> np.ndarray:
    """The float32 values a tensor holds once stored in ``dtype`` (identity for fp32)."""
    if dtype == PT_F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    return bf16_to_f32(bf16_bits(x)).reshape(x.shape)


def make_weights(cfg: PTConfig, seed: int, tracks: Optional[range] = None) -> Dict[str, np.ndarray]:
    """All weights of a PT model as float32 arrays already rounded to ``cfg.dtype``.

    Logical layouts (``x @ W`` convention): ``wq [T,L,d,H*hd]``, ``wk, wv [T,L,d,Hkv*hd]``,
    ``wo [T,L,H*hd,d]``, ``wg, wu [T,L,d,f]``, ``wd [T,L,f,d]``, norm gains
    ``g1, g2 [T,L,d]`` and ``gf [d]`` (all ones), ``embed [V,d]``, ``head [d,V]``
    (the last two only when ``cfg.vocab > 0``).  A PT-MoE model (``cfg.n_experts = E > 0``) has
    ``wg, wu [T,L,E,d,f]``, ``wd [T,L,E,f,d]`` and the router ``wr [T,L,d,E]``.
    """
    T, L, d = cfg.n_tracks, cfg.n_layers, cfg.d_model
    hq, hk, f = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.d_ffn
    E = cfg.n_experts
    shapes = {
        "wq": (KIND_WQ, (d, hq)), "wk": (KIND_WK, (d, hk)), "wv": (KIND_WV, (d, hk)),
        "wo": (KIND_WO, (hq, d)), "wg": (KIND_WG, (d, f)), "wu": (KIND_WU, (d, f)),
        "wd": (KIND_WD, (f, d)),
    }
    if E > 0:
        shapes["wr"] = (KIND_WR, (d, E))
    W: Dict[str, np.ndarray] = {}
    for name, (kind, shp) in shapes.items():
        per_expert = E > 0 and name in ("wg", "wu", "wd")
        arr = np.empty((T, L) + ((E,) if per_expert else ()) + shp, dtype=np.float32)
        for i in range(T):
            for l in range(L):
                if per_expert:
                    for e in range(E):
                        arr[i, l, e] = round_to_dtype(normal_tensor(
                            stream_key(seed, kind, i, expert_layer(l, e)), shp, cfg.init_std), cfg.dtype)
                else:
                    arr[i, l] = round_to_dtype(
                        normal_tensor(stream_key(seed, kind, i, l), shp, cfg.init_std), cfg.dtype)
        W[name] = arr
    W["g1"] = np.ones((T, L, d), dtype=np.float32)
    W["g2"] = np.ones((T, L, d), dtype=np.float32)
    W["gf"] = np.ones((d,), dtype=np.float32)
    if cfg.vocab > 0:
        W["embed"] = round_to_dtype(
            normal_tensor(stream_key(seed, KIND_EMBED), (cfg.vocab, d), cfg.init_std), cfg.dtype)
        W["head"] = round_to_dtype(
            normal_tensor(stream_key(seed, KIND_HEAD), (d, cfg.vocab), cfg.init_std), cfg.dtype)
    return W


class LazyWeights:
    """The weights of make_weights(cfg, seed), generated tensor by tensor on demand: ``W["wq"][i, l]`` (or
    ``W["wg"][i, l, e]`` for a PT-MoE model) builds that one tensor from its stream.  For models whose weights do not
    fit host memory at once; a consumer that walks layers in order holds one tensor at a time."""

    class _Indexer:
        def __init__(self, make):
            self._make = make

        def __getitem__(self, idx):
            return self._make(*idx) if isinstance(idx, tuple) else self._make(idx)

    def __init__(self, cfg: PTConfig, seed: int, on_tensor=None):
        """on_tensor(name, track, layer), when given, is called before a per-layer tensor is generated (a long
        consumer reports its progress through it)."""
        self.cfg, self.seed, self.on_tensor = cfg, seed, on_tensor
        d = cfg.d_model
        hq, hk, f = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim, cfg.d_ffn
        self._shapes = {"wq": (KIND_WQ, (d, hq)), "wk": (KIND_WK, (d, hk)), "wv": (KIND_WV, (d, hk)),
                        "wo": (KIND_WO, (hq, d)), "wg": (KIND_WG, (d, f)), "wu": (KIND_WU, (d, f)),
                        "wd": (KIND_WD, (f, d)), "wr": (KIND_WR, (d, cfg.n_experts))}
        self._global = {}

    def _tensor(self, name, track, layer, expert=None):
        kind, shp = self._shapes[name]
        if self.on_tensor is not None:
            self.on_tensor(name, track, layer)
        lay = layer if expert is None else expert_layer(layer, expert)
        return round_to_dtype(normal_tensor(stream_key(self.seed, kind, track, lay), shp, self.cfg.init_std), self.cfg.dtype)

    def __getitem__(self, name):
        cfg = self.cfg
        if name in ("g1", "g2"):
            return LazyWeights._Indexer(lambda i, l: np.ones((cfg.d_model,), dtype=np.float32))
        if name in ("gf", "embed", "head"):
            if name not in self._global:
                if name == "gf":
                    self._global[name] = np.ones((cfg.d_model,), dtype=np.float32)
                else:
                    kind, shp = ((KIND_EMBED, (cfg.vocab, cfg.d_model)) if name == "embed"
                                 else (KIND_HEAD, (cfg.d_model, cfg.vocab)))
                    self._global[name] = round_to_dtype(normal_tensor(stream_key(self.seed, kind), shp, cfg.init_std),
                                                        cfg.dtype)
            return self._global[name]
        if name not in self._shapes or (name == "wr" and cfg.n_experts == 0):
            raise KeyError(name)
        return LazyWeights._Indexer(lambda i, l, e=None: self._tensor(name, i, l, e))


def make_tokens(seed: int, batch: int, seq: int, vocab: int, stream: int = 0) -> np.ndarray:
    """int32 ``[batch, seq]`` token ids, uniform over the vocabulary."""
    key = stream_key(seed, KIND_TOKENS, stream, 0)
    z = raw_bits(key, np.arange(batch * seq, dtype=np.uint64))
    return (z % np.uint64(vocab)).astype(np.int32).reshape(batch, seq)


def make_hidden(seed: int, track: int, tokens: int, d: int, dtype: int = PT_BF16,
                std: float = 1.0) -> np.ndarray:
    """float32 ``[tokens, d]`` hidden states ~ N(0, std), rounded to ``dtype``."""
    key = stream_key(seed, KIND_HIDDEN, track, 0)
    return round_to_dtype(normal_tensor(key, (tokens, d), std), dtype)


# The benchmark configurations (index = position in the list of named workloads).
def config_tiny() -> PTConfig:
    return PTConfig(n_tracks=2, n_layers=4, block_depth=2, d_model=128, n_heads=4, n_kv_heads=4,
                    head_dim=32, d_ffn=512, vocab=512, max_batch=1, max_seq=64, dtype=PT_F32)


def config_mid(max_batch: int = 4, max_seq: int = 1024) -> PTConfig:
    return PTConfig(n_tracks=4, n_layers=16, block_depth=4, d_model=1024, n_heads=16, n_kv_heads=16,
                    head_dim=64, d_ffn=4096, vocab=32000, max_batch=max_batch, max_seq=max_seq,
                    dtype=PT_BF16)


def config_large(max_batch: int = 8, max_seq: int = 4096, n_kv_heads: int = 16) -> PTConfig:
    return PTConfig(n_tracks=8, n_layers=32, block_depth=8, d_model=2048, n_heads=16,
                    n_kv_heads=n_kv_heads, head_dim=128, d_ffn=8192, vocab=32000,
                    max_batch=max_batch, max_seq=max_seq, dtype=PT_BF16)


def config_large_moe(max_batch: int = 8, max_seq: int = 4096, n_kv_heads: int = 16) -> PTConfig:
    """PT-MoE variant of the Large PT workload (Section 2.2 and the Conclusion: MoE sparsity inside every track).  The
    paper gives no PT-MoE shapes: here every track's feed-forward network becomes 8 experts of width 4096 with 2
    experts per token, so a token activates the same 8192 hidden units as in the dense Large model while the
    feed-forward parameters grow fourfold (about 56 B parameters, 112 GB in bf16)."""
    return dataclasses.replace(config_large(max_batch, max_seq, n_kv_heads), d_ffn=4096, n_experts=8, top_k=2)


def config_paper30b(block_depth: int = 8, max_batch: int = 1, max_seq: int = 4096) -> PTConfig:
    """Shape of the paper's 30B PT model (Section 3.1, Table 1): 8 tracks, 48 layers, 8 query heads and 1 KV
    head per track, track block depth 2, 4 or 8.  The paper prints no widths: per-track d_model 3072,
    head_dim 128 and FFN 8192 are chosen here so that the 8 tracks hold about 31.7 B parameters."""
    return PTConfig(n_tracks=8, n_layers=48, block_depth=block_depth, d_model=3072, n_heads=8,
                    n_kv_heads=1, head_dim=128, d_ffn=8192, vocab=32000, max_batch=max_batch,
                    max_seq=max_seq, dtype=PT_BF16)


def config_dense30b(max_batch: int = 1, max_seq: int = 4096) -> PTConfig:
    """Dense counterpart of config_paper30b with the same layer, head and KV-head totals (Table 1: 48 layers,
    64 query heads, 8 KV heads) and a matched parameter count (31.4 B): one track that merges after every
    layer is a standard decoder.  Width 8192 and FFN 20480 are this build's choice."""
    return PTConfig(n_tracks=1, n_layers=48, block_depth=1, d_model=8192, n_heads=64, n_kv_heads=8,
                    head_dim=128, d_ffn=20480, vocab=32000, max_batch=max_batch, max_seq=max_seq,
                    dtype=PT_BF16)


def config_share(max_batch: int = 2, max_seq: int = 4096) -> PTConfig:
    return PTConfig(n_tracks=1, n_layers=8, block_depth=8, d_model=8192, n_heads=64, n_kv_heads=64,
                    head_dim=128, d_ffn=28672, vocab=0, max_batch=max_batch, max_seq=max_seq,
                    dtype=PT_BF16)
