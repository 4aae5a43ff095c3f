"""Thin ctypes binding of libpt.so (include/pt.h).  Argument marshalling only: every step of the
forward pass runs in the library's HIP kernels.  torch is used for device memory and streams.

The module fails loudly when the library is missing; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

from .inputs import PT_BF16, PT_F32, PTConfig

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpt.so")

PT_LOGITS_NONE, PT_LOGITS_LAST, PT_LOGITS_ALL = 0, 1, 2
PT_FAMILY_GENERIC, PT_FAMILY_COUNT = 0, 4
PT_TUNE_GEMM_TILE_CONFIG, PT_TUNE_SKINNY_PLAN, PT_TUNE_FOLD_RMSNORM, PT_TUNE_ATTN_PREFILL = 0, 1, 2, 3
PT_PATH_AUTO, PT_PATH_GENERIC = 0, 1
PT_W_EMBED, PT_W_HEAD, PT_W_Q, PT_W_K, PT_W_V, PT_W_O, PT_W_G, PT_W_U, PT_W_D, PT_W_G1, PT_W_G2, PT_W_GF, PT_W_ROUTER = range(1, 14)
WEIGHT_IDS = {"embed": PT_W_EMBED, "head": PT_W_HEAD, "wq": PT_W_Q, "wk": PT_W_K, "wv": PT_W_V,
              "wo": PT_W_O, "wg": PT_W_G, "wu": PT_W_U, "wd": PT_W_D, "g1": PT_W_G1, "g2": PT_W_G2,
              "gf": PT_W_GF, "wr": PT_W_ROUTER}


def pt_expert_layer(layer: int, expert: int) -> int:
    """PT_EXPERT_LAYER of include/pt.h: the `layer` argument that addresses expert `expert`'s WG / WU / WD."""
    return layer | ((expert + 1) << 12)

PT_OK = 0
PT_ERR_INVALID_CONFIG, PT_ERR_NULL_POINTER, PT_ERR_ARENA_TOO_SMALL, PT_ERR_CAPACITY = -1, -2, -3, -4
PT_ERR_BAD_STATE, PT_ERR_HIP, PT_ERR_INVALID_ARGUMENT = -5, -6, -7

EXPORTS = [
    "pt_query_bytes", "pt_create", "pt_destroy", "pt_init_weights", "pt_set_weight", "pt_get_weight",
    "pt_prefill", "pt_decode_step", "pt_track_merge", "pt_set_taps", "pt_set_kernel_path", "pt_reset",
    "pt_merge_count", "pt_seq_len", "pt_last_error", "pt_profile_enable", "pt_profile_read",
    "pt_profile_reset", "pt_profile_paths", "pt_sync_status", "pt_set_tuning", "pt_argmax", "pt_decode_step_static", "pt_prefill_ragged", "pt_seq_lens",
    "pt_set_moe_routes",
]

KERNEL_CLASSES = ["embed", "rmsnorm", "gemm_qkv", "attn_prefill", "attn_decode", "gemm_out",
                  "gemm_gateup", "gemm_down", "merge", "gemm_head", "other", "gemm_router", "moe"]


class pt_config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_tracks", "n_layers", "block_depth", "d_model", "n_heads", "n_kv_heads", "head_dim",
        "d_ffn", "vocab", "max_batch", "max_seq", "dtype")] + [
        (n, C.c_float) for n in ("merge_scale", "rms_eps", "rope_theta", "init_std")] + [
        (n, C.c_int32) for n in ("n_experts", "top_k")]


class PTError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__("libpt error %d: %s" % (code, msg))
        self.code = code


_lib = None


def lib() -> C.CDLL:
    """Loads libpt.so (built by ``python -m paper_2602_07306_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with `python -m paper_2602_07306_amd.build` "
                          "(there is no fallback path)" % LIB_PATH)
    L = C.CDLL(LIB_PATH)
    vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
    cfgp = C.POINTER(pt_config)
    L.pt_query_bytes.argtypes = [cfgp, C.POINTER(sz), C.POINTER(sz), C.POINTER(sz)]
    L.pt_create.argtypes = [cfgp, vp, sz, vp, sz, vp, sz, vp, C.POINTER(vp)]
    L.pt_destroy.argtypes = [vp]
    L.pt_init_weights.argtypes = [vp, C.c_uint64]
    L.pt_set_weight.argtypes = [vp, i32, i32, i32, vp]
    L.pt_get_weight.argtypes = [vp, i32, i32, i32, vp]
    L.pt_prefill.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp]
    L.pt_decode_step.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    L.pt_decode_step_static.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    L.pt_prefill_ragged.argtypes = [vp, vp, vp, i32, i32, C.POINTER(i32), i32, vp, vp]
    L.pt_seq_lens.argtypes = [vp, C.POINTER(i32)]
    L.pt_track_merge.argtypes = [C.POINTER(vp), i32, i64, i32, i32, C.c_float, vp, vp]
    L.pt_set_taps.argtypes = [vp, vp, vp]
    L.pt_set_moe_routes.argtypes = [vp, vp, vp]
    L.pt_set_kernel_path.argtypes = [vp, i32]
    L.pt_reset.argtypes = [vp]
    L.pt_merge_count.argtypes = [vp]
    L.pt_merge_count.restype = i64
    L.pt_seq_len.argtypes = [vp]
    L.pt_seq_len.restype = i32
    L.pt_profile_enable.argtypes = [vp, C.c_uint32]
    L.pt_profile_read.argtypes = [vp, i32, C.POINTER(C.c_double), C.POINTER(i64)]
    L.pt_profile_reset.argtypes = [vp]
    L.pt_profile_paths.argtypes = [vp, i32, C.POINTER(i64)]
    L.pt_sync_status.argtypes = [vp]
    L.pt_set_tuning.argtypes = [i32, i32]
    L.pt_argmax.argtypes = [vp, i32, i32, vp, vp]
    L.pt_last_error.argtypes = []
    L.pt_last_error.restype = C.c_char_p
    for name in EXPORTS:
        if name not in ("pt_merge_count", "pt_seq_len", "pt_last_error"):
            getattr(L, name).restype = C.c_int
    _lib = L
    return L


def _check(rc: int) -> None:
    if rc != 0:
        raise PTError(rc, lib().pt_last_error().decode())


def to_c_config(cfg: PTConfig) -> pt_config:
    return pt_config(cfg.n_tracks, cfg.n_layers, cfg.block_depth, cfg.d_model, cfg.n_heads,
                     cfg.n_kv_heads, cfg.head_dim, cfg.d_ffn, cfg.vocab, cfg.max_batch, cfg.max_seq,
                     cfg.dtype, cfg.merge_scale, cfg.rms_eps, cfg.rope_theta, cfg.init_std, cfg.n_experts,
                     cfg.top_k)


def pt_last_error() -> str:
    return lib().pt_last_error().decode()


def pt_set_tuning(knob: int, value: int) -> None:
    _check(lib().pt_set_tuning(knob, value))


def pt_query_bytes(cfg: PTConfig):
    """(weight_bytes, kv_bytes, workspace_bytes); host only."""
    w, kv, ws = C.c_size_t(), C.c_size_t(), C.c_size_t()
    c = to_c_config(cfg)
    _check(lib().pt_query_bytes(C.byref(c), C.byref(w), C.byref(kv), C.byref(ws)))
    return w.value, kv.value, ws.value


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def pt_track_merge(tracks, scale: float, out=None, stream=None):
    """out = scale * sum(tracks) through the library's merge kernel.  tracks: list of device
    tensors [tokens, d], all float32 or all bfloat16."""
    import torch
    t0 = tracks[0]
    dtype = PT_F32 if t0.dtype == torch.float32 else PT_BF16
    assert all(t.dtype == t0.dtype and t.shape == t0.shape and t.is_contiguous() for t in tracks)
    if out is None:
        out = torch.empty_like(t0)
    arr = (C.c_void_p * len(tracks))(*[t.data_ptr() for t in tracks])
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    tokens, d = (t0.shape[0], t0.shape[1]) if t0.dim() == 2 else (t0.numel() // t0.shape[-1], t0.shape[-1])
    _check(lib().pt_track_merge(arr, len(tracks), tokens, d, dtype, float(scale), out.data_ptr(), st))
    return out


def pt_argmax(logits, out=None, stream=None):
    """out[r] = argmax of logits[r, :] (float32 device tensor [rows, vocab]), lowest id on ties."""
    import torch
    assert logits.dtype == torch.float32 and logits.is_contiguous() and logits.dim() == 2
    if out is None:
        out = torch.empty((logits.shape[0],), dtype=torch.int32, device=logits.device)
    st = torch.cuda.current_stream().cuda_stream if stream is None else getattr(stream, "cuda_stream", stream)
    _check(lib().pt_argmax(logits.data_ptr(), logits.shape[0], logits.shape[1], out.data_ptr(), st))
    return out


class PTModel:
    """A pt_handle plus the torch tensors that back its three arenas."""

    def __init__(self, cfg: PTConfig, device: str = "cuda:0", stream=None):
        import torch
        self.torch = torch
        self.cfg = cfg
        self.device = torch.device(device)
        wb, kb, sb = pt_query_bytes(cfg)
        self.bytes = (wb, kb, sb)
        self._w = torch.empty(wb, dtype=torch.uint8, device=self.device)
        self._kv = torch.empty(kb, dtype=torch.uint8, device=self.device)
        self._ws = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.stream = torch.cuda.current_stream(self.device) if stream is None else stream
        h = C.c_void_p()
        c = to_c_config(cfg)
        _check(lib().pt_create(C.byref(c), self._w.data_ptr(), wb, self._kv.data_ptr(), kb,
                               self._ws.data_ptr(), sb, self.stream.cuda_stream, C.byref(h)))
        self.h = h
        self._taps = None

    def close(self):
        if self.h:
            lib().pt_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- weights -------------------------------------------------------------------------------
    def pt_init_weights(self, seed: int):
        _check(lib().pt_init_weights(self.h, seed))

    def pt_set_weight(self, name: str, track: int, layer: int, array):
        t = self.torch.as_tensor(np.ascontiguousarray(array, dtype=np.float32)).to(self.device)
        _check(lib().pt_set_weight(self.h, WEIGHT_IDS[name], track, layer, t.data_ptr()))
        self.torch.cuda.synchronize(self.device)

    def pt_get_weight(self, name: str, track: int, layer: int, shape):
        t = self.torch.empty(shape, dtype=self.torch.float32, device=self.device)
        _check(lib().pt_get_weight(self.h, WEIGHT_IDS[name], track, layer, t.data_ptr()))
        self.torch.cuda.synchronize(self.device)
        return t.cpu().numpy()

    def load_weights(self, W):
        """Uploads a dict of logical weights (layouts of inputs.make_weights)."""
        cfg = self.cfg
        E = cfg.n_experts
        for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2") + (("wr",) if E > 0 else ()):
            for i in range(cfg.n_tracks):
                for l in range(cfg.n_layers):
                    if E > 0 and name in ("wg", "wu", "wd"):
                        for e in range(E):
                            self.pt_set_weight(name, i, pt_expert_layer(l, e), W[name][i, l, e])
                    else:
                        self.pt_set_weight(name, i, l, W[name][i, l])
        self.pt_set_weight("gf", 0, 0, W["gf"])
        if cfg.vocab > 0:
            self.pt_set_weight("embed", 0, 0, W["embed"])
            self.pt_set_weight("head", 0, 0, W["head"])

    # -- forward -------------------------------------------------------------------------------
    def pt_set_taps(self, rows: int, track_taps: bool = False):
        cfg, torch = self.cfg, self.torch
        taps = torch.zeros((cfg.n_merges, rows, cfg.d_model), dtype=torch.float32, device=self.device)
        tt = (torch.zeros((cfg.n_merges, cfg.n_tracks, rows, cfg.d_model), dtype=torch.float32,
                          device=self.device) if track_taps else None)
        _check(lib().pt_set_taps(self.h, taps.data_ptr(), _ptr(tt)))
        self._taps = (taps, tt)
        return taps, tt

    def pt_clear_taps(self):
        _check(lib().pt_set_taps(self.h, None, None))
        self._taps = None

    def pt_set_moe_routes(self, rows: int, forced=None, observe: bool = True):
        """PT-MoE: observe and / or prescribe the expert selection of later forward calls over `rows` rows.
        forced: int array [n_layers, n_tracks, rows, top_k].  Returns the int32 device tensor that receives the
        selection (or None)."""
        cfg, torch = self.cfg, self.torch
        shape = (cfg.n_layers, cfg.n_tracks, rows, cfg.top_k)
        out = torch.full(shape, -1, dtype=torch.int32, device=self.device) if observe else None
        fin = None
        if forced is not None:
            fin = torch.as_tensor(np.ascontiguousarray(forced, dtype=np.int32)).to(self.device)
            assert tuple(fin.shape) == shape
        _check(lib().pt_set_moe_routes(self.h, _ptr(out), _ptr(fin)))
        self._routes = (out, fin)
        return out

    def pt_clear_moe_routes(self):
        _check(lib().pt_set_moe_routes(self.h, None, None))
        self._routes = None

    def pt_set_kernel_path(self, path: int):
        _check(lib().pt_set_kernel_path(self.h, path))

    def pt_prefill(self, tokens=None, hidden_in=None, logits_mode: int = PT_LOGITS_LAST,
                   want_hidden: bool = False, logits_out=None):
        """tokens: int32 device tensor [B, S]; hidden_in: float32 device tensor [B, S, d] or
        [T, B, S, d].  Returns (logits or None, hidden or None) as device tensors."""
        cfg, torch = self.cfg, self.torch
        if tokens is not None:
            B, S = tokens.shape
            ht = 1
        else:
            ht = 1 if hidden_in.dim() == 3 else hidden_in.shape[0]
            B, S = hidden_in.shape[-3], hidden_in.shape[-2]
        logits = logits_out
        if logits_mode != PT_LOGITS_NONE and logits is None:
            rows = B if logits_mode == PT_LOGITS_LAST else B * S
            logits = torch.empty((rows, cfg.vocab), dtype=torch.float32, device=self.device)
        hidden = torch.empty((B, S, cfg.d_model), dtype=torch.float32, device=self.device) if want_hidden else None
        _check(lib().pt_prefill(self.h, _ptr(tokens), _ptr(hidden_in), ht, B, S, logits_mode,
                                _ptr(logits), _ptr(hidden)))
        return logits, hidden

    def pt_prefill_ragged(self, lens, tokens=None, hidden_in=None, logits_mode: int = PT_LOGITS_LAST,
                          want_hidden: bool = False, logits_out=None):
        """Prefill of sequences of different lengths.  lens: host list of B lengths; tokens: int32 device tensor
        [sum(lens)] (packed); hidden_in: float32 device tensor [sum(lens), d] or [T, sum(lens), d].  Returns
        (logits or None, hidden or None) as device tensors, packed the same way."""
        cfg, torch = self.cfg, self.torch
        B, n = len(lens), int(sum(lens))
        ht = 1
        if tokens is None:
            ht = 1 if hidden_in.dim() == 2 else hidden_in.shape[0]
            assert hidden_in.shape[-2] == n
        else:
            assert tokens.numel() == n
        logits = logits_out
        if logits_mode != PT_LOGITS_NONE and logits is None:
            logits = torch.empty((B if logits_mode == PT_LOGITS_LAST else n, cfg.vocab), dtype=torch.float32, device=self.device)
        hidden = torch.empty((n, cfg.d_model), dtype=torch.float32, device=self.device) if want_hidden else None
        arr = (C.c_int32 * B)(*[int(x) for x in lens])
        _check(lib().pt_prefill_ragged(self.h, _ptr(tokens), _ptr(hidden_in), ht, B, arr, logits_mode, _ptr(logits), _ptr(hidden)))
        return logits, hidden

    def pt_seq_lens(self):
        B = 0
        arr = (C.c_int32 * max(self.cfg.max_batch, 1))()
        _check(lib().pt_seq_lens(self.h, arr))
        return list(arr)

    def pt_decode_step(self, tokens=None, hidden_in=None, want_logits: bool = True,
                       want_hidden: bool = False, want_argmax: bool = False, logits_out=None,
                       argmax_out=None, hidden_out=None, static_scratch: bool = False):
        """One decode step.  static_scratch=True calls pt_decode_step_static (temporaries in the library's
        static device array instead of the workspace arena); the output tensors are still the caller's."""
        cfg, torch = self.cfg, self.torch
        if tokens is not None:
            B, ht = tokens.shape[0], 1
        else:
            ht = 1 if hidden_in.dim() == 2 else hidden_in.shape[0]
            B = hidden_in.shape[-2]
        logits = logits_out
        if logits is None and (want_logits or want_argmax) and cfg.vocab > 0:
            logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device=self.device)
        hidden = hidden_out
        if hidden is None and want_hidden:
            hidden = torch.empty((B, cfg.d_model), dtype=torch.float32, device=self.device)
        amax = argmax_out
        if amax is None and want_argmax:
            amax = torch.empty((B,), dtype=torch.int32, device=self.device)
        fn = lib().pt_decode_step_static if static_scratch else lib().pt_decode_step
        _check(fn(self.h, _ptr(tokens), _ptr(hidden_in), ht, B, _ptr(logits), _ptr(hidden), _ptr(amax)))
        return logits, hidden, amax

    def pt_profile_enable(self, classes):
        """classes: iterable of kernel-class names (KERNEL_CLASSES) to time; empty = off."""
        mask = 0
        for c in classes:
            mask |= 1 << KERNEL_CLASSES.index(c)
        _check(lib().pt_profile_enable(self.h, mask))

    def pt_profile_read(self, cls: str):
        """(total milliseconds, launches) of one kernel class since the last reset."""
        ms, n = C.c_double(), C.c_int64()
        _check(lib().pt_profile_read(self.h, KERNEL_CLASSES.index(cls), C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def pt_profile_reset(self):
        _check(lib().pt_profile_reset(self.h))

    def pt_profile_paths(self, cls: str):
        """Launches of one kernel class per kernel family since the last pt_profile_reset
        (index 0: the shape-generic kernel; see include/pt.h)."""
        counts = (C.c_int64 * PT_FAMILY_COUNT)()
        _check(lib().pt_profile_paths(self.h, KERNEL_CLASSES.index(cls), counts))
        return list(counts)

    def pt_sync_status(self):
        """Synchronises the stream; raises PTError if a forward call met an out-of-range token id."""
        _check(lib().pt_sync_status(self.h))

    def pt_reset(self):
        _check(lib().pt_reset(self.h))

    def pt_merge_count(self) -> int:
        return lib().pt_merge_count(self.h)

    def pt_seq_len(self) -> int:
        return lib().pt_seq_len(self.h)
