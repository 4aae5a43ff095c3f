"""Shared helpers of the GPU parity tests."""
import dataclasses

import numpy as np

from oracle import pt_oracle as O
from paper_2602_07306_amd import inputs as I

FP32_TOL = 1e-4   # max relative error on logits, fp32 path
BF16_TOL = 2e-2   # bf16 path


def rel_err(got, ref) -> float:
    """max |got - ref| / max |ref| over the tensor (per-element relative error is undefined
    near zero logits)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.max(np.abs(got - ref)) / max(np.max(np.abs(ref)), 1e-30))


def row_rel_err(got, ref) -> float:
    """The worst row of the same measure taken row by row (rows = the last axis):
    max over rows of max |got_row - ref_row| / max |ref_row|.  A wrong row of small magnitude
    cannot hide under the largest entry of the tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    num = np.max(np.abs(got - ref), axis=-1)
    den = np.maximum(np.max(np.abs(ref), axis=-1), 1e-30)
    return float(np.max(num / den))


def assert_close(got, ref, tol, what=""):
    """Both error measures within tol: over the whole tensor and for every row."""
    e, er = rel_err(got, ref), row_rel_err(got, ref)
    assert e <= tol and er <= tol, "%s: relative error %.3g (tensor), %.3g (worst row) exceeds %g" % (what, e, er, tol)
    return e, er


GEMM_CLASSES = ("gemm_qkv", "gemm_out", "gemm_gateup", "gemm_down", "gemm_head")
PATH_CLASSES = GEMM_CLASSES + ("attn_prefill", "attn_decode")


def path_counts(model):
    """{kernel class: launches per kernel family} since the last pt_profile_reset."""
    return {c: model.pt_profile_paths(c) for c in PATH_CLASSES}


def argmax_agrees(got_logits, ref_logits, tol) -> bool:
    """ids must match on every row whose oracle top-2 gap exceeds tol * max|row|."""
    ref = np.asarray(ref_logits, dtype=np.float64)
    got = np.asarray(got_logits)
    top2 = np.sort(ref, axis=-1)[:, -2:]
    decided = (top2[:, 1] - top2[:, 0]) > tol * np.max(np.abs(ref), axis=-1)
    return bool(np.all(np.argmax(got, -1)[decided] == np.argmax(ref, -1)[decided]))


def oracle_prefill(cfg, W, tokens=None, hidden_in=None, max_seq=None, taps=True):
    if tokens is not None:
        B, S = tokens.shape
    else:
        B, S = hidden_in.shape[-3], hidden_in.shape[-2]
    st = O.PTState(cfg, B, max_seq or cfg.max_seq)
    out = O.pt_prefill(cfg, W, st, tokens=tokens, hidden_in=hidden_in, collect_taps=taps)
    return out, st


def small_bf16_config(**kw) -> I.PTConfig:
    base = dict(n_tracks=2, n_layers=4, block_depth=2, d_model=256, n_heads=4, n_kv_heads=4,
                head_dim=64, d_ffn=512, vocab=1024, max_batch=2, max_seq=256, dtype=I.PT_BF16)
    base.update(kw)
    return I.PTConfig(**base)
