"""Host-side logic of the C-ABI library: it loads without a GPU, exports every symbol that
include/pt.h declares, validates configurations and reports arena sizes.  No kernel is launched."""
import ctypes as C
import dataclasses
import os
import re

import pytest

from paper_2602_07306_amd import binding as PB
from paper_2602_07306_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pt_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    L = PB.lib()
    names = declared_functions()
    assert {"pt_init_weights", "pt_prefill", "pt_decode_step", "pt_track_merge"} <= set(names)
    for n in names:
        assert hasattr(L, n), n
    assert sorted(PB.EXPORTS) == names


def test_dynamic_symbol_table_holds_only_the_declared_functions():
    """The library is linked with hidden visibility and an export list: no internal launcher, tuning
    variable or kernel stub is reachable from outside."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", PB.LIB_PATH], capture_output=True, text=True, check=True).stdout
    exported = sorted(line.split()[-1] for line in out.splitlines() if line.strip())
    assert exported == declared_functions()


def test_benchmark_library_exports_what_its_header_declares():
    """libpt_ceilings.so (bare-loop ceilings and the stamped GEMM tile) loads without a GPU and exports the functions
    of include/pt_ceilings.h."""
    text = open(os.path.join(ROOT, "include", "pt_ceilings.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(pt_[a-z_0-9]+)\s*\(", text)))
    assert "pt_ceiling_mfma_bf16" in names and "pt_gemm_tile_clocks" in names
    L = C.CDLL(os.path.join(ROOT, "paper_2602_07306_amd", "libpt_ceilings.so"))
    for n in names:
        assert hasattr(L, n), n


def test_tuning_knobs_are_validated():
    assert PB.lib().pt_set_tuning(99, 0) == PB.PT_ERR_INVALID_ARGUMENT
    assert "knob" in PB.pt_last_error()
    PB.pt_set_tuning(PB.PT_TUNE_GEMM_TILE_CONFIG, -1)
    PB.pt_set_tuning(PB.PT_TUNE_SKINNY_PLAN, 0)


def test_config_struct_matches_the_header():
    text = open(os.path.join(ROOT, "include", "pt.h")).read()
    body = text[text.index("typedef struct pt_config {"):text.index("} pt_config;")]
    fields = re.findall(r"^\s*(?:int32_t|float)\s+([a-z_]+);", body, flags=re.M)
    assert fields == [f[0] for f in PB.pt_config._fields_]


@pytest.mark.parametrize("change,code", [
    (dict(n_layers=5), PB.PT_ERR_INVALID_CONFIG),          # L % D != 0: Algorithm 1's output undefined
    (dict(n_kv_heads=3), PB.PT_ERR_INVALID_CONFIG),
    (dict(n_tracks=0), PB.PT_ERR_INVALID_CONFIG),
    (dict(n_tracks=17), PB.PT_ERR_INVALID_CONFIG),
    (dict(head_dim=30), PB.PT_ERR_INVALID_CONFIG),
    (dict(d_model=100), PB.PT_ERR_INVALID_CONFIG),
    (dict(d_ffn=100), PB.PT_ERR_INVALID_CONFIG),
    (dict(vocab=511), PB.PT_ERR_INVALID_CONFIG),
    (dict(dtype=7), PB.PT_ERR_INVALID_CONFIG),
    (dict(max_seq=0), PB.PT_ERR_INVALID_CONFIG),
    (dict(block_depth=0), PB.PT_ERR_INVALID_CONFIG),
])
def test_invalid_configs_are_rejected(change, code):
    cfg = dataclasses.replace(I.config_tiny(), **change)
    with pytest.raises(PB.PTError) as e:
        PB.pt_query_bytes(cfg)
    assert e.value.code == code and str(e.value)


def test_arena_sizes():
    cfg = I.config_mid()
    w, kv, ws = PB.pt_query_bytes(cfg)
    T, L, d, f, V = 4, 16, 1024, 4096, 32000
    params = T * L * (4 * d * d + 3 * d * f) + 2 * V * d
    rope_table = 1024 * 64 * 4          # max_seq x head_dim/2 x (cos, sin), kept with the weights
    assert params * 2 <= w <= params * 2 + T * L * 2 * d * 4 + d * 4 + rope_table + 64 * 1024
    tokens = 4 * 1024
    assert kv >= 2 * T * L * tokens * 16 * 64 * 2
    assert kv <= 2.2 * T * L * tokens * 16 * 64 * 2
    assert ws >= T * tokens * d * 4
    # fp32 storage doubles the weights
    w32, _, _ = PB.pt_query_bytes(dataclasses.replace(cfg, dtype=I.PT_F32))
    assert 1.9 * w < w32 < 2.1 * w
    # the MHA cache of the large configuration at decode batch 64 exceeds one GPU's 288 GB
    _, kv_large, _ = PB.pt_query_bytes(I.config_large(max_batch=64, max_seq=4224))
    assert kv_large > 288e9


def _create(cfg, wb, kb, sb, wptr=0x1000000, kptr=0x2000000, sptr=0x3000000):
    h = C.c_void_p()
    c = PB.to_c_config(cfg)
    rc = PB.lib().pt_create(C.byref(c), wptr, wb, kptr, kb, sptr, sb, None, C.byref(h))
    return rc, h


def test_create_checks_arenas_without_touching_them():
    cfg = I.config_tiny()
    w, kv, ws = PB.pt_query_bytes(cfg)
    rc, h = _create(cfg, w, kv, ws)          # fake, never dereferenced device addresses
    assert rc == 0 and h.value
    L = PB.lib()
    assert L.pt_merge_count(h) == 0 and L.pt_seq_len(h) == 0
    # forward before weights exist, decode before prefill, capacity: all host-side refusals
    assert L.pt_prefill(h, 0x10, None, 1, 1, 8, PB.PT_LOGITS_NONE, None, None) == PB.PT_ERR_BAD_STATE
    assert L.pt_decode_step(h, 0x10, None, 1, 1, None, None, None) == PB.PT_ERR_BAD_STATE
    assert L.pt_prefill(h, 0x10, None, 1, 2, 8, PB.PT_LOGITS_NONE, None, None) == PB.PT_ERR_CAPACITY
    assert L.pt_prefill(h, 0x10, None, 1, 1, 65, PB.PT_LOGITS_NONE, None, None) == PB.PT_ERR_CAPACITY
    assert "max_seq" in PB.pt_last_error()
    assert L.pt_prefill(h, 0x10, None, 1, 1, 8, PB.PT_LOGITS_LAST, None, None) == PB.PT_ERR_NULL_POINTER
    assert L.pt_set_kernel_path(h, 9) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_set_weight(h, 99, 0, 0, 0x10) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_set_weight(h, PB.PT_W_Q, 2, 0, 0x10) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_destroy(h) == 0
    assert _create(cfg, w - 1, kv, ws)[0] == PB.PT_ERR_ARENA_TOO_SMALL
    assert _create(cfg, w, kv - 1, ws)[0] == PB.PT_ERR_ARENA_TOO_SMALL
    assert _create(cfg, w, kv, ws - 1)[0] == PB.PT_ERR_ARENA_TOO_SMALL
    assert _create(cfg, w, kv, ws, wptr=0)[0] == PB.PT_ERR_NULL_POINTER
    assert _create(cfg, w, kv, ws, kptr=0x2000010)[0] == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_destroy(None) == PB.PT_ERR_NULL_POINTER


def test_track_merge_argument_checks():
    L = PB.lib()
    arr = (C.c_void_p * 2)(0x1000, 0x2000)
    assert L.pt_track_merge(arr, 0, 4, 8, PB.PT_F32, 1.0, 0x3000, None) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_track_merge(arr, 17, 4, 8, PB.PT_F32, 1.0, 0x3000, None) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_track_merge(arr, 2, 4, 12, PB.PT_F32, 1.0, 0x3000, None) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_track_merge(arr, 2, 4, 8, 5, 1.0, 0x3000, None) == PB.PT_ERR_INVALID_ARGUMENT
    assert L.pt_track_merge(arr, 2, 4, 8, PB.PT_F32, 1.0, None, None) == PB.PT_ERR_NULL_POINTER
    assert L.pt_track_merge(arr, 2, 4, 8, PB.PT_F32, 1.0, 0x3004, None) == PB.PT_ERR_INVALID_ARGUMENT
    bad = (C.c_void_p * 2)(0x1000, None)
    assert L.pt_track_merge(bad, 2, 4, 8, PB.PT_F32, 1.0, 0x3000, None) == PB.PT_ERR_NULL_POINTER
    assert L.pt_track_merge(arr, 2, 0, 8, PB.PT_F32, 1.0, 0x3000, None) == 0      # empty input: no launch
