#!/usr/bin/env python3
"""Benchmark of the PT forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--legs LIST]

A step is one whole prefill pass (embedding, L layers of T tracks with a merge every D layers, final norm
and head on the last positions) over one batch of the "Large PT" workload, the largest single-GPU
configuration: T=8 tracks, 32 layers/track, merge every 8 layers, d_model 2048, 16 heads x 128, FFN 8192,
vocab 32000, bf16, batch 8 x 4096 uniform-random tokens (seed 3), weights N(0, 0.02) (seed 3).  Inputs are
resident in HBM before the timed region.  One JSON line is printed on stdout:

  value         prefill tokens/s of that workload (whole job, one GPU)
  roofline      its dominant kernel class (gate/up GEMM with the SwiGLU epilogue): algorithmic FLOPs of one
                launch / its mean duration, measured with HIP events around exactly those launches inside
                the timed region, against the dense bf16 MFMA peak
  decode        the decode legs (ms per step, algorithmic bytes per step against the HBM peak, and a roofline
                for the decode-attention kernel from in-run events): Large PT at batch 64, context 4096 with
                2 KV heads per track (as written, with 16 KV heads, the cache would need 550 GB), Large PT as
                written at batch 16, and one GPU's share of the wide model at batch 64, context 8192
  legs          the other workloads on the same kernels: share prefill 2 x 4096, the share-shape block-end merge
                (8 x [8192, 8192] bf16 through pt_track_merge), Mid PT prefill 4 x 1024, Mid PT
                decode (batch 32, 2048-token prompts, 128 steps) and the throughput mode (Mid PT, batch 256 of
                mixed lengths: ragged prefill and decode)
  cpu_baseline  the CPU oracle (numpy float64) on a stated, bounded sample of the headline workload

--legs selects a subset (comma list of moe-prefill, moe-decode, large-prefill, large-decode-gqa, large-decode-mha, share-prefill,
share-decode, share-merge, mid-prefill, mid-decode, throughput, cpu; default all), which is how the per-kernel profiles under
profiles/ are taken.  Other modes: --paper-sweep (batch-1 latency over input lengths), --ceilings (sustained
MFMA and HBM-read rates of two bare loops), --tile-clocks (where the time of a prefill GEMM tile goes: the tile
kernel built from the same source with shader-clock stamps).
"""
import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0

ALL_LEGS = ["large-prefill", "large-decode-gqa", "large-decode-mha", "share-prefill", "share-decode", "share-merge",
            "mid-prefill", "mid-decode", "throughput", "moe-prefill", "moe-decode", "cpu"]
PREFILL_CLASSES = ["embed", "rmsnorm", "gemm_qkv", "attn_prefill", "gemm_out", "gemm_router", "moe", "gemm_gateup",
                   "gemm_down", "merge", "gemm_head"]
DECODE_CLASSES = ["embed", "rmsnorm", "gemm_qkv", "attn_decode", "gemm_out", "gemm_router", "moe", "gemm_gateup",
                  "gemm_down", "merge", "gemm_head"]
FAMILY_NAMES = {
    "gemm": ["shape-generic", "MFMA tile kernel", "weight-streaming kernel", "matrix-vector kernel"],
    "attn_prefill": ["shape-generic", "flash kernel, LDS key/value tiles", "flash kernel, register operands", ""],
    "attn_decode": ["shape-generic", "matrix-core split-K kernel", "vector split-K kernel", ""],
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def prefill_flops(cfg, B, S, head_rows):
    """Algorithmic FLOPs of one prefill: GEMMs, causal attention at half the dense S^2 work, and the head on
    head_rows rows."""
    T, L, d, f = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn
    hq, hk = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    rows = B * S
    k = cfg.top_k if cfg.n_experts else 1     # PT-MoE: every token runs top_k experts of width d_ffn
    per_class = {
        "gemm_qkv": 2.0 * rows * d * (hq + 2 * hk) * T,
        "gemm_out": 2.0 * rows * hq * d * T,
        "gemm_gateup": 2.0 * rows * k * d * 2 * f * T,
        "gemm_down": 2.0 * rows * k * f * d * T,
        "attn_prefill": 2.0 * S * S * hq * B * T,
    }
    if cfg.n_experts:
        per_class["gemm_router"] = 2.0 * rows * d * cfg.n_experts * T
    total = L * sum(per_class.values()) + 2.0 * head_rows * d * cfg.vocab
    return total, per_class


def decode_bytes(cfg, B, ctx):
    """Algorithmic HBM bytes of one decode step: every weight once, the KV cache once."""
    T, L, d, f = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn
    hq, hk = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    if cfg.n_experts:
        # expected number of distinct experts the B * top_k assignments of a (track, layer) touch, uniform routing
        E = cfg.n_experts
        touched = E * (1.0 - (1.0 - cfg.top_k / E) ** B)
        ffn = touched * 3 * d * f + d * E
    else:
        ffn = 3 * d * f
    weights = T * L * (d * (hq + 2 * hk) + hq * d + ffn) * 2.0
    kv_per_launch = T * B * ctx * 2 * hk * 2.0
    return weights, kv_per_launch * L, kv_per_launch


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def family_report(model, cls):
    """Which kernel family served the launches of a class since the last reset (in-run evidence of the kernel
    behind a roofline figure)."""
    counts = model.pt_profile_paths(cls)
    names = FAMILY_NAMES["gemm" if cls.startswith("gemm") else cls]
    return {names[i]: n for i, n in enumerate(counts) if n}


def traffic_from_profiles(name):
    """HBM-side bytes per launch of a kernel from the rocprofv3 --pmc passes whose summary is kept under
    profiles/ (counters cannot be read inside a timing run).  Returns (bytes or None, provenance)."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None, None
    rec = json.load(open(path))
    return rec.get("traffic_bytes_per_launch"), "profiles/%s (separate rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes)" % name


def hidden_batch(torch, I, seed, B, S, d):
    """[B, S, d] seeded N(0,1) hidden states rounded to bf16 (the recipe of the share workload), on the device.
    Generated per sequence so that the host never holds more than one sequence in float64."""
    out = torch.empty((B, S, d), dtype=torch.float32, device="cuda")
    for b in range(B):
        out[b].copy_(torch.from_numpy(I.make_hidden(seed, b, S, d)))
    return out


def run_prefill_leg(torch, PB, I, name, cfg, B, S, seed, steps, warmup, traffic_file=None):
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    if cfg.vocab:
        tokens = torch.from_numpy(I.make_tokens(seed, B, S, cfg.vocab)).cuda()
        logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        run = lambda: model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
        head_rows = B
    else:
        hid = hidden_batch(torch, I, seed, B, S, cfg.d_model)
        run = lambda: model.pt_prefill(hidden_in=hid, logits_mode=PB.PT_LOGITS_NONE)
        head_rows = 0
    torch.cuda.synchronize()
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    model.pt_profile_reset()
    model.pt_profile_enable(["gemm_gateup"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev[0].record(model.stream)
    for i in range(steps):
        run()
        ev[i + 1].record(model.stream)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    model.pt_sync_status()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    ms_dom, n_dom = model.pt_profile_read("gemm_gateup")
    fam = family_report(model, "gemm_gateup")
    total_flops, per_class = prefill_flops(cfg, B, S, head_rows)
    ms_step = dt / steps * 1e3
    achieved = per_class["gemm_gateup"] / (ms_dom / n_dom * 1e-3) / 1e12
    traffic, tsrc = traffic_from_profiles(traffic_file) if traffic_file else (None, None)
    roofline = {"bound": "mfma", "kernel": "gemm_gateup: gate/up GEMM with the SwiGLU epilogue, one launch = one "
                "layer of all %d tracks" % cfg.n_tracks, "kernel_family": fam,
                "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic, "traffic_source": tsrc,
                "launches": n_dom, "avg_launch_ms": ms_dom / n_dom, "flops_per_launch": per_class["gemm_gateup"]}
    # per-class breakdown on extra, untimed steps
    extra = 1 if ms_step > 200 else 2
    model.pt_profile_reset()
    model.pt_profile_enable(PREFILL_CLASSES)
    for _ in range(extra):
        run()
    breakdown = {}
    for c in PREFILL_CLASSES:
        ms, n = model.pt_profile_read(c)
        if n:
            e = {"ms_per_step": ms / extra, "launches_per_step": n // extra}
            if c in per_class:
                e["tflops"] = per_class[c] / (ms / n * 1e-3) / 1e12
            if c.startswith("gemm") or c == "attn_prefill":
                e["kernel_family"] = family_report(model, c)
            breakdown[c] = e
    model.pt_profile_enable([])
    model.close()
    del model
    torch.cuda.empty_cache()
    tflops = total_flops / (ms_step * 1e-3) / 1e12
    rec = {"workload": name, "batch": B, "seq_len": S, "steps": steps, "warmup": warmup, "ms_per_step": ms_step,
           "ms_per_step_median": median(per), "ms_per_step_min": min(per),
           "tokens_per_s": B * S / (ms_step * 1e-3),
           "end_to_end": {"algorithmic_TFLOP": total_flops / 1e12, "TFLOP/s": tflops,
                          "frac_of_mfma_peak": tflops / MFMA_BF16_PEAK_TFLOPS},
           "roofline": roofline, "kernel_breakdown": breakdown}
    log("%s: %.2f ms/step, %.0f tokens/s, %.0f TFLOP/s (%.1f%% of bf16 MFMA peak); gate/up GEMM %.0f TFLOP/s" % (
        name, ms_step, rec["tokens_per_s"], tflops, 100 * tflops / MFMA_BF16_PEAK_TFLOPS, achieved))
    return rec


def run_decode_leg(torch, PB, I, name, cfg, B, ctx, seed, steps, warmup, token_seed=None, traffic_file=None,
                   note=None):
    """KV cache filled by a real prefill of B prompts of ctx tokens, then `warmup` untimed and `steps` timed
    KV-cached decode steps (greedy: each step feeds the argmax of the previous one)."""
    model = PB.PTModel(cfg)
    model.pt_init_weights(seed)
    t0 = time.perf_counter()
    if cfg.vocab:
        tokens = torch.from_numpy(I.make_tokens(seed if token_seed is None else token_seed, B, ctx, cfg.vocab)).cuda()
        logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
        nxt = torch.empty((B,), dtype=torch.int32, device="cuda")
        model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
        PB.pt_argmax(logits, nxt, model.stream)
        step = lambda: model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
        del tokens
    else:
        hid = hidden_batch(torch, I, seed, B, ctx, cfg.d_model)
        model.pt_prefill(hidden_in=hid, logits_mode=PB.PT_LOGITS_NONE)
        del hid
        x = torch.from_numpy(I.make_hidden(seed + 100, 0, B, cfg.d_model)).cuda()
        hout = torch.empty((B, cfg.d_model), dtype=torch.float32, device="cuda")
        step = lambda: model.pt_decode_step(hidden_in=x, want_logits=False, hidden_out=hout)
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    model.pt_profile_reset()
    model.pt_profile_enable(["attn_decode"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record(model.stream)
    for i in range(steps):
        step()
        ev[i + 1].record(model.stream)
    torch.cuda.synchronize()
    model.pt_sync_status()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    ms_attn, n_attn = model.pt_profile_read("attn_decode")
    fam = family_report(model, "attn_decode")
    wbytes, kv_step, kv_launch = decode_bytes(cfg, B, ctx + warmup + steps // 2)
    gbs = kv_launch / (ms_attn / n_attn * 1e-3) / 1e9
    med = median(per)
    traffic, tsrc = traffic_from_profiles(traffic_file) if traffic_file else (None, None)
    # per-class breakdown on extra, untimed steps
    extra = 4
    model.pt_profile_reset()
    model.pt_profile_enable(DECODE_CLASSES)
    for _ in range(extra):
        step()
    breakdown = {}
    for c in DECODE_CLASSES:
        ms, n = model.pt_profile_read(c)
        if n:
            e = {"ms_per_step": ms / extra, "launches_per_step": n // extra}
            if c.startswith("gemm") or c == "attn_decode":
                e["kernel_family"] = family_report(model, c)
            breakdown[c] = e
    model.pt_profile_enable([])
    model.close()
    del model
    torch.cuda.empty_cache()
    rec = {"workload": name, "batch": B, "context": ctx, "steps": steps, "warmup": warmup,
           "ms_per_step_median": med, "ms_per_step_min": min(per), "ms_per_token": med / B,
           "prompt_prefill_s": prefill_s,
           "step_bytes_GB": (wbytes + kv_step) / 1e9, "step_GBs": (wbytes + kv_step) / (med * 1e-3) / 1e9,
           "step_frac_of_hbm_peak": (wbytes + kv_step) / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "roofline": {"bound": "hbm", "kernel": "attn_decode: split-K decode attention, one launch = one layer's "
                        "K and V^T of all tracks, sequences and heads", "kernel_family": fam, "achieved": gbs,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                        "traffic_source": tsrc, "launches": n_attn, "avg_launch_ms": ms_attn / n_attn,
                        "bytes_per_launch": kv_launch},
           "kernel_breakdown": breakdown}
    if note:
        rec["note"] = note
    log("%s: %.3f ms/step median, %.0f GB/s of algorithmic bytes (%.1f%% of HBM peak), attention %.0f GB/s" % (
        name, med, rec["step_GBs"], 100 * rec["step_frac_of_hbm_peak"], gbs))
    return rec


def run_throughput_leg(torch, PB, I, steps):
    """Throughput-mode shape of the paper's serving tables (Section 3.3, Tables 5 and 8: maximum batch 256, inputs
    of mixed lengths) on the Mid PT model: 256 sequences of 64 .. 2048 tokens (seeded, uniform) in one ragged
    prefill, then KV-cached decode steps at batch 256, every sequence at its own position."""
    import numpy as np
    B = 256
    cfg = I.config_mid(max_batch=B, max_seq=2048 + steps + 8)
    lens = [int(x) for x in 64 + I.make_tokens(6, 1, B, 2048 - 64 + 1)[0]]
    n = sum(lens)
    padded = sum((x + 63) // 64 * 64 for x in lens)
    tok = I.make_tokens(6, 1, n, cfg.vocab, stream=1)[0]
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    tokens = torch.from_numpy(tok).cuda()
    logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
    nxt = torch.empty((B,), dtype=torch.int32, device="cuda")
    run = lambda: model.pt_prefill_ragged(lens, tokens=tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
    run()
    torch.cuda.synchronize()
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        run()
    torch.cuda.synchronize()
    pre_s = (time.perf_counter() - t0) / reps
    PB.pt_argmax(logits, nxt, model.stream)
    step = lambda: model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
    for _ in range(2):
        step()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record(model.stream)
    for i in range(steps):
        step()
        ev[i + 1].record(model.stream)
    torch.cuda.synchronize()
    model.pt_sync_status()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]
    med = median(per)
    # algorithmic work: GEMMs on the real tokens, causal attention over each sequence's own length
    T, L, d, f = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn
    hq, hk = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    flops = T * L * (2.0 * n * (d * (hq + 2 * hk) + hq * d + 3 * d * f) + 2.0 * sum(x * x for x in lens) * hq) + 2.0 * B * d * cfg.vocab
    ctx = sum(lens) / B + 2 + steps / 2
    wbytes, kv_step, _ = decode_bytes(cfg, B, ctx)
    fam = {c: family_report(model, c) for c in ("attn_prefill", "attn_decode", "gemm_gateup")}
    model.close()
    del model
    torch.cuda.empty_cache()
    rec = {"workload": "Mid PT, throughput mode: batch 256, input lengths uniform in 64..2048 (seed 6), ragged prefill "
                       "then %d decode steps" % steps,
           "batch": B, "tokens": n, "padded_rows": padded, "min_len": min(lens), "max_len": max(lens),
           "prefill_ms": pre_s * 1e3, "prefill_tokens_per_s": n / pre_s, "prefill_TFLOP/s": flops / pre_s / 1e12,
           "prefill_frac_of_mfma_peak": flops / pre_s / 1e12 / MFMA_BF16_PEAK_TFLOPS,
           "decode_ms_per_step_median": med, "decode_ms_per_step_min": min(per), "decode_tokens_per_s": B / (med * 1e-3),
           "decode_step_GBs": (wbytes + kv_step) / (med * 1e-3) / 1e9,
           "decode_frac_of_hbm_peak": (wbytes + kv_step) / (med * 1e-3) / 1e9 / HBM_PEAK_GBS, "kernel_family": fam}
    log("throughput mode (batch 256, %d tokens): prefill %.1f ms, %.0f tokens/s (%.1f%% of MFMA peak); decode %.2f ms/step, "
        "%.0f tokens/s (%.1f%% of HBM peak)" % (n, rec["prefill_ms"], rec["prefill_tokens_per_s"], 100 * rec["prefill_frac_of_mfma_peak"],
                                                med, rec["decode_tokens_per_s"], 100 * rec["decode_frac_of_hbm_peak"]))
    return rec


def run_merge_leg(torch, PB, I, reps=50):
    """The block-end merge at the one-GPU share shape: own hidden state plus 7 peers', seeded N(0,1) bf16 tensors of
    [8192 tokens, 8192], through pt_track_merge (T reads and one write of 134 MB each)."""
    tokens, d, n = 8192, 8192, 8
    tracks = [torch.from_numpy(I.make_hidden(4, i, tokens, d)).cuda().to(torch.bfloat16) for i in range(n)]
    out = torch.empty_like(tracks[0])
    for _ in range(5):
        PB.pt_track_merge(tracks, 1.0, out=out)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
    ev[0].record()
    for i in range(reps):
        PB.pt_track_merge(tracks, 1.0, out=out)
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = [ev[i].elapsed_time(ev[i + 1]) for i in range(reps)]
    nbytes = (n + 1) * tokens * d * 2.0
    med = median(per)
    rec = {"workload": "track merge of 8 x [8192, 8192] bf16 (one-GPU share, block end)", "reps": reps,
           "ms_median": med, "ms_min": min(per), "bytes": nbytes, "GBs": nbytes / (med * 1e-3) / 1e9,
           "frac_of_hbm_peak": nbytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBS}
    log("share merge 8 x [8192, 8192] bf16: %.3f ms, %.0f GB/s (%.1f%% of HBM peak)" % (med, rec["GBs"], 100 * rec["frac_of_hbm_peak"]))
    del tracks, out
    torch.cuda.empty_cache()
    return rec


def run_cpu_baseline(I):
    """The oracle, as it stands, on a bounded sample of the headline workload: sequence 0 of the 8 x 4096 batch
    through the first layer of each of the 8 tracks and the merge that follows (1/32 of the model's depth; all
    32 layers have the same shape), and the final norm + head on the last position.  The full-depth rate is the
    measured layer time scaled by 32 plus the head time; the scaling is stated in `sample`."""
    import numpy as np
    from oracle import pt_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    full = I.config_large(max_batch=1, max_seq=4096)
    cfg = dataclasses.replace(full, n_layers=1, block_depth=1)
    t0 = time.perf_counter()
    W = I.make_weights(cfg, 3)
    log("cpu_baseline: weights of one layer of 8 tracks generated in %.1f s" % (time.perf_counter() - t0))
    tokens = I.make_tokens(3, 8, 4096, cfg.vocab)[:1]
    body = dataclasses.replace(cfg, vocab=0)
    x = W["embed"][tokens[0]][None].astype(np.float64)            # [1, S, d]: the embedding input of Algorithm 1
    st = O.PTState(body, 1, 4096)
    t0 = time.perf_counter()
    out = O.pt_prefill(body, W, st, hidden_in=x)
    t_layer = time.perf_counter() - t0
    t0 = time.perf_counter()
    O.logits_from_hidden(cfg, W, out["hidden"][:, -1])
    t_head = time.perf_counter() - t0
    t_full = t_layer * full.n_layers + t_head
    return {"value": 4096 / t_full, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "sequence 0 (4096 tokens) of the Large PT batch through layer 0 of all 8 tracks and the merge "
                      "after it: %.1f s; final norm and head on the last position: %.3f s; value = 4096 tokens / "
                      "(32 layers x %.1f s + %.3f s), i.e. the measured one-layer time scaled to the model's 32 "
                      "equal layers, not a measurement of the full depth" % (t_layer, t_head, t_layer, t_head)}


def run_tile_clocks(torch):
    """Where the time of a 256 x 256 tile of the prefill GEMM goes at the Large shapes (libpt_ceilings.so,
    pt_gemm_tile_clocks: the forward library's tile kernel compiled from the same source with shader-clock
    stamps): entry to first MFMA, K loop, barrier, epilogue, per wavefront, averaged over the launch."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2602_07306_amd", "libpt_ceilings.so")
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2602_07306_amd.build`" % path)
    L = C.CDLL(path)
    vp, i32 = C.c_void_p, C.c_int32
    L.pt_gemm_tile_clocks.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, C.c_size_t, vp,
                                      C.POINTER(C.c_double)]
    st = torch.cuda.current_stream().cuda_stream
    gen = torch.Generator(device="cuda")
    gen.manual_seed(11)
    T, M = 8, 8 * 4096
    shapes = [("gate/up (SwiGLU epilogue, folded-norm row factors)", 2, 16384, 2048),
              ("down (residual epilogue with the folded-norm outputs)", 1, 2048, 8192),
              ("out-projection (residual epilogue with the folded-norm outputs)", 1, 2048, 2048),
              ("out-projection shape, fp32 store only", 0, 2048, 2048)]
    out = []
    for name, epi, N, K in shapes:
        a = torch.randn((T, M, K), generator=gen, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        w = (0.02 * torch.randn((T, N, K), generator=gen, device="cuda", dtype=torch.float32)).to(torch.bfloat16)
        o = torch.zeros((T, M, N), dtype=torch.float32, device="cuda")
        tiles = T * (M // 256) * (N // 256)
        stamps = torch.zeros(tiles * 32, dtype=torch.int64, device="cuda")
        rf = torch.ones((T, M), dtype=torch.float32, device="cuda") if epi == 2 else None
        ob = torch.empty((T, M, N), dtype=torch.bfloat16, device="cuda") if epi == 1 else None
        gain = torch.ones((T, N), dtype=torch.float32, device="cuda") if epi == 1 else None
        sums = torch.empty((T, M, N // 128), dtype=torch.float32, device="cuda") if epi == 1 else None
        res = (C.c_double * 10)()
        ptr = lambda t: t.data_ptr() if t is not None else None
        rc = L.pt_gemm_tile_clocks(epi, a.data_ptr(), w.data_ptr(), o.data_ptr(), ptr(ob), ptr(rf), ptr(gain), ptr(sums),
                                   M, N, K, T, stamps.data_ptr(), stamps.numel() * 8, st, res)
        if rc != 0:
            raise RuntimeError("pt_gemm_tile_clocks failed with %d" % rc)
        r = list(res)
        ms = r[9]
        rec = {"gemm": name, "M": M, "N": N, "K": K, "batch": T, "ms_per_launch": ms,
               "TFLOPs": 2.0 * M * N * K * T / (ms * 1e-3) / 1e12,
               "clocks": {"entry_to_first_mfma": r[0], "k_loop": r[1], "barrier": r[2], "epilogue": r[3], "tile": r[4]},
               "tile_us": r[5] / 1e3, "shader_clock_GHz": r[4] / r[5], "stamped_launch_span_ms": r[6] / 1e6,
               "tiles": int(r[7]), "tiles_per_cu": r[7] / 256.0, "k_loop_clocks_at_mfma_rate": 2.0 * 256 * 256 * K / 4069.0}
        out.append(rec)
        log("%s: %.2f ms/launch (%.0f TFLOP/s); per tile %.1f k clocks = first MFMA after %.1f k + K loop %.1f k "
            "(%.1f k at the MFMA rate) + barrier %.1f k + epilogue %.1f k; clock %.2f GHz"
            % (name, ms, rec["TFLOPs"], r[4] / 1e3, r[0] / 1e3, r[1] / 1e3, rec["k_loop_clocks_at_mfma_rate"] / 1e3,
               r[2] / 1e3, r[3] / 1e3, rec["shader_clock_GHz"]))
        del a, w, o, stamps, rf, ob, gain, sums
        torch.cuda.empty_cache()
    return out


def run_ceilings(torch, I):
    """Sustained rates of bare loops on this GPU (libpt_ceilings.so, include/pt_ceilings.h): the matrix-core loop
    on all-zero operands and on operands distributed like the model's (N(0,1) activations against N(0,0.02)
    weights), a streaming read, a streaming copy and an LDS read loop.  Context for the roofline fractions: the
    published peaks are what a kernel is priced against, these are what the chip holds under load."""
    import ctypes as C
    import numpy as np
    path = os.path.join(ROOT, "paper_2602_07306_amd", "libpt_ceilings.so")
    if not os.path.exists(path):
        raise ImportError("%s is missing: build it with `python -m paper_2602_07306_amd.build`" % path)
    L = C.CDLL(path)
    vp, i32, dbl = C.c_void_p, C.c_int32, C.c_double
    L.pt_ceiling_mfma_bf16.argtypes = [vp, vp, i32, i32, i32, vp, C.POINTER(dbl)]
    L.pt_ceiling_hbm_read.argtypes = [vp, C.c_size_t, vp, i32, vp, C.POINTER(dbl)]
    L.pt_ceiling_hbm_copy.argtypes = [vp, vp, C.c_size_t, i32, vp, C.POINTER(dbl)]
    L.pt_ceiling_lds_read.argtypes = [vp, i32, i32, i32, vp, dbl, C.POINTER(dbl), C.POINTER(dbl)]
    st = torch.cuda.current_stream().cuda_stream
    sink = torch.zeros(1 << 20, dtype=torch.float32, device="cuda")
    x = I.make_hidden(9, 0, 8192, 1024).reshape(-1, 8, 8)        # 8 Mi values: 16-byte entries in groups of 8
    x[:, 4:, :] *= 0.02                                          # entries 4..7 of a group feed the weight operand
    ops = {"zeros": torch.zeros(1 << 23, dtype=torch.bfloat16, device="cuda"),
           "model-like (N(0,1) x N(0,0.02))": torch.from_numpy(I.round_to_dtype(x.reshape(-1), I.PT_BF16)).cuda().to(torch.bfloat16)}
    out = {"mfma_bf16_TFLOPs": {}, "published": {"mfma_bf16_TFLOPs": MFMA_BF16_PEAK_TFLOPS, "hbm_GBs": HBM_PEAK_GBS}}

    def check(rc):
        if rc != 0:
            raise RuntimeError("libpt_ceilings call failed with %d" % rc)

    for name, buf in ops.items():
        for wps in (1, 2):
            v = dbl()
            check(L.pt_ceiling_mfma_bf16(buf.data_ptr(), sink.data_ptr(), wps, 40000, 5, st, C.byref(v)))
            out["mfma_bf16_TFLOPs"]["%s, %d wavefront(s) per SIMD" % (name, wps)] = v.value
            log("MFMA loop, %s, %d wavefront(s) per SIMD: %.0f TFLOP/s" % (name, wps, v.value))
    nbytes = 8 << 30
    src = torch.ones(nbytes // 4, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    v = dbl()
    check(L.pt_ceiling_hbm_read(src.data_ptr(), nbytes, sink.data_ptr(), 10, st, C.byref(v)))
    out["hbm_read_GBs"] = v.value
    check(L.pt_ceiling_hbm_copy(src.data_ptr(), dst.data_ptr(), nbytes, 10, st, C.byref(v)))
    out["hbm_copy_GBs_read_plus_write"] = v.value
    log("streaming read %.0f GB/s, copy %.0f GB/s (read + write)" % (out["hbm_read_GBs"], v.value))
    out["lds_read"] = {}
    for wps in (1, 2, 4):
        bpc, g = dbl(), dbl()
        check(L.pt_ceiling_lds_read(sink.data_ptr(), wps, 20000, 3, st, 2.4, C.byref(bpc), C.byref(g)))
        out["lds_read"]["%d wavefront(s) per SIMD" % wps] = {"bytes_per_clk_per_cu_at_2.4GHz": bpc.value, "GBs": g.value}
        log("LDS ds_read_b128, %d wavefront(s) per SIMD: %.0f B/clk/CU at 2.4 GHz" % (wps, bpc.value))
    return out


def run_paper_sweep(args, torch, PB, I):
    """Latency-mode shape of the paper's serving tables (Section 3.3: batch 1, input lengths 1024 ... 63488,
    30B-shaped PT model, track block depth 1, 2, 4, 8, and the dense model of matched size) on one GPU with all 8
    tracks resident: time to first token
    = one prefill, time per output token = mean of the KV-cached decode steps that follow.  Widths are this
    build's choice (inputs.config_paper30b); the paper's numbers are for 8 GPUs and are context only."""
    lengths = [int(x) for x in args.sweep_lengths.split(",")]
    out = []
    for D in [int(x) for x in args.sweep_depths.split(",")]:   # 0 = the dense model of matched size
        max_seq = max(lengths) + args.sweep_decode_steps + 8
        cfg = (I.config_paper30b(block_depth=D, max_batch=1, max_seq=max_seq) if D > 0
               else I.config_dense30b(max_batch=1, max_seq=max_seq))
        model = PB.PTModel(cfg)
        model.pt_init_weights(5)
        logits = torch.empty((1, cfg.vocab), dtype=torch.float32, device="cuda")
        nxt = torch.zeros((1,), dtype=torch.int32, device="cuda")
        warm = torch.from_numpy(I.make_tokens(5, 1, 256, cfg.vocab)).cuda()
        model.pt_prefill(warm, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
        torch.cuda.synchronize()
        for S in lengths:
            tokens = torch.from_numpy(I.make_tokens(5, 1, S, cfg.vocab)).cuda()
            model.pt_reset()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
            torch.cuda.synchronize()
            ttft = time.perf_counter() - t0
            PB.pt_argmax(logits, nxt, model.stream)
            model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.sweep_decode_steps):
                model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
            torch.cuda.synchronize()
            tpot = (time.perf_counter() - t0) / args.sweep_decode_steps
            flops, _ = prefill_flops(cfg, 1, S, 1)
            wbytes, kv_step, _ = decode_bytes(cfg, 1, S + 1 + args.sweep_decode_steps // 2)
            rec = {"model": "PT 8 tracks" if D > 0 else "dense", "block_depth": D if D > 0 else None, "input_len": S, "ttft_ms": ttft * 1e3, "tpot_ms": tpot * 1e3,
                   "prefill_TFLOPs": flops / ttft / 1e12, "decode_GBs": (wbytes + kv_step) / tpot / 1e9,
                   "merges_per_forward": cfg.n_layers // cfg.block_depth if D > 0 else 0}
            log("paper sweep D=%d input %6d: TTFT %9.2f ms (%.0f TFLOP/s), TPOT %6.2f ms (%.0f GB/s)" % (
                D, S, rec["ttft_ms"], rec["prefill_TFLOPs"], rec["tpot_ms"], rec["decode_GBs"]))
            out.append(rec)
            del tokens
        model.close()
        del model
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10, help="timed prefill steps of the headline workload")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--legs", default="all", help="comma list of " + ", ".join(ALL_LEGS) + "; default all")
    ap.add_argument("--decode-steps", type=int, default=16, help="timed decode steps of the large decode legs")
    ap.add_argument("--mid-decode-steps", type=int, default=128)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy kernel (reference for the HBM byte counters of a rocprofv3 --pmc pass)")
    ap.add_argument("--tile-clocks", action="store_true",
                    help="per-phase shader clocks of the prefill GEMM's 256x256 tile at the Large shapes")
    ap.add_argument("--ceilings", action="store_true",
                    help="instead of the benchmark: sustained MFMA / HBM / LDS rates of bare loops (one JSON line)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="instead of the benchmark: TTFT / TPOT at batch 1 over input lengths for the "
                         "30B-shaped PT model at track block depth 2, 4, 8 (one JSON line)")
    ap.add_argument("--sweep-lengths", default="1024,4096,16384,63488")
    ap.add_argument("--sweep-depths", default="0,1,2,4,8",
                    help="track block depths of the sweep; 0 = the dense model of matched parameter count")
    ap.add_argument("--sweep-decode-steps", type=int, default=32)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the PT forward on ONE GPU (all tracks resident); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    legs = ALL_LEGS if args.legs == "all" else [x for x in args.legs.split(",") if x]
    for x in legs:
        if x not in ALL_LEGS:
            print("bench.py: unknown leg %r" % x, file=sys.stderr)
            sys.exit(2)
    import torch
    from paper_2602_07306_amd import binding as PB
    from paper_2602_07306_amd import inputs as I
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    PB.lib()
    if args.copy_calibration:
        # the plain copy kernel of known size that the HBM byte counters are scaled by: 1 GiB read, 1 GiB written
        import ctypes as C
        L = C.CDLL(os.path.join(ROOT, "paper_2602_07306_amd", "libpt_ceilings.so"))
        L.pt_ceiling_hbm_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32, C.c_void_p, C.POINTER(C.c_double)]
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        v = C.c_double()
        if L.pt_ceiling_hbm_copy(src.data_ptr(), dst.data_ptr(), 1 << 30, 2, torch.cuda.current_stream().cuda_stream, C.byref(v)) != 0:
            raise RuntimeError("copy calibration failed")
        torch.cuda.synchronize()
        del src, dst
    if args.tile_clocks:
        print(json.dumps({"gemm_tile_clocks": run_tile_clocks(torch), "n_gpus": 1, "dtype": "bf16", "data": "synthetic"}),
              flush=True)
        return
    if args.ceilings:
        print(json.dumps({"ceilings": run_ceilings(torch, I), "n_gpus": 1, "dtype": "bf16", "data": "synthetic"}), flush=True)
        return
    if args.paper_sweep:
        print(json.dumps({"paper_sweep": run_paper_sweep(args, torch, PB, I), "n_gpus": 1, "dtype": "bf16",
                          "data": "synthetic",
                          "workload": "30B-shaped PT model (8 tracks x 48 layers, 8 query heads / 1 KV head per "
                                      "track, head_dim 128, per-track d_model 3072, FFN 8192), batch 1"}), flush=True)
        return

    large = None
    decode, other = {}, {}
    if "large-prefill" in legs:
        large = run_prefill_leg(torch, PB, I, "Large PT prefill 8 x 4096", I.config_large(max_batch=8, max_seq=4096),
                                8, 4096, 3, args.steps, args.warmup, "large_prefill_gateup_traffic.json")
    if "large-decode-gqa" in legs:
        decode["large_2_kv_heads"] = run_decode_leg(
            torch, PB, I, "Large PT decode, 2 KV heads per track, batch 64, context 4096",
            I.config_large(max_batch=64, max_seq=4096 + 64, n_kv_heads=2), 64, 4096, 3, args.decode_steps, 2,
            traffic_file="large_decode_attn_traffic.json",
            note="capacity deviation: as written (16 KV heads per track) batch 64 x context 4096 needs a 550 GB cache")
    if "large-decode-mha" in legs:
        decode["large_as_written_batch_16"] = run_decode_leg(
            torch, PB, I, "Large PT decode, 16 KV heads per track (as written), batch 16, context 4096",
            I.config_large(max_batch=16, max_seq=4096 + 64), 16, 4096, 3, args.decode_steps, 2,
            note="capacity deviation: batch 16 is the largest that fits one GPU's HBM; the workload states batch 64")
    if "share-prefill" in legs:
        other["share_prefill"] = run_prefill_leg(
            torch, PB, I, "one-GPU share prefill 2 x 4096", I.config_share(max_batch=2, max_seq=4096), 2, 4096, 4,
            max(args.steps, 10), args.warmup)
    if "share-decode" in legs:
        decode["share"] = run_decode_leg(
            torch, PB, I, "one-GPU share decode, batch 64, context 8192",
            I.config_share(max_batch=64, max_seq=8192 + 64), 64, 8192, 4, args.decode_steps, 2,
            traffic_file="share_decode_traffic.json")
    if "share-merge" in legs:
        other["share_merge"] = run_merge_leg(torch, PB, I)
    if "mid-prefill" in legs:
        other["mid_prefill"] = run_prefill_leg(
            torch, PB, I, "Mid PT prefill 4 x 1024", I.config_mid(max_batch=4, max_seq=1024), 4, 1024, 1,
            max(args.steps, 20), args.warmup, "mid_prefill_gateup_traffic.json")
    if "mid-decode" in legs:
        other["mid_decode"] = run_decode_leg(
            torch, PB, I, "Mid PT decode: batch 32, 2048-token prompts, %d KV-cached steps" % args.mid_decode_steps,
            I.config_mid(max_batch=32, max_seq=2048 + args.mid_decode_steps + 64), 32, 2048, 1,
            args.mid_decode_steps, 2, token_seed=2, traffic_file="mid_decode_attn_traffic.json")
    if "throughput" in legs:
        other["throughput_mode"] = run_throughput_leg(torch, PB, I, 16)
    if "moe-prefill" in legs:
        other["moe_prefill"] = run_prefill_leg(
            torch, PB, I, "Large PT-MoE prefill 8 x 4096 (8 experts of width 4096 per track and layer, top-2)",
            I.config_large_moe(max_batch=8, max_seq=4096), 8, 4096, 3, max(args.steps // 2, 3), 1)
    if "moe-decode" in legs:
        decode["large_moe"] = run_decode_leg(
            torch, PB, I, "Large PT-MoE decode, 2 KV heads per track, batch 64, context 4096",
            I.config_large_moe(max_batch=64, max_seq=4096 + 64, n_kv_heads=2), 64, 4096, 3, args.decode_steps, 2)
    cpu = run_cpu_baseline(I) if "cpu" in legs else None

    cfg = I.config_large()
    out = {
        "metric": "PT prefill tokens/s", "value": large["tokens_per_s"] if large else None, "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": large["ms_per_step"] if large else None,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "Large PT prefill: T=8 tracks, 32 layers/track, merge every 8 layers, d_model 2048, "
                               "16 heads x 128, FFN 8192, vocab 32000, batch 8 x 4096 tokens, seed 3",
                   "n_tracks": cfg.n_tracks, "n_layers": cfg.n_layers, "block_depth": cfg.block_depth,
                   "batch": 8, "seq_len": 4096},
        "legs_run": legs,
    }
    if large:
        out.update({"ms_per_step_median": large["ms_per_step_median"], "ms_per_step_min": large["ms_per_step_min"],
                    "end_to_end": large["end_to_end"], "roofline": large["roofline"],
                    "kernel_breakdown": large["kernel_breakdown"]})
    out["decode"] = decode or None
    out["legs"] = other or None
    out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
