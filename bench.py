#!/usr/bin/env python3
"""Benchmark of the PT forward hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--skip-decode] [--skip-cpu]

A step is one whole prefill pass (embedding, L layers of T tracks with a merge every D layers,
final norm and head on the last positions) over one batch of the "Mid PT prefill" workload:
T=4 tracks, 16 layers/track, merge every 4 layers, d_model 1024, 16 heads x 64, FFN 4096,
vocab 32000, bf16, batch 4 x 1024 uniform-random tokens (seed 1), weights N(0, 0.02) (seed 1).
Inputs are resident in HBM before the timed region.  One JSON line is printed on stdout:

  value      prefill tokens/s (whole job, one GPU)
  roofline   the dominant kernel (gate/up GEMM with the SwiGLU epilogue): algorithmic FLOPs of one
             launch / its mean duration, measured with HIP events around exactly those launches
             inside the timed region, against the dense bf16 MFMA peak
  decode     the "Mid PT decode" workload (same model, batch 32, 2048-token prompts, 128 KV-cached
             steps): ms per step and the decode-attention kernel's KV bytes / duration against HBM peak
  cpu_baseline  the CPU oracle (numpy float64) timed on one of the four sequences of the same
             prefill workload on this host's cores
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0   # MI355X dense bf16
HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def prefill_flops(cfg, B, S, head_rows):
    """Algorithmic FLOPs of one prefill: GEMMs, causal attention at half the dense S^2 work,
    and the head on head_rows rows."""
    T, L, d, f = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn
    hq, hk = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    rows = B * S
    per_class = {
        "gemm_qkv": 2.0 * rows * d * (hq + 2 * hk) * T,
        "gemm_out": 2.0 * rows * hq * d * T,
        "gemm_gateup": 2.0 * rows * d * 2 * f * T,
        "gemm_down": 2.0 * rows * f * d * T,
        "attn_prefill": 2.0 * S * S * hq * B * T,
    }
    total = L * sum(per_class.values()) + 2.0 * head_rows * d * cfg.vocab
    return total, per_class


def decode_bytes(cfg, B, ctx):
    """Algorithmic HBM bytes of one decode step: every weight once, the KV cache once."""
    T, L, d, f = cfg.n_tracks, cfg.n_layers, cfg.d_model, cfg.d_ffn
    hq, hk = cfg.n_heads * cfg.head_dim, cfg.n_kv_heads * cfg.head_dim
    weights = T * L * (d * (hq + 2 * hk) + hq * d + 3 * d * f) * 2.0
    kv_per_launch = T * B * ctx * 2 * hk * 2.0
    return weights, kv_per_launch * L, kv_per_launch


def run_prefill(args, torch, PB, I):
    cfg = I.config_mid(max_batch=4, max_seq=1024)
    B, S = 4, 1024
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    tokens = torch.from_numpy(I.make_tokens(1, B, S, cfg.vocab)).cuda()
    logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    for _ in range(args.warmup):
        model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
    torch.cuda.synchronize()
    model.pt_profile_reset()
    model.pt_profile_enable(["gemm_gateup"])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_dom, n_dom = model.pt_profile_read("gemm_gateup")
    total_flops, per_class = prefill_flops(cfg, B, S, B)
    ms_step = dt / args.steps * 1e3
    achieved = per_class["gemm_gateup"] / (ms_dom / n_dom * 1e-3) / 1e12
    traffic = None   # HBM-side bytes per launch from the rocprofv3 --pmc passes kept under profiles/
    tpath = os.path.join(ROOT, "profiles", "mid_prefill_gateup_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")
    roofline = {"bound": "mfma", "kernel": "gemm_dl_kernel<256, 256, 4, 2, EPI_SWIGLU> (gate/up GEMM)",
                "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / MFMA_BF16_PEAK_TFLOPS, "traffic": traffic,
                "launches": n_dom, "avg_launch_ms": ms_dom / n_dom,
                "flops_per_launch": per_class["gemm_gateup"]}
    # per-class breakdown on two extra, untimed steps
    model.pt_profile_reset()
    classes = ["embed", "rmsnorm", "gemm_qkv", "attn_prefill", "gemm_out", "gemm_gateup", "gemm_down",
               "merge", "gemm_head"]
    model.pt_profile_enable(classes)
    for _ in range(2):
        model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
    breakdown = {}
    for c in classes:
        ms, n = model.pt_profile_read(c)
        if n:
            e = {"ms_per_step": ms / 2, "launches_per_step": n // 2}
            if c in per_class:
                e["tflops"] = per_class[c] / (ms / n * 1e-3) / 1e12
            breakdown[c] = e
    model.pt_profile_enable([])
    model.close()
    del model
    torch.cuda.empty_cache()
    return {"cfg": cfg, "B": B, "S": S, "ms_step": ms_step, "tokens_per_s": B * S / (ms_step * 1e-3),
            "total_flops": total_flops, "roofline": roofline, "breakdown": breakdown}


def run_decode(args, torch, PB, I):
    B, prompt, steps = 32, 2048, args.decode_steps
    cfg = I.config_mid(max_batch=B, max_seq=prompt + steps + 64)
    model = PB.PTModel(cfg)
    model.pt_init_weights(1)
    tokens = torch.from_numpy(I.make_tokens(2, B, prompt, cfg.vocab)).cuda()
    logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
    nxt = torch.empty((B,), dtype=torch.int32, device="cuda")
    t0 = time.perf_counter()
    model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_LAST, logits_out=logits)
    nxt.copy_(logits.argmax(dim=-1).to(torch.int32))
    torch.cuda.synchronize()
    prefill_s = time.perf_counter() - t0
    model.pt_profile_reset()
    model.pt_profile_enable(["attn_decode"])
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
    ev[0].record()
    for i in range(steps):
        model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = sorted(ev[i].elapsed_time(ev[i + 1]) for i in range(steps))
    ms_attn, n_attn = model.pt_profile_read("attn_decode")
    wbytes, kv_step, kv_launch = decode_bytes(cfg, B, prompt + steps // 2)
    gbs = kv_launch / (ms_attn / n_attn * 1e-3) / 1e9
    med = per[len(per) // 2]
    traffic = None   # HBM-side bytes per launch from the rocprofv3 --pmc passes kept under profiles/
    tpath = os.path.join(ROOT, "profiles", "mid_decode_attn_traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get("traffic_bytes_per_launch")
    out = {"workload": "Mid PT decode: batch 32, 2048-token prompts, %d KV-cached steps" % steps,
           "ms_per_step_median": med, "ms_per_step_min": per[0], "ms_per_token": med / B,
           "prompt_prefill_s": prefill_s,
           "step_bytes_GB": (wbytes + kv_step) / 1e9, "step_GBs": (wbytes + kv_step) / (med * 1e-3) / 1e9,
           "step_frac_of_hbm_peak": (wbytes + kv_step) / (med * 1e-3) / 1e9 / HBM_PEAK_GBS,
           "roofline": {"bound": "hbm", "kernel": "attn_decode_tiled_kernel<64>", "achieved": gbs,
                        "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS, "traffic": traffic,
                        "launches": n_attn, "avg_launch_ms": ms_attn / n_attn,
                        "bytes_per_launch": kv_launch}}
    model.close()
    del model
    torch.cuda.empty_cache()
    return out


def run_cpu_baseline(I):
    """The oracle, as it stands, on sequence 0 of the prefill workload (sequences are independent)."""
    import numpy as np
    from oracle import pt_oracle as O
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    cfg = I.config_mid(max_batch=1, max_seq=1024)
    t0 = time.perf_counter()
    W = I.make_weights(cfg, 1)
    log("cpu_baseline: weights generated in %.1f s" % (time.perf_counter() - t0))
    tokens = I.make_tokens(1, 4, 1024, cfg.vocab)[:1]
    st = O.PTState(cfg, 1, 1024)
    t0 = time.perf_counter()
    O.pt_prefill(cfg, W, st, tokens=tokens)
    dt = time.perf_counter() - t0
    return {"value": 1024 / dt, "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "sequence 0 of the 4 x 1024-token batch (1024 tokens, full model), %.1f s" % dt}


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
            nxt.copy_(logits.argmax(dim=-1).to(torch.int32))
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


def run_large_configs(args, torch, PB, I):
    """The two large BASELINE configurations on the same kernels: Large PT (T=8, L=32, D=8, d=2048, 16 heads x
    128, FFN 8192) and one GPU's share of the wide model (one track, 8 layers, d=8192, 64 heads x 128, FFN
    28672).  Prefill at the stated batch; decode at the stated batch and context, except that Large's decode
    as written (MHA, batch 64, context 4096) needs a 550 GB KV cache: it runs with 2 KV heads per track at
    batch 64 and as written (MHA) at batch 16."""
    classes = ["rmsnorm", "gemm_qkv", "attn_prefill", "attn_decode", "gemm_out", "gemm_gateup", "gemm_down", "merge"]
    out = []

    def breakdown(model, nsteps):
        r = {}
        for c in classes:
            ms, n = model.pt_profile_read(c)
            if n:
                r[c] = ms / nsteps
        return r

    def prefill_case(name, cfg, B, S, seed):
        model = PB.PTModel(cfg)
        model.pt_init_weights(seed)
        if cfg.vocab:
            kw = dict(tokens=torch.from_numpy(I.make_tokens(seed, B, S, cfg.vocab)).cuda(),
                      logits_mode=PB.PT_LOGITS_LAST,
                      logits_out=torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda"))
            head_rows = B
        else:
            kw = dict(tokens=None, hidden_in=torch.randn((B, S, cfg.d_model), device="cuda"),
                      logits_mode=PB.PT_LOGITS_NONE)
            head_rows = 0
        total, _ = prefill_flops(cfg, B, S, head_rows)
        tokens = kw.pop("tokens")
        run = lambda: model.pt_prefill(tokens, **kw)
        run()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(2):
            run()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / 2
        model.pt_profile_reset()
        model.pt_profile_enable(classes)
        run()
        rec = {"workload": name, "kind": "prefill", "batch": B, "seq_len": S, "ms": dt * 1e3,
               "tokens_per_s": B * S / dt, "TFLOP/s": total / dt / 1e12,
               "frac_of_mfma_peak": total / dt / 1e12 / MFMA_BF16_PEAK_TFLOPS, "kernel_ms": breakdown(model, 1)}
        log("%s: %.1f ms, %.0f tokens/s, %.0f TFLOP/s (%.1f%% of peak)" % (
            name, rec["ms"], rec["tokens_per_s"], rec["TFLOP/s"], 100 * rec["frac_of_mfma_peak"]))
        out.append(rec)
        model.close()
        del model, kw, tokens
        torch.cuda.empty_cache()

    def decode_case(name, cfg, B, ctx, seed):
        model = PB.PTModel(cfg)
        model.pt_init_weights(seed)
        if cfg.vocab:
            tokens = torch.from_numpy(I.make_tokens(seed, B, ctx, cfg.vocab)).cuda()
            model.pt_prefill(tokens, logits_mode=PB.PT_LOGITS_NONE)
            nxt = torch.zeros((B,), dtype=torch.int32, device="cuda")
            logits = torch.empty((B, cfg.vocab), dtype=torch.float32, device="cuda")
            step = lambda: model.pt_decode_step(nxt, logits_out=logits, argmax_out=nxt, want_argmax=True)
            del tokens
        else:
            hid = torch.randn((B, ctx, cfg.d_model), device="cuda")
            model.pt_prefill(hidden_in=hid, logits_mode=PB.PT_LOGITS_NONE)
            del hid
            x = torch.randn((B, cfg.d_model), device="cuda")
            step = lambda: model.pt_decode_step(hidden_in=x, want_logits=False, want_hidden=True)
        for _ in range(2):
            step()
        torch.cuda.synchronize()
        n = 8
        t0 = time.perf_counter()
        for _ in range(n):
            step()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / n
        wb, kvstep, kvl = decode_bytes(cfg, B, ctx + 6)
        model.pt_profile_reset()
        model.pt_profile_enable(classes)
        step()
        br = breakdown(model, 1)
        ms_attn, n_attn = model.pt_profile_read("attn_decode")
        rec = {"workload": name, "kind": "decode", "batch": B, "context": ctx, "ms_per_step": dt * 1e3,
               "step_bytes_GB": (wb + kvstep) / 1e9, "step_GBs": (wb + kvstep) / dt / 1e9,
               "frac_of_hbm_peak": (wb + kvstep) / dt / 1e9 / HBM_PEAK_GBS,
               "attention_GBs": kvl / (ms_attn / n_attn * 1e-3) / 1e9, "kernel_ms": br}
        log("%s: %.2f ms/step, %.0f GB/s (%.1f%% of peak), attention %.0f GB/s" % (
            name, rec["ms_per_step"], rec["step_GBs"], 100 * rec["frac_of_hbm_peak"], rec["attention_GBs"]))
        out.append(rec)
        model.close()
        del model
        torch.cuda.empty_cache()

    which = args.large_configs.split(",")
    if "large-prefill" in which:
        prefill_case("Large PT prefill 8 x 4096", I.config_large(max_batch=8, max_seq=4096), 8, 4096, 3)
    if "share-prefill" in which:
        prefill_case("one-GPU share prefill 2 x 4096", I.config_share(max_batch=2, max_seq=4096), 2, 4096, 4)
    if "large-decode-gqa" in which:
        decode_case("Large PT decode, 2 KV heads per track, batch 64, context 4096",
                    I.config_large(max_batch=64, max_seq=4096 + 64, n_kv_heads=2), 64, 4096, 3)
    if "large-decode-mha" in which:
        decode_case("Large PT decode, MHA, batch 16, context 4096",
                    I.config_large(max_batch=16, max_seq=4096 + 64), 16, 4096, 3)
    if "share-decode" in which:
        decode_case("one-GPU share decode, batch 64, context 8192",
                    I.config_share(max_batch=64, max_seq=8192 + 64), 64, 8192, 4)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--skip-decode", action="store_true")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--decode-steps", type=int, default=128,
                    help="KV-cached decode steps of the decode leg (a counter pass uses a handful)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy three times (reference for the HBM byte counters)")
    ap.add_argument("--paper-sweep", action="store_true",
                    help="instead of the benchmark: TTFT / TPOT at batch 1 over input lengths for the "
                         "30B-shaped PT model at track block depth 2, 4, 8 (one JSON line)")
    ap.add_argument("--large-configs", default="",
                    help="instead of the benchmark: comma list of large-prefill, share-prefill, large-decode-gqa, "
                         "large-decode-mha, share-decode (one JSON line)")
    ap.add_argument("--sweep-lengths", default="1024,4096,16384,63488")
    ap.add_argument("--sweep-depths", default="0,1,2,4,8",
                    help="track block depths of the sweep; 0 = the dense model of matched parameter count")
    ap.add_argument("--sweep-decode-steps", type=int, default=32)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the PT forward on ONE GPU (all tracks resident); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_07306_amd import binding as PB
    from paper_2602_07306_amd import inputs as I
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    PB.lib()
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.large_configs:
        print(json.dumps({"large_configs": run_large_configs(args, torch, PB, I), "n_gpus": 1, "dtype": "bf16",
                          "data": "synthetic"}), flush=True)
        return
    if args.paper_sweep:
        print(json.dumps({"paper_sweep": run_paper_sweep(args, torch, PB, I), "n_gpus": 1, "dtype": "bf16",
                          "data": "synthetic",
                          "workload": "30B-shaped PT model (8 tracks x 48 layers, 8 query heads / 1 KV head per "
                                      "track, head_dim 128, per-track d_model 3072, FFN 8192), batch 1"}), flush=True)
        return
    pre = run_prefill(args, torch, PB, I)
    log("prefill: %.3f ms/step, %.0f tokens/s, %.1f%% of bf16 MFMA peak end to end" % (
        pre["ms_step"], pre["tokens_per_s"],
        100 * pre["total_flops"] / (pre["ms_step"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS))
    dec = None if args.skip_decode else run_decode(args, torch, PB, I)
    if dec:
        log("decode: %.3f ms/step median, attention %.0f GB/s" % (dec["ms_per_step_median"], dec["roofline"]["achieved"]))
    cpu = None if args.skip_cpu else run_cpu_baseline(I)
    cfg = pre["cfg"]
    e2e_tflops = pre["total_flops"] / (pre["ms_step"] * 1e-3) / 1e12
    out = {
        "metric": "PT prefill tokens/s", "value": pre["tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": pre["ms_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "Mid PT prefill: T=4 tracks, 16 layers/track, merge every 4 layers, d_model 1024, "
                               "16 heads x 64, FFN 4096, vocab 32000, batch 4 x 1024 tokens, seed 1",
                   "n_tracks": cfg.n_tracks, "n_layers": cfg.n_layers, "block_depth": cfg.block_depth,
                   "batch": pre["B"], "seq_len": pre["S"]},
        "end_to_end": {"algorithmic_TFLOP": pre["total_flops"] / 1e12, "TFLOP/s": e2e_tflops,
                       "frac_of_mfma_peak": e2e_tflops / MFMA_BF16_PEAK_TFLOPS},
        "roofline": pre["roofline"],
        "kernel_breakdown": pre["breakdown"],
        "decode": dec,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
