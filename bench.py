#!/usr/bin/env python3
"""Benchmark of the decoder-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C3|C4|C5]

One step = one pass of the whole hot path over one micro-batch of synthetic input:
  taw_weight_stage   the other layer's weight chunk is copied owner-store -> staging buffer on a
                     side stream while this step computes (double buffered, two events)
  taw_layer_fwd      on the chunk staged during the previous step
  taw_layer_bwd      weight gradients written into a local fp32 gradient buffer (two, used in turn)
  taw_grad_accum     owner-side aggregation of that buffer into the fp32 gradient shard, on a second
                     side stream: like the weights coming in, the gradients going out are off the
                     compute stream (ready / consumed events per buffer), so the aggregation of step k
                     runs beside the forward pass of step k+1
Inputs are resident in HBM before the timed region.  The metric is model TFLOP/s of the layer's
forward+backward: GEMMs 6 T H (4H+3I) + attention 12 B (S(S+1)/2) H (causal pairs, backward
counted as 2x forward; the score recomputation inside the tiled backward is not credited).

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel (the bf16 MFMA GEMM): algorithmic FLOPs of the step's 12 GEMM
                shapes / their summed launch durations, each launched on its own and measured
                with HIP events on the launch stream, against the 2.5 PFLOP/s dense bf16 MFMA peak
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on a bounded sample
  kernels       per-kernel-class rates measured the same way (attention, bandwidth kernels)
  overlap       step time with and without the staging copy running beside it, and with the
                gradient aggregation on the compute stream instead of its side stream
  recompute     the same step in activation-checkpointing mode (TAW_RECOMPUTE): same model FLOPs
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per GEMM launch (average of the 12 shapes of a step), from two rocprofv3 --pmc runs of this file
# (FETCH_SIZE, WRITE_SIZE; each scaled by what the counter reads for the staging copy kernel, a plain copy of
# known size): profiles/gemm_C2_hbm_traffic.md.  Only measured for the workload named.
GEMM_TRAFFIC_BYTES_PER_LAUNCH = {"C2": 1459.7e6}
# the paper's throughput table (Experiments, Throughput and Memory Usage): micro-batch size per sequence length and
# TawPipe's tokens per GPU per second on its own hardware
PAPER_TABLE_B = {4096: 16, 8192: 8, 16384: 4}
PAPER_TABLE_TAWPIPE = {(1024, 4096): 13629.2, (1024, 8192): 11738.2, (1024, 16384): 8913.7, (2048, 4096): 5040.0,
                       (2048, 8192): 4636.6, (2048, 16384): 4175.7, (4096, 4096): 1567.7, (4096, 8192): 1511.5,
                       (4096, 16384): 1377.6}


def model_flops(cfg):
    T = cfg.B * cfg.S
    gemm = 6.0 * T * cfg.H * (4 * cfg.H + 3 * cfg.I)
    attn = 12.0 * cfg.B * (cfg.S * (cfg.S + 1) / 2.0) * cfg.H
    return gemm, attn


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="C2",
                    help="C2 (default), C3, C4, C5, or a shape of the paper's throughput table as P-<H>-<S> "
                         "(H in 1024/2048/4096, S in 4096/8192/16384; micro-batch size as in that table)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-leg", action="store_true")
    ap.add_argument("--no-recompute-leg", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one device's share of the weight pipeline); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2511_09741_amd.binding as taw
    from paper_2511_09741_amd import inputs as I

    taw.load()
    torch.cuda.set_device(0)
    sweep = None
    if args.workload in I.CONFIGS and args.workload != "C1":
        cfg = I.CONFIGS[args.workload]
    else:
        # the paper's throughput table: 48-layer LLaMA-style models, heads of 128, I = 8H/3 rounded up to 256
        try:
            _, h_, s_ = args.workload.split("-")
            h_, s_ = int(h_), int(s_)
            b_ = PAPER_TABLE_B[s_]
            assert h_ % 128 == 0
        except Exception:
            print(f"bench.py: unknown workload {args.workload!r}", file=sys.stderr)
            sys.exit(2)
        cfg = I.LayerConfig(args.workload, I.BF16, b_, s_, h_, h_ // 128, 128, (8 * h_ // 3 + 255) // 256 * 256)
        sweep = {"layers": 48, "paper_tawpipe_tokens_per_s_per_gpu": PAPER_TABLE_TAWPIPE.get((h_, s_)),
                 "paper_setup": "24 x A800, NVLink + 10GbE, fp16, activation checkpointing (context, not the target)"}
    desc_acc = taw.desc_from_config(cfg, 0)   # bwd overwrites the local gradient buffer
    L = taw.taw_layer_weight_layout(desc_acc)
    P = L["total_elems"]

    def dev_bf16(a):
        return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda().view(torch.bfloat16)

    # ---- synthetic inputs, resident in HBM
    store = []                                # the owner's store: two layers' chunks
    for layer in range(2):
        w = I.make_weights(cfg, seed=0, layer=layer)
        store.append(dev_bf16(I.pack_chunk(w, L, P, cfg.dtype)))
        del w
    x_np, dy_np = I.make_activations(cfg, seed=0)
    x, dy = dev_bf16(x_np), dev_bf16(dy_np)
    del x_np, dy_np
    y, dx = torch.empty_like(x), torch.empty_like(x)
    stage_buf = [torch.empty_like(store[0]) for _ in range(2)]
    g_locals = [torch.zeros(P, dtype=torch.float32, device="cuda") for _ in range(2)]
    g_local = g_locals[0]
    G_shard = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx = torch.empty(taw.taw_layer_ctx_bytes(desc_acc), dtype=torch.uint8, device="cuda")
    desc_rc = taw.desc_from_config(cfg, taw.TAW_RECOMPUTE)      # activation checkpointing (extra leg below)
    ws_bytes_rc = taw.taw_layer_workspace_bytes(desc_rc)
    ws_bytes = taw.taw_layer_workspace_bytes(desc_acc)
    ws = torch.empty(ws_bytes if args.no_recompute_leg else ws_bytes_rc, dtype=torch.uint8, device="cuda")
    rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc_acc, rope)

    compute = torch.cuda.current_stream()
    copy_stream = torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    chunk_bytes = P * 2
    agg_stream = torch.cuda.Stream()
    g_ready = [torch.cuda.Event() for _ in range(2)]
    g_consumed = [torch.cuda.Event() for _ in range(2)]

    state = {"cur": 0, "layer": 0, "n": 0}
    taw.taw_weight_stage(stage_buf[0], store[0], chunk_bytes, copy_stream, None, ready[0])
    consumed[1].record(compute)

    def step(staging=True, agg_side=True):
        cur, nxt = state["cur"], state["cur"] ^ 1
        gi = state["n"] & 1
        state["n"] += 1
        if staging:
            taw.taw_weight_stage(stage_buf[nxt], store[(state["layer"] + 1) & 1], chunk_bytes, copy_stream,
                                 consumed[nxt], ready[nxt])
            compute.wait_event(ready[cur])
        taw.taw_layer_fwd(desc_acc, stage_buf[cur], rope, x, y, ctx, ws, ws_bytes, compute)
        compute.wait_event(g_consumed[gi])      # the aggregation of two steps ago has read this buffer
        taw.taw_layer_bwd(desc_acc, stage_buf[cur], rope, x, dy, ctx, dx, g_locals[gi], ws, ws_bytes, compute)
        consumed[cur].record(compute)
        if agg_side:
            g_ready[gi].record(compute)
            agg_stream.wait_event(g_ready[gi])
            taw.taw_grad_accum(G_shard, g_locals[gi], taw.TAW_F32, P, 1.0, agg_stream)
            g_consumed[gi].record(agg_stream)
        else:
            taw.taw_grad_accum(G_shard, g_locals[gi], taw.TAW_F32, P, 1.0, compute)
        if staging:
            state["cur"] = nxt
            state["layer"] += 1

    def timed(nsteps, staging=True, agg_side=True):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(nsteps):
            step(staging, agg_side)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / nsteps

    for _ in range(args.warmup):
        step()
    ms = timed(args.steps)
    gemm_fl, attn_fl = model_flops(cfg)
    flops = gemm_fl + attn_fl
    value = flops / ms / 1e9            # TFLOP/s

    # ---- staging overlap: same steps with no copy running beside them
    copy_stream.synchronize()
    torch.cuda.synchronize()
    # make both buffers valid, then time without staging
    stage_buf[0].copy_(store[0]); stage_buf[1].copy_(store[1])
    ms_nostage = timed(max(3, args.steps // 2), staging=False)
    ms_stage = timed(max(3, args.steps // 2), staging=True)
    ms_agg_serial = timed(max(3, args.steps // 2), staging=True, agg_side=False)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(copy_stream)
    taw.taw_weight_stage(stage_buf[state["cur"] ^ 1], store[0], chunk_bytes, copy_stream, None, None)
    e1.record(copy_stream)
    torch.cuda.synchronize()
    copy_ms = e0.elapsed_time(e1)
    overlap = {"ms_per_step_staging": round(ms_stage, 4), "ms_per_step_no_staging": round(ms_nostage, 4),
               "delta_frac": round(ms_stage / ms_nostage - 1.0, 4),
               "ms_per_step_aggregation_on_compute_stream": round(ms_agg_serial, 4), "copy_alone_ms": round(copy_ms, 4),
               "copy_alone_GBs": round(2 * chunk_bytes / copy_ms / 1e6, 1)}

    # ---- activation-checkpointing mode: same model FLOPs, the backward re-runs the forward first
    recompute = None
    if not args.no_recompute_leg:
        def step_rc():
            taw.taw_layer_fwd(desc_rc, stage_buf[0], rope, x, y, None, ws, ws_bytes_rc, compute)
            gi = state["n"] & 1
            state["n"] += 1
            compute.wait_event(g_consumed[gi])
            taw.taw_layer_bwd(desc_rc, stage_buf[0], rope, x, dy, None, dx, g_locals[gi], ws, ws_bytes_rc, compute)
            g_ready[gi].record(compute)
            agg_stream.wait_event(g_ready[gi])
            taw.taw_grad_accum(G_shard, g_locals[gi], taw.TAW_F32, P, 1.0, agg_stream)
            g_consumed[gi].record(agg_stream)
        step_rc()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n_rc = max(3, args.steps // 2)
        for _ in range(n_rc):
            step_rc()
        torch.cuda.synchronize()
        ms_rc = (time.perf_counter() - t0) * 1e3 / n_rc
        recompute = {"ms_per_step": round(ms_rc, 4), "model_TFLOPs": round(flops / ms_rc / 1e9, 2),
                     "ctx_bytes_saved": int(taw.taw_layer_ctx_bytes(desc_acc))}

    if sweep is not None and recompute is not None:
        # what one GPU's compute alone allows for the paper's 48-layer model in its training mode
        # (activation checkpointing): tokens of a micro-batch / (48 x this layer's checkpointed step)
        sweep["tokens_per_s_per_gpu_compute_only"] = round(cfg.B * cfg.S / (48 * recompute["ms_per_step"] * 1e-3), 1)

    # ---- per-kernel leg: HIP events on the launch stream around each launch
    def ev_time(fn, reps=5):
        fn()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record(compute)
        for _ in range(reps):
            fn()
        e.record(compute)
        e.synchronize()
        return s.elapsed_time(e) / reps

    roofline, kernels = None, {}
    if not args.no_kernel_leg:
        T, H, Iw, BF = cfg.B * cfg.S, cfg.H, cfg.I, taw.TAW_BF16
        Wqkv, Wo = store[0][L["w_qkv"]:], store[0][L["w_o"]:]
        Wgu, Wd = store[0][L["w_gate_up"]:], store[0][L["w_down"]:]
        bufA = torch.empty(T * max(3 * H, 2 * Iw), dtype=torch.bfloat16, device="cuda").normal_()
        bufB = torch.empty(T * max(3 * H, 2 * Iw), dtype=torch.bfloat16, device="cuda").normal_()
        bufC = torch.empty(T * max(3 * H, 2 * Iw), dtype=torch.bfloat16, device="cuda").normal_()
        Gq, Go = g_local[L["w_qkv"]:], g_local[L["w_o"]:]
        Ggu, Gd = g_local[L["w_gate_up"]:], g_local[L["w_down"]:]
        NT, NN, TN, F32 = taw.TAW_GEMM_NT, taw.TAW_GEMM_NN, taw.TAW_GEMM_TN, taw.TAW_F32
        gemms = [  # (name, mode, M, N, K, A, lda, B, ldb, C, ldc, c_dtype)
            ("qkv", NT, T, 3 * H, H, bufA, H, Wqkv, H, bufB, 3 * H, BF),
            ("o_proj", NT, T, H, H, bufA, H, Wo, H, bufB, H, BF),
            ("gate_up", NT, T, 2 * Iw, H, bufA, H, Wgu, H, bufB, 2 * Iw, BF),
            ("down", NT, T, H, Iw, bufA, Iw, Wd, Iw, bufB, H, BF),
            ("d_a", NN, T, Iw, H, bufA, H, Wd, Iw, bufB, Iw, BF),
            ("d_hn", NN, T, H, 2 * Iw, bufA, 2 * Iw, Wgu, H, bufB, H, BF),
            ("d_o", NN, T, H, H, bufA, H, Wo, H, bufB, H, BF),
            ("d_xn", NN, T, H, 3 * H, bufA, 3 * H, Wqkv, H, bufB, H, BF),
            ("G.w_down", TN, H, Iw, T, bufA, H, bufB, Iw, Gd, Iw, F32),
            ("G.w_gate_up", TN, 2 * Iw, H, T, bufA, 2 * Iw, bufB, H, Ggu, H, F32),
            ("G.w_o", TN, H, H, T, bufA, H, bufB, H, Go, H, F32),
            ("G.w_qkv", TN, 3 * H, H, T, bufA, 3 * H, bufB, H, Gq, H, F32),
        ]
        tot_fl, tot_ms, per = 0.0, 0.0, {}
        for (name, mode, M, N, K, A, lda, Bm, ldb, Cm, ldc, cd) in gemms:
            t = ev_time(lambda: taw.taw_op_gemm(BF, mode, M, N, K, A, lda, Bm, ldb, Cm, ldc, cd, 0, None, 0,
                                                taw.TAW_IMPL_MFMA, compute))
            fl = 2.0 * M * N * K
            tot_fl += fl; tot_ms += t
            per[name] = {"ms": round(t, 4), "TFLOPs": round(fl / t / 1e9, 1)}
        achieved = tot_fl / tot_ms / 1e9
        roofline = {"kernel": "gemm_pipe_kernel (bf16 MFMA GEMM; the 12 GEMM shapes of a step, one launch each; inside "
                              "taw_layer_bwd the 8 backward shapes run pairwise in one grid, gemm_dual_kernel)", "bound": "mfma",
                    "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": GEMM_TRAFFIC_BYTES_PER_LAUNCH.get(args.workload),
                    "traffic_unit": "bytes per launch (L2 fills + write-backs, rocprofv3 FETCH_SIZE/WRITE_SIZE)",
                    "algorithmic_bytes_per_launch": sum((M * K + N * K) * 2 + M * N * (4 if cd == F32 else 2) for (_, _, M, N, K, *_r, cd) in gemms) / len(gemms),
                    "avg_launch_ms": round(tot_ms / len(gemms), 4), "flops_per_launch_avg": tot_fl / len(gemms)}
        kernels["gemm"] = per
        # attention
        qkv = bufA[: T * 3 * H]
        o = torch.empty(T * H, dtype=torch.bfloat16, device="cuda")
        dO = torch.empty(T * H, dtype=torch.bfloat16, device="cuda").normal_()
        dqkv = bufB[: T * 3 * H]
        lse = torch.empty(cfg.B * cfg.n_heads * cfg.S, dtype=torch.float32, device="cuda")
        scr = torch.empty(taw.taw_op_attn_bwd_scratch_floats(cfg.B, cfg.S, cfg.n_heads), dtype=torch.float32, device="cuda")
        tf = ev_time(lambda: taw.taw_op_attn_fwd(BF, cfg.B, cfg.S, cfg.n_heads, cfg.head_dim, qkv, o, lse, taw.TAW_IMPL_MFMA, compute), 3)
        tb = ev_time(lambda: taw.taw_op_attn_bwd(BF, cfg.B, cfg.S, cfg.n_heads, cfg.head_dim, qkv, o, dO, lse, dqkv, scr, None, taw.TAW_IMPL_MFMA, compute), 3)
        kernels["attn_fwd"] = {"ms": round(tf, 4), "model_TFLOPs": round(attn_fl / 3 / tf / 1e9, 1)}
        kernels["attn_bwd"] = {"ms": round(tb, 4), "model_TFLOPs": round(attn_fl * 2 / 3 / tb / 1e9, 1)}
        # bandwidth kernels: algorithmic bytes / time
        e = 2
        r = torch.empty(T, dtype=torch.float32, device="cuda")
        gam = store[0][L["gamma_attn"]:]
        t = ev_time(lambda: taw.taw_op_rmsnorm_fwd(BF, T, H, bufA, gam, 1e-6, bufB, r, compute))
        kernels["rmsnorm_fwd"] = {"ms": round(t, 4), "GBs": round(2 * T * H * e / t / 1e6, 1)}
        scratch = torch.empty(taw.taw_op_rmsnorm_bwd_scratch_floats(H), dtype=torch.float32, device="cuda")
        dgam = torch.zeros(H, dtype=torch.float32, device="cuda")
        t = ev_time(lambda: taw.taw_op_rmsnorm_bwd(BF, T, H, bufA, x, r, gam, dy, bufB, dgam, 0, scratch, compute))
        kernels["rmsnorm_bwd"] = {"ms": round(t, 4), "GBs": round(4 * T * H * e / t / 1e6, 1)}
        t = ev_time(lambda: taw.taw_op_rope(BF, cfg.B, cfg.S, 2 * H, cfg.head_dim, bufA, 3 * H, rope, 0, compute))
        kernels["rope"] = {"ms": round(t, 4), "GBs": round(4 * T * H * e / t / 1e6, 1)}
        t = ev_time(lambda: taw.taw_op_swiglu_fwd(BF, T, Iw, bufA, bufB, compute))
        kernels["swiglu_fwd"] = {"ms": round(t, 4), "GBs": round(3 * T * Iw * e / t / 1e6, 1)}
        t = ev_time(lambda: taw.taw_op_swiglu_bwd(BF, T, Iw, bufA, bufC, bufB, compute))
        kernels["swiglu_bwd"] = {"ms": round(t, 4), "GBs": round(5 * T * Iw * e / t / 1e6, 1)}
        t = ev_time(lambda: taw.taw_grad_accum(G_shard, g_local, taw.TAW_F32, P, 1.0, compute))
        kernels["grad_accum"] = {"ms": round(t, 4), "GBs": round(12 * P / t / 1e6, 1)}
        # owner-side AdamW over the whole shard: reads G, m, v, master (16 B), writes m, v, master, bf16 chunk, zeroed G (18 B)
        master = torch.empty(P, dtype=torch.float32, device="cuda").normal_()
        om, ov = torch.zeros_like(master), torch.zeros_like(master)
        t = ev_time(lambda: taw.taw_optimizer_step(stage_buf[0], BF, master, om, ov, g_local, P, 1, zero_grad=True, stream=compute), 3)
        kernels["optimizer_step"] = {"ms": round(t, 4), "GBs": round(34 * P / t / 1e6, 1)}
        del master, om, ov
        del bufA, bufB, bufC

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import decoder_layer as O
        S_s = min(4096, cfg.S)       # about 10 s of host work
        scfg = cfg.with_(B=1, S=S_s)
        w64 = I.weights_to_f64(I.make_weights(scfg, seed=0), cfg.dtype)
        xs, dys = I.make_activations(scfg, seed=0)
        xs, dys = I.to_f64(xs, cfg.dtype), I.to_f64(dys, cfg.dtype)
        t0 = time.perf_counter()
        ys, cache = O.layer_fwd(w64, xs, scfg.n_heads, scfg.rope_theta, scfg.rms_eps)
        O.layer_bwd(w64, cache, dys)
        dt = time.perf_counter() - t0
        sg, sa = model_flops(scfg)
        cpu = {"value": round((sg + sa) / dt / 1e12, 4), "unit": "TFLOP/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
               "kind": "oracle", "seconds": round(dt, 2),
               "sample": f"fp64 numpy oracle, one forward+backward of the same layer widths on B=1, S={S_s} tokens "
                         f"({S_s}/{cfg.B * cfg.S} of the workload's tokens; attention cost per token is lower at this S)"}
        del w64, cache

    out = {
        "metric": "layer fwd+bwd TFLOP/s (model FLOPs; fraction of the bf16 MFMA peak in config), H=4096 S=8192 (C2) or S=32768 (--workload C3)", "value": round(value, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: bf16 decoder layer fwd+bwd, B={cfg.B} S={cfg.S} H={cfg.H} heads={cfg.n_heads}x{cfg.head_dim} "
                               f"I={cfg.I}, + weight staging and fp32 grad-shard aggregation on side streams",
                   "model_flops_per_step": flops, "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4)},
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels, "overlap": overlap, "recompute": recompute, "paper_sweep": sweep,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
