#!/usr/bin/env python3
"""Benchmark of the decoder-layer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload default|C2|C3|C4|C5|P-<H>-<S>|paper-sweep|diag]

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

The default run measures both lengths the metric is quoted on, in one process: the target
configuration C3 (S = 32768) at the top level of the JSON line and C2 (S = 8192) under "c2", each
with its own step time, fraction of the bf16 MFMA peak and roofline of its dominant kernel.
C4 runs four distinct layers (forward 0..3, backward 3..0, every chunk arriving through the staging
buffers); C5 runs four micro-batches through one layer, accumulating into one fp32 shard while the
next layer's chunk is staged; paper-sweep runs the nine shapes of the paper's throughput table.

Steps are timed with HIP events on the compute stream (one per step boundary): the K timed steps sit
between a synchronisation on both sides, `ms_per_step` is their mean, median and minimum are beside it.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline      the dominant kernel of the top-level workload, measured live with HIP events on the
                launch stream: at C3 the attention backward (credited and executed FLOP/s against the
                2.5 PFLOP/s dense bf16 MFMA peak), at C2 the bf16 MFMA GEMM (the 12 GEMM shapes of a
                step, one launch each); "rooflines" holds both, plus the attention forward
  cpu_baseline  the fp64 CPU oracle timed on this machine's host cores on one whole C2 layer
  kernels       per-kernel-class rates measured the same way (attention, bandwidth kernels)
  overlap       step time with and without the staging copy running beside it, with the gradient
                aggregation on the compute stream instead of its side stream, and the event timestamps
                of the copies against the steps that consume them
  recompute     the same step in activation-checkpointing mode (TAW_RECOMPUTE): same model FLOPs
  measured_ceiling  a loop of nothing but bf16 MFMAs on random operands, timed in the same run: what the matrix cores
                sustain under the part's power limit; every TFLOP/s roofline carries its fraction of that too
--workload diag prints the probes of include/taw_diag.h instead (MFMA loop alone, with LDS reads, with loads; LDS read
rate; dQ-update rates with atomics, stores, load-add-store; vector stores beside MFMAs; the GEMM kernel on 64 / 256 / 1024 tiles and over K).
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0
# HBM-side bytes per launch of the dominant kernel from two rocprofv3 --pmc runs of this file (FETCH_SIZE, WRITE_SIZE; each
# scaled by what the counter reads for the staging copy kernel, a plain copy of known size).  Precomputed: a counter run is a
# separate profiler invocation, not part of a timed run.  (workload, kernel) -> (bytes, file under profiles/ it comes from)
TRAFFIC_BYTES_PER_LAUNCH = {
    ("C2", "gemm"): (1442.9e6, "profiles/gemm_C2_hbm_traffic.md"),
    ("C3", "gemm"): (5424.2e6, "profiles/attn_C3_kernels.md"),
    ("C3", "attn_bwd"): (81.1e9, "profiles/attn_C3_kernels.md"),
}
# the paper's throughput table (Experiments, Throughput and Memory Usage): micro-batch size per sequence length and
# TawPipe's tokens per GPU per second on its own hardware
PAPER_TABLE_B = {4096: 16, 8192: 8, 16384: 4}
PAPER_TABLE_TAWPIPE = {(1024, 4096): 13629.2, (1024, 8192): 11738.2, (1024, 16384): 8913.7, (2048, 4096): 5040.0,
                       (2048, 8192): 4636.6, (2048, 16384): 4175.7, (4096, 4096): 1567.7, (4096, 8192): 1511.5,
                       (4096, 16384): 1377.6}
PAPER_SETUP = "24 x A800, NVLink + 10GbE, fp16, activation checkpointing, 48 layers (context, not the target)"
# matrix products the attention backward executes per (query tile, key tile) pair; 4 are credited (dV, dP, dK, dQ) and the
# score recomputation is a fifth that every tiled backward needs
ATTN_BWD_PRODUCTS_EXECUTED = 5


def model_flops(cfg):
    T = cfg.B * cfg.S
    gemm = 6.0 * T * cfg.H * (4 * cfg.H + 3 * cfg.I)
    attn = 12.0 * cfg.B * (cfg.S * (cfg.S + 1) / 2.0) * cfg.H
    return gemm, attn


def _stats(ms_list):
    return {"mean": sum(ms_list) / len(ms_list), "median": statistics.median(ms_list), "min": min(ms_list)}


class Env:
    """torch, the binding, the inputs module and small device helpers, imported once"""

    def __init__(self):
        import numpy as np
        import torch
        import paper_2511_09741_amd.binding as taw
        from paper_2511_09741_amd import inputs as I
        taw.load()
        torch.cuda.set_device(0)
        self.np, self.torch, self.taw, self.I = np, torch, taw, I
        self.compute = torch.cuda.current_stream()

    def dev_bf16(self, a):
        return self.torch.from_numpy(self.np.ascontiguousarray(a).view(self.np.int16)).cuda().view(self.torch.bfloat16)

    def timed_steps(self, fn, n):
        """n calls of fn between two synchronisations, one HIP event per step boundary on the compute
        stream: per-step durations in ms"""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        torch.cuda.synchronize()
        ev[0].record(self.compute)
        for i in range(n):
            fn()
            ev[i + 1].record(self.compute)
        torch.cuda.synchronize()
        return [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]

    def ev_time(self, fn, reps=5):
        """average launch duration of fn over reps back-to-back launches (HIP events on the launch stream)"""
        torch = self.torch
        fn()
        s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        s.record(self.compute)
        for _ in range(reps):
            fn()
        e.record(self.compute)
        e.synchronize()
        return s.elapsed_time(e) / reps

    def free(self):
        import gc
        gc.collect()
        self.torch.cuda.empty_cache()


def paper_cfg(I, name):
    """P-<H>-<S>: a shape of the paper's throughput table (48-layer LLaMA-style models, heads of 128,
    I = 8H/3 rounded up to 256, micro-batch size as in that table)"""
    _, h_, s_ = name.split("-")
    h_, s_ = int(h_), int(s_)
    b_ = PAPER_TABLE_B[s_]
    assert h_ % 128 == 0
    return I.LayerConfig(name, I.BF16, b_, s_, h_, h_ // 128, 128, (8 * h_ // 3 + 255) // 256 * 256)


# =============================================================================== one layer, one micro-batch per step
def run_layer_workload(env, cfg, steps, warmup, kernel_leg=True, recompute_leg=True, overlap_leg=True):
    np, torch, taw, I = env.np, env.torch, env.taw, env.I
    compute = env.compute
    desc = taw.desc_from_config(cfg, 0)       # bwd overwrites the local gradient buffer
    L = taw.taw_layer_weight_layout(desc)
    P = L["total_elems"]

    # ---- synthetic inputs, resident in HBM
    store = []                                # the owner's store: two layers' chunks
    for layer in range(2):
        w = I.make_weights(cfg, seed=0, layer=layer)
        store.append(env.dev_bf16(I.pack_chunk(w, L, P, cfg.dtype)))
        del w
    x_np, dy_np = I.make_activations(cfg, seed=0)
    x, dy = env.dev_bf16(x_np), env.dev_bf16(dy_np)
    del x_np, dy_np
    y, dx = torch.empty_like(x), torch.empty_like(x)
    stage_buf = [torch.empty_like(store[0]) for _ in range(2)]
    g_locals = [torch.zeros(P, dtype=torch.float32, device="cuda") for _ in range(2)]
    G_shard = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx = torch.empty(taw.taw_layer_ctx_bytes(desc), dtype=torch.uint8, device="cuda")
    desc_rc = taw.desc_from_config(cfg, taw.TAW_RECOMPUTE)      # activation checkpointing (extra leg below)
    ws_bytes_rc = taw.taw_layer_workspace_bytes(desc_rc)
    ws_bytes = taw.taw_layer_workspace_bytes(desc)
    ws = torch.empty(ws_bytes_rc if recompute_leg else ws_bytes, dtype=torch.uint8, device="cuda")
    rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, rope)

    copy_stream, agg_stream = torch.cuda.Stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    g_ready = [torch.cuda.Event() for _ in range(2)]
    g_consumed = [torch.cuda.Event() for _ in range(2)]
    chunk_bytes = P * 2

    state = {"cur": 0, "layer": 0, "n": 0, "trace": None}
    taw.taw_weight_stage(stage_buf[0], store[0], chunk_bytes, copy_stream, None, ready[0])
    consumed[1].record(compute)

    def step(staging=True, agg_side=True):
        cur, nxt = state["cur"], state["cur"] ^ 1
        gi = state["n"] & 1
        state["n"] += 1
        tr = state["trace"]
        if tr is not None:                     # timestamps for the overlap object
            rec = {k: torch.cuda.Event(enable_timing=True) for k in ("step_start", "copy_start", "copy_end", "fwd_start", "step_end")}
            rec["step_start"].record(compute)
        if staging:
            if tr is not None:
                copy_stream.wait_event(consumed[nxt])
                rec["copy_start"].record(copy_stream)
            taw.taw_weight_stage(stage_buf[nxt], store[(state["layer"] + 1) & 1], chunk_bytes, copy_stream,
                                 consumed[nxt], ready[nxt])
            if tr is not None:
                rec["copy_end"].record(copy_stream)
            compute.wait_event(ready[cur])
        if tr is not None:
            rec["fwd_start"].record(compute)
        taw.taw_layer_fwd(desc, stage_buf[cur], rope, x, y, ctx, ws, ws_bytes, compute)
        compute.wait_event(g_consumed[gi])      # the aggregation of two steps ago has read this buffer
        taw.taw_layer_bwd(desc, stage_buf[cur], rope, x, dy, ctx, dx, g_locals[gi], ws, ws_bytes, compute)
        consumed[cur].record(compute)
        if agg_side:
            g_ready[gi].record(compute)
            agg_stream.wait_event(g_ready[gi])
            taw.taw_grad_accum(G_shard, g_locals[gi], taw.TAW_F32, P, 1.0, agg_stream)
            g_consumed[gi].record(agg_stream)
        else:
            taw.taw_grad_accum(G_shard, g_locals[gi], taw.TAW_F32, P, 1.0, compute)
        if tr is not None:
            rec["step_end"].record(compute)
            tr.append(rec)
        if staging:
            state["cur"] = nxt
            state["layer"] += 1

    for _ in range(warmup):
        step()
    per_step = env.timed_steps(step, steps)
    st = _stats(per_step)
    gemm_fl, attn_fl = model_flops(cfg)
    flops = gemm_fl + attn_fl
    value = flops / st["mean"] / 1e9            # TFLOP/s
    res = {"name": cfg.name, "ms_per_step": round(st["mean"], 4), "ms_per_step_median": round(st["median"], 4),
           "ms_per_step_min": round(st["min"], 4), "value": round(value, 2),
           "model_TFLOPs_at_median": round(flops / st["median"] / 1e9, 2),
           "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4), "model_flops_per_step": flops,
           "workload": f"{cfg.name}: bf16 decoder layer fwd+bwd, B={cfg.B} S={cfg.S} H={cfg.H} heads={cfg.n_heads}x{cfg.head_dim} "
                       f"I={cfg.I}, + weight staging and fp32 grad-shard aggregation on side streams"}

    # ---- staging overlap: same steps with no copy running beside them, and the copies' timestamps
    if overlap_leg:
        n_ov = max(3, steps // 2)
        copy_stream.synchronize()
        torch.cuda.synchronize()
        stage_buf[0].copy_(store[0]); stage_buf[1].copy_(store[1])      # both buffers valid, then time without staging
        ms_nostage = _stats(env.timed_steps(lambda: step(staging=False), n_ov))["median"]
        ms_stage = _stats(env.timed_steps(lambda: step(staging=True), n_ov))["median"]
        ms_agg_serial = _stats(env.timed_steps(lambda: step(staging=True, agg_side=False), n_ov))["median"]
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record(copy_stream)
        taw.taw_weight_stage(stage_buf[state["cur"] ^ 1], store[0], chunk_bytes, copy_stream, None, None)
        e1.record(copy_stream)
        torch.cuda.synchronize()
        copy_ms = e0.elapsed_time(e1)
        # event timestamps: for every traced step, when its copy of the NEXT step's chunk started and ended relative to
        # the step, and how long the compute stream waited for its own chunk (fwd_start - step_start: 0 when the copy
        # issued during the previous step had finished before this step began)
        state["trace"] = []
        step(); step()
        torch.cuda.synchronize()
        state["trace"] = []
        for _ in range(4):
            step()
        torch.cuda.synchronize()
        tr = state["trace"]
        state["trace"] = None
        stamps = []
        for r in tr:
            s0 = r["step_start"]
            stamps.append({"step_ms": round(s0.elapsed_time(r["step_end"]), 4),
                           "wait_for_own_chunk_ms": round(s0.elapsed_time(r["fwd_start"]), 4),
                           "next_chunk_copy_start_ms": round(s0.elapsed_time(r["copy_start"]), 4),
                           "next_chunk_copy_end_ms": round(s0.elapsed_time(r["copy_end"]), 4)})
        hidden = all(s["next_chunk_copy_end_ms"] < s["step_ms"] and s["wait_for_own_chunk_ms"] < 0.05 for s in stamps)
        res["overlap"] = {"ms_per_step_staging": round(ms_stage, 4), "ms_per_step_no_staging": round(ms_nostage, 4),
                          "delta_frac": round(ms_stage / ms_nostage - 1.0, 4),
                          "ms_per_step_aggregation_on_compute_stream": round(ms_agg_serial, 4), "copy_alone_ms": round(copy_ms, 4),
                          "copy_alone_GBs": round(2 * chunk_bytes / copy_ms / 1e6, 1),
                          "timestamps_relative_to_step_start": stamps,
                          "every_copy_ends_inside_the_step_before_its_consumer": bool(hidden)}

    # ---- activation-checkpointing mode: same model FLOPs, the backward re-runs the forward first
    if recompute_leg:
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
        ms_rc = _stats(env.timed_steps(step_rc, max(3, steps // 2)))["median"]
        res["recompute"] = {"ms_per_step": round(ms_rc, 4), "model_TFLOPs": round(flops / ms_rc / 1e9, 2),
                            "ctx_bytes_saved": int(taw.taw_layer_ctx_bytes(desc))}

    # ---- per-kernel leg: HIP events on the launch stream around each launch
    if kernel_leg:
        torch.cuda.synchronize()
        ev_time = env.ev_time
        g_local = g_locals[0]
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
        traffic = TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, "gemm"), (None, None))
        rooflines = {"gemm": {
            "kernel": "gemm_pipe_kernel (bf16 MFMA GEMM; the 12 GEMM shapes of a step, one launch each; inside "
                      "taw_layer_bwd the 8 backward shapes run pairwise in one grid, gemm_dual_kernel)", "bound": "mfma",
            "achieved": round(achieved, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_BF16_TFLOPS, 4), "traffic": traffic[0],
            "traffic_unit": "bytes per launch (L2 fills + write-backs, rocprofv3 FETCH_SIZE/WRITE_SIZE)",
            "traffic_source": (traffic[1] + " (precomputed by separate counter runs of this file, not measured in this run)") if traffic[1] else None,
            "algorithmic_bytes_per_launch": sum((M * K + N * K) * 2 + M * N * (4 if cd == F32 else 2) for (_, _, M, N, K, *_r, cd) in gemms) / len(gemms),
            "avg_launch_ms": round(tot_ms / len(gemms), 4), "flops_per_launch_avg": tot_fl / len(gemms),
            "share_of_step": round(tot_ms / st["mean"], 3)}}
        kernels = {"gemm": per}
        # attention
        qkv = bufA[: T * 3 * H]
        o = torch.empty(T * H, dtype=torch.bfloat16, device="cuda")
        dO = torch.empty(T * H, dtype=torch.bfloat16, device="cuda").normal_()
        dqkv = bufB[: T * 3 * H]
        lse = torch.empty(cfg.B * cfg.n_heads * cfg.S, dtype=torch.float32, device="cuda")
        scr = torch.empty(taw.taw_op_attn_bwd_scratch_floats(cfg.B, cfg.S, cfg.n_heads), dtype=torch.float32, device="cuda")
        tf = ev_time(lambda: taw.taw_op_attn_fwd(BF, cfg.B, cfg.S, cfg.n_heads, cfg.head_dim, qkv, o, lse, taw.TAW_IMPL_MFMA, compute), 3)
        tb = ev_time(lambda: taw.taw_op_attn_bwd(BF, cfg.B, cfg.S, cfg.n_heads, cfg.head_dim, qkv, o, dO, lse, dqkv, scr, rope, taw.TAW_IMPL_MFMA_STORED, compute), 3)
        # the other forms of the backward, for the record
        scr_all = scr
        forms = {"two kernels, dS stored by the dK/dV kernel and read back by the dQ kernel (default; 5 products)": round(tb, 4)}
        for fname, impl in (("two kernels, the dQ kernel recomputes the scores (TAW_ATTN_BWD_RECOMPUTE; 7 products)", taw.TAW_IMPL_MFMA),
                            ("fused, dQ slots (TAW_ATTN_BWD_FUSED; 5 products, no atomics)", taw.TAW_IMPL_MFMA_FUSED),
                            ("fused, fp32 atomics (5 products)", taw.TAW_IMPL_MFMA_ATOMIC)):
            tt_ = ev_time(lambda: taw.taw_op_attn_bwd(BF, cfg.B, cfg.S, cfg.n_heads, cfg.head_dim, qkv, o, dO, lse, dqkv, scr_all, rope, impl, compute), 2)
            forms[fname] = round(tt_, 4)
        kernels["attn_bwd_forms_ms"] = forms
        kernels["attn_fwd"] = {"ms": round(tf, 4), "model_TFLOPs": round(attn_fl / 3 / tf / 1e9, 1)}
        kernels["attn_bwd"] = {"ms": round(tb, 4), "model_TFLOPs": round(attn_fl * 2 / 3 / tb / 1e9, 1)}
        prod = attn_fl / 6.0                   # one S x S x d product over the causal pairs
        nprod = ATTN_BWD_PRODUCTS_EXECUTED
        tr_b = TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, "attn_bwd"), (None, None))
        rooflines["attn_bwd"] = {
            "kernel": "attention backward (taw_op_attn_bwd: row statistics + the tiled dK/dV/dQ kernels), all heads of the micro-batch in one call",
            "bound": "mfma", "achieved": round(4 * prod / tb / 1e9, 1), "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": round(4 * prod / tb / 1e9 / PEAK_BF16_TFLOPS, 4),
            "credited_products": 4, "executed_products": nprod,
            "executed_TFLOPs": round(nprod * prod / tb / 1e9, 1), "executed_frac": round(nprod * prod / tb / 1e9 / PEAK_BF16_TFLOPS, 4),
            "avg_launch_ms": round(tb, 4), "flops_per_launch": 4 * prod, "traffic": tr_b[0],
            "traffic_source": (tr_b[1] + " (precomputed by separate counter runs of this file)") if tr_b[1] else None,
            "algorithmic_bytes_per_launch": 2.0 * T * H * (3 + 1 + 1 + 3) + 4.0 * cfg.B * cfg.n_heads * cfg.S,
            "ds_handover_bytes_per_launch": 2.0 * (2.0 * cfg.B * cfg.n_heads * (((cfg.S + 255) // 256) * ((cfg.S + 255) // 256 + 1) // 2) * 65536),
            "share_of_step": round(tb / st["mean"], 3)}
        rooflines["attn_fwd"] = {
            "kernel": "attn_fwd_kernel", "bound": "mfma", "achieved": round(2 * prod / tf / 1e9, 1), "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": round(2 * prod / tf / 1e9 / PEAK_BF16_TFLOPS, 4), "avg_launch_ms": round(tf, 4),
            "flops_per_launch": 2 * prod, "traffic": None, "share_of_step": round(tf / st["mean"], 3)}
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
        res["kernels"] = kernels
        res["rooflines"] = rooflines
        # the dominant kernel: the single launch that takes the largest share of the step
        dom = "attn_bwd" if tb > tot_ms / len(gemms) * 4 else "gemm"
        res["roofline"] = dict(rooflines[dom], dominant_because=(
            "one attention-backward call is the longest launch of the step" if dom == "attn_bwd"
            else "the GEMM launches together are the largest share of the step and no other launch is longer than four of them"))
    torch.cuda.synchronize()
    return res


# =============================================================================== C4: four chained layers
def run_c4(env, cfg, steps, warmup):
    """Four distinct layers: forward 0 -> 3, then backward 3 -> 0, every layer's chunk arriving through one of
    two staging buffers on a side stream while the previous layer computes.  One step = the whole sweep."""
    np, torch, taw, I = env.np, env.torch, env.taw, env.I
    compute = env.compute
    nl = cfg.n_layers
    desc = taw.desc_from_config(cfg, 0)
    L = taw.taw_layer_weight_layout(desc)
    P = L["total_elems"]
    store = []
    for layer in range(nl):
        w = I.make_weights(cfg, seed=0, layer=layer)
        store.append(env.dev_bf16(I.pack_chunk(w, L, P, cfg.dtype)))
        del w
    x_np, dy_np = I.make_activations(cfg, seed=0)
    acts = [env.dev_bf16(x_np)] + [None] * nl
    dy = env.dev_bf16(dy_np)
    del x_np, dy_np
    for l in range(nl):
        acts[l + 1] = torch.empty_like(acts[0])
    grads = [torch.empty_like(dy) for _ in range(2)]
    stage_buf = [torch.empty_like(store[0]) for _ in range(2)]
    G = [torch.zeros(P, dtype=torch.float32, device="cuda") for _ in range(nl)]
    ctx = [torch.empty(taw.taw_layer_ctx_bytes(desc), dtype=torch.uint8, device="cuda") for _ in range(nl)]
    ws_bytes = taw.taw_layer_workspace_bytes(desc)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, rope)
    side = torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    order = list(range(nl)) + list(reversed(range(nl)))
    chunk_bytes = P * 2

    def layer_call(i, l, chunk):
        if i < nl:
            taw.taw_layer_fwd(desc, chunk, rope, acts[l], acts[l + 1], ctx[l], ws, ws_bytes, compute)
        else:                                   # the gradient buffers alternate: layer l reads what layer l + 1 wrote
            g_in = dy if l == nl - 1 else grads[(l + 1) & 1]
            taw.taw_layer_bwd(desc, chunk, rope, acts[l], g_in, ctx[l], grads[l & 1], G[l], ws, ws_bytes, compute)

    def sweep(staging=True):
        if not staging:                         # all four chunks sit in the store already: compute reads them in place
            for i, l in enumerate(order):
                layer_call(i, l, store[l])
            return
        for b in range(2):
            consumed[b].record(compute)
        taw.taw_weight_stage(stage_buf[0], store[order[0]], chunk_bytes, side, consumed[0], ready[0])
        for i, l in enumerate(order):
            buf = i & 1
            if i + 1 < len(order):              # the next step's chunk into the other buffer, once its last reader is done
                taw.taw_weight_stage(stage_buf[buf ^ 1], store[order[i + 1]], chunk_bytes, side, consumed[buf ^ 1], ready[buf ^ 1])
            compute.wait_event(ready[buf])
            layer_call(i, l, stage_buf[buf])
            consumed[buf].record(compute)

    for _ in range(warmup):
        sweep()
    st = _stats(env.timed_steps(sweep, steps))
    n_ov = max(2, steps // 2)
    ms_nostage = _stats(env.timed_steps(lambda: sweep(False), n_ov))["median"]
    ms_stage = _stats(env.timed_steps(lambda: sweep(True), n_ov))["median"]
    gemm_fl, attn_fl = model_flops(cfg)
    flops = (gemm_fl + attn_fl) * nl
    value = flops / st["mean"] / 1e9
    return {"name": cfg.name, "ms_per_step": round(st["mean"], 4), "ms_per_step_median": round(st["median"], 4),
            "ms_per_step_min": round(st["min"], 4), "ms_per_layer": round(st["mean"] / nl, 4), "value": round(value, 2),
            "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4), "model_flops_per_step": flops,
            "workload": f"{cfg.name}: {nl} distinct bf16 decoder layers, forward 0..{nl - 1} then backward {nl - 1}..0, B={cfg.B} S={cfg.S} "
                        f"H={cfg.H} heads={cfg.n_heads}x{cfg.head_dim} I={cfg.I}; each layer's chunk staged on a side stream into one of two buffers",
            "overlap": {"ms_per_step_staging": round(ms_stage, 4), "ms_per_step_no_staging": round(ms_nostage, 4),
                        "delta_frac": round(ms_stage / ms_nostage - 1.0, 4)}}


# =============================================================================== C5: four micro-batches, one shard
def run_c5(env, cfg, steps, warmup):
    """One layer, four independent micro-batches: forward + backward of each, the weight gradients accumulated by
    the backward into ONE fp32 shard (TAW_ACCUMULATE), while the next layer's chunk is staged on a side stream.
    One step = the four micro-batches."""
    np, torch, taw, I = env.np, env.torch, env.taw, env.I
    compute = env.compute
    nmb = cfg.n_microbatches
    desc = taw.desc_from_config(cfg, taw.TAW_ACCUMULATE)
    L = taw.taw_layer_weight_layout(desc)
    P = L["total_elems"]
    store = []
    for layer in range(2):
        w = I.make_weights(cfg, seed=0, layer=layer)
        store.append(env.dev_bf16(I.pack_chunk(w, L, P, cfg.dtype)))
        del w
    xs, dys = [], []
    for mb in range(nmb):
        x_np, dy_np = I.make_activations(cfg, seed=0, mb=mb)
        xs.append(env.dev_bf16(x_np)); dys.append(env.dev_bf16(dy_np))
        del x_np, dy_np
    y, dx = torch.empty_like(xs[0]), torch.empty_like(xs[0])
    staged = torch.empty_like(store[0])
    G = torch.zeros(P, dtype=torch.float32, device="cuda")
    ctx = torch.empty(taw.taw_layer_ctx_bytes(desc), dtype=torch.uint8, device="cuda")
    ws_bytes = taw.taw_layer_workspace_bytes(desc)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda")
    rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, rope)
    side = torch.cuda.Stream()
    start_ev, ready = torch.cuda.Event(), torch.cuda.Event()
    chunk_bytes = P * 2

    def minibatch(staging=True):
        if staging:                               # the next layer's chunk arrives while this layer's micro-batches compute
            start_ev.record(compute)
            taw.taw_weight_stage(staged, store[1], chunk_bytes, side, start_ev, ready)
        for mb in range(nmb):
            taw.taw_layer_fwd(desc, store[0], rope, xs[mb], y, ctx, ws, ws_bytes, compute)
            taw.taw_layer_bwd(desc, store[0], rope, xs[mb], dys[mb], ctx, dx, G, ws, ws_bytes, compute)
        if staging:
            compute.wait_event(ready)             # the next layer would start here

    for _ in range(warmup):
        minibatch()
    st = _stats(env.timed_steps(minibatch, steps))
    n_ov = max(2, steps // 2)
    ms_nostage = _stats(env.timed_steps(lambda: minibatch(False), n_ov))["median"]
    ms_stage = _stats(env.timed_steps(lambda: minibatch(True), n_ov))["median"]
    gemm_fl, attn_fl = model_flops(cfg)
    flops = (gemm_fl + attn_fl) * nmb
    value = flops / st["mean"] / 1e9
    return {"name": cfg.name, "ms_per_step": round(st["mean"], 4), "ms_per_step_median": round(st["median"], 4),
            "ms_per_step_min": round(st["min"], 4), "ms_per_microbatch": round(st["mean"] / nmb, 4), "value": round(value, 2),
            "frac_of_bf16_mfma_peak": round(value / PEAK_BF16_TFLOPS, 4), "model_flops_per_step": flops,
            "workload": f"{cfg.name}: one bf16 decoder layer, {nmb} micro-batches fwd+bwd accumulating into one fp32 gradient shard, B={cfg.B} "
                        f"S={cfg.S} H={cfg.H} heads={cfg.n_heads}x{cfg.head_dim} I={cfg.I}; the next layer's chunk staged on a side stream",
            "overlap": {"ms_per_step_staging": round(ms_stage, 4), "ms_per_step_no_staging": round(ms_nostage, 4),
                        "delta_frac": round(ms_stage / ms_nostage - 1.0, 4)}}


# =============================================================================== what the part sustains
def mfma_ceiling(env):
    """A loop of nothing but bf16 MFMAs on random operands (and on zeros): the rate the matrix cores sustain under the
    part's power limit, measured in this run.  Every roofline fraction is quoted against this as well as against the
    published peak."""
    taw = env.taw
    r = taw.taw_diag_mfma_loop(taw.TAW_DIAG_MFMA_RANDOM, 20000)
    z = taw.taw_diag_mfma_loop(taw.TAW_DIAG_MFMA_ZERO, 20000)
    return {"mfma_loop_random_operands_TFLOPs": round(r["TFLOPs"], 1), "clock_GHz": round(r["clock_GHz"], 3),
            "mfma_loop_zero_operands_TFLOPs": round(z["TFLOPs"], 1), "clock_GHz_zero_operands": round(z["clock_GHz"], 3),
            "what": "256 workgroups x 4 wavefronts issuing v_mfma_f32_32x32x16_bf16 back to back from registers (taw_diag_mfma_loop)"}


def run_diag(env):
    """The probes of include/taw_diag.h and the GEMM kernel on a quarter of the chip against the whole chip."""
    torch, taw = env.torch, env.taw
    src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
    src.view(torch.int32).random_(0, 1 << 30)
    names = {taw.TAW_DIAG_MFMA_RANDOM: "mfma_only_random_operands", taw.TAW_DIAG_MFMA_ZERO: "mfma_only_zero_operands",
             taw.TAW_DIAG_MFMA_LDS: "mfma_plus_lds_fragment_reads", taw.TAW_DIAG_MFMA_LDS_LOADS: "mfma_plus_lds_reads_plus_global_to_lds_loads"}
    out = {"mfma_loop": {}, "lds_read_bytes_per_clock_per_cu": {}, "issue_cycles_per_mfma_slot": {}, "dq_update": {}, "gemm_by_tiles": []}
    # vector instructions beside MFMAs: cycles per slot of {1 MFMA + n vector instructions} (32 = the matrix pipe never idles)
    mode_names = ("one wavefront per SIMD, interleaved", "two wavefronts per SIMD, each interleaved (64 = pipe never idles)",
                  "two wavefronts per SIMD, one MFMAs only, one vector instructions only")
    for mode, mname in enumerate(mode_names):
        for kind, kname in enumerate(("v_fma_f32", "v_exp_f32")):
            for n in (0, 2, 4, 8):
                if n == 0 and kind == 1:
                    continue
                r = taw.taw_diag_issue_rate(mode, kind, n)
                key = f"{mname}; {n} x {kname}" if n else f"{mname}; MFMAs only"
                out["issue_cycles_per_mfma_slot"][key] = {"mfma_wavefront": round(r["cycles_per_slot_mfma_wave"], 1),
                                                            "last_wavefront": round(r["cycles_per_slot_last_wave"], 1)}
    for kind, name in names.items():
        r = taw.taw_diag_mfma_loop(kind, 20000, src)
        out["mfma_loop"][name] = {k: round(v, 3) for k, v in r.items()}
    for instr, iname in enumerate(("ds_read_b128", "ds_read_b64", "ds_read_b64_tr_b16")):
        for waves in (4, 8):
            r = taw.taw_diag_lds_read_rate(instr, waves)
            out["lds_read_bytes_per_clock_per_cu"][f"{iname}, {waves} wavefronts"] = round(r["bytes_per_clock_per_cu"], 1)
    del src
    for S in (8192, 32768):
        buf = torch.empty(S * 32 * 128, dtype=torch.float32, device="cuda")
        for mode, mname in enumerate(("fp32 atomic add (no return)", "plain store", "load + add + store")):
            r = taw.taw_diag_dq_update_rate(buf, S, 32, mode)
            out["dq_update"][f"S={S}, 32 heads, {mname}"] = {"ms": round(r["ms"], 3), "G_updates_per_s": round(r["updates_per_s"] / 1e9, 1)}
        del buf
    # vector stores amid MFMAs: ns per trip of {16 or 64 MFMAs, then n stores of one KiB} per wavefront, 4 or 8 wavefronts per compute unit
    nb = taw.taw_diag_store_cost_bytes()
    buf = torch.empty(nb, dtype=torch.uint8, device="cuda")
    out["store_cost_ns_per_trip"] = {}
    for waves in (4, 8):
        for mf in (16, 64):
            row = {f"{n} stores": round(taw.taw_diag_store_cost(buf, nb, waves, mf, n), 1) for n in (0, 1, 2, 4)}
            out["store_cost_ns_per_trip"][f"{waves} wavefronts per compute unit, {mf} MFMAs per trip"] = row
    del buf
    # the product GEMM (NT, bf16, K = 4096) on 64, 256 and 1024 output tiles: the same kernel and the same work per tile; what changes
    # is how many compute units draw power at once
    BF = taw.TAW_BF16
    for (M, N) in ((2048, 2048), (4096, 4096), (8192, 8192)):
        K = 4096
        A = torch.empty(M * K, dtype=torch.bfloat16, device="cuda").normal_()
        Bm = torch.empty(N * K, dtype=torch.bfloat16, device="cuda").normal_()
        Cm = torch.empty(M * N, dtype=torch.bfloat16, device="cuda")
        t = env.ev_time(lambda: taw.taw_op_gemm(BF, taw.TAW_GEMM_NT, M, N, K, A, K, Bm, K, Cm, N, BF, 0, None, 0, taw.TAW_IMPL_MFMA, env.compute), 20)
        tiles = (M // 256) * (N // 256)
        tf = 2.0 * M * N * K / t / 1e9
        out["gemm_by_tiles"].append({"M": M, "N": N, "K": K, "tiles": tiles, "ms": round(t, 4), "TFLOPs": round(tf, 1),
                                     "TFLOPs_per_busy_compute_unit": round(tf / min(tiles, 256), 2)})
        del A, Bm, Cm
    # the same kernel over K at fixed M, N (8 rounds of 256 tiles): the time per round is a fixed cost per tile (prologue and
    # epilogue) plus K / 64 main-loop steps; a straight line through the two shortest K gives the fixed cost
    out["gemm_by_K"] = []
    M, N = 32768, 4096
    Cm = torch.empty(M * N, dtype=torch.bfloat16, device="cuda")
    for K in (1024, 2048, 4096, 8192, 16384):
        A = torch.empty(M * K, dtype=torch.bfloat16, device="cuda").normal_()
        Bm = torch.empty(N * K, dtype=torch.bfloat16, device="cuda").normal_(std=0.02)
        t = env.ev_time(lambda: taw.taw_op_gemm(BF, taw.TAW_GEMM_NT, M, N, K, A, K, Bm, K, Cm, N, BF, 0, None, 0, taw.TAW_IMPL_MFMA, env.compute), 10)
        rounds = (M // 256) * (N // 256) / 256
        out["gemm_by_K"].append({"M": M, "N": N, "K": K, "ms": round(t, 4), "TFLOPs": round(2.0 * M * N * K / t / 1e9, 1),
                                 "us_per_round_of_tiles": round(1e3 * t / rounds, 2)})
        del A, Bm
    g = out["gemm_by_K"]
    per_1024 = g[1]["us_per_round_of_tiles"] - g[0]["us_per_round_of_tiles"]
    out["gemm_fixed_us_per_tile"] = round(g[0]["us_per_round_of_tiles"] - per_1024, 2)
    return out


# =============================================================================== CPU oracle beside it
def cpu_baseline(env):
    """The fp64 numpy oracle, as it stands, on one whole C2 layer (forward + backward), all host cores numpy uses."""
    from oracle import decoder_layer as O
    I = env.I
    scfg = I.CONFIGS["C2"]
    w64 = I.weights_to_f64(I.make_weights(scfg, seed=0), scfg.dtype)
    xs, dys = I.make_activations(scfg, seed=0)
    xs, dys = I.to_f64(xs, scfg.dtype), I.to_f64(dys, scfg.dtype)
    t0 = time.perf_counter()
    _, cache = O.layer_fwd(w64, xs, scfg.n_heads, scfg.rope_theta, scfg.rms_eps)
    O.layer_bwd(w64, cache, dys)
    dt = time.perf_counter() - t0
    sg, sa = model_flops(scfg)
    return {"value": round((sg + sa) / dt / 1e12, 4), "unit": "TFLOP/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": "fp64 numpy oracle, one forward+backward of the whole C2 layer (B=1, S=8192, H=4096, I=11008: 11.6 model TFLOP); "
                      "C3 has four times the tokens at four times the attention length, where the oracle's rate is no higher"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="default",
                    help="default (C3 at the top level and C2 beside it), C2, C3, C4, C5, a shape of the paper's throughput table as "
                         "P-<H>-<S> (H in 1024/2048/4096, S in 4096/8192/16384; micro-batch size as in that table), or paper-sweep (all nine)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-leg", action="store_true")
    ap.add_argument("--no-recompute-leg", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (one device's share of the weight pipeline); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    env = Env()
    I = env.I
    wl = args.workload
    if wl == "diag":
        print(json.dumps({"diag": run_diag(env)}))
        return
    extra = {}
    kl, rl = not args.no_kernel_leg, not args.no_recompute_leg
    if wl == "default":
        top = run_layer_workload(env, I.CONFIGS["C3"], args.steps, args.warmup, kl, rl)
        env.free()
        c2 = run_layer_workload(env, I.CONFIGS["C2"], args.steps, args.warmup, kl, rl)
        env.free()
        extra["c2"] = c2
    elif wl in ("C2", "C3"):
        top = run_layer_workload(env, I.CONFIGS[wl], args.steps, args.warmup, kl, rl)
    elif wl == "C4":
        top = run_c4(env, I.CONFIGS["C4"], args.steps, args.warmup)
    elif wl == "C5":
        top = run_c5(env, I.CONFIGS["C5"], args.steps, args.warmup)
    elif wl == "paper-sweep":
        rows = []
        for h_ in (1024, 2048, 4096):
            for s_ in (4096, 8192, 16384):
                cfg = paper_cfg(I, f"P-{h_}-{s_}")
                r = run_layer_workload(env, cfg, max(3, args.steps // 2), 2, kernel_leg=False, recompute_leg=True, overlap_leg=False)
                env.free()
                rows.append({"H": h_, "S": s_, "B": cfg.B, "I": cfg.I, "ms_per_step": r["ms_per_step"], "model_TFLOPs": r["value"],
                             "frac_of_bf16_mfma_peak": r["frac_of_bf16_mfma_peak"],
                             "ms_per_step_checkpointing": r["recompute"]["ms_per_step"],
                             # what one GPU's compute alone allows for the paper's 48-layer model in its training mode
                             # (activation checkpointing): tokens of a micro-batch / (48 x this layer's checkpointed step)
                             "tokens_per_s_per_gpu_compute_only": round(cfg.B * cfg.S / (48 * r["recompute"]["ms_per_step"] * 1e-3), 1),
                             "paper_tawpipe_tokens_per_s_per_gpu": PAPER_TABLE_TAWPIPE[(h_, s_)]})
                print(f"bench.py: {cfg.name} done", file=sys.stderr, flush=True)
                top = r                           # the last shape, (4096, 16384): the paper's largest setting
        extra["paper_sweep"] = {"rows": rows, "paper_setup": PAPER_SETUP}
    else:
        try:
            cfg = paper_cfg(I, wl)
        except Exception:
            print(f"bench.py: unknown workload {wl!r}", file=sys.stderr)
            sys.exit(2)
        top = run_layer_workload(env, cfg, args.steps, args.warmup, kl, True)
        extra["paper_sweep"] = {"rows": [{"H": cfg.H, "S": cfg.S, "B": cfg.B, "ms_per_step_checkpointing": top["recompute"]["ms_per_step"],
                                          "tokens_per_s_per_gpu_compute_only": round(cfg.B * cfg.S / (48 * top["recompute"]["ms_per_step"] * 1e-3), 1),
                                          "paper_tawpipe_tokens_per_s_per_gpu": PAPER_TABLE_TAWPIPE.get((cfg.H, cfg.S))}],
                                "paper_setup": PAPER_SETUP}

    ceiling = mfma_ceiling(env)
    for obj in [top.get("roofline")] + list((top.get("rooflines") or {}).values()) + [extra.get("c2", {}).get("roofline")] + \
            list((extra.get("c2", {}).get("rooflines") or {}).values()):
        if obj and obj.get("unit") == "TFLOP/s":
            obj["frac_of_measured_mfma_loop"] = round(obj["achieved"] / ceiling["mfma_loop_random_operands_TFLOPs"], 4)
    cpu = None if args.no_cpu_baseline else cpu_baseline(env)

    metric = "layer fwd+bwd TFLOP/s (model FLOPs; fraction of the bf16 MFMA peak in config)"
    if wl == "default":
        metric += ", H=4096: S=32768 (C3) at the top level, S=8192 (C2) under c2"
    out = {
        "metric": metric, "value": top["value"], "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": top["ms_per_step"],
        "ms_per_step_median": top["ms_per_step_median"], "ms_per_step_min": top["ms_per_step_min"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": top["workload"], "model_flops_per_step": top["model_flops_per_step"],
                   "frac_of_bf16_mfma_peak": top["frac_of_bf16_mfma_peak"]},
        "roofline": top.get("roofline"), "cpu_baseline": cpu, "measured_ceiling": ceiling,
    }
    for k in ("rooflines", "kernels", "overlap", "recompute", "ms_per_layer", "ms_per_microbatch"):
        if k in top:
            out[k] = top[k]
    out.update(extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
