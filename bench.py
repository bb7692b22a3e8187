#!/usr/bin/env python3
"""Benchmark of the fused ROSAQ linear on one MI355X.

Headline workload (`config.workload` = "llama7b_attn_qkvo_M64_int4_headwise"): the four
attention projections q/k/v/o of a LLaMA-7B-shaped layer, D = N = 4096, 32 heads
x 128, x [64 x 4096] fp16, K = 128 FP16 salient channels, INT4 g128 for the rest,
head-wise block-diagonal rotation.  One step = one decode step of the attention
linears of a 32-layer model = 128 linears.  Per layer the q, k, v projections share
their input and PCA rotation and go through one rosaq_linear_batch call; the output
projection has its own input and goes through rosaq_linear_headwise (`--unbatched`
issues four separate rosaq_linear_headwise calls instead).  The calls cycle over
`--layers` x 4 distinct packed weights whose total size exceeds the 256 MB
last-level cache, so every linear streams its weights from HBM.

Prints ONE JSON line; `value` is algorithmic GB/s from the median step time with all
inputs resident in HBM.  Every step is timed with its own pair of HIP events on the
stream the kernels run on; median, p10 and p90 are reported (the paper's throughput
appendix defines decode speed from the median time per token).  The same line carries
two more measurements, each bounded to a few seconds of GPU time:
  "sweep"   single calls of the INT3 7B MLP shapes at M = 64 and of the INT4 13B MLP shapes at M = 1, 16, 64, 256
  "decode"  the 7 linears x 32 layers of a 7B-shaped decode step, 256 steps, against fp16 GEMMs
Weights, activations and the 512-row calibration sets are synthetic (seeded); the head-wise
rotations are the PCA of the calibration sets, computed on the GPU by rosaq_pca_headwise
before the timed region; dense rotations are seeded random orthogonal matrices.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

D = N = 4096
M = 64
K = 128
BITS = 4
GROUP = 128
HEADS = 32
CALLS_PER_STEP = 128
HBM_PEAK_GBS = 8000.0

# HBM bytes one launch of the main GEMM moves, from rocprofv3 FETCH_SIZE (KiB, x 2.0: the factor a
# 256 MiB device copy gives for this counter) and WRITE_SIZE (KiB, x 1.0), keyed by what the launch
# is: (layers in the launch, mt, nt, waves, depth, splits) as rosaq_launch_shape reports it.
# Source: profiles/gemm_kernel_llama7b_attn_M64_int4.md.  A launch shape without an entry reports
# traffic = null rather than another shape's number.
MEASURED_TRAFFIC_KIB = {
    (1, 2, 2, 8, 1, 1): (13697, 512),     # one 4096 x 4096 layer, 32 x 32 tiles
    (3, 4, 3, 8, 1, 1): (32657, 1536),    # q, k, v in one launch, 64 x 48 tiles
}


def row_bytes(d_in, bits):
    """Stored bytes of one output row: fp16 salient block, codes, fp16 scale + zero per group."""
    return 2 * K + (d_in - K) * bits // 8 + 4 * (d_in - K) // GROUP


def algorithmic_bytes():
    """Bytes the method itself must move per call: packed weights, rotation, x, y."""
    weights = row_bytes(D, BITS) * N
    rot = 2 * 128 * 128 * HEADS
    xy = 2 * M * (D + N)
    return dict(weights=weights, rotation=rot, xy=xy, call=weights + rot + xy,
                gemm_kernel=weights + 2 * M * D + 2 * M * N,
                gemm_kernel_qkv=3 * weights + 2 * M * D + 3 * 2 * M * N)


def pct(v, q):
    return float(np.percentile(np.asarray(v, dtype=np.float64), q))


class Timer:
    """Captures `fn` into one hipGraph (unless eager) and times replays, each between its own events."""

    def __init__(self, torch, stream, eager=False):
        self.torch, self.stream, self.eager = torch, stream, eager

    def prepare(self, fn):
        torch = self.torch
        with torch.cuda.stream(self.stream):
            fn()                                   # eager once: first-use work happens outside the graph
            self.stream.synchronize()
            if self.eager:
                return fn
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.stream):
                fn()
        return g.replay

    def run(self, fn, steps, warmup):
        """Returns dict(ms median / p10 / p90 per step from events, wall_ms mean per step)."""
        torch = self.torch
        run = self.prepare(fn)
        with torch.cuda.stream(self.stream):
            for _ in range(warmup):
                run()
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                  for _ in range(steps)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for e0, e1 in ev:
                e0.record(self.stream)
                run()
                e1.record(self.stream)
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
        ms = [e0.elapsed_time(e1) for e0, e1 in ev]
        return {"median": pct(ms, 50), "p10": pct(ms, 10), "p90": pct(ms, 90), "wall": wall / steps * 1e3}


def cpu_baseline(seconds_target=12.0):
    """The CPU oracle's reference linear (fp64 numpy) on a bounded sample of the same calls."""
    from oracle import rosaq_oracle as O
    from paper_2506_13472_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    W = synth.make_weight(100, N, D)
    Qb = synth.random_orthogonal_blocks(200, HEADS)
    lam = synth.descending_spectrum(300, D, HEADS)
    x = synth.make_activations(400, M, D)
    ref = O.pack(W, Qb, lam, K, BITS, O.MODE_HEADWISE)      # offline, not timed
    O.linear_ref(x, Qb, ref)                                  # warm-up
    n, t0 = 0, time.perf_counter()
    while True:
        O.linear_ref(x, Qb, ref)
        n += 1
        dt = time.perf_counter() - t0
        if dt >= seconds_target or n >= 64:
            break
    gbs = algorithmic_bytes()["call"] * n / dt / 1e9
    out = {"value": round(gbs, 4), "unit": "GB/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{n} of the {CALLS_PER_STEP} calls of one step (oracle linear_ref, fp64 numpy), "
                     f"{dt / n * 1e3:.1f} ms per call"}
    try:                                     # one more call on a single thread, for scale
        from threadpoolctl import threadpool_limits
        with threadpool_limits(limits=1):
            t1 = time.perf_counter()
            O.linear_ref(x, Qb, ref)
            out["single_thread_ms_per_call"] = round((time.perf_counter() - t1) * 1e3, 1)
    except Exception:
        pass
    return out


SWEEP_SHAPES = [
    # name, D, N, bits, q_mode ("headwise" | "full" | "none"), M values
    ("7B attn q/k/v/o, head-wise, INT4", 4096, 4096, 4, "headwise", (1, 16, 64, 256)),
    ("7B gate/up, full 4096^2 rotation, INT3", 4096, 11008, 3, "full", (64,)),
    ("7B down, no rotation (paper's setting), INT3", 11008, 4096, 3, "none", (64,)),
    ("7B down, full 11008^2 rotation, INT3", 11008, 4096, 3, "full", (64,)),
    ("13B up, full 5120^2 rotation, INT4", 5120, 13824, 4, "full", (1, 16, 64, 256)),
    ("13B down, no rotation, INT4", 13824, 5120, 4, "none", (1, 16, 64, 256)),
    ("13B down, full 13824^2 rotation, INT4", 13824, 5120, 4, "full", (64,)),
    # not one of the benchmark's configs: a large streaming launch (7B-shaped vocabulary projection)
    ("vocab 4096->32000, no rotation, INT4", 4096, 32000, 4, "none", (1, 16, 64)),
]
# the rows the default run carries in its JSON line: the M = 64 calls of the two MLP configs
BOUNDED_SWEEP = ("7B gate/up", "7B down", "13B up", "13B down")


def shape_sweep(torch, shapes, ms_override, reps, emit):
    """us per call of the library against a fp16 torch.matmul for each (shape, M), both cycling over
    enough distinct copies of the weights to stay out of the last-level cache; 32 calls per hipGraph
    replay, median over `reps` replays.  `emit` receives one dict per row."""
    from paper_2506_13472_amd import binding as B, synth, torch_glue as T
    dev = torch.device("cuda:0")
    timer = Timer(torch, torch.cuda.Stream())
    modes = {"headwise": B.Q_HEADWISE, "full": B.Q_FULL, "none": B.Q_NONE}
    calls = 32
    for name, D_, N_, bits, mode, Ms in shapes:
        W = synth.make_weight(11, N_, D_)
        lam = synth.descending_spectrum(13, D_, D_ // 128 if mode == "headwise" else 1)
        Q = None
        if mode == "headwise":
            Q = synth.random_orthogonal_blocks(12, D_ // 128)
        elif mode == "full":
            Q = synth.random_orthogonal_dense(12, D_)
        t0 = time.perf_counter()
        base = B.rosaq_pack_weights(W, Q, lam, K, bits, modes[mode])
        t_pack = time.perf_counter() - t0
        copies = [base]
        while sum(h.device_bytes for h in copies) < (320 << 20) or len(copies) < 2:
            copies.append(B.rosaq_packed_clone(base))
        w16 = torch.from_numpy(W).to(dev)
        n16 = max(2, (320 << 20) // (2 * N_ * D_) + 1)
        W16 = [w16.clone() for _ in range(n16)]
        rot_bytes = {"headwise": 2 * 128 * D_, "full": 2 * D_ * D_, "none": 0}[mode]
        for M_ in (ms_override or Ms):
            x = torch.from_numpy(synth.make_activations(17, M_, D_)).to(dev)
            y = torch.empty((M_, N_), dtype=torch.float16, device=dev)
            ws = T.alloc_workspace(base, M_)

            def step():
                for i in range(calls):
                    T.linear(copies[i % len(copies)], x, y, ws)

            def step16():
                for i in range(calls):
                    torch.matmul(x, W16[i % n16].t(), out=y)
            t_all = timer.run(step, reps, 3)
            B.rosaq_tune("stages", 2)
            t_gemm = timer.run(step, reps, 3)
            B.rosaq_tune("stages", 3)
            t16 = timer.run(step16, reps, 3)
            us = t_all["median"] * 1e3 / calls
            us16 = t16["median"] * 1e3 / calls
            nbytes = row_bytes(D_, bits) * N_ + rot_bytes + 2 * M_ * (D_ + N_)
            emit({"shape": name, "D": D_, "N": N_, "M": M_, "bits": bits, "rotation": mode,
                  "us_per_call": round(us, 2), "us_per_call_p10": round(t_all["p10"] * 1e3 / calls, 2),
                  "us_per_call_p90": round(t_all["p90"] * 1e3 / calls, 2),
                  "us_main_gemm": round(t_gemm["median"] * 1e3 / calls, 2),
                  "algorithmic_MB": round(nbytes / 1e6, 2),
                  "GBps": round(nbytes / us / 1e3, 1),
                  "frac_of_hbm_peak": round(nbytes / us / 1e3 / HBM_PEAK_GBS, 4),
                  "tflops": round(2.0 * M_ * N_ * D_ / us / 1e6, 1),
                  "fp16_matmul_us": round(us16, 2), "speedup_vs_fp16": round(us16 / us, 2),
                  "launch_shape_main_gemm": list(B.rosaq_launch_shape(M_, -(-N_ // 16) * 16, D_, bits)),
                  "distinct_copies": len(copies), "pack_s": round(t_pack, 2)})
        for h in copies:
            h.free()
        del W16, w16


def decode_workload(torch, steps, warmup, absorbed=False, chained_mlp=True):
    """The linears of a LLaMA-7B-shaped decode step at batch 64, INT4 g128, K = 128: per layer
    q/k/v (one batched call, shared head-wise rotation), o (head-wise), gate/up (one batched call
    sharing one dense 4096 x 4096 rotation) and down (no rotation, the paper's setting for W_D);
    32 layers per step, every layer its own device copy of weights and rotations.  With `chained_mlp`
    the three FFN linears are one rosaq_mlp_swiglu call (the gated product goes straight into the down
    projection's input fragments); without it, rosaq_linear_swiglu and rosaq_linear(down) on a buffer
    of the same shape.  Returns a dict with the time per step next to the same linears as fp16
    torch.matmul calls."""
    from paper_2506_13472_amd import binding as B, synth, torch_glue as T
    dev = torch.device("cuda:0")
    timer = Timer(torch, torch.cuda.Stream())
    d, f, L = 4096, 11008, 32
    t0 = time.perf_counter()
    Qh_a, Qh_o = synth.random_orthogonal_blocks(21, d // 128), synth.random_orthogonal_blocks(22, d // 128)
    lam_h = synth.descending_spectrum(23, d, d // 128)
    Qf, lam_f = synth.random_orthogonal_dense(24, d), synth.descending_spectrum(25, d, 1)
    lam_n = synth.descending_spectrum(26, f, 1)
    base = {}
    ab = bool(absorbed)      # rotations folded into the producing layers offline (weight-splitting appendix)
    for j, name in enumerate("qkv"):
        base[name] = B.rosaq_pack_weights(synth.make_weight(40 + j, d, d), Qh_a, lam_h, K, 4, B.Q_HEADWISE,
                                          rotation_absorbed=ab)
    base["o"] = B.rosaq_pack_weights(synth.make_weight(43, d, d), Qh_o, lam_h, K, 4, B.Q_HEADWISE,
                                     rotation_absorbed=ab)
    for j, name in enumerate(("gate", "up")):
        base[name] = B.rosaq_pack_weights(synth.make_weight(44 + j, f, d), Qf, lam_f, K, 4, B.Q_FULL,
                                          rotation_absorbed=ab)
    base["down"] = B.rosaq_pack_weights(synth.make_weight(46, d, f), None, lam_n, K, 4, B.Q_NONE)
    t_pack = time.perf_counter() - t0
    layers = [base] + [{k: B.rosaq_packed_clone(h) for k, h in base.items()} for _ in range(L - 1)]
    packed_bytes = sum(h.device_bytes for lay in layers for h in lay.values())

    x = torch.from_numpy(synth.make_activations(7, M, d)).to(dev)
    xh = torch.from_numpy(synth.make_activations(8, M, f)).to(dev)
    y_d = [torch.empty((M, d), dtype=torch.float16, device=dev) for _ in range(4)]
    y_f = [torch.empty((M, f), dtype=torch.float16, device=dev) for _ in range(2)]
    ws_bytes = max([B.rosaq_workspace_bytes(h, M) for h in base.values()] +
                   [B.rosaq_workspace_bytes_batch([base[n] for n in "qkv"], M),
                    B.rosaq_workspace_bytes_batch([base["gate"], base["up"]], M),
                    B.rosaq_workspace_bytes_mlp(base["gate"], base["up"], base["down"], M)])
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    qkv = [B.BatchArgs([lay[n] for n in "qkv"], [y.data_ptr() for y in y_d[:3]], [y.stride(0) for y in y_d[:3]])
           for lay in layers]

    def step():
        sp = T.current_stream_ptr()
        for l, lay in enumerate(layers):
            B.rosaq_linear_batch(qkv[l], x.data_ptr(), M, x.stride(0), ws.data_ptr(), ws.numel(), sp)
            T.linear(lay["o"], x, y_d[3], ws)
            if chained_mlp:
                # gate and up in one launch, silu(gate) * up applied in its epilogue and written as the
                # down projection's input fragments; then the down projection
                B.rosaq_mlp_swiglu(lay["gate"], lay["up"], lay["down"], x.data_ptr(), M, x.stride(0),
                                   y_d[3].data_ptr(), y_d[3].stride(0), ws.data_ptr(), ws.numel(), sp)
            else:
                B.rosaq_linear_swiglu(lay["gate"], lay["up"], x.data_ptr(), M, x.stride(0), y_f[0].data_ptr(),
                                      y_f[0].stride(0), ws.data_ptr(), ws.numel(), sp)
                T.linear(lay["down"], xh, y_d[3], ws)

    # fp16: the same seven linears per layer as separate vendor GEMMs, and with q/k/v and gate/up fused
    W_qkv = [torch.randn((3 * d, d), dtype=torch.float16, device=dev) * 0.02 for _ in range(L)]
    W_o = [torch.randn((d, d), dtype=torch.float16, device=dev) * 0.02 for _ in range(L)]
    W_gu = [torch.randn((2 * f, d), dtype=torch.float16, device=dev) * 0.02 for _ in range(L)]
    W_dn = [torch.randn((d, f), dtype=torch.float16, device=dev) * 0.02 for _ in range(L)]
    y_qkv = torch.empty((M, 3 * d), dtype=torch.float16, device=dev)
    y_gu = torch.empty((M, 2 * f), dtype=torch.float16, device=dev)

    def step16_fused():
        for l in range(L):
            torch.matmul(x, W_qkv[l].t(), out=y_qkv)
            torch.matmul(x, W_o[l].t(), out=y_d[3])
            torch.matmul(x, W_gu[l].t(), out=y_gu)
            torch.matmul(xh, W_dn[l].t(), out=y_d[3])

    def step16_separate():
        for l in range(L):
            for j in range(3):
                torch.matmul(x, W_qkv[l][j * d:(j + 1) * d].t(), out=y_d[j])
            torch.matmul(x, W_o[l].t(), out=y_d[3])
            for j in range(2):
                torch.matmul(x, W_gu[l][j * f:(j + 1) * f].t(), out=y_f[j])
            torch.matmul(xh, W_dn[l].t(), out=y_d[3])

    t = timer.run(step, steps, warmup)
    B.rosaq_tune("stages", 2)
    t_gemm = timer.run(step, steps, warmup)
    B.rosaq_tune("stages", 3)
    t16f = timer.run(step16_fused, steps, warmup)
    t16s = timer.run(step16_separate, steps, warmup)

    per_layer = (4 * d * row_bytes(d, 4) + 2 * f * row_bytes(d, 4) + d * row_bytes(f, 4)   # packed weights
                 + (0 if ab else 2 * 2 * 128 * d + 2 * d * d)                       # two head-wise + one dense rotation
                 + 2 * M * (4 * d + 4 * d) + 2 * M * (d + f) + 2 * M * (f + d))      # x and y of the four calls
    fp16_layer = 2 * (4 * d * d + 3 * d * f) + 2 * M * (2 * d + 4 * d) + 2 * M * (d + 2 * f) + 2 * M * (f + d)
    ms = t["median"]
    ffn = ("rosaq_mlp_swiglu(gate,up,down; silu(gate)*up written as down's input fragments)" if chained_mlp else
           "rosaq_linear_swiglu(gate,up; silu(gate)*up in the epilogue) + rosaq_linear(down)")
    out = {
        "workload": "llama7b_decode_linears_M64_int4" + ("_rotations_absorbed" if ab else ""),
        "layers": L, "linears_per_step": 7 * L, "M": M,
        "calls_per_layer": (("rosaq_linear_batch(q,k,v) + rosaq_linear(o) + " + ffn +
                             ": inputs arrive rotated, run time only permutes them") if ab else
                            ("rosaq_linear_batch(q,k,v; head-wise) + rosaq_linear_headwise(o) + " + ffn +
                             "; gate/up behind one dense 4096^2 rotation, down without rotation")),
        "steps_timed": steps, "ms_per_step": round(ms, 4), "ms_per_step_p10": round(t["p10"], 4),
        "ms_per_step_p90": round(t["p90"], 4), "total_s": round(ms * steps * 1e-3, 4),
        "tokens_per_s": round(M / (ms * 1e-3), 1),
        "ms_per_step_main_gemms_only": round(t_gemm["median"], 4),
        "algorithmic_GB_per_step": round(per_layer * L / 1e9, 3),
        "GBps": round(per_layer * L / ms / 1e6, 1),
        "frac_of_hbm_peak": round(per_layer * L / ms / 1e6 / HBM_PEAK_GBS, 4),
        "packed_GB_resident": round(packed_bytes / 1e9, 3),
        "setup_s_one_layer_incl_synthetic_weights": round(t_pack, 1),
        "fp16": {"impl": "torch.matmul fp16 (vendor GEMM), one hipGraph per step; no activation kernel",
                 "ms_per_step_4_gemms_per_layer_fused_qkv_gateup": round(t16f["median"], 4),
                 "ms_per_step_7_gemms_per_layer": round(t16s["median"], 4),
                 "GB_per_step": round(fp16_layer * L / 1e9, 3),
                 "GBps_fused": round(fp16_layer * L / t16f["median"] / 1e6, 1)},
        "speedup_vs_fp16_fused": round(t16f["median"] / ms, 3),
        "speedup_vs_fp16_separate": round(t16s["median"] / ms, 3),
        "data": "synthetic"}
    for lay in layers:
        for h in lay.values():
            h.free()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--layers", type=int, default=10, help="distinct layers (x4 packed weights)")
    ap.add_argument("--unbatched", action="store_true", help="one call per linear (no q/k/v batching)")
    ap.add_argument("--only", choices=["qkv", "o"], default=None,
                    help="tuning aid: issue only the batched q/k/v call or only the o call of each layer")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of one hipGraph per step")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fp16", action="store_true", help="skip the fp16 GEMM comparison")
    ap.add_argument("--no-probe", action="store_true", help="skip the pure read-stream ceiling")
    ap.add_argument("--no-sweep", action="store_true", help="skip the bounded MLP sweep of the default line")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode step of the default line")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the bench, time every MLP / attention shape of the task's configs "
                         "(one JSON line each)")
    ap.add_argument("--decode", action="store_true",
                    help="instead of the bench, time the seven linears x 32 layers of a 7B-shaped decode step "
                         "at batch 64 against fp16 vendor GEMMs (one JSON line)")
    ap.add_argument("--decode-steps", type=int, default=256)
    ap.add_argument("--absorbed", action="store_true",
                    help="with --decode: pack every layer with rotation_absorbed (the paper's deployment: "
                         "rotations folded into the producing layers offline, no rotation at run time)")
    ap.add_argument("--unchained-mlp", action="store_true",
                    help="with --decode: rosaq_linear_swiglu + rosaq_linear(down) instead of rosaq_mlp_swiglu")
    ap.add_argument("--sweep-filter", default="", help="substring of the shape names to run")
    ap.add_argument("--sweep-m", default="", help="comma-separated M values replacing each shape's own list")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="instead of the bench, run 20 plain device copies of this size "
                         "(reference for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--mt", type=int, default=0, help="tuning aid: 16-row tiles per workgroup")
    ap.add_argument("--nt", type=int, default=0, help="tuning aid: 16-channel tiles per workgroup")
    ap.add_argument("--wpb", type=int, default=0, help="tuning aid: waves per workgroup (8 or 16)")
    ap.add_argument("--depth", type=int, default=0, help="tuning aid: units in flight per wave (2-4)")
    ap.add_argument("--splits", type=int, default=0, help="tuning aid: workgroups per output tile (1-16)")
    ap.add_argument("--rot", default="", help="tuning aid: mt,nt,depth of the dense-rotation launch")
    ap.add_argument("--rot-splits", type=int, default=0, help="tuning aid: slabs of the contraction for the dense rotation of 17-64 rows (2-16)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (--gpus 1); no multi-GPU path exists", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2506_13472_amd import binding as B, synth, torch_glue as T

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.copy_calibration:
        n = args.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": n, "bytes_written": n, "copies": 20}))
        return
    B.lib()
    for key in ("mt", "nt", "wpb", "depth", "splits"):
        B.rosaq_tune(key, getattr(args, key))
    if args.rot:
        for key, v in zip(("rot_mt", "rot_nt", "rot_depth"), args.rot.split(",")):
            B.rosaq_tune(key, int(v))
    B.rosaq_tune("rot_splits", args.rot_splits)
    if args.sweep:
        shapes = [s for s in SWEEP_SHAPES if not args.sweep_filter or args.sweep_filter in s[0]]
        ms = [int(v) for v in args.sweep_m.split(",")] if args.sweep_m else None
        shape_sweep(torch, shapes, ms, 20, lambda row: print(json.dumps(row), flush=True))
        return
    if args.decode:
        print(json.dumps(decode_workload(torch, args.decode_steps, args.warmup, args.absorbed, not args.unchained_mlp)), flush=True)
        return

    # ---- synthetic layers: calibrate (PCA per head on the GPU), pack, all through the C ABI ------
    # q, k, v read the same activations, hence share one PCA; o has its own input and PCA.
    t_pack = 0.0
    t_pca = 0.0
    handles = []
    rot_first = None
    for layer in range(args.layers):
        rot = []
        for which in range(2):
            xc = torch.from_numpy(synth.make_activations(5000 + 2 * layer + which, 512, D)).to(dev)
            t0 = time.perf_counter()
            rot.append(B.rosaq_pca_headwise(xc.data_ptr(), 512, D, xc.stride(0)))
            t_pca += time.perf_counter() - t0
        if rot_first is None:
            rot_first = rot[0]
        for j in range(4):
            W = synth.make_weight(1000 + 4 * layer + j, N, D)
            Qb, lam = rot[0] if j < 3 else rot[1]
            t0 = time.perf_counter()
            handles.append(B.rosaq_pack_weights(W, Qb, lam, K, BITS, B.Q_HEADWISE))
            t_pack += time.perf_counter() - t0
    packed_bytes = sum(h.device_bytes for h in handles)
    x = torch.from_numpy(synth.make_activations(7, M, D)).to(dev)
    ys = [torch.empty((M, N), dtype=torch.float16, device=dev) for _ in range(4)]
    ws = torch.empty(B.rosaq_workspace_bytes_batch(handles[:3], M), dtype=torch.uint8, device=dev)

    timer = Timer(torch, torch.cuda.Stream(), eager=args.no_graph)
    calls = [(handles[i % len(handles)], ys[i % 4]) for i in range(CALLS_PER_STEP)]
    n_layers = CALLS_PER_STEP // 4
    qkv = [B.BatchArgs([handles[(4 * l + j) % len(handles)] for j in range(3)],
                       [ys[j].data_ptr() for j in range(3)], [ys[j].stride(0) for j in range(3)])
           for l in range(n_layers)]
    wo = [handles[(4 * l + 3) % len(handles)] for l in range(n_layers)]

    def issue_step():
        if args.unbatched:
            for h, y in calls:
                T.linear(h, x, y, ws)
            return
        sp = T.current_stream_ptr()
        for l in range(n_layers):
            if args.only != "o":
                B.rosaq_linear_batch(qkv[l], x.data_ptr(), M, x.stride(0), ws.data_ptr(), ws.numel(), sp)
            if args.only != "qkv":
                T.linear(wo[l], x, ys[3], ws)

    t_step = timer.run(issue_step, args.steps, args.warmup)
    # dominant kernel alone (main GEMM; xhat fragments left in the workspace by the runs above)
    B.rosaq_tune("stages", 2)
    t_gemm = timer.run(issue_step, args.steps, args.warmup)
    B.rosaq_tune("stages", 1)
    t_rot = timer.run(issue_step, args.steps, args.warmup)
    B.rosaq_tune("stages", 3)

    ab = algorithmic_bytes()
    calls_per_step = CALLS_PER_STEP if not args.only else CALLS_PER_STEP // 4 * (3 if args.only == "qkv" else 1)
    us_call = t_step["median"] * 1e3 / calls_per_step
    gbs = ab["call"] * calls_per_step / (t_step["median"] * 1e-3) / 1e9
    # per launch of the dominant kernel: unbatched, every launch is one linear; batched, a
    # layer issues one q/k/v launch and one o launch (the mean launch moves half of both)
    shape_one = tuple(B.rosaq_launch_shape(M, N, D, BITS))
    shape_qkv = tuple(B.rosaq_launch_shape(M, 3 * N, D, BITS))
    launch_kinds = {"o": [(1, shape_one, ab["gemm_kernel"])], "qkv": [(3, shape_qkv, ab["gemm_kernel_qkv"])]}
    if args.unbatched:
        kinds, launches = launch_kinds["o"], CALLS_PER_STEP
    elif args.only:
        kinds, launches = launch_kinds[args.only], n_layers
    else:
        kinds, launches = launch_kinds["qkv"] + launch_kinds["o"], 2 * n_layers
    gemm_bytes = sum(k[2] for k in kinds) // len(kinds)
    us_gemm = t_gemm["median"] * 1e3 / launches
    gemm_gbs = gemm_bytes / (us_gemm * 1e-6) / 1e9
    measured = [MEASURED_TRAFFIC_KIB.get((k[0],) + k[1]) for k in kinds]
    if all(m is not None for m in measured):
        traffic = sum((m[0] + m[1]) * 1024 for m in measured) // len(measured)
        traffic_note = "rocprofv3 FETCH_SIZE x 2.0 + WRITE_SIZE, mean over the launch kinds of a step"
    else:
        traffic = None
        traffic_note = ("no rocprofv3 measurement on file for launch shape(s) " +
                        ", ".join(str((k[0],) + k[1]) for k, m in zip(kinds, measured) if m is None))

    # ---- fp16 dense GEMM on the same shape, same cold-weight protocol ----------------
    fp16 = None
    if not args.no_fp16:
        n_w = max(8, (len(handles) * ab["weights"]) // (2 * N * D) + 1)
        Ws = [torch.randn((N, D), dtype=torch.float16, device=dev) * 0.02 for _ in range(n_w)]
        yb = torch.empty((M, N), dtype=torch.float16, device=dev)

        def fp16_step():
            for i in range(CALLS_PER_STEP):
                torch.matmul(x, Ws[i % n_w].t(), out=yb)
        us16 = timer.run(fp16_step, args.steps, args.warmup)["median"] * 1e3 / CALLS_PER_STEP
        fp16 = {"us_per_call": round(us16, 3),
                "GBps": round((2 * N * D + ab["xy"]) / (us16 * 1e-6) / 1e9, 1),
                "rosaq_speedup": round(us16 / us_call, 3), "impl": "torch.matmul fp16 (vendor GEMM)"}
        del Ws
        # the library's own all-fp16 path: the same layer packed with K = D (every channel salient),
        # four calls per layer like the unbatched workload
        h16 = [B.rosaq_pack_weights(synth.make_weight(1000, N, D), *rot_first, D, BITS, B.Q_HEADWISE)]
        while len(h16) < n_w:
            h16.append(B.rosaq_packed_clone(h16[0]))

        def own16_step():
            for i in range(CALLS_PER_STEP):
                T.linear(h16[i % n_w], x, yb, ws)
        fp16["own_all_salient_us_per_call"] = round(
            timer.run(own16_step, args.steps, args.warmup)["median"] * 1e3 / CALLS_PER_STEP, 3)
        for h in h16:
            h.free()

    # ---- the memory system's own ceiling: a pure read stream of one linear's size ------
    probe = None
    if not args.no_probe:
        pb = 10 << 20                                     # ~ one packed 4096 x 4096 INT4 layer
        n_src = max(8, packed_bytes // pb + 1)
        srcs = [torch.ones(pb, dtype=torch.uint8, device=dev) for _ in range(n_src)]
        shared = torch.ones(512 << 10, dtype=torch.uint8, device=dev)       # = 64 x 4096 fp16
        sink = torch.zeros(256 * 8 * 1024, dtype=torch.uint8, device=dev)
        probe = {"bytes_per_launch": pb, "launch": "256 workgroups x 512 threads"}
        for name, per_wg in (("weights_only_us", 0), ("with_256KiB_shared_per_workgroup_us", 256 << 10)):
            def probe_step():
                sp = T.current_stream_ptr()
                for i in range(CALLS_PER_STEP):
                    B.rosaq_stream_probe(srcs[i % n_src].data_ptr(), pb, shared.data_ptr(), shared.numel(),
                                         per_wg, 256, 512, sink.data_ptr(), sink.numel(), sp)
            probe[name] = round(timer.run(probe_step, args.steps, args.warmup)["median"] * 1e3 / CALLS_PER_STEP, 3)
        probe["weights_only_GBps"] = round(pb / (probe["weights_only_us"] * 1e-6) / 1e9, 1)
        del srcs

    out = {
        "metric": "fused ROSAQ linear HBM GB/s at M=64 (algorithmic bytes / time)",
        "value": round(gbs, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(t_step["wall"], 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f16 x int4 -> f32 accumulate", "data": "synthetic",
        "config": {"workload": "llama7b_attn_qkvo_M64_int4_headwise", "D": D, "N": N, "M": M, "K": K,
                   "bits": BITS, "group": GROUP, "heads": HEADS, "calls_per_step": calls_per_step,
                   "distinct_packed_weights": len(handles), "packed_MB": round(packed_bytes / 1e6, 1),
                   "launch": "eager" if args.no_graph else "hipGraph per step",
                   "calls": "4 x rosaq_linear_headwise per layer" if args.unbatched else
                            "rosaq_linear_batch(q,k,v) + rosaq_linear_headwise(o) per layer",
                   "tiles": {k: getattr(args, k) or "heuristic" for k in ("mt", "nt", "wpb", "depth", "splits")},
                   "launch_shape_mt_nt_waves_depth_splits": {"one_layer": list(shape_one), "qkv": list(shape_qkv)}},
        "timing": "each step between its own pair of HIP events on the launch stream; value, us_per_linear and "
                  "frac_of_hbm_peak use the median step; ms_per_step is host wall time over all steps / steps",
        "step_ms": {"median": round(t_step["median"], 5), "p10": round(t_step["p10"], 5),
                    "p90": round(t_step["p90"], 5)},
        "us_per_linear": round(us_call, 3),
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "tflops": round(2.0 * M * N * (D + 128) / (us_call * 1e-6) / 1e12, 2),
        "rotation_kernel_us": round(t_rot["median"] * 1e3 / launches, 3),
        "pack_seconds_per_layer": round(t_pack / len(handles), 3),
        "pca_seconds_per_rotation": round(t_pca / (2 * args.layers), 4),
        "fp16_gemm": fp16,
        "stream_probe": probe,
        "roofline": {"kernel": "gemm_kernel", "bound": "hbm", "achieved": round(gemm_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(gemm_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_note": traffic_note, "bytes_per_launch": gemm_bytes,
                     "launches_per_step": launches, "us_per_launch": round(us_gemm, 3),
                     "us_per_launch_p10": round(t_gemm["p10"] * 1e3 / launches, 3),
                     "us_per_launch_p90": round(t_gemm["p90"] * 1e3 / launches, 3)},
    }
    for h in handles:
        h.free()
    del handles, qkv, wo, calls
    torch.cuda.empty_cache()
    if not args.no_sweep:
        rows = []
        # the INT3 7B MLP at M = 64; the INT4 13B MLP at its whole M sweep (the shape's own list)
        shape_sweep(torch, [s for s in SWEEP_SHAPES if s[0].startswith("7B") and s[0].startswith(BOUNDED_SWEEP)],
                    [64], 10, rows.append)
        shape_sweep(torch, [s for s in SWEEP_SHAPES if s[0].startswith("13B")], None, 10, rows.append)
        out["sweep"] = {"what": "single calls of the INT3 7B MLP shapes at M = 64 and of the INT4 13B MLP shapes at "
                                "M = 1, 16, 64, 256 (dense 13824^2 rotation: M = 64), K = 128, median of 10 replays "
                                "of 32 calls over distinct weight copies (cold HBM)",
                        "rows": rows}
        torch.cuda.empty_cache()
    if not args.no_decode:
        out["decode"] = decode_workload(torch, args.decode_steps, args.warmup)
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
