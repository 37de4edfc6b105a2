#!/usr/bin/env python3
"""MoBA forward+backward benchmark on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic input that
is already resident in HBM: key conv (if any) + centroids -> gate scores + top-k +
key-block lists -> forward attention -> backward (D, dQ, dK/dV).  The default
workload is the N = 32768, B = 32, top-k 64 configuration the headline metric is
quoted on.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--no-cpu-baseline]
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

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3      # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch (fetch + write) of a kernel come from the rocprofv3 --pmc summaries kept
# under profiles/ (FETCH_SIZE and WRITE_SIZE per dispatch, already scaled there by what the same
# counters read for a plain copy of known size): profiles/config<N>_hbm_traffic.txt, one row per
# kernel, last column = bytes per launch.  Not measured -> None.
PROFILED_KERNEL = {"topk": "topk_mfma_kernel", "forward": ("forward_mfma_kernel", "fwd_km_kernel"),
                   "bwd_dq": ("dq_mfma_kernel", "dq_km_kernel"), "bwd_dkdv": "dkdv_mfma_kernel"}


def measured_traffic(config, kernel):
    path = os.path.join(ROOT, "profiles", "config%d_hbm_traffic.txt" % config)
    names = PROFILED_KERNEL.get(kernel)
    if names is None or not os.path.exists(path):
        return None
    names = (names,) if isinstance(names, str) else names
    for line in open(path):
        f = line.split()
        if len(f) == 4 and f[0] in names:
            try:
                return float(f[3])
            except ValueError:
                pass
    return None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--rotate-inputs", type=int, default=1, metavar="SETS",
                    help="cycle through SETS copies of the input tensors, one per step, so that a step "
                         "does not find its inputs in the 256 MB Infinity Cache (for the HBM-bound "
                         "stage rates; default 1: the same tensors every step)")
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="benchmark configuration 1..5")
    ap.add_argument("--shape", default="",
                    help="instead of --config: batch,heads,N,d,B,k[,fwd] (bf16, no conv), e.g. the "
                         "paper's latency sweep 2,16,65536,64,128,8")
    ap.add_argument("--reference-kernels", action="store_true",
                    help="force the plain (non-MFMA) kernels")
    ap.add_argument("--attention", choices=["auto", "tiles", "keymajor"], default="auto",
                    help="force the query-tile or the key-block-major attention kernels")
    ap.add_argument("--latency-sweep", default="",
                    help="instead of one workload: the paper's latency sweep (Section 5.3: batch 2, "
                         "B = 128, top-k 8, forward + backward; here 16 heads of d = 64) over the "
                         "comma-separated sequence lengths given, e.g. 8192,16384,...,524288; "
                         "prints one JSON line with one point per length")
    ap.add_argument("--dense-upto", type=int, default=0,
                    help="with --latency-sweep: for sequence lengths up to this one also time the "
                         "same kernels with every past block kept (top-k = n: full causal attention), "
                         "the reference line of the sweep")
    ap.add_argument("--kv-heads", type=int, default=0,
                    help="grouped-query attention: key/value heads of the workload (0 = as many as "
                         "query heads)")
    ap.add_argument("--decode", type=int, default=0, metavar="Q_LEN",
                    help="instead of a training-shaped step: time the decode-shaped forward for the "
                         "last Q_LEN positions of the workload's sequence plus 37 tokens (a ragged "
                         "last block); prints one JSON line")
    ap.add_argument("--varlen", default="", metavar="L1,L2,...",
                    help="a packed variable-length batch of these sequence lengths instead of one "
                         "sequence (heads, d, B, top-k of --config / --shape): pad, centroids, gate top-k "
                         "per sequence, forward, backward, unpad")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed steps, copy 1 GiB device to device once (a kernel of "
                         "known HBM traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--separate-workspaces", action="store_true",
                    help="give forward and backward a workspace each (every call then makes its own copies "
                         "of K and V) instead of one shared workspace prepared by the forward call")
    ap.add_argument("--microbench", action="store_true",
                    help="also run the library's two ceiling measurements once (a plain 1 GiB copy kernel, "
                         "a register-only bf16 MFMA loop) and report the fractions of those measured "
                         "ceilings next to the fractions of the published peaks")
    ap.add_argument("--cpu-max-slices", type=int, default=0,
                    help="cap on the (batch, head) slices of the CPU-baseline sample")
    return ap.parse_args()


def cpu_baseline(w, t, target_seconds=15.0, max_slices=0):
    """Times the CPU oracle, as it stands, on a bounded sample of the same workload: whole
    (batch, head) slices, starting with slice 0 and adding slices until about
    `target_seconds` of CPU work.  Each sampled slice runs the full chain (conv if any,
    centroids, gate top-k, lists, forward, and for backward workloads D, dQ and dK/dV).
    The rate uses the same effective flop count as the GPU metric (4d per attended pair
    forward, 10d backward)."""
    import numpy as np
    import workloads
    from oracle import moba_oracle as orc

    def run(lo, hi):
        b, h = w.batch, w.heads
        sl = [(s // h, s % h) for s in range(lo, hi)]
        pick = lambda x: np.stack([workloads.to_f64(t[x][bi:bi + 1, hi_:hi_ + 1])[0] for bi, hi_ in sl])
        Q, K, V, dO = (pick(x) for x in ("Q", "K", "V", "dO"))
        t0 = time.perf_counter()
        Kp = K
        if w.conv_width:
            mode = orc.ROUND_BF16 if w.dtype == "bf16" else orc.ROUND_F32
            cw = t["conv_w"].double().numpy()
            Kp = np.stack([orc.key_conv(K[i:i + 1], cw[hh:hh + 1], 1, mode)[0]
                           for i, (_, hh) in enumerate(sl)])
        C = orc.centroids(Kp, w.B)
        idx, _ = orc.topk(Q, C, w.B, w.k)
        O, lse = orc.attn_fwd(Q, Kp, V, idx, w.B, w.scale)
        if w.backward:
            Dv = (dO * O).sum(-1)
            off, ql = orc.csr(idx, w.B)
            orc.attn_bwd_dq(Q, Kp, V, idx, dO, lse, Dv, w.B, w.scale)
            orc.attn_bwd_dkdv(Q, Kp, V, dO, lse, Dv, off, ql, w.B, w.scale)
        return time.perf_counter() - t0

    dt = run(0, 1)
    ns = 1
    extra = min(w.bh - 1, int(target_seconds / max(dt, 1e-3)) - 1)
    if max_slices:
        extra = min(extra, max_slices - 1)
    if extra > 0:
        dt += run(1, 1 + extra)
        ns += extra
    pairs = ns * workloads.attended_pairs_per_slice(w.N, w.B, w.k)
    flops = (4 + (10 if w.backward else 0)) * w.d * pairs
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": orc.num_threads(), "kind": "oracle",
        "seconds": dt, "build": orc.BUILD_COMMAND,
        "sample": "%d of %d (batch, head) slices, whole chain (%scentroids, gate top-k, lists, "
                  "forward%s); %d attended pairs" % (
                      ns, w.bh, "key conv, " if w.conv_width else "",
                      ", backward" if w.backward else "", pairs),
    }


def measure(w, a, moba, binding, workloads, torch):
    """Times a.steps passes of the whole path over workload w (inputs resident in HBM)."""
    t = workloads.generate(w)
    d = {k: (v.cuda() if v is not None else None) for k, v in t.items()}
    sets = [d] + [{k: (v.clone() if v is not None else None) for k, v in d.items()}
                  for _ in range(max(a.rotate_inputs, 1) - 1)]
    flags = binding.FLAG_REFERENCE_KERNELS if a.reference_kernels else 0
    flags |= {"auto": 0, "tiles": binding.FLAG_QUERY_TILES, "keymajor": binding.FLAG_KEY_MAJOR}[a.attention]
    if w.backward and not a.separate_workspaces:
        flags |= binding.FLAG_SHARED_WORKSPACE      # forward and backward share the prepared copies of K and V
    sh = moba.Shape(w.batch, w.heads, w.N, w.d, w.B, w.k, w.conv_width,
                    binding.BF16 if w.dtype == "bf16" else binding.F32, 0.0, flags, w.kv_heads)
    R = moba.routes_per_slice(sh)
    sizes = moba.workspace_bytes(sh)
    ws_topk = torch.empty(max(sizes[0], 256), dtype=torch.uint8, device="cuda")
    if flags & binding.FLAG_SHARED_WORKSPACE:
        ws_fwd = ws_bwd = torch.empty(max(sizes[1], sizes[2], 256), dtype=torch.uint8, device="cuda")
    else:
        ws_fwd, ws_bwd = (torch.empty(max(x, 256), dtype=torch.uint8, device="cuda") for x in sizes[1:])
    dev = torch.device("cuda")
    Keff = torch.empty_like(d["K"]) if w.conv_width else None
    cent = torch.empty((w.batch, w.hkv, w.n, w.d), dtype=torch.float32, device=dev)
    O = torch.empty_like(d["Q"])
    lse = torch.empty((w.batch, w.heads, w.N), dtype=torch.float32, device=dev)
    grads = (torch.empty_like(d["Q"]), torch.empty_like(d["K"]), torch.empty_like(d["V"]))

    stages = ["centroids", "topk_lists", "forward", "bwd_pre", "bwd_dq", "bwd_dkdv"]
    if not w.backward:
        stages = stages[:3]

    def step(events=None, d=d):
        def mark(i):
            if events is not None:
                events[i].record()
        mark(0)
        Ke, c = moba.centroids(sh, d["K"], d["conv_w"], K_eff=Keff, out=cent)
        mark(1)
        idx, lists = moba.topk(sh, d["Q"], c, ws=ws_topk)
        mark(2)
        moba.forward(sh, d["Q"], Ke, d["V"], idx, lists, ws=ws_fwd, O=O, lse=lse)
        mark(3)
        if w.backward:
            for i, part in enumerate((binding.BWD_PREPROCESS, binding.BWD_DQ, binding.BWD_DKDV)):
                moba.backward(sh, d["Q"], Ke, d["V"], O, lse, d["dO"], idx, lists, ws=ws_bwd,
                              out=grads, parts=part)
                mark(4 + i)

    for s in range(a.warmup):
        step(None, sets[s % len(sets)])
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)]
          for _ in range(a.steps)]
    torch.cuda.synchronize()
    moba.profile_begin()          # HIP events around every main kernel, on its launch stream
    t0 = time.perf_counter()
    for s in range(a.steps):
        step(ev[s], sets[s % len(sets)])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kernel_ms = {name: (tot / max(n, 1)) for name, (tot, n) in moba.profile_end().items() if n}
    ms_step = 1e3 * wall / a.steps
    stage_ms = {name: sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(a.steps)) / a.steps
                for i, name in enumerate(stages)}

    return {"t": t, "d": d, "sh": sh, "R": R, "dev": dev, "ms_step": ms_step, "stage_ms": stage_ms,
            "kernel_ms": kernel_ms, "stages": stages}


def decode_bench(w, a, moba, binding, torch):
    """Latency of moba_decode_forward: q_len queries at the end of N = w.N + 37 keys (so that the
    own block is ragged), centroids of the complete blocks resident as a caller's cache would
    hold them.  HBM-side work per call: the centroids, and k + 1 blocks of K and V per query."""
    q_len, N = a.decode, w.N + 37
    dt = w.torch_dtype
    es = 2 if w.dtype == "bf16" else 4
    g = torch.Generator(device="cuda").manual_seed(w.seed)
    Q = torch.randn((w.batch, w.heads, q_len, w.d), generator=g, device="cuda").to(dt)
    K = torch.randn((w.batch, w.hkv, N, w.d), generator=g, device="cuda").to(dt)
    V = torch.randn((w.batch, w.hkv, N, w.d), generator=g, device="cuda").to(dt)
    npast = (N - 1) // w.B
    cent = K[:, :, :npast * w.B].float().reshape(w.batch, w.hkv, npast, w.B, w.d).mean(3).contiguous()
    sh = moba.Shape(w.batch, w.heads, N, w.d, w.B, w.k, 0,
                    binding.BF16 if w.dtype == "bf16" else binding.F32, 0.0, 0, w.kv_heads)
    for _ in range(max(a.warmup, 1)):
        moba.decode_forward(sh, q_len, Q, K, V, cent, want_idx=False)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = max(a.steps, 1) * 20
    e0.record()
    for _ in range(reps):
        moba.decode_forward(sh, q_len, Q, K, V, cent, want_idx=False)
    e1.record()
    torch.cuda.synchronize()
    us = 1e3 * e0.elapsed_time(e1) / reps
    bytes_call = w.bh * q_len * (npast * w.d * 4 + 2 * (min(w.k, npast) + 1) * w.B * w.d * es)
    print(json.dumps({
        "metric": "moba_decode_forward_latency", "value": us, "unit": "us", "n_gpus": 1, "steps": reps,
        "warmup": max(a.warmup, 1), "higher_is_better": False, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "decode: batch %d, heads %d (%d key/value heads), %d queries at the end of "
                               "%d keys, d %d, B %d, top-k %d, I/O %s" % (
                                   w.batch, w.heads, w.hkv, q_len, N, w.d, w.B, w.k, w.dtype)},
        "roofline": {"kernel": "decode", "bound": "hbm", "achieved": bytes_call / (us * 1e-6) / 1e9,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": bytes_call / (us * 1e-6) / 1e9 / PEAK_HBM_GBS,
                     "bytes_per_launch": bytes_call, "traffic": None}}))


def varlen_bench(w, a, moba, binding, torch):
    """One step = the whole path over a packed batch: copy into the padded layout, centroids, gate
    top-k with per-sequence candidates + lists, forward, backward, copy results back."""
    lens = [int(x) for x in a.varlen.split(",")]
    offs = [0]
    for L in lens:
        offs.append(offs[-1] + L)
    T = offs[-1]
    lay = moba.VarlenLayout(offs, w.B)
    Tp = lay.padded_tokens
    dt = w.torch_dtype
    g = torch.Generator(device="cuda").manual_seed(w.seed)
    Q, dO = (torch.randn((1, w.heads, T, w.d), generator=g, device="cuda").to(dt) for _ in range(2))
    K, V = (torch.randn((1, w.hkv, T, w.d), generator=g, device="cuda").to(dt) for _ in range(2))
    flags = binding.FLAG_SHARED_WORKSPACE
    sh = moba.Shape(1, w.heads, Tp, w.d, w.B, w.k, 0, binding.BF16 if w.dtype == "bf16" else binding.F32,
                    0.0, flags, w.kv_heads)
    sizes = moba.workspace_bytes(sh)
    ws_topk = torch.empty(max(sizes[0], 256), dtype=torch.uint8, device="cuda")
    ws_att = torch.empty(max(sizes[1], sizes[2], 256), dtype=torch.uint8, device="cuda")
    stages = ["pad", "centroids", "topk_lists", "forward", "backward", "unpad"]

    def step(ev=None):
        def mark(i):
            if ev is not None:
                ev[i].record()
        mark(0)
        Qp, Kp, Vp, dOp = (lay.pad(x) for x in (Q, K, V, dO))
        mark(1)
        _, cent = moba.centroids(sh, Kp)
        mark(2)
        idx, lists = moba.topk_varlen(sh, lay, Qp, cent, ws=ws_topk)
        mark(3)
        O, lse = moba.forward(sh, Qp, Kp, Vp, idx, lists, ws=ws_att)
        mark(4)
        grads = moba.backward(sh, Qp, Kp, Vp, O, lse, dOp, idx, lists, ws=ws_att)
        mark(5)
        out = [lay.unpad(x) for x in (O, lse) + tuple(grads)]
        mark(6)
        return out

    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)] for _ in range(a.steps)]
    t0 = time.perf_counter()
    for s in range(a.steps):
        step(ev[s])
    torch.cuda.synchronize()
    ms = 1e3 * (time.perf_counter() - t0) / a.steps
    stage_ms = {n: sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(a.steps)) / a.steps
                for i, n in enumerate(stages)}
    import workloads
    pairs = w.heads * sum(workloads.ragged_pairs(L, w.B, w.k) for L in lens)
    print(json.dumps({
        "metric": "moba_fwd_bwd_effective_tflops", "value": 14.0 * w.d * pairs / (ms * 1e-3) / 1e12,
        "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms,
        "higher_is_better": True, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "packed batch of %d sequences (%s tokens, %d in all, %d after padding to "
                               "blocks), heads %d (%d key/value heads), d %d, B %d, top-k %d, "
                               "forward+backward" % (len(lens), a.varlen, T, Tp, w.heads, w.hkv, w.d, w.B, w.k)},
        "stage_ms": stage_ms, "attended_pairs": pairs}))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every (batch, head) slice is independent; "
              "sharding them over several GPUs is designed, not built). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads
    import paper_2511_11571_amd as moba
    from paper_2511_11571_amd import binding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if a.latency_sweep:
        points = []
        for N_ in (int(x) for x in a.latency_sweep.split(",")):
            w = workloads.Workload("sweep_N%d" % N_, 2, 16, N_, 64, 128, 8, backward=True, seed=9100)
            m = measure(w, a, moba, binding, workloads, torch)
            points.append({"N": N_, "ms_per_step": m["ms_step"], "stage_ms": m["stage_ms"],
                           "kernel_ms": m["kernel_ms"],
                           "effective_tflops": 14.0 * w.d * w.bh * workloads.attended_pairs_per_slice(
                               w.N, w.B, w.k) / (m["ms_step"] * 1e-3) / 1e12})
            del m
            torch.cuda.empty_cache()
            if N_ <= a.dense_upto:
                wd = workloads.Workload("dense_N%d" % N_, 2, 16, N_, 64, 128, N_ // 128, backward=True, seed=9100)
                m = measure(wd, a, moba, binding, workloads, torch)
                points[-1]["dense_ms_per_step"] = m["ms_step"]
                points[-1]["dense_stage_ms"] = m["stage_ms"]
                del m
                torch.cuda.empty_cache()
        print(json.dumps({
            "metric": "moba_fwd_bwd_latency_sweep", "unit": "ms", "n_gpus": 1, "steps": a.steps,
            "warmup": a.warmup, "higher_is_better": False, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "batch 2, heads 16, d 64, B 128, top-k 8, forward+backward "
                                   "(gate + top-k + lists + attention + gradients)",
                       "attention": a.attention},
            "points": points}))
        return
    w = workloads.CONFIGS[a.config]
    if a.shape:
        f = a.shape.split(",")
        b_, h_, N_, d_, B_, k_ = (int(x) for x in f[:6])
        w = workloads.Workload("shape_%s" % a.shape.replace(",", "_"), b_, h_, N_, d_, B_, k_,
                               backward=not (len(f) > 6 and f[6] == "fwd"), seed=9000)
        a.config = 0
    if a.kv_heads:
        w = w.scaled(kv_heads=a.kv_heads, name=w.name + "_kv%d" % a.kv_heads)
        a.config = 0
    if a.decode:
        decode_bench(w, a, moba, binding, torch)
        return
    if a.varlen:
        varlen_bench(w, a, moba, binding, torch)
        return
    m = measure(w, a, moba, binding, workloads, torch)
    t, d, sh, R, dev = m["t"], m["d"], m["sh"], m["R"], m["dev"]
    ms_step, stage_ms, kernel_ms, stages = m["ms_step"], m["stage_ms"], m["kernel_ms"], m["stages"]

    pairs = w.bh * workloads.attended_pairs_per_slice(w.N, w.B, w.k)
    fwd_flop = 4.0 * w.d * pairs
    bwd_flop = 10.0 * w.d * pairs if w.backward else 0.0
    value = (fwd_flop + bwd_flop) / (ms_step * 1e-3) / 1e12

    # Roofline of the dominant kernel = the one with the longest launch among the four main
    # kernels, timed by the library with HIP events around each launch (kernel_ms; the stage
    # times above also hold the small preparation kernels of a stage).  The dK/dV kernel
    # executes 4 of the backward's matrix products (S, dP, dV, dK = 8d flop per attended pair),
    # the dQ kernel 3 (S, dP, dQ = 6d), the forward 2 (4d): bf16 MFMA work.  The gate/top-k
    # kernel is priced against HBM: it has to read Q and the centroids and write the routing.
    es = 2 if w.dtype == "bf16" else 4
    mfma = (w.dtype == "bf16") and not a.reference_kernels
    work = {"forward": ("flop", fwd_flop), "bwd_dq": ("flop", 6.0 * w.d * pairs),
            "bwd_dkdv": ("flop", 8.0 * w.d * pairs),
            "topk": ("byte", float(w.bh * (w.N * w.d * es + w.n * w.d * 4 + w.N * w.k * 4)))}
    timed = {k: v for k, v in kernel_ms.items() if k in work and (w.backward or not k.startswith("bwd"))}
    if timed:
        dom = max(timed, key=timed.get)
        dom_ms = timed[dom]
    else:                               # plain kernels: no event hooks, fall back to stage times
        dom = max((s for s in stages if s in work), key=lambda s: stage_ms[s])
        dom_ms = stage_ms[dom]
    kind, amount = work[dom]
    if kind == "flop":
        peak = PEAK_BF16_TFLOPS if mfma else PEAK_FP32_TFLOPS
        ach = amount / (dom_ms * 1e-3) / 1e12
        roofline = {"kernel": dom, "bound": "mfma" if mfma else "alu", "achieved": ach, "peak": peak,
                    "unit": "TFLOP/s", "frac": ach / peak, "flop_per_launch": amount}
    else:
        ach = amount / (dom_ms * 1e-3) / 1e9
        roofline = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": ach / PEAK_HBM_GBS, "bytes_per_launch": amount}
    roofline["ms_per_launch"] = dom_ms
    # every timed attention kernel against the same peak (algorithmic flop of its products / launch time)
    kernel_frac = {}
    if mfma:
        for kname, kms in timed.items():
            if work[kname][0] == "flop" and kms > 0:
                tf = work[kname][1] / (kms * 1e-3) / 1e12
                kernel_frac[kname] = {"tflops": tf, "frac_of_mfma_peak": tf / PEAK_BF16_TFLOPS}
    # the backward as the metric counts it: 10d flop per attended pair over both of its kernels (the
    # per-kernel figures above count what each kernel executes: S and dP are computed in both)
    if mfma and "bwd_dq" in timed and "bwd_dkdv" in timed:
        for kname in ("bwd_dq", "bwd_dkdv"):
            kernel_frac[kname]["counts"] = "executed flop of this kernel (%dd per attended pair)" % (
                6 if kname == "bwd_dq" else 8)
        bms = timed["bwd_dq"] + timed["bwd_dkdv"]
        tf = bwd_flop / (bms * 1e-3) / 1e12
        kernel_frac["backward"] = {"tflops": tf, "frac_of_mfma_peak": tf / PEAK_BF16_TFLOPS, "ms": bms,
                                   "counts": "algorithmic flop of the backward (10d per attended pair) over "
                                             "the dQ and the dK/dV kernel"}
        ams = bms + timed.get("forward", 0.0)
        tf = (fwd_flop + bwd_flop) / (ams * 1e-3) / 1e12
        kernel_frac["attention_stage"] = {"tflops": tf, "frac_of_mfma_peak": tf / PEAK_BF16_TFLOPS, "ms": ams,
                                          "counts": "algorithmic flop, forward + backward kernels"}
    roofline["traffic"] = measured_traffic(a.config, dom) if not a.reference_kernels else None
    # HBM-bound stages, for the record: algorithmic bytes / measured time
    cent_bytes = w.bh * (w.N * w.d * es * (2 if w.conv_width else 1) + w.n * w.d * 4)
    topk_bytes = w.bh * (w.N * w.d * es + w.n * w.d * 4 + w.N * w.k * 4 + R * 4 + (w.n + 1) * 4)
    hbm = {"centroids_GBs": cent_bytes / (stage_ms["centroids"] * 1e-3) / 1e9,
           "topk_lists_GBs": topk_bytes / (stage_ms["topk_lists"] * 1e-3) / 1e9,
           "peak_GBs": PEAK_HBM_GBS}

    out = {
        "metric": "moba_fwd_bwd_effective_tflops" if w.backward else "moba_fwd_effective_tflops",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": "%s: batch %d, heads %d%s, N %d, d %d, B %d, top-k %d%s, %s" % (
            w.name, w.batch, w.heads, " (%d key/value heads)" % w.hkv if w.hkv != w.heads else "",
            w.N, w.d, w.B, w.k,
            ", key conv W=%d" % w.conv_width if w.conv_width else "",
            "forward+backward" if w.backward else "forward"),
            "kernels": "plain" if a.reference_kernels else "default", "attention": a.attention,
            "attended_pairs": pairs, "fwd_gflop": fwd_flop / 1e9, "bwd_gflop": bwd_flop / 1e9},
        "stage_ms": stage_ms,
        "kernel_ms": kernel_ms,
        "roofline": roofline,
        "attention_kernels": kernel_frac,
        "hbm_stages": hbm,
    }
    if w.conv_width:
        # Not part of a step (the benchmark workloads with a convolution are forward-only): the
        # convolution's backward, timed on its own with a synthetic dK_eff.  HBM-bound: it has
        # to read K and dK_eff and write dK.
        G = torch.randn(d["K"].shape, device=dev, dtype=torch.float32).to(d["K"].dtype)
        nws = __import__("ctypes").c_size_t(0)
        moba.lib().moba_key_conv_backward_workspace(__import__("ctypes").byref(sh.c()),
                                                    __import__("ctypes").byref(nws))
        ws_cb = torch.empty(nws.value, dtype=torch.uint8, device=dev)
        for _ in range(2):
            moba.key_conv_backward(sh, d["K"], d["conv_w"], G, ws=ws_cb)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(5):
            moba.key_conv_backward(sh, d["K"], d["conv_w"], G, ws=ws_cb)
        e1.record()
        torch.cuda.synchronize()
        cb_ms = e0.elapsed_time(e1) / 5
        cb_bytes = 3 * w.bh * w.N * w.d * es
        out["key_conv_backward"] = {"ms": cb_ms, "GBs": cb_bytes / (cb_ms * 1e-3) / 1e9,
                                    "frac_of_hbm_peak": cb_bytes / (cb_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}
    if a.microbench:
        mb = moba.microbench()
        best = max(mb["mfma_tflops"].values())
        out["microbench"] = {
            "copy_GBs": mb["copy_GBs"], "copy_frac_of_hbm_peak": mb["copy_GBs"] / PEAK_HBM_GBS,
            "mfma_loop_tflops_by_waves_per_simd": mb["mfma_tflops"],
            "mfma_loop_frac_of_peak": best / PEAK_BF16_TFLOPS,
            "roofline_frac_of_measured": (roofline["achieved"] / best if roofline["bound"] == "mfma"
                                          else roofline["achieved"] / mb["copy_GBs"] if roofline["bound"] == "hbm"
                                          else None),
            "attention_kernels_frac_of_measured_mfma": {k: v["tflops"] / best for k, v in kernel_frac.items()},
            "hbm_stages_frac_of_measured_copy": {k: v / mb["copy_GBs"] for k, v in hbm.items() if k != "peak_GBs"},
        }
    if a.calibration_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)      # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    if not a.no_cpu_baseline and w.hkv == w.heads:      # (the CPU leg times the multi-head form only)
        out["cpu_baseline"] = cpu_baseline(w, t, max_slices=a.cpu_max_slices)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
