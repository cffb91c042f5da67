#!/usr/bin/env python3
"""Benchmark of the LinFusion token mixer hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

A step is one pass of the whole hot path (feature map, split-N state reduction, combine,
apply + normalize: one linfusion_attn_fwd_ex call) over one batch of seeded synthetic Q/K/V
that is already resident in HBM.  Prints ONE JSON line: tokens/s for the whole job, the HBM
roofline of the dominant kernel measured live with HIP events recorded on the launch stream
between the library's kernels, and the fp64 CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak
DEFAULT_WORKLOAD = "sd15_16k_f16"   # 16384x8192 image, SD-v1.5 top level: B=1 H=8 N=2,097,152 d=40 fp16


class HipEvents:
    """hipEvent_t handles created through the HIP runtime directly (ctypes), for per-kernel timing."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventSynchronize.argtypes = [ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.ev.append(e.value)

    def elapsed_ms(self, a, b):
        ms = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(ms), self.ev[a], self.ev[b])
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return ms.value

    def sync(self, i):
        self.hip.hipEventSynchronize(self.ev[i])

    def close(self):
        for e in self.ev:
            self.hip.hipEventDestroy(e)
        self.ev = []


def _oracle_sample(q, k, v, cfg, n, threads):
    """Times the oracle as it stands on the first n tokens of head (0, 0) with the BLAS pool limited to `threads`
    (None = as the library starts it).  Returns (seconds, threads actually used)."""
    import numpy as np
    from oracle import linattn_oracle as orc
    from paper_2409_02097_amd import workloads as wl
    qs = wl.stored_numpy(q[0, 0, :n])
    ks = wl.stored_numpy(k[0, 0, :n])
    vs = wl.stored_numpy(v[0, 0, :n])
    from threadpoolctl import threadpool_info, threadpool_limits
    with threadpool_limits(limits=threads):
        used = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        t0 = time.perf_counter()
        ref = orc.attention_linear_stored(qs, ks, vs, cfg["dtype"], 0, wl.EPS)
        dt = time.perf_counter() - t0
    assert np.all(np.isfinite(ref))
    return dt, int(used)


def cpu_baseline(q, k, v, cfg, sample_tokens):
    """The oracle as it stands, timed on the host in two modes: all cores (its BLAS pool as it starts: the figure
    reported as `cpu_baseline`) and a single thread.  Sample: one (batch, head) slice, the first `sample_tokens`
    tokens for the all-core run and an eighth of that for the single-thread run; tokens/s counts a token once it
    has passed through all H heads, as the GPU figure does."""
    n_all = min(sample_tokens, cfg["N"])
    n_one = max(min(n_all // 8, cfg["N"]), 1)
    dt_all, used_all = _oracle_sample(q, k, v, cfg, n_all, None)
    dt_one, used_one = _oracle_sample(q, k, v, cfg, n_one, 1)
    host = os.cpu_count()
    base = {"value": n_all / (dt_all * cfg["H"]), "unit": "tokens/s", "cores": used_all, "kind": "oracle",
            "sample": f"fp64 numpy oracle on the first {n_all} tokens of one (batch, head) slice of the same "
                      f"tensors ({dt_all:.1f} s); scaled to all {cfg['H']} heads per token; host has "
                      f"{host} logical cores, BLAS threads = {used_all}",
            "single_thread": {"value": n_one / (dt_one * cfg["H"]), "unit": "tokens/s", "cores": used_one,
                              "sample": f"the same on the first {n_one} tokens with the BLAS pool limited to one "
                                        f"thread ({dt_one:.1f} s)"}}
    return base


def hbm_ceilings(nbytes=1342177280, reps=20):
    """What plain streaming reaches on this device with the access pattern of the library's kernels
    (linfusion_hbm_probe: 128-bit non-temporal accesses, workgroups sweeping one moving window): read-only
    streams (the state reduction's pattern), one read + one write stream (apply's pattern), and the 3 : 1 mix
    of a whole step.  Best launch size per pattern; every byte crosses HBM (streams of 1.34 GB each)."""
    import torch
    import paper_2409_02097_amd as lf
    bufs = [torch.randint(0, 255, (nbytes,), dtype=torch.uint8, device="cuda") for _ in range(3)]
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    rows = []
    for reads, writes in ((1, 0), (2, 0), (1, 1), (3, 1), (2, 1), (0, 1)):
        best = None
        for wgs in (512, 1024, 2048, 4096, 8192, 16384):
            def call():
                lf.linfusion_hbm_probe(reads, writes, bufs[0], bufs[1], bufs[2], dst, nbytes, wgs, sink)
            for _ in range(5):
                call()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(reps):
                call()
            ev[1].record()
            torch.cuda.synchronize()
            us = ev[0].elapsed_time(ev[1]) * 1e3 / reps
            gbps = (reads + writes) * nbytes / us / 1e3
            if best is None or gbps > best["gbps"]:
                best = {"reads": reads, "writes": writes, "bytes_per_stream": nbytes, "workgroups": wgs,
                        "avg_us": round(us, 1), "gbps": round(gbps, 1), "frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4)}
        rows.append(best)
    del bufs, dst
    return rows


def launch_floor(reps=200):
    """Cost of launching by itself: one empty kernel, three dependent empty kernels (the split path's chain), and
    one HIP-graph replay of those three; microseconds per chain, back to back on one stream, host-timed."""
    import torch
    import paper_2409_02097_amd as lf
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    res = {}
    for label, n, wgs in (("one_empty_kernel", 1, 512), ("three_empty_kernels", 3, 512), ("three_empty_kernels_1wg", 3, 1)):
        for _ in range(20):
            lf.linfusion_launch_probe(n, wgs, sink)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            lf.linfusion_launch_probe(n, wgs, sink)
        torch.cuda.synchronize()
        res[label + "_us"] = round((time.perf_counter() - t0) / reps * 1e6, 2)
    g = torch.cuda.CUDAGraph()
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        lf.linfusion_launch_probe(3, 512, sink)
        torch.cuda.synchronize()
        with torch.cuda.graph(g, stream=st):
            lf.linfusion_launch_probe(3, 512, sink)
    for _ in range(20):
        g.replay()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        g.replay()
    torch.cuda.synchronize()
    res["graph_of_three_empty_kernels_us"] = round((time.perf_counter() - t0) / reps * 1e6, 2)
    return res


PATH_NAMES = {0: "three kernels", 1: "single launch with barriers", 2: "replicated-state single launch"}
PAPER_CONFIGS = ["sd15_256_f32", "sd15_512_f16", "sd21_768_f16", "sd21_768_f16_peaky", "sdxl_2048_A_bf16",
                 "sdxl_2048_B_bf16"]


def latency_rows(names, paths=(("auto", 0),), steps=200):
    """Per-call latency of small and medium workloads (they fit the 256 MB memory-side cache):
    'hot' = the same buffers back to back, 'cold' = rotating through enough independent buffer sets
    (> 768 MB in total) that every call streams from HBM.  Calls are issued back to back from the host and the
    whole batch is timed, so a figure is the larger of the device time and the host's time per call."""
    import torch
    import paper_2409_02097_amd as lf
    from paper_2409_02097_amd import workloads as wl
    rows = []
    for name in names:
        cfg = wl.CONFIGS[name]
        B, H, N, d, dtype = cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["dtype"]
        code = wl.DTYPE_CODE[dtype]
        nbytes = wl.algorithmic_bytes(B, H, N, d, dtype)
        nsets = max(2, int(768e6 // nbytes) + 1)
        q0, k0, v0 = wl.make_config(name, device="cuda")
        sets = [(q0, k0, v0, torch.empty_like(q0))] + [
            (q0.clone(), k0.clone(), v0.clone(), torch.empty_like(q0)) for _ in range(nsets - 1)]
        ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
        row = {"workload": name, "B": B, "H": H, "N": N, "d": d, "dtype": dtype, "algorithmic_bytes": nbytes,
               "ideal_us_at_8TBps": round(nbytes / 8e6, 2), "buffer_sets_cold": nsets}
        for label, flags in paths:
            try:
                plan = lf.linfusion_attn_plan(B, H, N, d, code, flags)
            except lf.LinFusionError:          # no single launch for the widest heads
                continue
            for mode in ("hot", "cold"):
                use = sets[:1] if mode == "hot" else sets
                # arguments marshalled once per buffer set (the binding's per-call checks cost the host ~5 us,
                # more than the difference between the paths at these sizes); the status of every call is checked
                calls = [lf.linfusion_attn_fwd_ex_bound(q, k, v, o, lf.PHI_ELU_PLUS_ONE, wl.EPS, flags, ws)
                         for q, k, v, o in use]
                for i in range(20):
                    if calls[i % len(calls)]() != 0:
                        raise RuntimeError(f"{name}: the library returned an error")
                torch.cuda.synchronize()
                bad = 0
                t0 = time.perf_counter()
                for i in range(steps):
                    bad |= calls[i % len(calls)]()
                torch.cuda.synchronize()
                us = (time.perf_counter() - t0) / steps * 1e6
                if bad:
                    raise RuntimeError(f"{name}: the library returned an error")
                pre = "" if label == "auto" else label + "_"
                row[f"{pre}{mode}_us"] = round(us, 2)
                row[f"{pre}{mode}_tokens_per_s"] = round(B * N / us * 1e6)
                row[f"{pre}{mode}_gbps"] = round(nbytes / us / 1e3, 1)
                row[f"{pre}{mode}_frac_of_peak"] = round(nbytes / us / 1e3 / HBM_PEAK_GBPS, 4)
            row[("" if label == "auto" else label + "_") + "path"] = PATH_NAMES[plan["path"]]
        rows.append(row)
        del sets
    return rows


def latency_table(steps=200):
    """Every small and medium workload on the automatic, the three-kernel and the single-launch path; one JSON
    line per workload on stderr."""
    import paper_2409_02097_amd as lf
    from paper_2409_02097_amd import workloads as wl
    names = [n for n, c in wl.CONFIGS.items()
             if n != DEFAULT_WORKLOAD and wl.algorithmic_bytes(c["B"], c["H"], c["N"], c["d"], c["dtype"]) <= 512e6]
    for row in latency_rows(names, (("auto", 0), ("split", lf.FLAG_FORCE_SPLIT), ("fused", lf.FLAG_FORCE_FUSED), ("solo", lf.FLAG_FORCE_SOLO)), steps):
        print(json.dumps(row), file=sys.stderr, flush=True)


def settle(step, batch=10, max_calls=300, tol=0.01):
    """Runs the step untimed until its duration has stopped drifting: batches of `batch` calls, each timed with the
    host clock around a synchronisation, until two consecutive batches agree within `tol` (or `max_calls`).
    After any idle time -- a fresh process, input generation, even 50 ms without work -- this device runs the first
    tens of milliseconds of a memory-bound load slower (the third to about the 25th call of this workload, the
    read-only reduction up to 1.5x) before it reaches the steady state a long-running job sees; a warm-up of a
    few calls would put that transient inside the timed region.  Returns (calls made, last batch ms per call)."""
    import torch
    calls, prev, cur = 0, None, None
    while calls < max_calls:
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(batch):
            step()
        torch.cuda.synchronize()
        cur = (time.perf_counter() - t0) / batch * 1e3
        calls += batch
        if prev is not None and abs(cur - prev) <= tol * prev and calls >= 3 * batch:
            break
        prev = cur
    return calls, cur


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=25)
    ap.add_argument("--workload", default=DEFAULT_WORKLOAD)
    ap.add_argument("--profile-steps", type=int, default=20)
    ap.add_argument("--cpu-sample-tokens", type=int, default=1 << 21)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--layout", choices=["head_major", "token_major"], default="head_major",
                    help="memory layout of q, k, v, out: contiguous [B, H, N, d] (the headline workload) or the "
                         "UNet's [B, N, H*d] handed over as strided views")
    ap.add_argument("--backward", action="store_true",
                    help="also time linfusion_attn_bwd on the same workload (fp16 / bf16 only); reported in an extra "
                         "`backward` object of the result line")
    ap.add_argument("--mlp", action="store_true",
                    help="also time linfusion_attn_fwd_mlp (the mixer fed by the two-branch MLPs' results, token-major) "
                         "on the same shape, next to the unfused route (q and k formed by torch ops, then the "
                         "strided mixer); reported in an extra `mlp` object of the result line")
    ap.add_argument("--d-qk", type=int, default=0,
                    help="also time linfusion_attn_fwd_qv with this feature width of q and k (the workload's d stays "
                         "the value width); reported in an extra `qv` object of the result line")
    ap.add_argument("--latency-table", action="store_true",
                    help="also time the small and medium workloads, hot and cold cache, both launch paths "
                         "(JSON lines on stderr; the one-line result on stdout is unchanged)")
    ap.add_argument("--no-settle", action="store_true",
                    help="skip the untimed settling calls before the warm-up (see settle())")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the per-call latencies of the other paper-shaped workloads (`configs` in the result)")
    ap.add_argument("--ceilings", action="store_true",
                    help="also measure what plain streaming kernels reach on this device (read-only, copy, 3:1 mix) "
                         "and what empty launches cost; reported in extra `hbm_ceilings` and `launch_floor` objects")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain device copy of one tensor (known size) so that a rocprofv3 --pmc "
                         "run of this command holds the reference reading for FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the hot path is a single-device kernel "
              "sequence and every box has one GPU; no multi-GPU figure exists). Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2409_02097_amd as lf
    from paper_2409_02097_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the hot path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    cfg = wl.config(args.workload)
    B, H, N, d, dtype = cfg["B"], cfg["H"], cfg["N"], cfg["d"], cfg["dtype"]
    q, k, v = wl.make_config(args.workload, device="cuda")
    if args.layout == "token_major":
        tm = lambda t: t.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)   # [B, N, H, d] in memory
        qd, kd, vd = tm(q), tm(k), tm(v)
    else:
        qd, kd, vd = q, k, v
    out = torch.empty_like(qd)          # keeps the strides of qd
    code = wl.DTYPE_CODE[dtype]
    ws = torch.empty(lf.linfusion_attn_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")
    plan = lf.linfusion_attn_plan(B, H, N, d, code, args.flags)

    def step():
        lf.linfusion_attn_fwd_strided(qd, kd, vd, out, lf.PHI_ELU_PLUS_ONE, wl.EPS, args.flags, ws)

    if args.calibrate_copy:
        out.copy_(qd)            # reads and writes B*H*N*d*itemsize bytes exactly once each
        torch.cuda.synchronize()
    settle_calls, settle_ms = (0, None) if args.no_settle else settle(step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = B * N / (dt / args.steps)
    alg_bytes = wl.algorithmic_bytes(B, H, N, d, dtype)

    # per-kernel durations, HIP events recorded on the launch stream between the kernels
    evs = HipEvents(4)
    acc = [0.0, 0.0, 0.0]
    for _ in range(args.profile_steps):
        lf.linfusion_attn_fwd_profile(qd, kd, vd, out, lf.PHI_ELU_PLUS_ONE, wl.EPS, args.flags, ws, evs.ev)
        evs.sync(3)
        for i in range(3):
            acc[i] += evs.elapsed_ms(i, i + 1)
    evs.close()
    kms = [a / max(args.profile_steps, 1) for a in acc]
    tag = {"f16": "<F16", "bf16": "<BF16", "f32": ""}[dtype]
    rname = ("state_reduce32" if dtype == "f32" else "state_reduce16") + tag
    aname = lf.linfusion_attn_apply_kernel(B, H, N, d, code, args.flags) + tag
    mid = "combine_state + pack_state16" if aname.startswith("apply16_packed") else "combine_state"
    if d > 80:
        rname = rname.replace("state_reduce16<", "state_reduce16_wide<")
        if (N + 31) // 32 <= 2:
            mid = "(no combine: one workgroup per head wrote the state)"
    elif args.layout == "token_major" and dtype != "f32" and (d * 2) % 128 != 0 and H >= 4:
        # heads adjacent in memory and rows that are not whole 128-byte lines: the row-piece kernels run
        rname = rname.replace("state_reduce16<", "state_reduce16_rows<")
        aname = "apply16_rows" + tag
        mid = "combine_state + pack_state16"
    half = alg_bytes / 2      # K+V read by the reduction; Q read + out written by apply
    kernels = [
        {"name": rname, "ms": kms[0], "alg_bytes": half},
        {"name": mid, "ms": kms[1], "alg_bytes": 0},
        {"name": aname, "ms": kms[2], "alg_bytes": half},
    ]
    for kk in kernels:
        kk["gbps"] = kk["alg_bytes"] / (kk["ms"] * 1e-3) / 1e9 if kk["ms"] > 0 else None
    dom = max((kernels[0], kernels[2]), key=lambda x: x["ms"])
    roofline = {"bound": "hbm", "kernel": dom["name"], "achieved": dom["gbps"], "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": dom["gbps"] / HBM_PEAK_GBPS, "traffic": None,
                "avg_launch_ms": dom["ms"], "kernels": kernels}
    # HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if there is one
    tname = args.workload + ("_token_major" if args.layout == "token_major" else "")
    tpath = os.path.join(ROOT, "profiles", f"hbm_traffic_{tname}.json")
    if os.path.exists(tpath):
        with open(tpath) as f:
            tr = json.load(f)
        ent = tr.get("kernels", {}).get(dom["name"].split("<")[0])
        if ent:
            roofline["traffic"] = ent["hbm_bytes_per_launch"]
            roofline["traffic_source"] = f"profiles/{os.path.basename(tpath)}"

    result = {
        "metric": "non-causal linear-attn tokens/s + achieved HBM GB/s (% of peak), 1 GPU",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype, "data": "synthetic",
        "config": {"workload": args.workload, "B": B, "H": H, "N": N, "d": d, "eps": wl.EPS,
                   "feature_map": "elu+1", "layout": args.layout, "plan": plan},
        "hbm_gbps": alg_bytes / (dt / args.steps) / 1e9,
        "hbm_frac_of_peak": alg_bytes / (dt / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "roofline": roofline,
        "settle": {"untimed_calls_before_warmup": settle_calls, "last_batch_ms_per_call": settle_ms,
                   "why": "after idle time the device runs the first ~25 ms of this load slower; see bench.py: settle"},
    }
    if args.backward:
        # gradient tensors resident in HBM; minimal traffic = q, k, v, dout read + dq, dk, dv written (7 tensors);
        # the kernels read k, v twice when they recompute the forward state (9 tensor passes); token-major bf16 and
        # token-major d = 56 / 80 also read q and dout twice (11 passes plus 16 bytes per token-head of scalars)
        # (--layout token_major: all seven tensors as strided views of [B, N, H*d] memory)
        g = torch.empty_like(qd).copy_(torch.randn_like(q))   # keeps the strides of qd
        grads = [torch.empty_like(qd) for _ in range(3)]
        bws = torch.empty(lf.linfusion_attn_bwd_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")

        # A training step runs the forward pass first, which leaves the fp32 head states (52 KB here) in its workspace;
        # handing them to the backward call saves its own pass over k and v.  Both ways are timed: `ms_per_step` is
        # the call a training step makes (state handed over), `ms_per_step_state_recomputed` the stand-alone call.
        step()
        off = lf.linfusion_attn_workspace_state_offset(B, H, N, d, code)
        nstate = B * H * (d * d + d)
        saved = ws[off:off + 4 * nstate].view(torch.float32).clone()
        tensor_bytes = alg_bytes / 4
        # dQ and the state gradient in one kernel: always on contiguous heads; on token-major tensors whose head
        # rows are no whole cache lines only where its row-piece form exists (fp16, d <= 48)
        merged = args.layout == "head_major" or (d * 2) % 128 == 0 or (dtype == "f16" and d <= 48)
        timings = {}
        for label, state in (("with_state", saved), ("recomputed", None)):
            def bstep():
                lf.linfusion_attn_bwd_strided(qd, kd, vd, g, *grads, lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, bws, state=state)
            for _ in range(max(args.warmup // 2, 2)):
                bstep()
            torch.cuda.synchronize()
            tb = time.perf_counter()
            bsteps = max(args.steps // 2, 1)
            for _ in range(bsteps):
                bstep()
            torch.cuda.synchronize()
            timings[label] = (time.perf_counter() - tb) / bsteps
        bdt = timings["with_state"]
        # tensor passes of the kernels with the state handed over: the minimum of 7 (q, k, v, dout read; dq, dk, dv
        # written) with the merged kernel; the separate kernels read q and dout twice and move 16 bytes of scalars
        # per token-head; recomputing the state reads k and v once more
        passes = (7 if merged else 9)
        kbytes = passes * tensor_bytes + (0 if merged else 16.0 * B * H * N)
        result["backward"] = {"layout": args.layout, "ms_per_step": bdt * 1e3, "tokens_per_s": B * N / bdt,
                              "ms_per_step_state_recomputed": timings["recomputed"] * 1e3,
                              "kernel_tensor_passes": passes,
                              "min_traffic_gbps": 7 * tensor_bytes / bdt / 1e9,
                              "kernel_traffic_gbps": kbytes / bdt / 1e9,
                              "frac_of_peak_kernel_traffic": kbytes / bdt / 1e9 / HBM_PEAK_GBPS}
        del g, grads, bws
    if args.mlp:
        # algorithmic traffic: a_k, t_k, v read by the reduction; a_q, t_q read and out written by apply
        ins = wl.make_mlp_inputs(B, H, N, d, dtype, idx=cfg["idx"], device="cuda")
        mout = torch.empty_like(ins[0])
        mws = torch.empty(lf.linfusion_attn_mlp_workspace_bytes(B, H, N, d, code), dtype=torch.uint8, device="cuda")

        def mstep(events=None):
            lf.linfusion_attn_fwd_mlp(*ins[:5], mout, *ins[5:], H, lf.PHI_ELU_PLUS_ONE, wl.EPS, 1e-5, 0.01, 0, mws,
                                      events=events)
        for _ in range(max(args.warmup // 2, 2)):
            mstep()
        torch.cuda.synchronize()
        tm0 = time.perf_counter()
        msteps = max(args.steps // 2, 1)
        for _ in range(msteps):
            mstep()
        torch.cuda.synchronize()
        mdt = (time.perf_counter() - tm0) / msteps
        mev = HipEvents(4)
        macc = [0.0, 0.0, 0.0]
        for _ in range(args.profile_steps):
            mstep(mev.ev)
            mev.sync(3)
            for i in range(3):
                macc[i] += mev.elapsed_ms(i, i + 1)
        mev.close()
        mk = [a / max(args.profile_steps, 1) for a in macc]
        tensor_bytes = alg_bytes / 4

        def unfused():
            F = torch.nn.functional
            C = H * d
            qq = ins[0] + F.leaky_relu(F.layer_norm(ins[1], (C,), ins[5].to(ins[1].dtype), ins[6].to(ins[1].dtype), 1e-5), 0.01)
            kk = ins[2] + F.leaky_relu(F.layer_norm(ins[3], (C,), ins[7].to(ins[3].dtype), ins[8].to(ins[3].dtype), 1e-5), 0.01)
            hv = lambda t: t.view(B, N, H, d).permute(0, 2, 1, 3)
            lf.linfusion_attn_fwd_strided(hv(qq), hv(kk), hv(ins[4]), hv(mout), lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, ws)
        for _ in range(3):
            unfused()
        torch.cuda.synchronize()
        tu0 = time.perf_counter()
        usteps = max(args.steps // 4, 1)
        for _ in range(usteps):
            unfused()
        torch.cuda.synchronize()
        udt = (time.perf_counter() - tu0) / usteps
        # the same call on column blocks of one [B, N, 5 C] buffer (the layout one wide projection writes)
        wide = torch.cat(ins[:5], dim=2)
        views = [wide[:, :, i * H * d:(i + 1) * H * d] for i in range(5)]
        for _ in range(3):
            lf.linfusion_attn_fwd_mlp_strided(*views, mout, *ins[5:], H, lf.PHI_ELU_PLUS_ONE, wl.EPS, 1e-5, 0.01, 0, mws)
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        for _ in range(msteps):
            lf.linfusion_attn_fwd_mlp_strided(*views, mout, *ins[5:], H, lf.PHI_ELU_PLUS_ONE, wl.EPS, 1e-5, 0.01, 0, mws)
        torch.cuda.synchronize()
        sdt = (time.perf_counter() - ts0) / msteps
        del wide, views
        # shapes whose token rows fit one workgroup run two big kernels; the others a statistics pass (reads t_q and
        # t_k once more) and per-head kernels: the first timed interval then covers statistics + reduction
        whole_rows = ((H == 8 and d <= 48) or (H == 4 and (d <= 64 or d == 80))) and \
            os.environ.get("LINFUSION_MLP_ROUTE", "0") != "1"
        forced = os.environ.get("LINFUSION_MLP_ROUTE", "0")
        if whole_rows and forced != "2":
            route, rname, aname = "whole token rows per workgroup", "state_reduce16_mlp", "apply16_mlp"
        elif forced != "1" and H % 4 == 0 and (d <= 56 or d == 80):
            route = "statistics pass + row-piece kernels on groups of four heads"
            rname, aname = "mlp_rowstats16 + state_reduce16_mlp<PRE>", "apply16_mlpg"
            whole_rows = False
        elif d > 80:
            route = "statistics pass + wide kernels"
            rname = "mlp_rowstats16 + state_reduce16_wide_mlp"
            aname = "apply16_wave_mlp"
        else:
            route = "statistics pass + per-head kernels"
            rname, aname = "mlp_rowstats16 + state_reduce16_mlph", "apply16_mlph"
        rpasses = 3 if whole_rows else 5
        result["mlp"] = {
            "route": route,
            "kernel_tensor_passes": 6 if whole_rows else 8,
            "ms_per_step": mdt * 1e3, "interleaved_ms_per_step": sdt * 1e3, "tokens_per_s": B * N / mdt, "alg_bytes": 6 * tensor_bytes,
            "hbm_gbps": 6 * tensor_bytes / mdt / 1e9, "hbm_frac_of_peak": 6 * tensor_bytes / mdt / 1e9 / HBM_PEAK_GBPS,
            "kernels": [
                {"name": rname, "ms": mk[0], "alg_bytes": rpasses * tensor_bytes,
                 "gbps": rpasses * tensor_bytes / (mk[0] * 1e-3) / 1e9 if mk[0] > 0 else None},
                {"name": "combine_state + pack_state16", "ms": mk[1], "alg_bytes": 0, "gbps": 0.0},
                {"name": aname, "ms": mk[2], "alg_bytes": 3 * tensor_bytes,
                 "gbps": 3 * tensor_bytes / (mk[2] * 1e-3) / 1e9 if mk[2] > 0 else None}],
            "unfused_ms_per_step": udt * 1e3,
            "unfused": "q, k formed by torch layer_norm + leaky_relu + add (16-bit), then linfusion_attn_fwd_strided",
        }
        del ins, mout, mws
    if args.d_qk:
        dk = args.d_qk
        qq, kk, vv = wl.make_qkv_widths(B, H, N, dk, d, dtype, idx=cfg["idx"], device="cuda")
        qout = torch.empty_like(vv)
        qws = torch.empty(lf.linfusion_attn_qv_workspace_bytes(B, H, N, dk, d, code), dtype=torch.uint8, device="cuda")
        for _ in range(max(args.warmup // 2, 2)):
            lf.linfusion_attn_fwd_qv(qq, kk, vv, qout, lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, qws)
        torch.cuda.synchronize()
        tq0 = time.perf_counter()
        qsteps = max(args.steps // 2, 1)
        for _ in range(qsteps):
            lf.linfusion_attn_fwd_qv(qq, kk, vv, qout, lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, qws)
        torch.cuda.synchronize()
        qdt = (time.perf_counter() - tq0) / qsteps
        qev = HipEvents(4)
        qacc = [0.0, 0.0, 0.0]
        for _ in range(args.profile_steps):
            lf.linfusion_attn_fwd_qv(qq, kk, vv, qout, lf.PHI_ELU_PLUS_ONE, wl.EPS, 0, qws, events=qev.ev)
            qev.sync(3)
            for i in range(3):
                qacc[i] += qev.elapsed_ms(i, i + 1)
        qev.close()
        qk = [a / max(args.profile_steps, 1) for a in qacc]
        per_elem = B * H * N * wl.ITEMSIZE[dtype]
        rb, ab = (dk + d) * per_elem, (dk + d) * per_elem      # k + v read; q read + out written
        result["qv"] = {
            "d_qk": dk, "d_v": d, "ms_per_step": qdt * 1e3, "tokens_per_s": B * N / qdt, "alg_bytes": rb + ab,
            "hbm_gbps": (rb + ab) / qdt / 1e9, "hbm_frac_of_peak": (rb + ab) / qdt / 1e9 / HBM_PEAK_GBPS,
            "kernels": [
                {"name": "state_reduce16_qv", "ms": qk[0], "alg_bytes": rb, "gbps": rb / (qk[0] * 1e-3) / 1e9 if qk[0] > 0 else None},
                {"name": "combine_state", "ms": qk[1], "alg_bytes": 0, "gbps": 0.0},
                {"name": "apply16_qv", "ms": qk[2], "alg_bytes": ab, "gbps": ab / (qk[2] * 1e-3) / 1e9 if qk[2] > 0 else None}]}
        del qq, kk, vv, qout, qws
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(q, k, v, cfg, args.cpu_sample_tokens)
    if not args.no_configs and args.workload == DEFAULT_WORKLOAD and args.layout == "head_major":
        # the other paper-shaped workloads: per-call latency hot and cold, then this run's own line for the table
        rows = latency_rows(PAPER_CONFIGS)
        rows.append({"workload": args.workload, "B": B, "H": H, "N": N, "d": d, "dtype": dtype,
                     "algorithmic_bytes": alg_bytes, "ideal_us_at_8TBps": round(alg_bytes / 8e6, 2),
                     "cold_us": round(ms_per_step * 1e3, 2), "cold_tokens_per_s": round(tokens_per_s),
                     "cold_gbps": round(alg_bytes / (dt / args.steps) / 1e9, 1),
                     "cold_frac_of_peak": round(alg_bytes / (dt / args.steps) / 1e9 / HBM_PEAK_GBPS, 4),
                     "path": PATH_NAMES[plan["path"]],
                     "note": "5.4 GB per call: every call streams from HBM"})
        result["configs"] = rows
    if args.ceilings:
        result["hbm_ceilings"] = hbm_ceilings()
        result["launch_floor"] = launch_floor()
    if args.latency_table:
        del q, k, v, qd, kd, vd, out
        torch.cuda.empty_cache()
        latency_table()
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
