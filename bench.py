#!/usr/bin/env python3
"""Benchmark of the mHC-lite hyper-connection hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all
tensors resident in HBM: mhcl_fwd_coeffs_pre, mhcl_post (the two forward calls
around the caller's layer function) and mhcl_bwd_fused.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tokens T]
                    [--no-cpu-baseline] [--detail] [--graph] [--copy-calibration]
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0   # MI355X published HBM3E peak

STAGES = {1: "fwd_proj", 2: "fwd_pre", 3: "post", 4: "bwd_reduce", 5: "bwd_out", 6: "bwd_gw"}


def stage_bytes(stage: int, n: int, C: int, T: int, e: int) -> int:
    """Algorithmic HBM bytes of one launch of a stage: every stream tensor the
    stage consumes or produces crosses HBM once (U = C*e bytes per token row);
    per-token coefficients and W (MiBs) are ignored."""
    U = C * e
    per_token = {
        1: n * U,                # read x
        2: (n + 1) * U,          # read x, write h
        3: (2 * n + 1) * U,      # read x, y; write x_out
        4: (2 * n + 2) * U,      # read x, g_xout, y, g_h
        5: (3 * n + 2) * U,      # read x, g_xout, g_h; write g_x, g_y (g_W rides on the same read)
        6: n * U,                # separate g_W kernel (paths where it is not fused): read x
    }[stage]
    return per_token * T


# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (scaled by the copy
# kernel's readings; profiles/n4_c4096_bench_step.md), valid only for the kernel sources whose
# digest is recorded with them: {workload: (csrc digest, {stage: bytes})}
MEASURED_TRAFFIC = {
    "n4_c4096": ("cd0cb42336ae1ba0", {
        1: int(1040.8 * 2**20 + 4.1 * 2**20),
        2: int(1028.0 * 2**20 + 256.0 * 2**20),
        3: int(1292.3 * 2**20 + 1024.0 * 2**20),
        4: int(2691.1 * 2**20 + 7.1 * 2**20),
        5: int(2433.5 * 2**20 + 1296.2 * 2**20),
    }),
}

def csrc_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2601_05732_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, stage: int):
    digest, table = MEASURED_TRAFFIC.get(workload, ("", {}))
    return table.get(stage) if digest == csrc_digest() else None


def _hip_runtime():
    """The HIP runtime this process already has loaded (torch's)."""
    path = None
    with open("/proc/self/maps") as f:
        for line in f:
            if "libamdhip64" in line:
                path = line.split()[-1]
                break
    return ctypes.CDLL(path or "libamdhip64.so")


class HipEvents:
    def __init__(self, count):
        self.rt = _hip_runtime()
        self.rt.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.rt.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p,
                                                ctypes.c_void_p]
        self.rt.hipEventDestroy.argtypes = [ctypes.c_void_p]
        self.ev = []
        for _ in range(count):
            h = ctypes.c_void_p()
            if self.rt.hipEventCreate(ctypes.byref(h)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.ev.append(h)

    def elapsed_ms(self, i, j):
        ms = ctypes.c_float()
        rc = self.rt.hipEventElapsedTime(ctypes.byref(ms), self.ev[i], self.ev[j])
        if rc != 0:
            self.rt.hipGetLastError()     # reset the runtime's sticky error state
            raise RuntimeError(f"hipEventElapsedTime failed ({rc})")
        return ms.value

    def close(self):
        for h in self.ev:
            self.rt.hipEventDestroy(h)


def cpu_baseline(inp, wl, sample_tokens):
    """The fp64 oracle, as it stands, on the first `sample_tokens` tokens of the
    same workload (forward + backward), timed on the host cores."""
    import numpy as np
    import torch

    import oracle
    f64 = lambda t: t[:sample_tokens].detach().to("cpu", torch.float64).numpy()
    full = lambda t: t.detach().to("cpu", torch.float64).numpy()
    x, y = f64(inp["x"]), f64(inp["y"])
    W, b, al = full(inp["W"]), full(inp["b"]), full(inp["alpha"])
    kw = dict(eps=wl.eps, res_mode=wl.res_mode, iters=wl.sk_iters)
    if wl.res_mode == "subset":
        kw["sigma"] = inp["perm"].cpu().numpy().astype(np.int32)
    if wl.backward:
        gxo, gh = f64(inp["g_xout"]), f64(inp["g_h"])
        run = lambda k: oracle.backward(x[:k], W, b, al, y[:k], gxo[:k], gh[:k], **kw)
    else:
        run = lambda k: oracle.forward(x[:k], W, b, al, y[:k], **kw)
    run(8)                               # loads the library, warms the caches
    t0 = time.perf_counter()
    run(sample_tokens)
    dt = time.perf_counter() - t0
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample_tokens} of {wl.T} tokens, "
                      f"{'forward+backward' if wl.backward else 'forward'}, fp64, "
                      f"{dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="n4_c4096")
    ap.add_argument("--tokens", type=int, default=0,
                    help="run the workload's shape with this many tokens instead of its own count "
                         "(a scaling aid; the headline figure is the default)")
    ap.add_argument("--cpu-sample", type=int, default=16384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="per-stage times on stderr")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (for launch-bound small "
                         "shapes); the dominant kernel's time then comes from the eager warmup probe")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run the library's plain copy kernel on 1 GiB five times (a dispatch "
                         "of known traffic, to scale hardware byte counters with)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this benchmark runs on one GPU only (tokens are independent, so the path "
              "shards over tokens; no multi-GPU figure is produced). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2601_05732_amd as mhcl
    import synth_inputs as si

    wl = si.WORKLOADS[args.workload]
    if args.tokens > 0:
        import dataclasses
        wl = dataclasses.replace(wl, T=args.tokens)
    torch.cuda.set_device(0)
    inp = si.make_inputs(wl, seed=0, device="cuda:0")
    # the layer's stream tensors sit where the package's allocator puts them (layer.py)
    inp["x"] = mhcl.place_stream(inp["x"], mhcl.layer.PHASE_X)
    if "g_xout" in inp:
        inp["g_xout"] = mhcl.place_stream(inp["g_xout"], mhcl.layer.PHASE_G_XOUT)
    fwd_only = not wl.backward      # a forward-only workload times the two forward calls alone
    d = mhcl.desc_for(wl, perm=inp.get("perm"))
    L = mhcl.GpuLayer(d, inp)
    e = 2 if wl.io == "bf16" else 4
    lib = mhcl.lib()
    lib.mhcl_profile_next_call.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]

    def step(stage=0, ev=None, i0=0):
        """One pass; optionally bracket `stage` with events ev[i0], ev[i0+1]."""
        arm = lambda on: lib.mhcl_profile_next_call(stage if on else 0, ev.ev[i0] if on else None,
                                                    ev.ev[i0 + 1] if on else None)
        i, dd = L.inp, L.d
        arm(stage in (1, 2))
        mhcl.mhcl_fwd_coeffs_pre(dd, i["x"], i["W"], i["b"], i["alpha"], L.H_res, L.H_pre,
                                 L.H_post, L.h, L.ws)
        arm(stage == 3)
        mhcl.mhcl_post(dd, i["x"], i["y"], L.H_res, L.H_post, L.x_out)
        if fwd_only:
            return
        arm(stage in (4, 5, 6))
        mhcl.mhcl_bwd_fused(dd, i["x"], i["y"], i["W"], i["b"], i["alpha"], i["g_xout"], i["g_h"],
                            L.g_x, L.g_y, L.g_W, L.g_b, L.g_alpha, L.ws)

    if args.copy_calibration:
        lib.mhcl_debug_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t,
                                        ctypes.c_void_p]
        nbytes = 1 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0").fill_(1)
        dst = torch.empty_like(src)
        cev = HipEvents(2)
        rt = cev.rt
        rt.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
        stream = torch.cuda.current_stream().cuda_stream
        for it in range(5):
            if it == 1:
                rt.hipEventRecord(cev.ev[0], stream)
            lib.mhcl_debug_copy(dst.data_ptr(), src.data_ptr(), nbytes, stream)
        rt.hipEventRecord(cev.ev[1], stream)
        torch.cuda.synchronize()
        ms = cev.elapsed_ms(0, 1) / 4
        print(f"[copy] 1 GiB device copy: {ms:.3f} ms, {2 * nbytes / ms / 1e6:.1f} GB/s "
              "(read + write)", file=sys.stderr)
        cev.close()
        del src, dst

    # warmup; the last warmup passes also find the stage that takes longest
    probe = HipEvents(2 * len(STAGES))
    for _ in range(max(0, args.warmup - len(STAGES))):
        step()
    stage_ms = {}
    for i, st in enumerate(STAGES):
        if fwd_only and st > 3:
            continue
        step(st, probe, 2 * i)
        torch.cuda.synchronize()
        try:
            stage_ms[st] = probe.elapsed_ms(2 * i, 2 * i + 1)
        except RuntimeError:
            pass          # this stage is fused into another kernel for this workload
    probe.close()
    dominant = max(stage_ms, key=stage_ms.get)
    if args.detail:
        for st, ms in stage_ms.items():
            gbs = stage_bytes(st, wl.n, wl.C, wl.T, e) / ms / 1e6
            print(f"[stage] {STAGES[st]:>10}: {ms:8.3f} ms  {gbs:8.1f} GB/s algorithmic",
                  file=sys.stderr)

    if args.graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kern_ms = stage_ms[dominant]
    else:
        ev = HipEvents(2 * args.steps)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(dominant, ev, 2 * k)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kern_ms = sum(ev.elapsed_ms(2 * k, 2 * k + 1) for k in range(args.steps)) / args.steps
        ev.close()

    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = wl.T / (dt / args.steps)
    floor_bytes = ((3 * wl.n + 2) + (0 if fwd_only else 3 * wl.n + 3)) * wl.C * e * wl.T
    achieved = stage_bytes(dominant, wl.n, wl.C, wl.T, e) / kern_ms / 1e6
    out = {
        "metric": "tokens/s + achieved HBM GB/s, fused mHC-lite fwd+bwd, n=4 C=4096 32k tok"
                  if args.workload == "n4_c4096" and args.tokens <= 0 else
                  f"tokens/s, {'forward' if fwd_only else 'fused fwd+bwd'}, {args.workload}"
                  + (f" at {wl.T} tokens" if args.tokens > 0 else ""),
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if wl.io == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: n={wl.n} C={wl.C} T={wl.T} "
                               f"{wl.io} streams, fp32 accumulate, {wl.res_mode} H_res, "
                               "forward (coeffs+pre, post)" + ("" if fwd_only else " + fused backward")
                               + (", HIP graph replay" if args.graph else ""),
                   "path_hbm_gbs_algorithmic": floor_bytes / (dt / args.steps) / 1e9,
                   "path_frac_of_peak": floor_bytes / (dt / args.steps) / 1e9 / PEAK_HBM_GBS},
        "roofline": {"bound": "hbm", "kernel": STAGES[dominant], "achieved": achieved,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "kernel_ms": kern_ms,
                     "traffic": measured_traffic(args.workload, dominant) if args.tokens <= 0 else None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, wl, min(args.cpu_sample, wl.T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
