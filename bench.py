#!/usr/bin/env python3
"""Benchmark of the mHC-lite hyper-connection hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic input, all
tensors resident in HBM: mhcl_fwd_coeffs_pre, mhcl_post (the two forward calls
around the caller's layer function) and mhcl_bwd_fused.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--tokens T]
                    [--no-cpu-baseline] [--detail] [--graph] [--copy-calibration]
    python bench.py --memsys        (runs the memory-system probe, a separate executable, and exits)
    python bench.py --print-digest  (digest of the kernel sources, as recorded in profiles/)
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
FWD_ONCE = 12   # stages 1 and 2 in one kernel (single read of x): reported under stage 1's bracket


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
        FWD_ONCE: (n + 1) * U,   # read x once, write h
    }[stage]
    return per_token * T


# kernel that implements a stage (prefix of its name in the rocprofv3 tables under profiles/)
STAGE_KERNEL = {1: "proj_mfma_kernel", 2: "pre_kernel", 3: "post_kernel", 4: "bwd_reduce_kernel",
                5: "bwd_out_gw_kernel", 6: "bwd_gw", FWD_ONCE: "fwd_once_kernel"}


def profile_traffic(workload: str):
    """(digest, {kernel name: HBM bytes per launch}) from profiles/<workload>_bench_step.md: the
    rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings, scaled by the copy kernel's, that the file
    tabulates, and the digest of the kernel sources they were taken with."""
    path = os.path.join(ROOT, "profiles", f"{workload}_bench_step.md")
    digest, table = "", {}
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("csrc digest:"):
                    digest = line.split(":", 1)[1].strip()
                cells = [c.strip() for c in line.strip().strip("|").split("|")]
                if len(cells) == 5 and cells[0] and cells[0] != "kernel":
                    try:
                        table[cells[0]] = int((float(cells[3]) + float(cells[4])) * 2**20)
                    except ValueError:
                        pass
    except OSError:
        pass
    return digest, table


def csrc_digest() -> str:
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2601_05732_amd", "csrc")
    for name in sorted(os.listdir(d)):
        with open(os.path.join(d, name), "rb") as f:
            h.update(name.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload: str, stage: int):
    """HBM bytes per launch of the stage's kernel as tabulated under profiles/, or None when the
    kernel sources have changed since (or nothing was recorded)."""
    digest, table = profile_traffic(workload)
    if not digest or digest != csrc_digest():
        return None
    for name, nbytes in table.items():
        if name.startswith(STAGE_KERNEL.get(stage, "?")):
            return nbytes
    return None


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


def cpu_baseline(inp, wl, sample_tokens, threads=None):
    """The fp64 oracle, as it stands, on the first `sample_tokens` tokens of the
    same workload (forward + backward), timed on the host cores (`threads`: None =
    all the OpenMP runtime takes, else that many)."""
    import numpy as np
    import torch

    import oracle
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    if threads is not None:
        gomp = ctypes.CDLL("libgomp.so.1")      # the OpenMP runtime the oracle's library links
        gomp.omp_set_num_threads(int(threads))
        cores = int(threads)
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
    return {"value": sample_tokens / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"first {sample_tokens} of {wl.T} tokens, "
                      f"{'forward+backward' if wl.backward else 'forward'}, fp64, "
                      f"{dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default="n4_c4096")
    ap.add_argument("--tokens", type=int, default=0,
                    help="run the workload's shape with this many tokens instead of its own count "
                         "(a scaling aid; the headline figure is the default)")
    ap.add_argument("--cpu-sample", type=int, default=16384)
    ap.add_argument("--cpu-sample-1thread", type=int, default=1024)
    ap.add_argument("--memsys", action="store_true",
                    help="run the memory-system probe (traffic skeletons of the path's access "
                         "patterns; a separate executable) and exit")
    ap.add_argument("--print-digest", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--detail", action="store_true", help="per-stage times on stderr")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (for launch-bound small "
                         "shapes); the dominant kernel's time then comes from the eager warmup probe")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="accepted and ignored: the library's plain copy kernel now always runs on "
                         "1 GiB five times before the warm-up (its rate is reported, and under "
                         "rocprofv3 --pmc it is the dispatch of known traffic)")
    args = ap.parse_args()
    if args.print_digest:
        print(csrc_digest())
        return
    if args.memsys:
        import subprocess
        exe = os.path.join(ROOT, "paper_2601_05732_amd", "memsys_probe")
        if not os.path.exists(exe):
            sys.exit(f"{exe} is missing: build it with `python -m paper_2601_05732_amd.build`")
        sys.exit(subprocess.run([exe]).returncode)    # nothing in this process has touched the GPU
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

    # the library's plain copy kernel on 1 GiB: the yardstick beside the 8 TB/s peak (and, under
    # rocprofv3 --pmc, a dispatch of known traffic to scale hardware byte counters with)
    lib.mhcl_debug_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
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
    copy_gbs = 2 * nbytes / (cev.elapsed_ms(0, 1) / 4) / 1e6
    print(f"[copy] 1 GiB device copy: {copy_gbs:.1f} GB/s (read + write)", file=sys.stderr)
    cev.close()
    del src, dst

    # warmup; the last warmup passes also find the stage that takes longest
    probe = HipEvents(2 * len(STAGES))
    for _ in range(max(2, args.warmup - len(STAGES))):   # (first calls load code objects)
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
    # the single-read forward runs under stage 1's bracket and leaves stage 2's unrecorded
    fwd_once = 1 in stage_ms and 2 not in stage_ms
    kind = lambda st: FWD_ONCE if (st == 1 and fwd_once) else st
    label = lambda st: "fwd_once" if kind(st) == FWD_ONCE else STAGES[st]
    dominant = max(stage_ms, key=stage_ms.get)
    if args.detail:
        for st, ms in stage_ms.items():
            gbs = stage_bytes(kind(st), wl.n, wl.C, wl.T, e) / ms / 1e6
            print(f"[stage] {label(st):>10}: {ms:8.3f} ms  {gbs:8.1f} GB/s algorithmic",
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
    achieved = stage_bytes(kind(dominant), wl.n, wl.C, wl.T, e) / kern_ms / 1e6
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
                   "path_frac_of_peak": floor_bytes / (dt / args.steps) / 1e9 / PEAK_HBM_GBS,
                   "copy_kernel_gbs": copy_gbs,
                   "path_frac_of_copy": floor_bytes / (dt / args.steps) / 1e9 / copy_gbs},
        "roofline": {"bound": "hbm", "kernel": label(dominant), "achieved": achieved,
                     "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": achieved / PEAK_HBM_GBS,
                     "kernel_ms": kern_ms, "frac_of_copy": achieved / copy_gbs,
                     "traffic": measured_traffic(args.workload, kind(dominant)) if args.tokens <= 0 else None},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inp, wl, min(args.cpu_sample, wl.T))
        out["cpu_baseline_1thread"] = cpu_baseline(inp, wl, min(args.cpu_sample_1thread, wl.T), threads=1)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
