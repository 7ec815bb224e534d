"""Benchmark of the fused Signum step on the ResNet-50-sized workload (d = 25,557,032, M = 15).

A step is one pass of the whole hot path -- momentum, sign, majority vote, parameter update -- for
all M simulated workers: one call of ssv_signum_step on gradients that are already resident in HBM.
Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
BYTES_PER_COORD = 15 * 12 + 8  # per coordinate: M x (read g, read v, write v) fp32 + read/write x fp32


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workers", type=int, default=15)
    ap.add_argument("--d", type=int, default=25_557_032)
    ap.add_argument("--row-align", type=int, default=32,
                    help="round row strides up to a multiple of this many elements")
    ap.add_argument("--grad-sets", type=int, default=8, help="distinct pre-generated gradient sets that are cycled")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--other-kernels", action="store_true",
                    help="also time the packed vote (d = 2^30, M = 255), the fused vote+apply (resnet50 size) and "
                         "the large bf16 fused step (d = 1.5e9, M = 31, 23 chunk launches) and add them to the JSON line")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run a plain 1 GiB device-to-device copy three times "
                         "(known traffic: 1 GiB read + 1 GiB written per copy) to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters")
    ap.add_argument("--cpu-sample", type=int, default=1 << 22, help="coordinates in the oracle's timed sample")
    return ap.parse_args()


def read_traffic(name):
    """Measured HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("hbm_bytes_per_launch"):
                    return float(line.split()[1])
    except OSError:
        pass
    return None


def time_launches(torch, fn, iters, warmup=2):
    """Average milliseconds per call of fn() over `iters` back-to-back launches (events on the current stream)."""
    for i in range(warmup):
        fn(i)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        fn(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def other_kernels(torch, sv, wl, dev):
    """Secondary measurements: the kernels that are not the headline, at their own workloads."""
    out = {}
    # yardstick: the library's plain streaming copy (1:1 read/write), 1.5 GB like one gradient set
    src = wl.gaussian((15 * 25_557_056,), 1.0, seed=1, device=dev)
    dst = torch.empty_like(src)
    ms = time_launches(torch, lambda i: sv.bench_copy(src, dst), 20)
    b = 2.0 * src.numel() * 4
    out["stream_copy_1.5GB"] = {"ms": ms, "GB/s": b / ms / 1e6, "frac": b / ms / 1e6 / HBM_PEAK_GBS,
                                "note": "plain 16-byte non-temporal copy, bytes read + written"}
    del src, dst
    # packed majority vote, d = 2^30, M = 255 (uniform random bits: the kernel is data-oblivious)
    M, d = 255, 1 << 30
    W = sv.words_for(d)
    rows = wl.random_words((M, W), seed=5, device=dev)
    vote = torch.empty((W,), dtype=torch.int64, device=dev)
    ms = time_launches(torch, lambda i: sv.majority_vote(rows, d, vote), 10)
    b = (M + 1) / 8 * d
    out["majority_vote_d2^30_M255"] = {"ms": ms, "GB/s": b / ms / 1e6, "frac": b / ms / 1e6 / HBM_PEAK_GBS,
                                        "coords_per_s": d / ms * 1e3, "algorithmic_bytes": b}
    del rows, vote
    # fused vote + apply at the resnet50 size, 8 rotating buffer sets (2 GB, beyond the 256 MB Infinity Cache)
    M, d = 15, 25_557_032
    W = sv.words_for(d)
    sets = [(wl.random_words((M, W), seed=10 + k, device=dev), wl.gaussian((d,), 0.02, seed=20 + k, device=dev))
            for k in range(8)]
    ms = time_launches(torch, lambda i: sv.vote_apply(sets[i % 8][0], d, sets[i % 8][1], 1e-4), 80, warmup=8)
    b = (M / 8 + 8) * d
    out["vote_apply_resnet50_M15"] = {"ms": ms, "GB/s": b / ms / 1e6, "frac": b / ms / 1e6 / HBM_PEAK_GBS,
                                      "algorithmic_bytes": b, "note": "8 rotating buffer sets"}
    del sets
    # large bf16 fused step: d = 1.5e9, M = 31, fp32 momentum resident (186 GB), streamed in chunks of 2^26
    # coordinates (one launch per chunk, gradients double-buffered); one step = 23 launches
    M, d, chunk = 31, 1_500_000_000, 1 << 26
    free, _ = torch.cuda.mem_get_info()
    if free > (M * d * 4 + d * 2 + 2 * M * chunk * 2 + (4 << 30)):
        nch = (d + chunk - 1) // chunk
        v = torch.zeros((M, d), dtype=torch.float32, device=dev)
        x = wl.gaussian((chunk,), 0.02, seed=3, device=dev).to(torch.bfloat16).repeat(nch)[:d].contiguous()
        mu = wl.shared_mean(chunk, seed=4, device=dev)
        g = [wl.worker_gradients(mu, M, s, base_seed=7, dtype=torch.bfloat16) for s in range(2)]

        def large_step(i):
            for c in range(nch):
                c0, c1 = c * chunk, min(d, (c + 1) * chunk)
                sv.signum_step(g[c % 2][:, :c1 - c0], v[:, c0:c1], 0.9, x[c0:c1], 1e-5)

        ms = time_launches(torch, large_step, 3, warmup=1)
        b = (10 * M + 4) * d
        out["signum_step_bf16_d1.5e9_M31"] = {"ms": ms, "launches": nch, "GB/s": b / ms / 1e6,
                                              "frac": b / ms / 1e6 / HBM_PEAK_GBS,
                                              "worker_coords_per_s": M * d / ms * 1e3, "algorithmic_bytes": b}
        del v, x, g
    else:
        out["signum_step_bf16_d1.5e9_M31"] = {"skipped": "not enough free HBM for the 186 GB momentum"}
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (the M workers are M buffers on that GPU); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_1810_05291_amd as sv
    import workloads as wl

    if not os.path.exists(sv.library_path()):
        from paper_1810_05291_amd import build as hip_build
        hip_build.build()
    sv.load_library()
    dev = "cuda:0"
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            sv.bench_copy(src, dst)          # ssv::copy_kernel: exactly 1 GiB read + 1 GiB written per launch
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"copy_calibration": "3 launches of ssv::copy_kernel", "bytes_read_each": src.numel() * 4,
                          "bytes_written_each": src.numel() * 4}))
        return
    M, d, K, Wm = args.workers, args.d, args.steps, args.warmup
    beta, lr = 0.9, 1e-4
    stride = ((d + args.row_align - 1) // args.row_align) * args.row_align

    # ---- inputs resident in HBM before the timed region ---------------------------------------
    mu = wl.shared_mean(d, seed=1, device=dev)
    x = wl.gaussian((d,), 0.02, seed=2, device=dev)
    v = torch.zeros((M, stride), device=dev)[:, :d]
    nsets = max(1, min(args.grad_sets, K + Wm))
    grads = [wl.worker_gradients(mu, M, s, base_seed=1000, row_stride=stride) for s in range(nsets)]
    torch.cuda.synchronize()

    # ---- CPU oracle on a bounded sample of the same workload (also a parity check of the warmup) ----
    ds = min(args.cpu_sample, d)
    cpu = None
    x_ref = v_ref = None
    if not args.no_cpu_baseline:
        import oracle as ora
        x_ref = wl.to_numpy(x[:ds]).copy()
        v_ref = np.zeros((M, ds), np.float32)
        g_h = [np.ascontiguousarray(wl.to_numpy(grads[s % nsets][:, :ds].contiguous())) for s in range(min(Wm, nsets))]
        t_cpu, n_cpu = 0.0, 0
        for s in range(Wm):
            t0 = time.perf_counter()
            ora.signum_step(g_h[s % len(g_h)], v_ref, beta, x_ref, lr)
            t_cpu += time.perf_counter() - t0
            n_cpu += 1
        # keep timing (on copies, so the parity state is not disturbed) until about 10 s of CPU work
        xs, vs = x_ref.copy(), v_ref.copy()
        while t_cpu < 10.0 and n_cpu < 1000:
            t0 = time.perf_counter()
            ora.signum_step(g_h[n_cpu % len(g_h)], vs, beta, xs, lr)
            t_cpu += time.perf_counter() - t0
            n_cpu += 1
        cpu = {"value": M * ds * n_cpu / t_cpu, "unit": "worker-coordinates/s (M*d/s)", "cores": ora.max_threads(),
               "kind": "oracle",
               "sample": f"first {ds} of {d} coordinates, M={M}, {n_cpu} fused steps, {t_cpu:.1f} s of CPU time"}

    # ---- warmup (untimed) ------------------------------------------------------------------------
    for s in range(Wm):
        sv.signum_step(grads[s % nsets], v, beta, x, lr)
    torch.cuda.synchronize()
    parity = None
    if x_ref is not None and Wm <= nsets:
        ok = np.array_equal(wl.to_numpy(x[:ds]), x_ref) and \
            np.array_equal(wl.to_numpy(v[:, :ds].contiguous()), v_ref)
        parity = "bit-exact vs oracle on the sample after warmup" if ok else "MISMATCH vs oracle"

    # ---- timed region: exactly K steps ---------------------------------------------------------------
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0.record()                       # on the current stream, the one the library launches on
    for s in range(K):
        sv.signum_step(grads[(Wm + s) % nsets], v, beta, x, lr)
    ev1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / K
    kern_ms = ev0.elapsed_time(ev1) / K

    algo_bytes = float(M * 12 + 8) * d
    achieved = algo_bytes / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "voted coords/sec (M*d/s), fused Signum step (momentum + sign + majority vote + update)",
        "value": M * d / (wall_ms * 1e-3),
        "unit": "worker-coordinates/s (M*d/s)",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "resnet50-sized fused Signum step", "d": d, "M": M, "beta": beta, "lr": lr,
                   "grad_dtype": "f32", "weight_dtype": "f32", "row_stride": stride,
                   "gradient_sets_cycled": nsets, "kernel": "ssv_signum_step"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS,
                     "traffic": read_traffic("signum_step_resnet50_pmc.txt"),
                     "kernel_ms": kern_ms, "algorithmic_bytes_per_launch": algo_bytes},
        "cpu_baseline": cpu,
        "parity": parity,
    }
    if args.other_kernels:
        del grads, v, x, mu
        torch.cuda.empty_cache()
        out["other_kernels"] = other_kernels(torch, sv, wl, dev)
    print(json.dumps(out), flush=True)
    if parity is not None and parity.startswith("MISMATCH"):
        sys.exit(1)


if __name__ == "__main__":
    main()
