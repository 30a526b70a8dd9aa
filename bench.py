#!/usr/bin/env python3
"""Benchmark of the fine-grained FP8 linear layer on one MI355X.

One "step" is one pass of the hot path over one batch of synthetic input at the
DeepSeek-V3 dense-FFN up-projection shape (X[4096x7168] BF16, W[18432x7168]
BF16): 1x128 quantization of X, 128x128 quantization of W and the block-scaled
FP8 GEMM Y = X W^T in BF16.  Inputs are resident in HBM before the timed
region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg4|cfg3|cfg5|fused] [--pow2] [--no-cpu-baseline]

The headline `value` is 2*M*N*K per step time (quantizers included) of the
default workload; `kernels` lists every kernel of the step with its own
roofline figure, measured with HIP events inside the timed steps.
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

PEAK_FP8_TFLOPS = 5000.0     # MI355X dense FP8 MFMA, published
PEAK_HBM_GBS = 8000.0        # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=500)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--settle-ms", type=float, default=250.0,
                    help="before the warmup steps, run untimed steps for this long so that the GPU has left its "
                         "idle power state and its clocks have settled (the first ~15 ms after idle run 15-20%% slower)")
    ap.add_argument("--event-every", type=int, default=8,
                    help="bracket the kernels with HIP events on every n-th timed step only (1 = every step)")
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5", "fused"])
    ap.add_argument("--unfused-swiglu", action="store_true", help="cfg3: separate SwiGLU and 1x128 quantizer kernels")
    ap.add_argument("--swiglu-kernel", action="store_true",
                    help="cfg3: SwiGLU and the 1x128 quantizer as one kernel behind the gate|up GEMM (default: in its epilogue)")
    ap.add_argument("--wgrad-from-cache", action="store_true",
                    help="cfg4: the Wgrad activation operand is re-tiled from the FP8 1x128 cache instead of re-quantized from BF16")
    ap.add_argument("--dual-weight-quant", action="store_true",
                    help="cfg4: the Dgrad weight codes come from the quantizer that writes W and W^T from one read of W")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the two machine probes (sustained MFMA rate, L2->LDS feed)")
    ap.add_argument("--gemm-variant", type=int, default=-1)
    ap.add_argument("--pow2", action="store_true",
                    help="power-of-two scaling factors (Section 3.3.3): the *_pow2 quantizers and the GEMM that lets "
                         "the matrix instruction apply the scales; not the headline configuration")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run three plain 256 MiB device copies and exit (scales the FETCH_SIZE / WRITE_SIZE counters)")
    return ap.parse_args()


class Timed:
    """A kernel launch bracketed by HIP events on the launching (current) stream."""

    def __init__(self, name, fn, unit, work, bound, peak, also=None):
        import torch
        self.name, self.fn, self.unit, self.work, self.bound, self.peak = name, fn, unit, work, bound, peak
        self.also = also                         # (bound, unit, work, peak): the kernel against its other roofline
        self.pairs = []
        self._torch = torch

    def __call__(self, record: bool):
        if record:
            e0 = self._torch.cuda.Event(enable_timing=True)
            e1 = self._torch.cuda.Event(enable_timing=True)
            e0.record()
            self.fn()
            e1.record()
            self.pairs.append((e0, e1))
        else:
            self.fn()

    def summary(self):
        ms = sorted(a.elapsed_time(b) for a, b in self.pairs)
        avg = sum(ms) / len(ms)
        achieved = self.work / (avg * 1e-3)
        out = dict(name=self.name, avg_us=avg * 1e3, min_us=ms[0] * 1e3, bound=self.bound, achieved=achieved,
                   peak=self.peak, unit=self.unit, frac=achieved / self.peak)
        if self.also:
            b, u, w, pk = self.also
            out["also"] = dict(bound=b, unit=u, achieved=w / (avg * 1e-3), peak=pk, frac=w / (avg * 1e-3) / pk)
        return out


def build_cfg2(ds3, torch, wl, dev, variant, pow2=False):
    """Dense FFN up-projection Fprop.  Two input sets are rotated so that the
    quantizers stream from HBM rather than from the 256 MB last-level cache."""
    M, N, K = 4096, wl.DENSE_INTER, wl.HIDDEN
    nsets_x, nsets_w = 10, 3                     # 587 MB of X, 793 MB of W: more than twice the last-level cache each
    x = wl.cfg2_x()
    w = wl.cfg2_w()
    xs = [torch.from_numpy(x).to(dev).to(torch.bfloat16) for _ in range(nsets_x)]
    ws = [torch.from_numpy(w).to(dev).to(torch.bfloat16) for _ in range(nsets_w)]
    del x, w
    state = {"i": 0}
    qa, sa = (ds3.ds3_quant_act_1x128_pow2 if pow2 else ds3.ds3_quant_act_1x128)(xs[0])
    qb, sb = (ds3.ds3_quant_w_128x128_pow2 if pow2 else ds3.ds3_quant_w_128x128)(ws[0])
    y = torch.empty((M, N), dtype=torch.bfloat16, device=dev)
    L = ds3._L()
    st = torch.cuda.current_stream().cuda_stream
    c_quant_x = L.ds3_quant_act_1x128_pow2 if pow2 else L.ds3_quant_act_1x128
    c_quant_w = L.ds3_quant_w_128x128_pow2 if pow2 else L.ds3_quant_w_128x128
    c_gemm = L.ds3_gemm_fp8_bs_pow2 if pow2 else L.ds3_gemm_fp8_bs_v

    def quant_x():
        xi = xs[state["i"] % nsets_x]
        c_quant_x(xi.data_ptr(), ds3.DS3_BF16, M, K, K, qa.data_ptr(), K, sa.data_ptr(), sa.stride(0), sa.stride(1), st)

    def quant_w():
        wi = ws[state["i"] % nsets_w]
        c_quant_w(wi.data_ptr(), ds3.DS3_BF16, N, K, K, qb.data_ptr(), K, sb.data_ptr(), st)

    def gemm():
        r = c_gemm(variant, M, N, K, qa.data_ptr(), K, sa.data_ptr(), sa.stride(0), sa.stride(1),
                   qb.data_ptr(), K, sb.data_ptr(), sb.stride(0), sb.stride(1), ds3.DS3_BSCALE_128x128,
                   y.data_ptr(), ds3.DS3_BF16, N, 0, None, 0, st)
        assert r == 0, r

    bx = M * K * (2 + 1) + M * (K // 128) * 4
    bw = N * K * (2 + 1) + (N // 128) * (K // 128) * 4
    kernels = [
        Timed("quant_act_1x128", quant_x, "GB/s", bx / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_w_128x128", quant_w, "GB/s", bw / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("gemm_fp8_bs", gemm, "TFLOP/s", 2.0 * M * N * K / 1e12, "mfma", PEAK_FP8_TFLOPS),
    ]

    def step(record):
        for k in kernels:
            k(record)
        state["i"] += 1

    cfg = {"workload": "cfg2: dense FFN up-projection Fprop, X[4096x7168] BF16 (1% outlier channels x50), "
                       "W[18432x7168] BF16 ~N(0,0.02); quant 1x128 + quant 128x128 + block-scaled FP8 GEMM, BF16 out",
           "M": M, "N": N, "K": K, "gemm_variant": variant}
    if pow2:
        cfg["workload"] += "; power-of-two scaling factors, scales applied by the matrix instruction"
        cfg["scales"] = "pow2"
    return step, kernels, 2.0 * M * N * K, cfg, "gemm_fp8_bs"


def library_context(torch, dev, M=4096, N=18432, K=7168):
    """Context only: what the vendor GEMM library reaches on this machine for the cfg2 shape WITHOUT block
    scaling (one scale per tensor) and in BF16.  Nothing of the product runs through it."""
    out = {}

    def rate(fn):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while time.perf_counter() - t0 < 0.25:
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(50):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return 2.0 * M * N * K / (e0.elapsed_time(e1) / 50 * 1e-3) / 1e12

    try:
        a = torch.randn(M, K, device=dev).to(torch.float8_e4m3fn)
        b = torch.randn(N, K, device=dev).to(torch.float8_e4m3fn)
        one = torch.tensor(1.0, device=dev)
        out["fp8_per_tensor_scale_gemm_tflops"] = rate(
            lambda: torch._scaled_mm(a, b.t(), scale_a=one, scale_b=one, out_dtype=torch.bfloat16))
        del a, b
    except Exception as e:                       # the call is private API of the installed torch
        out["fp8_per_tensor_scale_gemm_tflops"] = None
        out["fp8_error"] = repr(e)[:120]
    a = torch.randn(M, K, device=dev, dtype=torch.bfloat16)
    b = torch.randn(N, K, device=dev, dtype=torch.bfloat16)
    out["bf16_gemm_tflops"] = rate(lambda: a @ b.t())
    out["shape"] = [M, N, K]
    return out


def machine_probes(ds3, torch, dev):
    """What this chip sustains: FP8 MFMA rate from registers, and L2 -> LDS feed rate per compute unit."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    out_f = torch.empty(cus * 8, dtype=torch.float32, device=dev)
    out_i = torch.empty(cus, dtype=torch.int32, device=dev)
    src = torch.zeros(64 << 20, dtype=torch.uint8, device=dev)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        best = 1e30
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            best = min(best, e0.elapsed_time(e1) * 1e-3)
        return best

    iters = 4000
    t = timed(lambda: ds3.ds3_probe_mfma_fp8(iters, cus, out_f))
    mfma = cus * 8 * iters * 32 * 65536.0 / t / 1e12
    t = timed(lambda: ds3.ds3_probe_lds_feed(src, 7168, iters, cus, out_i))
    feed = iters * 65536.0 / t / 1e9
    lib = library_context(torch, dev)
    return {"library_context": lib, "mfma_fp8_register_loop_tflops": mfma, "mfma_fp8_register_loop_frac_of_peak": mfma / PEAK_FP8_TFLOPS,
            "l2_to_lds_feed_gbs_per_cu": feed, "l2_to_lds_feed_tbs_total": feed * cus / 1e3,
            "feed_needed_gbs_per_cu_at_register_loop_rate": 65536.0 / (2.0 * 256 * 256 * 128 / (mfma * 1e12 / cus)) / 1e9,
            "note": "a 256x256 FP8 tile consumes 64 KiB of operands per 128-deep K-step (2*256*256*128 flop); the feed probe "
                    "keeps one K-step of LDS-bound loads queued behind the one it waits for, as the GEMM does"}


def cpu_baseline(wl):
    """The oracle as it stands on a bounded sample of the same workload."""
    import numpy as np
    from threadpoolctl import threadpool_info
    from oracle import ds3_oracle as orc
    ms, ns, k = 4096, wl.DENSE_INTER, wl.HIDDEN      # the whole cfg2 problem: about 10 s on the GPU machine's host
    x = wl.cfg2_x(m=ms)
    w = wl.cfg2_w(n=ns)
    t0 = time.perf_counter()
    qa, sa = orc.quant_act_1x128(x)
    qb, sb = orc.quant_w_128x128(w)
    y = orc.gemm_fp8_bs(qa, sa, qb, sb)
    dt = time.perf_counter() - t0
    assert np.isfinite(y).all()
    threads = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
    return {"value": 2.0 * ms * ns * k / dt / 1e12, "unit": "TFLOP/s", "cores": threads, "kind": "oracle",
            "seconds": dt,
            "sample": f"the whole cfg2 step once: oracle quant 1x128 of X[{ms}x{k}] + quant 128x128 of W[{ns}x{k}] + "
                      f"FP64 GEMM {ms}x{ns}x{k}; numpy elementwise (1 thread) + OpenBLAS dgemm ({threads} threads)"}


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures the single-GPU hot path only; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    import paper_2412_19437_amd as ds3
    from synth import workloads as wl
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    ds3._L()                                     # fail loudly if libds3.so has not been built
    dev = "cuda:0"
    if args.calibrate_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 256 << 20, "copy_bytes_written": 256 << 20, "launches": 3}))
        return
    if args.workload != "cfg2":
        import bench_extra
        step, kernels, flops, cfg, dominant = bench_extra.build(args.workload, ds3, torch, wl, dev, args.gemm_variant,
                                                                args.pow2, args.unfused_swiglu, args.wgrad_from_cache,
                                                                args.dual_weight_quant, args.swiglu_kernel)
    else:
        step, kernels, flops, cfg, dominant = build_cfg2(ds3, torch, wl, dev, args.gemm_variant, args.pow2)

    t_settle = time.perf_counter()
    while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
        for _ in range(8):
            step(False)
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    every = max(1, min(args.event_every, args.steps // 8 if args.steps >= 16 else 1))
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i % every == 0)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ksum = [k.summary() for k in kernels]
    dom = next(k for k in ksum if k["name"] == dominant)
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tfile):
        entry = json.load(open(tfile)).get(args.workload + ("_pow2" if args.pow2 else ""), {}).get(dominant)
        traffic = entry["total_bytes"] if entry else None     # HBM-side bytes per launch, from profiles/
    out = {
        "metric": "block-scaled FP8 GEMM TFLOP/s + % FP8 MFMA peak; quantizer GB/s + % HBM peak",
        "value": flops * args.steps / dt / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "settle_ms": args.settle_ms,
        "event_timed_steps": len(kernels[0].pairs),
        "ms_per_step": dt / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp8_e4m3 (fp32 accumulate)", "data": "synthetic",
        "config": cfg,
        "roofline": {"bound": dom["bound"], "achieved": dom["achieved"], "peak": dom["peak"], "unit": dom["unit"],
                     "frac": dom["frac"], "traffic": traffic, "kernel": dom["name"], "avg_us": dom["avg_us"]},
        "kernels": ksum,
    }
    if not args.no_probes:
        out["machine"] = machine_probes(ds3, torch, dev)
    if not args.no_cpu_baseline and not args.pow2:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
