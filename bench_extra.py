"""Benchmark workloads beyond the headline one (bench.py --workload cfg3|cfg4|cfg5).

Each builder returns (step, kernels, flops_per_step, config, dominant_kernel)
with the same meaning as bench.build_cfg2: `step(record)` enqueues one pass of
the workload on the current stream, timing every kernel with HIP events when
`record` is set.  Inputs are synthetic, seeded and resident in HBM.
"""
from __future__ import annotations

import numpy as np

PEAK_FP8_TFLOPS = 5000.0
PEAK_HBM_GBS = 8000.0


def _timed():
    from bench import Timed
    return Timed


def _quant_bytes(rows, cols, groups):
    return rows * cols * 3 + groups * 4


_UNFUSED_SWIGLU = False
_SWIGLU_KERNEL = False
_WGRAD_FROM_CACHE = False
_DUAL_WEIGHT_QUANT = False


class _Pow2:
    """The binding with every quantizer and GEMM replaced by its power-of-two-scale form."""

    def __init__(self, ds3):
        self._ds3 = ds3

    def __getattr__(self, name):
        if name.startswith(("ds3_quant_", "ds3_gemm_fp8_bs", "ds3_grouped_gemm_fp8_bs", "ds3_grouped_gemm_swiglu_quant_fp8_bs",
                            "ds3_swiglu_quant", "ds3_retile_")) \
                and not name.endswith("_pow2"):
            return getattr(self._ds3, name + "_pow2")
        return getattr(self._ds3, name)


def build(workload, ds3, torch, wl, dev, variant, pow2=False, unfused_swiglu=False, wgrad_from_cache=False,
          dual_weight_quant=False, swiglu_kernel=False):
    global _UNFUSED_SWIGLU, _WGRAD_FROM_CACHE, _DUAL_WEIGHT_QUANT, _SWIGLU_KERNEL
    _UNFUSED_SWIGLU, _WGRAD_FROM_CACHE, _DUAL_WEIGHT_QUANT = unfused_swiglu, wgrad_from_cache, dual_weight_quant
    _SWIGLU_KERNEL = swiglu_kernel
    step, kernels, flops, cfg, dominant = {"cfg3": _cfg3, "cfg4": _cfg4, "cfg5": _cfg5, "fused": _fused}[workload](
        _Pow2(ds3) if pow2 else ds3, torch, wl, dev, variant)
    if pow2:
        cfg["workload"] += "; power-of-two scaling factors, scales applied by the matrix instruction"
        cfg["scales"] = "pow2"
    return step, kernels, flops, cfg, dominant


def _bf16(torch, x, dev):
    return torch.from_numpy(x).to(dev).to(torch.bfloat16)


def _cfg3(ds3, torch, wl, dev, variant):
    """MoE expert FFN forward of one GPU's 32 experts: quant 1x128 -> grouped
    gate|up GEMM -> SwiGLU -> quant 1x128 -> grouped down GEMM.  By default the
    middle three run as one kernel (SwiGLU and the cast in the GEMM's epilogue,
    on a gate|up weight interleaved in blocks of 128 rows)."""
    Timed = _timed()
    G, H, I = wl.LOCAL_EXPERTS, wl.HIDDEN, wl.MOE_INTER
    sizes, off, _ = wl.cfg3_routing()
    rows = int(off[-1])
    x = _bf16(torch, wl.cfg3_tokens(rows), dev)
    gen = torch.Generator(device=dev).manual_seed(wl.seed_for(3, 2))
    w13 = (torch.randn((G * 2 * I, H), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
    w2 = (torch.randn((G * H, I), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
    offd = torch.from_numpy(off).to(dev)
    q13, s13 = ds3.ds3_quant_w_128x128(w13)
    q2, s2 = ds3.ds3_quant_w_128x128(w2)
    q13v, s13v = q13.view(G, 2 * I, H), s13.view(G, 2 * I // 128, H // 128)
    q2v, s2v = q2.view(G, H, I), s2.view(G, H // 128, I // 128)
    in_gemm = not (_UNFUSED_SWIGLU or _SWIGLU_KERNEL)
    if in_gemm:
        # whole 128-row blocks move: the interleaved weight's codes and scales are those of w13, reordered
        q13i = q13v.view(G, 2, I // 128, 128, H).transpose(1, 2).contiguous().view(G, 2 * I, H)
        s13i = s13v.view(G, 2, I // 128, H // 128).transpose(1, 2).contiguous().view(G, 2 * I // 128, H // 128)
    st = {}

    def quant_x():
        st["qx"], st["sx"] = ds3.ds3_quant_act_1x128(x)

    def quant_w():
        ds3.ds3_quant_w_128x128(w13)
        ds3.ds3_quant_w_128x128(w2)

    def gemm1():
        st["h"] = ds3.ds3_grouped_gemm_fp8_bs(st["qx"], st["sx"], offd, q13v, s13v, variant=variant)

    def swiglu():
        st["act"] = ds3.ds3_swiglu(st["h"])

    def quant_h():
        st["qh"], st["sh"] = ds3.ds3_quant_act_1x128(st["act"])

    def swiglu_quant():
        st["qh"], st["sh"] = ds3.ds3_swiglu_quant_1x128(st["h"])

    def gemm1_swiglu_quant():
        st["qh"], st["sh"] = ds3.ds3_grouped_gemm_swiglu_quant_fp8_bs(st["qx"], st["sx"], offd, q13i, s13i)

    def gemm2():
        st["y"] = ds3.ds3_grouped_gemm_fp8_bs(st["qh"], st["sh"], offd, q2v, s2v, variant=variant)

    f1, f2 = 2.0 * rows * 2 * I * H, 2.0 * rows * H * I
    # The grouped GEMMs at ~264 rows per expert are bound by the HBM stream of the expert weights (every weight
    # byte serves two or three row tiles): algorithmic bytes = codes + scales of both operands + the output, once.
    sc = lambda r, c: r * (c // 128) * 4
    b1_in = rows * H + sc(rows, H) + G * 2 * I * H + G * (2 * I // 128) * (H // 128) * 4
    b1 = b1_in + rows * 2 * I * 2                              # h in BF16
    b1_fused = b1_in + rows * I + sc(rows, I)                  # codes and scales of silu(gate) * up
    b2 = rows * I + sc(rows, I) + G * H * I + G * (H // 128) * (I // 128) * 4 + rows * H * 2
    mf = lambda f: ("mfma", "TFLOP/s", f / 1e12, PEAK_FP8_TFLOPS)
    wbytes = _quant_bytes(G * 2 * I, H, G * 2 * I * H // 16384) + _quant_bytes(G * H, I, G * H * I // 16384)
    kernels = [
        Timed("quant_act_1x128(x)", quant_x, "GB/s", _quant_bytes(rows, H, rows * H // 128) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_w_128x128(w13,w2)", quant_w, "GB/s", wbytes / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("grouped_gemm_fp8_bs(gate|up)", gemm1, "GB/s", b1 / 1e9, "hbm", PEAK_HBM_GBS, also=mf(f1)),
        Timed("swiglu", swiglu, "GB/s", rows * I * 6 / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_act_1x128(h)", quant_h, "GB/s", _quant_bytes(rows, I, rows * I // 128) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("grouped_gemm_fp8_bs(down)", gemm2, "GB/s", b2 / 1e9, "hbm", PEAK_HBM_GBS, also=mf(f2)),
    ]
    dominant = "grouped_gemm_fp8_bs(gate|up)"
    if in_gemm:
        dominant = "grouped_gemm_swiglu_quant_fp8_bs(gate|up)"
        kernels = kernels[:2] + [Timed(dominant, gemm1_swiglu_quant, "GB/s", b1_fused / 1e9, "hbm", PEAK_HBM_GBS,
                                       also=mf(f1))] + kernels[5:]
    elif _SWIGLU_KERNEL:
        # one pass: reads the gate|up output (4 B per activation), writes codes + scales (1.03 B)
        fused = Timed("swiglu_quant_1x128(fused)", swiglu_quant, "GB/s", (rows * I * 5 + rows * I // 128 * 4) / 1e9, "hbm",
                      PEAK_HBM_GBS)
        kernels = kernels[:3] + [fused] + kernels[5:]
    # rows the GEMM tiles cover / rows that hold tokens (128-row tiles unless a 256-row variant is forced)
    bm = 256 if variant == 0 else 128
    padded = int(sum((int(n) + bm - 1) // bm * bm for n in sizes))

    def step(record):
        for k in kernels:
            k(record)

    cfg = {"workload": "cfg3: MoE grouped Fprop, 32 local experts of 256, 8192 tokens top-8 (sigmoid affinity + bias), "
                       "gate|up [n_e x 7168]x[4096x7168]^T, SwiGLU, down [n_e x 2048]x[7168x2048]^T, BF16 out",
           "swiglu": ("separate SwiGLU and quantizer kernels" if _UNFUSED_SWIGLU else
                      "one kernel with the 1x128 quantizer" if _SWIGLU_KERNEL else
                      "in the gate|up GEMM's epilogue together with the 1x128 quantizer"),
           "padding_efficiency": rows / padded, "tile_rows": bm,
           "rows": rows, "group_sizes_min_med_max": [int(sizes.min()), int(np.median(sizes)), int(sizes.max())],
           "gemm_variant": variant}
    return step, kernels, f1 + f2, cfg, dominant


def _cfg4(ds3, torch, wl, dev, variant):
    """Backward of the dense FFN up-projection: Dgrad dX = dY W and Wgrad dW += dY^T X."""
    Timed = _timed()
    M, N, K = 4096, wl.DENSE_INTER, wl.HIDDEN
    x = _bf16(torch, wl.cfg2_x(), dev)
    dy = _bf16(torch, wl.cfg4_dy(), dev)
    wt = _bf16(torch, np.ascontiguousarray(wl.cfg2_w().T), dev)          # W^T [K][N]: the Dgrad weight operand
    dw = torch.zeros((N, K), dtype=torch.float32, device=dev)
    st = {}

    def q_dy_row():
        st["qdy"], st["sdy"] = ds3.ds3_quant_act_1x128(dy)

    def q_wt():
        st["qwt"], st["swt"] = ds3.ds3_quant_w_128x128(wt)

    w_fwd = _bf16(torch, wl.cfg2_w(), dev) if _DUAL_WEIGHT_QUANT else None   # W [N][K] as the forward pass holds it

    def q_w_dual():
        _, _, st["qwt"], st["swt"] = ds3.ds3_quant_w_128x128_dual(w_fwd)

    def dgrad():
        st["dx"] = ds3.ds3_gemm_fp8_bs(st["qdy"], st["sdy"], st["qwt"], st["swt"], variant=variant)

    def q_dy_col():
        st["qdyt"], st["sdyt"] = ds3.ds3_quant_act_128x1(dy)

    def q_x_col():
        st["qxt"], st["sxt"] = ds3.ds3_quant_act_128x1(x)

    qx_cache, sx_cache = ds3.ds3_quant_act_1x128(x)                      # what Fprop left behind

    def retile_x():
        st["qxt"], st["sxt"] = ds3.ds3_retile_1x128_to_128x1(qx_cache, sx_cache)

    def wgrad():
        ds3.ds3_gemm_fp8_bs(st["qdyt"], st["sdyt"], st["qxt"], st["sxt"], sb_mode=ds3.DS3_BSCALE_PER_ROW, c=dw,
                            accumulate=True, variant=variant)

    fl = 2.0 * M * N * K
    kernels = [
        Timed("quant_act_1x128(dY)", q_dy_row, "GB/s", _quant_bytes(M, N, M * N // 128) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_w_128x128(W^T)", q_wt, "GB/s", _quant_bytes(K, N, K * N // 16384) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("gemm_fp8_bs(dgrad)", dgrad, "TFLOP/s", fl / 1e12, "mfma", PEAK_FP8_TFLOPS),
        Timed("quant_act_128x1(dY)", q_dy_col, "GB/s", _quant_bytes(M, N, M * N // 128) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_act_128x1(X)", q_x_col, "GB/s", _quant_bytes(M, K, M * K // 128) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("gemm_fp8_bs(wgrad, fp32 accumulate)", wgrad, "TFLOP/s", fl / 1e12, "mfma", PEAK_FP8_TFLOPS),
    ]
    if _DUAL_WEIGHT_QUANT:
        # one read of W, codes written in both layouts: 2 + 1 + 1 bytes per element
        kernels[1] = Timed("quant_w_128x128_dual(W -> W, W^T)", q_w_dual, "GB/s", (K * N * 4 + 2 * (K * N // 16384) * 4) / 1e9,
                           "hbm", PEAK_HBM_GBS)
    if _WGRAD_FROM_CACHE:
        # X comes from the FP8 1x128 cache of the forward pass: 1 B read + 1 B written per element, scales both ways
        kernels[4] = Timed("retile_1x128_to_128x1(X cache)", retile_x, "GB/s", (M * K * 2 + 2 * (M * K // 128) * 4) / 1e9,
                           "hbm", PEAK_HBM_GBS)

    def step(record):
        for k in kernels:
            k(record)

    cfg = {"workload": "cfg4: backward of the cfg2 layer; Dgrad dX[4096x7168] = dY[4096x18432] W (dY 1x128, W^T 128x128) "
                       "and Wgrad dW[18432x7168] += dY^T X over 4096 tokens (both operands 128x1), dW FP32",
           "M": M, "N": N, "K": K, "gemm_variant": variant,
           "dgrad_weight_codes": "from the dual-layout quantizer of W" if _DUAL_WEIGHT_QUANT else "quantizer run on a materialised W^T",
           "wgrad_x_source": "FP8 1x128 cache, re-tiled" if _WGRAD_FROM_CACHE else "BF16 X, quantized along tokens"}
    return step, kernels, 2 * fl, cfg, "gemm_fp8_bs(dgrad)"


def _cfg5(ds3, torch, wl, dev, variant):
    """The four MLA projections (Section 2.1.1) at 8192 tokens."""
    Timed = _timed()
    kernels, flops = [], 0.0
    for idx, (name, m, n, k) in enumerate(wl.cfg5_shapes()):
        gen = torch.Generator(device=dev).manual_seed(wl.seed_for(5, idx))
        x = torch.randn((m, k), generator=gen, device=dev).to(torch.bfloat16)
        w = (torch.randn((n, k), generator=gen, device=dev) * 0.02).to(torch.bfloat16)
        st = {}

        def qx(x=x, st=st):
            st["qa"], st["sa"] = ds3.ds3_quant_act_1x128(x)

        def qw(w=w, st=st):
            st["qb"], st["sb"] = ds3.ds3_quant_w_128x128(w)

        def gemm(st=st):
            st["y"] = ds3.ds3_gemm_fp8_bs(st["qa"], st["sa"], st["qb"], st["sb"], variant=variant)

        fl = 2.0 * m * n * k
        flops += fl
        kernels += [
            Timed(f"quant_act_1x128({name})", qx, "GB/s", _quant_bytes(m, k, m * k // 128) / 1e9, "hbm", PEAK_HBM_GBS),
            Timed(f"quant_w_128x128({name})", qw, "GB/s", _quant_bytes(n, k, n * k // 16384 + 1) / 1e9, "hbm", PEAK_HBM_GBS),
        ]
        gbytes = m * k + n * k + m * (k // 128) * 4 + (n // 128 + 1) * (k // 128) * 4 + m * n * 2
        if gbytes / PEAK_HBM_GBS > fl / 1e3 / PEAK_FP8_TFLOPS:      # kv_b: writing the BF16 output takes longer than the MFMAs
            kernels.append(Timed(f"gemm_fp8_bs({name} {m}x{n}x{k})", gemm, "GB/s", gbytes / 1e9, "hbm", PEAK_HBM_GBS,
                                 also=("mfma", "TFLOP/s", fl / 1e12, PEAK_FP8_TFLOPS)))
        else:
            kernels.append(Timed(f"gemm_fp8_bs({name} {m}x{n}x{k})", gemm, "TFLOP/s", fl / 1e12, "mfma", PEAK_FP8_TFLOPS))

    def step(record):
        for kk in kernels:
            kk(record)

    cfg = {"workload": "cfg5: MLA projections at 8192 tokens: q_a 7168->1536, kv_a 7168->576, q_b 1536->24576, "
                       "kv_b 512->32768; quant 1x128 + quant 128x128 + block-scaled FP8 GEMM each, BF16 out",
           "gemm_variant": variant}
    return step, kernels, flops, cfg, "gemm_fp8_bs(q_b 8192x24576x1536)"


def _fused(ds3, torch, wl, dev, variant):
    """The producer-fused and layout kernels around the Linear at the dense-layer shapes (4096 tokens):
    RMSNorm -> quant, SwiGLU -> quant, FP8 cache re-tiling, dual-layout weight quantizer.  All HBM-bound;
    there is no GEMM in this workload, so `value` counts no flops."""
    Timed = _timed()
    T, H, I = 4096, wl.HIDDEN, wl.DENSE_INTER
    x = _bf16(torch, wl.cfg2_x(), dev)
    gen = torch.Generator(device=dev).manual_seed(wl.seed_for(6, 0))
    gamma = 1.0 + 0.1 * torch.randn(H, generator=gen, device=dev)
    h = (torch.randn((T, 2 * I), generator=gen, device=dev) * 2.0).to(torch.bfloat16)
    w = _bf16(torch, wl.cfg2_w(), dev)
    dy = _bf16(torch, wl.cfg4_dy(), dev)
    qdy, sdy = ds3.ds3_quant_act_1x128(dy)
    groups = lambda r, c: r * ((c + 127) // 128)
    kernels = [
        Timed("rmsnorm_quant_1x128(X 4096x7168)", lambda: ds3.ds3_rmsnorm_quant_1x128(x, gamma, 1e-6), "GB/s",
              (T * H * 3 + groups(T, H) * 4 + H * 4) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("swiglu_quant_1x128(h 4096x36864)", lambda: ds3.ds3_swiglu_quant_1x128(h), "GB/s",
              (T * I * 5 + groups(T, I) * 4) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("retile_1x128_to_128x1(dY 4096x18432)", lambda: ds3.ds3_retile_1x128_to_128x1(qdy, sdy), "GB/s",
              (T * I * 2 + 2 * groups(T, I) * 4) / 1e9, "hbm", PEAK_HBM_GBS),
        Timed("quant_w_128x128_dual(W 18432x7168)", lambda: ds3.ds3_quant_w_128x128_dual(w), "GB/s",
              (I * H * 4 + 2 * (I * H // 16384) * 4) / 1e9, "hbm", PEAK_HBM_GBS),
    ]

    def step(record):
        for k in kernels:
            k(record)

    kernels.append(Timed("quant_act_1x128_e5m6(X 4096x7168)", lambda: ds3.ds3_quant_act_1x128_e5m6(x), "GB/s",
                         (T * H * 3.5 + groups(T, H) * 4) / 1e9, "hbm", PEAK_HBM_GBS))
    # AdamW with BF16 moments on the layer's 132 M parameters: 22 bytes of traffic per parameter
    nparam = I * H
    mw = torch.randn(nparam, generator=gen, device=dev) * 0.02
    gr = torch.randn(nparam, generator=gen, device=dev) * 1e-3
    m1 = torch.zeros(nparam, dtype=torch.bfloat16, device=dev)
    v1 = torch.zeros(nparam, dtype=torch.bfloat16, device=dev)
    wb = torch.empty(nparam, dtype=torch.bfloat16, device=dev)
    state = {"t": 0}

    def adamw():
        state["t"] += 1
        ds3.ds3_adamw_bf16_states(mw, gr, m1, v1, 2.2e-4, 0.9, 0.95, 1e-8, 0.1, state["t"], w_bf16=wb)

    kernels.append(Timed("adamw_bf16_states(132M parameters)", adamw, "GB/s", nparam * 22 / 1e9, "hbm", PEAK_HBM_GBS))

    cfg = {"workload": "fused: producer-fused quantizers and layout kernels at the dense-layer shapes, 4096 tokens "
                       "(RMSNorm->1x128, SwiGLU->1x128, 1x128 cache -> 128x1, W -> codes of W and W^T), and the AdamW step with "
                       "BF16 moments on the layer's parameters"}
    return step, kernels, 0.0, cfg, "quant_w_128x128_dual(W 18432x7168)"
