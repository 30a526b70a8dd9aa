"""Plain, slow, obviously-correct CPU oracle for the fine-grained FP8 linear layer.

THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and
the benchmark's ``cpu_baseline`` leg may import it; the GPU library never does,
and this file imports nothing from the GPU package.  It shares no code, table
or constant generator with the HIP kernels.

What it follows (DeepSeek-V3 technical report, arXiv 2412.19437):

* Section 3.3.2, "Fine-Grained Quantization": the max-abs of each group of
  elements is mapped to the largest representable FP8 value; activations are
  grouped 1x128 (per token, per 128 channels), weights 128x128.
* Section 3.3.2, "Mantissa over Exponents": every tensor uses E4M3.
* Section 3.3.2, "Online Quantization": the max-abs is taken from the data at
  hand, so the quantizers are stateless.
* Section 3.3.2, "Increasing Accumulation Precision": per-group scaling factors
  along the GEMM inner dimension are multiplied in as the de-quantisation step
  at every N_C = 128 interval; accumulation is high precision.
* Section 3.3.3, "Low-Precision Activation" (1): in the backward pass
  activations are tiled 128x1, i.e. the group of 128 runs along tokens.
* Section 3.3.1: GEMM outputs are BF16 or FP32 (the oracle leaves its result
  unrounded in FP64; the comparison tolerance covers the output rounding).

Readings where the paper is silent:

* the largest FP8 value that a group's max-abs is mapped to (Section 3.3.2) = 448, the OCP E4M3 maximum.
* The stored factor is the de-quantisation scale  s = fl32(amax / 448).
* Elements are scaled by one FP32 multiply with r = fl32(448 / amax), then
  rounded to nearest-even onto the E4M3 grid; magnitudes that would round
  above 448 saturate to 448; the sign bit is always copied.
* An all-zero group stores s = 1 and (signed) zero codes.
* A ragged trailing group is simply smaller.
* Inputs must be finite.
* Power-of-two ("round scaled", Section 3.3.3) factors: the smallest power
  of two >= amax / 448, elements multiplied by its exact reciprocal.

Pins (tests marked "not gpu"): closed form over all 256 codes, round trip of
all finite codes, every midpoint tie, brute-force nearest-neighbour search,
PyTorch's CPU float8_e4m3fn cast as a third opinion, an independent
exact-rational implementation of the quantizers and the GEMM on tiny shapes,
power-of-two exactness, scale-invariance, transposition identities, and the
"all scales 1 equals the plain product" identity; for the later additions:
the library optimizer in FP64 and the first step's closed form (AdamW), the
library RMSNorm, the library BF16 cast, composition identities of the fused
producers, and binary16's upper twelve bits plus brute-force nearest search
(E5M6 arithmetic).

PARITY UNPINNED: the bit layout and byte packing of the E5M6 cache format
(e5m6_* and quant_act_1x128_e5m6 / dequant_e5m6).  The report names the format
and its use but prints no layout; the one here is this build's proposal.  Its
arithmetic (rounding, scales, error bound) is pinned, its layout cannot be.
Every other function in this file is pinned.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0        # largest finite OCP E4M3 magnitude (S.1111.110)
TILE = 128              # N_C of Section 3.3.2


# --------------------------------------------------------------------------
# OCP E4M3 ("FN" flavour: no infinities, 0x7F / 0xFF are NaN)
# --------------------------------------------------------------------------
def e4m3_decode(codes) -> np.ndarray:
    """Exact value of each E4M3 code as float64.

    Format definition: 1 sign bit, 4 exponent bits (bias 7), 3 mantissa bits;
    exponent field 0 is subnormal (mantissa * 2^-9); S.1111.111 is NaN.
    """
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    sign = np.where((c & 0x80) != 0, -1.0, 1.0)
    efield = (c >> 3) & 0xF
    mant = (c & 0x7).astype(np.float64)
    normal = np.ldexp(1.0 + mant / 8.0, (efield - 7).astype(np.int64))
    subnormal = mant * 2.0 ** -9
    val = sign * np.where(efield == 0, subnormal, normal)
    return np.where((c & 0x7F) == 0x7F, np.nan, val)


def e4m3_encode_rne_sat(y) -> np.ndarray:
    """Round finite float values to the nearest E4M3 value, ties to the even
    code, saturating at +-448; returns the uint8 codes.  The sign bit of the
    input is always copied (so -0.0 and negative underflow give 0x80)."""
    y = np.asarray(y)
    if not np.all(np.isfinite(y)):
        raise ValueError("oracle precondition: finite inputs")
    neg = np.signbit(y)
    a = np.abs(y.astype(np.float64))
    # binade of a: a = m * 2^ex with m in [0.5, 1)  ->  floor(log2 a) = ex - 1
    _, ex = np.frexp(a)
    e = np.maximum(ex.astype(np.int64) - 1, -6)      # below 2^-6 the grid is the subnormal one
    quantum = np.ldexp(1.0, e - 3)                   # spacing of the grid in that binade
    n = np.rint(a / quantum)                         # exact division; rint is ties-to-even
    v = np.minimum(n * quantum, E4M3_MAX)            # a carry to 16*quantum is just the next binade
    # value -> code
    _, ex2 = np.frexp(v)
    e2 = ex2.astype(np.int64) - 1
    is_sub = v < 2.0 ** -6
    sub_code = np.rint(v * 2.0 ** 9).astype(np.int64)                 # 0..7
    mant = np.rint((v / np.ldexp(1.0, e2) - 1.0) * 8.0).astype(np.int64)
    norm_code = ((e2 + 7) << 3) | mant
    code = np.where(is_sub, sub_code, norm_code)
    code = np.where(neg, code | 0x80, code)
    return code.astype(np.uint8)


# --------------------------------------------------------------------------
# Quantizers (Section 3.3.2, Fine-Grained Quantization / Online Quantization)
# --------------------------------------------------------------------------
def _quant_groups(xg: np.ndarray, axes, pow2: bool = False):
    """Quantize groups.  ``xg`` is float32; the max-abs is taken over ``axes``
    (kept as size-1 axes for broadcasting).  Returns (codes, scales).

    ``pow2`` selects the "round scaled" factors of Section 3.3.3 (integral
    powers of two): the scale is the smallest power of two not below amax/448
    (reading: rounded up, so that nothing exceeds the E4M3 range), and the
    elements are multiplied by its exact reciprocal."""
    if xg.dtype != np.float32:
        raise TypeError("quantizer input must be float32 (BF16 widens exactly)")
    if not np.all(np.isfinite(xg)):
        raise ValueError("oracle precondition: finite inputs")
    amax = np.max(np.abs(xg), axis=axes, keepdims=True).astype(np.float32)
    zero = amax == np.float32(0)
    safe = np.where(zero, np.float32(1), amax)
    if pow2:
        ratio = safe.astype(np.float64) / E4M3_MAX           # exact enough: only its binade matters, ties are exact
        m, ex = np.frexp(ratio)                              # ratio = m * 2^ex, m in [0.5, 1)
        e = np.where(m == 0.5, ex - 1, ex)                   # smallest e with 2^e >= ratio
        s = np.where(zero, np.float32(1), np.ldexp(1.0, e)).astype(np.float32)
        r = np.where(zero, np.float32(0), np.ldexp(1.0, -e)).astype(np.float32)
    else:
        s = np.where(zero, np.float32(1), safe / np.float32(E4M3_MAX)).astype(np.float32)
        r = np.where(zero, np.float32(0), np.float32(E4M3_MAX) / safe).astype(np.float32)
    y = (xg * r).astype(np.float32)                  # one FP32 multiply per element
    return e4m3_encode_rne_sat(y), s


def _pad_to(x: np.ndarray, rows: int, cols: int) -> np.ndarray:
    out = np.zeros((rows, cols), dtype=x.dtype)
    out[: x.shape[0], : x.shape[1]] = x
    return out


def quant_act_1x128(x, pow2: bool = False):
    """1x128 tiles: per row (token), per 128 contiguous columns (channels).
    x: float32 [M][K].  Returns codes uint8 [M][K], scales float32 [M][ceil(K/128)].
    Zero padding of a ragged last tile changes neither its max-abs nor its
    codes, so padding implements "the group is simply smaller"."""
    x = np.asarray(x)
    m, k = x.shape
    kb = -(-k // TILE)
    xp = _pad_to(x, m, kb * TILE).reshape(m, kb, TILE)
    q, s = _quant_groups(xp, axes=(2,), pow2=pow2)
    return q.reshape(m, kb * TILE)[:, :k].copy(), s.reshape(m, kb)


def quant_act_128x1(x, pow2: bool = False):
    """128x1 tiles: the group of 128 runs along rows (tokens), one column
    (channel) wide.  x: float32 [T][C].  Returns the *transposed* results:
    codes uint8 [C][T] (token-contiguous) and scales float32 [C][ceil(T/128)],
    the layout the weight-gradient GEMM contracts over."""
    x = np.asarray(x)
    t, c = x.shape
    tb = -(-t // TILE)
    xp = _pad_to(x, tb * TILE, c).reshape(tb, TILE, c)
    q, s = _quant_groups(xp, axes=(1,), pow2=pow2)
    q = q.reshape(tb * TILE, c)[:t, :]
    return np.ascontiguousarray(q.T), np.ascontiguousarray(s.reshape(tb, c).T)


def quant_w_128x128(w, pow2: bool = False):
    """128x128 blocks: per 128 output channels (rows) per 128 input channels
    (columns).  w: float32 [N][K].  Returns codes uint8 [N][K] and scales
    float32 [ceil(N/128)][ceil(K/128)]."""
    w = np.asarray(w)
    n, k = w.shape
    nb, kb = -(-n // TILE), -(-k // TILE)
    wp = _pad_to(w, nb * TILE, kb * TILE).reshape(nb, TILE, kb, TILE)
    q, s = _quant_groups(wp, axes=(1, 3), pow2=pow2)
    return q.reshape(nb * TILE, kb * TILE)[:n, :k].copy(), s.reshape(nb, kb)


# --------------------------------------------------------------------------
# Block-scaled GEMM (Section 3.3.2, Increasing Accumulation Precision)
# --------------------------------------------------------------------------
def dequant_rows(codes, scales) -> np.ndarray:
    """decode(codes[i][k]) * scales[i][k // 128] in float64 (per-row, per-K-block scales)."""
    codes = np.asarray(codes, dtype=np.uint8)
    k = codes.shape[1]
    s = np.repeat(np.asarray(scales, dtype=np.float32).astype(np.float64), TILE, axis=1)[:, :k]
    return e4m3_decode(codes) * s


def dequant_blocks(codes, scales) -> np.ndarray:
    """decode(codes[n][k]) * scales[n // 128][k // 128] in float64 (128x128 block scales)."""
    codes = np.asarray(codes, dtype=np.uint8)
    n, k = codes.shape
    s = np.asarray(scales, dtype=np.float32).astype(np.float64)
    s = np.repeat(np.repeat(s, TILE, axis=0)[:n, :], TILE, axis=1)[:, :k]
    return e4m3_decode(codes) * s


def gemm_fp8_bs(a, sa, b, sb, sb_per_row: bool = False, c_in=None) -> np.ndarray:
    """Y[m][n] = sum_k (dec(a[m][k]) sa[m][k/128]) * (dec(b[n][k]) sb[..][k/128]) in float64.

    a: codes [M][K], sa: [M][K/128]; b: codes [N][K];
    sb: [ceil(N/128)][K/128] (weights, block scales) or, with ``sb_per_row``,
    [N][K/128] (the weight-gradient GEMM, where both operands carry 128x1
    tiles along the contracted token axis).  ``c_in`` (float) is added when
    given: gradients are accumulated in FP32 outside the FP8 domain
    (Section 3.3.3, optimizer states).  The result is left unrounded."""
    ad = dequant_rows(a, sa)
    bd = dequant_rows(b, sb) if sb_per_row else dequant_blocks(b, sb)
    y = ad @ bd.T
    if c_in is not None:
        y = y + np.asarray(c_in).astype(np.float64)
    return y


def grouped_gemm_fp8_bs(a, sa, group_offsets, b, sb) -> np.ndarray:
    """Per expert g: rows [off[g], off[g+1]) of ``a`` times expert g's weight
    b[g] ([N][K] codes) with block scales sb[g].  Section 2.1.2: experts see
    only the tokens routed to them; no token is dropped, so groups are ragged
    and may be empty."""
    a = np.asarray(a)
    off = np.asarray(group_offsets, dtype=np.int64)
    n = np.asarray(b).shape[1]
    y = np.zeros((a.shape[0], n), dtype=np.float64)
    for g in range(len(off) - 1):
        lo, hi = int(off[g]), int(off[g + 1])
        if hi > lo:
            y[lo:hi] = gemm_fp8_bs(a[lo:hi], np.asarray(sa)[lo:hi], b[g], sb[g])
    return y


def swiglu(h) -> np.ndarray:
    """SwiGLU of the fused gate|up projection output (Section 3.3.3 names the
    operator; the split is the reading: first half of the columns is the gate,
    second half is up).  out[r][j] = silu(h[r][j]) * h[r][I + j], float64."""
    h = np.asarray(h).astype(np.float64)
    inter = h.shape[1] // 2
    g, u = h[:, :inter], h[:, inter:]
    return g / (1.0 + np.exp(-g)) * u


def round_to_bf16(x) -> np.ndarray:
    """Round to the nearest BF16 value, ties to even; returned as float32.  The
    input is first brought to float32 (the producers compute in FP32)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(np.shape(x))


def swiglu_quant_1x128(h, pow2: bool = False):
    """The SwiGLU output as the down projection receives it (Section 3.3.3,
    Low-Precision Activation): the activation is a BF16 tensor (reading: rounded
    from the FP32 evaluation), quantized per 1x128 tile.  Defined as the
    composition of the two steps, which is what a fused kernel must equal."""
    return quant_act_1x128(round_to_bf16(swiglu(h)), pow2=pow2)


def retile_1x128_to_128x1(q, s, pow2: bool = False):
    """Re-tile a cached FP8 activation for the weight-gradient GEMM (Section
    3.5.2, transposed GEMM operations; Section 3.3.3 (1)): the 1x128-quantized
    matrix [T][C] is dequantized (one FP32 multiply per element), transposed,
    and re-quantized into 128x1 tiles along the token axis.  Returns what
    quant_act_128x1 returns: codes [C][T] and scales [C][ceil(T/128)]."""
    v = dequant_rows(q, s).astype(np.float32)          # dec(q) * s is exact in FP64, so this is ONE FP32 rounding
    return quant_act_128x1(v, pow2=pow2)


def quant_w_128x128_dual(w, pow2: bool = False):
    """The weight and its transpose, both 128x128-quantized (Section 3.3.1: Fprop
    uses W, Dgrad contracts over W's rows and needs W^T).  Each is quantized on its
    own here; that the second result is the transpose of the first is a property
    of block-wise tiles (Appendix B.2) which the tests pin rather than assume."""
    w = np.asarray(w)
    q, s = quant_w_128x128(w, pow2=pow2)
    q_t, s_t = quant_w_128x128(np.ascontiguousarray(w.T), pow2=pow2)
    return q, s, q_t, s_t


def rmsnorm(x, gamma, eps: float) -> np.ndarray:
    """RMSNorm (the normalisation DeepSeek-V3 applies before attention and FFN,
    Section 2 / Figure 2; Section 3.3 keeps it in its original precision):
    x[c] / sqrt(mean_c x[c]^2 + eps) * gamma[c], float64.  eps is the caller's
    (the report does not print it)."""
    x = np.asarray(x).astype(np.float64)
    g = np.asarray(gamma).astype(np.float64)
    return x / np.sqrt(np.mean(x * x, axis=1, keepdims=True) + float(eps)) * g[None, :]


def rmsnorm_quant_1x128(x, gamma, eps: float, pow2: bool = False):
    """RMSNorm output as the following Linear receives it: a BF16 tensor
    (reading), quantized per 1x128 tile.  The composition a fused kernel must equal."""
    return quant_act_1x128(round_to_bf16(rmsnorm(x, gamma, eps)), pow2=pow2)


def adamw_step(w, g, m, v, lr, beta1, beta2, eps, weight_decay, step, bf16_moments: bool = True):
    """One AdamW step (decoupled weight decay, bias-corrected moments) in float64,
    with the storage formats of Section 3.3.3: the moments are BF16 tensors (they
    arrive as BF16 values and are rounded to BF16 when stored), the master weights
    FP32.  The update uses the moments before their storage rounding (reading).
    Returns (w_new float32, m_new, v_new as float32 arrays holding the stored
    values, w_bf16 float32 array holding the BF16 copy).  With
    ``bf16_moments=False`` nothing is rounded and everything is returned in float64:
    the textbook algorithm, against which the function is pinned."""
    w = np.asarray(w).astype(np.float64)
    g = np.asarray(g).astype(np.float64)
    m = beta1 * np.asarray(m).astype(np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v).astype(np.float64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    w = w - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * w)
    if not bf16_moments:
        return w, m, v, w
    w32 = w.astype(np.float32)
    return w32, round_to_bf16(m), round_to_bf16(v), round_to_bf16(w32)


# --------------------------------------------------------------------------
# E5M6 activation cache (Section 3.3.3, Low-Precision Activation (1)).
# The report names the format (a customized 12-bit E5M6 for the inputs of the
# Linear after attention, with power-of-two 1x128 scaling factors) but gives no
# bit layout.  PROPOSED ENCODING of this build -- parity unpinned as far as the
# layout goes: 1 sign bit, 5 exponent bits (bias 15), 6 mantissa bits, i.e. the
# upper 12 bits of IEEE binary16: exponent field 0 is subnormal (mantissa *
# 2^-20), exponent field 31 is reserved and never produced, so the largest
# magnitude is (2 - 2^-6) * 2^15 = 65024.  Two codes a, b are packed into three
# bytes: a[7:0], a[11:8] | b[3:0] << 4, b[11:4].
# --------------------------------------------------------------------------
E5M6_MAX = 65024.0


def e5m6_decode(codes) -> np.ndarray:
    """Exact value of each 12-bit E5M6 code (uint16 array) as float64; reserved codes give NaN."""
    c = np.asarray(codes).astype(np.int64)
    sign = np.where((c & 0x800) != 0, -1.0, 1.0)
    efield = (c >> 6) & 0x1F
    mant = (c & 0x3F).astype(np.float64)
    normal = np.ldexp(1.0 + mant / 64.0, (efield - 15).astype(np.int64))
    val = sign * np.where(efield == 0, mant * 2.0 ** -20, normal)
    return np.where(efield == 31, np.nan, val)


def e5m6_encode_rne_sat(y) -> np.ndarray:
    """Round finite values to the nearest E5M6 value, ties to the even code,
    saturating at +-65024; the sign bit of the input is always copied."""
    y = np.asarray(y)
    if not np.all(np.isfinite(y)):
        raise ValueError("oracle precondition: finite inputs")
    neg = np.signbit(y)
    a = np.abs(y.astype(np.float64))
    _, ex = np.frexp(a)
    e = np.maximum(ex.astype(np.int64) - 1, -14)
    quantum = np.ldexp(1.0, e - 6)
    v = np.minimum(np.rint(a / quantum) * quantum, E5M6_MAX)
    _, ex2 = np.frexp(v)
    e2 = ex2.astype(np.int64) - 1
    sub = v < 2.0 ** -14
    sub_code = np.rint(v * 2.0 ** 20).astype(np.int64)
    mant = np.rint((v / np.ldexp(1.0, e2) - 1.0) * 64.0).astype(np.int64)
    code = np.where(sub, sub_code, ((e2 + 15) << 6) | mant)
    return np.where(neg, code | 0x800, code).astype(np.uint16)


def e5m6_pack(codes) -> np.ndarray:
    """[rows][k] 12-bit codes (k even) -> [rows][3k/2] bytes."""
    c = np.asarray(codes).astype(np.uint32)
    a, b = c[:, 0::2], c[:, 1::2]
    out = np.empty((c.shape[0], c.shape[1] // 2, 3), np.uint8)
    out[:, :, 0] = a & 0xFF
    out[:, :, 1] = (a >> 8) | ((b & 0xF) << 4)
    out[:, :, 2] = b >> 4
    return out.reshape(c.shape[0], -1)


def e5m6_unpack(packed) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8).astype(np.uint16).reshape(packed.shape[0], -1, 3)
    a = p[:, :, 0] | ((p[:, :, 1] & 0xF) << 8)
    b = (p[:, :, 1] >> 4) | (p[:, :, 2] << 4)
    return np.stack([a, b], axis=2).reshape(packed.shape[0], -1)


def quant_act_1x128_e5m6(x):
    """1x128 tiles, power-of-two scale = the smallest power of two >= amax / 65024
    (1 for an all-zero tile), elements times its exact reciprocal, rounded to
    E5M6.  x float32 [M][K], K even.  Returns (packed codes uint8 [M][3K/2],
    scales float32 [M][ceil(K/128)])."""
    x = np.asarray(x)
    if x.dtype != np.float32:
        raise TypeError("quantizer input must be float32 (BF16 widens exactly)")
    m, k = x.shape
    kb = (k + TILE - 1) // TILE
    xp = np.zeros((m, kb * TILE), np.float32)
    xp[:, :k] = x
    xg = xp.reshape(m, kb, TILE)
    amax = np.max(np.abs(xg), axis=2, keepdims=True)
    zero = amax == 0
    mant, ex = np.frexp(np.where(zero, 1.0, amax).astype(np.float64) / E5M6_MAX)
    e = np.where(mant == 0.5, ex - 1, ex)
    s = np.where(zero, 1.0, np.ldexp(1.0, e)).astype(np.float32)
    y = (xg * np.where(zero, 0.0, np.ldexp(1.0, -e)).astype(np.float32)).astype(np.float32)
    codes = e5m6_encode_rne_sat(y).reshape(m, kb * TILE)[:, :k]
    return e5m6_pack(codes), s.reshape(m, kb)


def dequant_e5m6(packed, scales) -> np.ndarray:
    """decode * scale, float64 [M][K]."""
    codes = e5m6_unpack(packed)
    k = codes.shape[1]
    s = np.repeat(np.asarray(scales, dtype=np.float32).astype(np.float64), TILE, axis=1)[:, :k]
    return e5m6_decode(codes) * s
