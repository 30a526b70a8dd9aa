// Online E4M3 quantizers for gfx950: 1x128 activation tiles, 128x128 weight
// blocks and 128x1 (token-axis) tiles -- Section 3.3.2 "Fine-Grained
// Quantization" / "Online Quantization" and Section 3.3.3 "Low-Precision
// Activation" (1) of the DeepSeek-V3 report.  All three are single-pass HBM
// scans: every input element is read once with 128-bit loads, the max-abs is
// reduced in registers / across lanes, and codes plus FP32 scales are written
// from the same registers.
#include "ds3_dev.h"
#include "ds3_internal.h"

namespace ds3 {

// The quantizers touch every byte once: loads and stores carry the non-temporal hint
// so that the streams do not displace each other in the L2 / last-level cache
// (measured on MI355X: 6.2 TB/s instead of 5.5 TB/s for a 2:1 read:write stream).
__device__ __forceinline__ u32x4 ld_stream(const uint8_t* p) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
template <typename V>
__device__ __forceinline__ void st_stream(uint8_t* p, V v) {
    *reinterpret_cast<V*>(p) = v;
}
// Non-temporal store: measured faster only where a kernel reads at least as much as it
// writes per element and the tensors are large (the fused producers, the optimizer step);
// the plain quantizers and the transposing kernels are 5-15% slower with it.
template <typename V>
__device__ __forceinline__ void st_nt(uint8_t* p, V v) {
    __builtin_nontemporal_store(v, reinterpret_cast<V*>(p));
}

// Byte offset inside a [128 rows][128 + 16 bytes] LDS tile whose 16-byte chunks are
// XOR-swizzled by a key taken from the row index (bits KS .. KS+2): the lanes of a
// wave that write the same chunk position of rows 2^KS apart then hit different banks
// (the row stride of 144 bytes alone repeats the bank every 16 rows).  `off` is the
// byte offset inside the row; accesses never straddle a 16-byte chunk.
template <int KS>
__device__ __forceinline__ int tile_off(int row, int off) {
    return row * 144 + ((((off >> 4) ^ (row >> KS)) & 7) << 4) + (off & 15);
}

// ----- element traits: how many elements one 16-byte load carries --------------
struct Bf16 { static constexpr int EPL = 8; };   // elements per 128-bit load
struct F32  { static constexpr int EPL = 4; };

// Widen the EPL elements of one 16-byte granule to FP32.
template <typename T> __device__ __forceinline__ void widen(const u32x4& g, float* v);
template <> __device__ __forceinline__ void widen<Bf16>(const u32x4& g, float* v) {
    v[0] = bf16_lo(g.x); v[1] = bf16_hi(g.x); v[2] = bf16_lo(g.y); v[3] = bf16_hi(g.y);
    v[4] = bf16_lo(g.z); v[5] = bf16_hi(g.z); v[6] = bf16_lo(g.w); v[7] = bf16_hi(g.w);
}
template <> __device__ __forceinline__ void widen<F32>(const u32x4& g, float* v) {
    v[0] = as_f32(g.x); v[1] = as_f32(g.y); v[2] = as_f32(g.z); v[3] = as_f32(g.w);
}

// max |element| of one granule, as the bit pattern of a non-negative float.
template <typename T> __device__ __forceinline__ unsigned int granule_amax_bits(const u32x4& g);
template <> __device__ __forceinline__ unsigned int granule_amax_bits<Bf16>(const u32x4& g) {
    unsigned int m = 0;
    const unsigned int w[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        m = umax(m, w[i] & 0x7fff0000u);
        m = umax(m, (w[i] << 16) & 0x7fff0000u);
    }
    return m;
}
template <> __device__ __forceinline__ unsigned int granule_amax_bits<F32>(const u32x4& g) {
    return umax(umax(g.x & 0x7fffffffu, g.y & 0x7fffffffu), umax(g.z & 0x7fffffffu, g.w & 0x7fffffffu));
}

// =============================================================================
// 1x128: one 16-lane DPP row per tile.  A workgroup is 16 rows of the matrix
// (one per DPP row of its 4 waves) by TPG consecutive tiles, so each lane has
// TPG independent 128-bit loads in flight and the 16 scales of one K-block
// land in 64 contiguous bytes of a K-block-major scale array.
// The grid is one-dimensional and walks along the rows first (`ngroups` tile
// groups per band of 16 rows): the workgroups that are resident together then
// cover whole bands of consecutive rows, and every DRAM page they open is used
// to its end (column strips across all rows ran at 60% of HBM peak where this
// order reaches 70-76%).
// =============================================================================
template <typename T, int TPG>
__global__ __launch_bounds__(256) void quant_act_1x128_kernel(
    const uint8_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx_bytes,
    uint8_t* __restrict__ q, int64_t ldq, float* __restrict__ s, int64_t ssr, int64_t ssk, int pow2, int ngroups) {
    constexpr int EPL = T::EPL;
    constexpr int GPT = 8 / EPL;                  // granules per lane per tile (16 lanes x 8 elements)
    constexpr int ESZ = 16 / EPL;                 // bytes per element
    const int lane16 = threadIdx.x & 15;
    const int64_t row = (int64_t)(blockIdx.x / (unsigned)ngroups) * 16 + (threadIdx.x >> 4);
    if (row >= rows) return;                      // a whole DPP row leaves together
    const int64_t kb0 = (int64_t)(blockIdx.x % (unsigned)ngroups) * TPG;
    const int64_t nkb = (cols + 127) >> 7;
    const uint8_t* xr = x + row * ldx_bytes;

    u32x4 g[TPG][GPT];
    bool ok[TPG][GPT];
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
#pragma unroll
        for (int h = 0; h < GPT; ++h) {
            // granule h of the lane covers elements [h*64 + lane16*EPL, +EPL) of the tile when GPT == 2
            const int64_t col = (kb0 + t) * 128 + h * (128 / GPT) + lane16 * EPL;
            ok[t][h] = col < cols;
            g[t][h] = u32x4{0u, 0u, 0u, 0u};
            if (ok[t][h]) g[t][h] = ld_stream(xr + col * ESZ);
        }
    }
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
        if (kb0 + t >= nkb) break;
        unsigned int m = 0;
#pragma unroll
        for (int h = 0; h < GPT; ++h) m = umax(m, granule_amax_bits<T>(g[t][h]));
        m = row16_max_bits(m);
        const GroupScale gs = group_scale(as_f32(m), pow2);
        if (lane16 == 0) s[row * ssr + (kb0 + t) * ssk] = gs.s;
#pragma unroll
        for (int h = 0; h < GPT; ++h) {
            float v[EPL];
            widen<T>(g[t][h], v);
#pragma unroll
            for (int i = 0; i < EPL; ++i) v[i] = v[i] * gs.r;
            const int64_t col = (kb0 + t) * 128 + h * (128 / GPT) + lane16 * EPL;
            uint8_t* dst = q + row * ldq + col;
            if (ok[t][h]) {
                if constexpr (EPL == 8) {
                    u32x2 w = {cvt4_e4m3(v[0], v[1], v[2], v[3]), cvt4_e4m3(v[4], v[5], v[6], v[7])};
                    st_stream(dst, w);
                } else {
                    st_stream(dst, cvt4_e4m3(v[0], v[1], v[2], v[3]));
                }
            }
        }
    }
}

// =============================================================================
// 128x128: one workgroup per block.  The whole block (32 KiB BF16 / 64 KiB
// FP32) is held in registers between the max-abs pass and the cast, so HBM is
// read exactly once.
// =============================================================================
template <typename T>
__global__ __launch_bounds__(256) void quant_w_128x128_kernel(
    const uint8_t* __restrict__ w, int64_t n, int64_t k, int64_t ldw_bytes,
    uint8_t* __restrict__ q, int64_t ldq, float* __restrict__ s, int64_t nkb, int pow2) {
    constexpr int EPL = T::EPL;
    constexpr int ESZ = 16 / EPL;
    constexpr int LPR = 128 / EPL;                // lanes per block row
    constexpr int RPP = 256 / LPR;                // rows per pass
    constexpr int NP = 128 / RPP;                 // passes
    __shared__ unsigned int red[16];
    const int64_t kb = blockIdx.x, nb = blockIdx.y;
    const int lc = threadIdx.x % LPR, lr = threadIdx.x / LPR;
    const int64_t col = kb * 128 + lc * EPL;
    const bool col_ok = col < k;

    u32x4 g[NP];
    unsigned int m = 0;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int64_t row = nb * 128 + p * RPP + lr;
        g[p] = u32x4{0u, 0u, 0u, 0u};
        if (col_ok && row < n) g[p] = ld_stream(w + row * ldw_bytes + col * ESZ);
    }
#pragma unroll
    for (int p = 0; p < NP; ++p) m = umax(m, granule_amax_bits<T>(g[p]));
    m = row16_max_bits(m);
    if ((threadIdx.x & 15) == 0) red[threadIdx.x >> 4] = m;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) m = umax(m, red[i]);
    const GroupScale gs = group_scale(as_f32(m), pow2);
    if (threadIdx.x == 0) s[nb * nkb + kb] = gs.s;
#pragma unroll
    for (int p = 0; p < NP; ++p) {
        const int64_t row = nb * 128 + p * RPP + lr;
        float v[EPL];
        widen<T>(g[p], v);
#pragma unroll
        for (int i = 0; i < EPL; ++i) v[i] = v[i] * gs.r;
        if (col_ok && row < n) {
            uint8_t* dst = q + row * ldq + col;
            if constexpr (EPL == 8) {
                u32x2 o = {cvt4_e4m3(v[0], v[1], v[2], v[3]), cvt4_e4m3(v[4], v[5], v[6], v[7])};
                st_stream(dst, o);
            } else {
                st_stream(dst, cvt4_e4m3(v[0], v[1], v[2], v[3]));
            }
        }
    }
}

// =============================================================================
// 128x128 with both layouts from one read: the codes of W [n][k] and of its
// transpose [k][n] (the Dgrad operand; a 128x128 block and its scale are
// transpose-invariant, so the transposed codes are the same bytes moved).
// A thread owns RPT consecutive rows of one 16-byte granule, so for every one of
// its columns it holds RPT consecutive codes of the transposed row; those go
// through an LDS tile [k][n] and leave as 16-byte stores.
// =============================================================================
template <typename T>
__global__ __launch_bounds__(256) void quant_w_128x128_dual_kernel(
    const uint8_t* __restrict__ w, int64_t n, int64_t k, int64_t ldw_bytes,
    uint8_t* __restrict__ q, int64_t ldq, float* __restrict__ s,
    uint8_t* __restrict__ qt, int64_t ldqt, float* __restrict__ st, int64_t nkb, int64_t nnb, int pow2) {
    constexpr int EPL = T::EPL;
    constexpr int ESZ = 16 / EPL;
    constexpr int LPR = 128 / EPL;                // lanes per block row
    constexpr int NRG = 256 / LPR;                // row groups
    constexpr int RPT = 128 / NRG;                // consecutive rows per thread (8 BF16, 16 FP32)
    constexpr int OST = 128 + 16;
    constexpr int KS = EPL == 8 ? 3 : 4;          // swizzle key: the lane index across the block row
    __shared__ unsigned int red[16];
    __shared__ __attribute__((aligned(16))) uint8_t tile[128 * OST];   // [k][n]
    const int64_t kb = blockIdx.x, nb = blockIdx.y;
    const int lc = threadIdx.x % LPR, rg = threadIdx.x / LPR;
    const int64_t col = kb * 128 + lc * EPL;
    const bool col_ok = col < k;

    u32x4 g[RPT];
    unsigned int m = 0;
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int64_t row = nb * 128 + rg * RPT + r;
        g[r] = u32x4{0u, 0u, 0u, 0u};
        if (col_ok && row < n) g[r] = ld_stream(w + row * ldw_bytes + col * ESZ);
    }
#pragma unroll
    for (int r = 0; r < RPT; ++r) m = umax(m, granule_amax_bits<T>(g[r]));
    m = row16_max_bits(m);
    if ((threadIdx.x & 15) == 0) red[threadIdx.x >> 4] = m;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16; ++i) m = umax(m, red[i]);
    const GroupScale gs = group_scale(as_f32(m), pow2);
    if (threadIdx.x == 0) {
        s[nb * nkb + kb] = gs.s;
        st[kb * nnb + nb] = gs.s;
    }
    // codes of this thread: cw[r][j] = word j (4 consecutive columns) of row r
    unsigned int cw[RPT][EPL / 4];
#pragma unroll
    for (int r = 0; r < RPT; ++r) {
        const int64_t row = nb * 128 + rg * RPT + r;
        float v[EPL];
        widen<T>(g[r], v);
#pragma unroll
        for (int i = 0; i < EPL; ++i) v[i] = v[i] * gs.r;
#pragma unroll
        for (int j = 0; j < EPL / 4; ++j) cw[r][j] = cvt4_e4m3(v[4 * j], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]);
        if (col_ok && row < n) {
            uint8_t* dst = q + row * ldq + col;
            if constexpr (EPL == 8) st_stream(dst, u32x2{cw[r][0], cw[r][1]});
            else st_stream(dst, cw[r][0]);
        }
    }
    // transposed: for column e of the granule, the RPT codes of rows rg*RPT .. are consecutive in [k][n]
#pragma unroll
    for (int e = 0; e < EPL; ++e) {
        unsigned int tw[RPT / 4];
#pragma unroll
        for (int x = 0; x < RPT / 4; ++x) {
            unsigned int wv = 0;
#pragma unroll
            for (int b = 0; b < 4; ++b) wv |= ((cw[4 * x + b][e >> 2] >> (8 * (e & 3))) & 0xffu) << (8 * b);
            tw[x] = wv;
        }
        uint8_t* dst = tile + tile_off<KS>(lc * EPL + e, rg * RPT);
        if constexpr (RPT == 8) *reinterpret_cast<u32x2*>(dst) = u32x2{tw[0], tw[1]};
        else *reinterpret_cast<u32x4*>(dst) = u32x4{tw[0], tw[1], tw[2], tw[3]};
    }
    __syncthreads();
    // 128 transposed rows (k) x 8 chunks of 16 codes (n)
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int kr = it * 32 + (threadIdx.x >> 3), chunk = threadIdx.x & 7;
        const int64_t kk = kb * 128 + kr, nn = nb * 128 + chunk * 16;
        if (kk >= k || nn >= n) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(tile + tile_off<KS>(kr, chunk * 16));
        uint8_t* dst = qt + kk * ldqt + nn;
        if (nn + 16 <= n) {
            st_stream(dst, v);
        } else {
            const unsigned int wds[4] = {v.x, v.y, v.z, v.w};
            for (int b = 0; b < 16 && nn + b < n; ++b) dst[b] = (uint8_t)(wds[b >> 2] >> (8 * (b & 3)));
        }
    }
}

// =============================================================================
// 128x1: a workgroup takes 128 tokens x 128 channels.  Each thread loads TPT
// consecutive tokens of one 16-byte channel granule, so after the column
// max-abs (registers, then LDS across the token slices) it owns TPT
// consecutive codes of each of its channels; these go through an LDS tile
// laid out [channel][token] and leave as 16-byte token-contiguous stores.
// =============================================================================
template <typename T>
__global__ __launch_bounds__(256, (T::EPL == 8 ? 7 : 4)) void quant_act_128x1_kernel(
    const uint8_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx_bytes,
    uint8_t* __restrict__ qt, int64_t ldq, float* __restrict__ st, int64_t ssc, int64_t sst, int pow2) {
    constexpr int EPL = T::EPL;
    constexpr int ESZ = 16 / EPL;
    constexpr int LPR = 128 / EPL;                // lanes across the 128 channels
    constexpr int NSL = 256 / LPR;                // token slices (16 for BF16, 8 for FP32)
    constexpr int TPT = 128 / NSL;                // consecutive tokens per thread (8 / 16)
    constexpr int OST = 128 + 16;                 // LDS row stride of the [channel][token] tile
    constexpr int KS = EPL == 8 ? 3 : 4;          // swizzle key: the lane index across the channels
    // the per-slice maxima are dead once the multipliers are known: they share the code tile's memory
    __shared__ __attribute__((aligned(16))) uint8_t tile[128 * OST];
    __shared__ float rmul[128];
    static_assert(NSL * 128 * 4 <= 128 * OST, "partial maxima fit in the code tile");
    unsigned int (*part)[128] = reinterpret_cast<unsigned int (*)[128]>(tile);

    const int64_t c0 = (int64_t)blockIdx.x * 128, t0 = (int64_t)blockIdx.y * 128;
    const int lc = threadIdx.x % LPR, sl = threadIdx.x / LPR;
    const int64_t col = c0 + lc * EPL;
    const bool col_ok = col < cols;

    u32x4 g[TPT];
#pragma unroll
    for (int p = 0; p < TPT; ++p) {
        const int64_t tok = t0 + sl * TPT + p;
        g[p] = u32x4{0u, 0u, 0u, 0u};
        if (col_ok && tok < rows) g[p] = ld_stream(x + tok * ldx_bytes + col * ESZ);
    }
    // per-channel max over this thread's tokens
    unsigned int cm[EPL];
#pragma unroll
    for (int i = 0; i < EPL; ++i) cm[i] = 0;
#pragma unroll
    for (int p = 0; p < TPT; ++p) {
        const unsigned int wds[4] = {g[p].x, g[p].y, g[p].z, g[p].w};
        if constexpr (EPL == 8) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                cm[2 * i] = umax(cm[2 * i], (wds[i] << 16) & 0x7fff0000u);
                cm[2 * i + 1] = umax(cm[2 * i + 1], wds[i] & 0x7fff0000u);
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) cm[i] = umax(cm[i], wds[i] & 0x7fffffffu);
        }
    }
#pragma unroll
    for (int i = 0; i < EPL; ++i) part[sl][lc * EPL + i] = cm[i];
    __syncthreads();
    if (threadIdx.x < 128) {
        unsigned int m = 0;
#pragma unroll
        for (int j = 0; j < NSL; ++j) m = umax(m, part[j][threadIdx.x]);
        const GroupScale gs = group_scale(as_f32(m), pow2);
        rmul[threadIdx.x] = gs.r;
        if (c0 + threadIdx.x < cols) st[(c0 + threadIdx.x) * ssc + (int64_t)blockIdx.y * sst] = gs.s;
    }
    __syncthreads();
    // cast, and gather each channel's TPT consecutive tokens into the LDS tile
    // one channel at a time: its TPT tokens are widened, scaled and packed straight from the raw granules
#pragma unroll
    for (int i = 0; i < EPL; ++i) {
        const float r = rmul[lc * EPL + i];
        uint8_t* dst = tile + tile_off<KS>(lc * EPL + i, sl * TPT);
#pragma unroll
        for (int p = 0; p < TPT; p += 8) {
            float y[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const unsigned int wds[4] = {g[p + k].x, g[p + k].y, g[p + k].z, g[p + k].w};
                float xv;
                if constexpr (EPL == 8) xv = (i & 1) ? bf16_hi(wds[i >> 1]) : bf16_lo(wds[i >> 1]);
                else xv = as_f32(wds[i]);
                y[k] = xv * r;
            }
            u32x2 o = {cvt4_e4m3(y[0], y[1], y[2], y[3]), cvt4_e4m3(y[4], y[5], y[6], y[7])};
            *reinterpret_cast<u32x2*>(dst + p) = o;
        }
    }
    __syncthreads();
    // 128 channels x 8 chunks of 16 tokens
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ch = it * 32 + (threadIdx.x >> 3), chunk = threadIdx.x & 7;
        const int64_t tok = t0 + chunk * 16;
        if (c0 + ch >= cols || tok >= rows) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(tile + tile_off<KS>(ch, chunk * 16));
        uint8_t* dst = qt + (c0 + ch) * ldq + tok;
        if (tok + 16 <= rows) {
            st_stream(dst, v);
        } else {
            const unsigned int wds[4] = {v.x, v.y, v.z, v.w};
            for (int b = 0; b < 16 && tok + b < rows; ++b) dst[b] = (uint8_t)(wds[b >> 2] >> (8 * (b & 3)));
        }
    }
}

// =============================================================================
// SwiGLU between the two expert GEMMs: out = silu(gate) * up in FP32, BF16 out.
// =============================================================================
__global__ __launch_bounds__(256) void swiglu_kernel(const uint8_t* __restrict__ h, int64_t rows, int64_t inter,
                                                     int64_t ldh_bytes, uint8_t* __restrict__ out, int64_t ldo_bytes) {
    const int64_t gpr = inter >> 3;                                  // 8-element granules per row
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * gpr) return;
    const int64_t row = idx / gpr, gi = idx - row * gpr;
    const u32x4 gg = ld_stream(h + row * ldh_bytes + gi * 16);
    const u32x4 uu = ld_stream(h + row * ldh_bytes + (inter + gi * 8) * 2);
    float g[8], u[8], o[8];
    widen<Bf16>(gg, g);
    widen<Bf16>(uu, u);
#pragma unroll
    for (int i = 0; i < 8; ++i) o[i] = silu_mul(g[i], u[i]);
    u32x4 w = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
    st_stream(out + row * ldo_bytes + gi * 16, w);
}

// =============================================================================
// Re-tiling of a cached FP8 activation for the weight-gradient GEMM: 1x128
// tiles [T][C] -> 128x1 tiles written transposed [C][T].  Same workgroup shape
// as the 128x1 quantizer (128 tokens x 128 channels), but the source is one
// byte per element plus one scale per token: a thread owns 16 channels of 4
// consecutive tokens, dequantizes them with one FP32 multiply each (the same
// values for the max-abs pass and for the cast), and packs the 4 tokens of a
// channel into one word of the [channel][token] LDS tile.
// =============================================================================
__device__ __forceinline__ void dec4_e4m3(unsigned int w, float* v) {
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, false);
    const f32x2 hi = __builtin_amdgcn_cvt_pk_f32_fp8((int)w, true);
    v[0] = lo.x; v[1] = lo.y; v[2] = hi.x; v[3] = hi.y;
}

__global__ __launch_bounds__(256) void retile_1x128_to_128x1_kernel(
    const uint8_t* __restrict__ q, int64_t rows, int64_t cols, int64_t ldq,
    const float* __restrict__ s, int64_t ssr, int64_t ssk,
    uint8_t* __restrict__ qt, int64_t ldqt, float* __restrict__ st, int64_t ssc, int64_t sst, int pow2) {
    constexpr int LPR = 8;                        // lanes across the 128 channels (16 codes each)
    constexpr int NSL = 32;                       // token slices
    constexpr int TPT = 4;                        // consecutive tokens per thread
    constexpr int OST = 128 + 16;
    __shared__ __attribute__((aligned(16))) uint8_t tile[128 * OST];
    __shared__ float rmul[128];
    static_assert(NSL * 128 * 4 <= 128 * OST, "partial maxima fit in the code tile");
    unsigned int (*part)[128] = reinterpret_cast<unsigned int (*)[128]>(tile);

    const int64_t c0 = (int64_t)blockIdx.x * 128, t0 = (int64_t)blockIdx.y * 128;
    const int lc = threadIdx.x % LPR, sl = threadIdx.x / LPR;
    const int64_t col = c0 + lc * 16;
    const bool col_ok = col < cols;

    u32x4 g[TPT];
    float sc[TPT];
#pragma unroll
    for (int p = 0; p < TPT; ++p) {
        const int64_t tok = t0 + sl * TPT + p;
        g[p] = u32x4{0u, 0u, 0u, 0u};
        sc[p] = 0.f;
        if (col_ok && tok < rows) {
            g[p] = ld_stream(q + tok * ldq + col);
            sc[p] = s[tok * ssr + (int64_t)blockIdx.x * ssk];
        }
    }
    // per-channel max over this thread's 4 tokens
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        unsigned int cm[4] = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int p = 0; p < TPT; ++p) {
            float v[4];
            dec4_e4m3(g[p][w], v);
#pragma unroll
            for (int i = 0; i < 4; ++i) cm[i] = umax(cm[i], as_u32(v[i] * sc[p]) & 0x7fffffffu);
        }
        *reinterpret_cast<u32x4*>(&part[sl][lc * 16 + w * 4]) = u32x4{cm[0], cm[1], cm[2], cm[3]};
    }
    __syncthreads();
    if (threadIdx.x < 128) {
        unsigned int m = 0;
#pragma unroll
        for (int j = 0; j < NSL; ++j) m = umax(m, part[j][threadIdx.x]);
        const GroupScale gs = group_scale(as_f32(m), pow2);
        rmul[threadIdx.x] = gs.r;
        if (c0 + threadIdx.x < cols) st[(c0 + threadIdx.x) * ssc + (int64_t)blockIdx.y * sst] = gs.s;
    }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        float y[TPT][4];
#pragma unroll
        for (int p = 0; p < TPT; ++p) {
            dec4_e4m3(g[p][w], y[p]);
#pragma unroll
            for (int i = 0; i < 4; ++i) y[p][i] = y[p][i] * sc[p];
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const float r = rmul[lc * 16 + w * 4 + i];
            *reinterpret_cast<unsigned int*>(tile + tile_off<4>(lc * 16 + w * 4 + i, sl * TPT)) =
                cvt4_e4m3(y[0][i] * r, y[1][i] * r, y[2][i] * r, y[3][i] * r);
        }
    }
    __syncthreads();
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int ch = it * 32 + (threadIdx.x >> 3), chunk = threadIdx.x & 7;
        const int64_t tok = t0 + chunk * 16;
        if (c0 + ch >= cols || tok >= rows) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(tile + tile_off<4>(ch, chunk * 16));
        uint8_t* dst = qt + (c0 + ch) * ldqt + tok;
        if (tok + 16 <= rows) {
            st_stream(dst, v);
        } else {
            const unsigned int wds[4] = {v.x, v.y, v.z, v.w};
            for (int b = 0; b < 16 && tok + b < rows; ++b) dst[b] = (uint8_t)(wds[b >> 2] >> (8 * (b & 3)));
        }
    }
}

// =============================================================================
// SwiGLU fused with the 1x128 quantizer of the down projection's input: the
// activation is rounded to BF16 exactly as swiglu_kernel writes it, but goes
// straight from registers into the max-abs / scale / cast steps of the 1x128
// quantizer, so the BF16 tensor never travels to HBM and back.
// =============================================================================
template <int TPG>
__global__ __launch_bounds__(256) void swiglu_quant_1x128_kernel(
    const uint8_t* __restrict__ h, int64_t rows, int64_t inter, int64_t ldh_bytes,
    uint8_t* __restrict__ q, int64_t ldq, float* __restrict__ s, int64_t ssr, int64_t ssk, int pow2, int ngroups) {
    const int lane16 = threadIdx.x & 15;
    const int64_t row = (int64_t)(blockIdx.x / (unsigned)ngroups) * 16 + (threadIdx.x >> 4);
    if (row >= rows) return;                      // a whole DPP row leaves together
    const int64_t kb0 = (int64_t)(blockIdx.x % (unsigned)ngroups) * TPG;
    const int64_t nkb = (inter + 127) >> 7;
    const uint8_t* hr = h + row * ldh_bytes;
    u32x4 gg[TPG], uu[TPG];
    bool ok[TPG];
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
        const int64_t col = (kb0 + t) * 128 + lane16 * 8;
        ok[t] = col < inter;
        gg[t] = u32x4{0u, 0u, 0u, 0u};
        uu[t] = u32x4{0u, 0u, 0u, 0u};
        if (ok[t]) {
            gg[t] = ld_stream(hr + col * 2);
            uu[t] = ld_stream(hr + (inter + col) * 2);
        }
    }
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
        if (kb0 + t >= nkb) break;
        float g[8], u[8], o[8];
        widen<Bf16>(gg[t], g);
        widen<Bf16>(uu[t], u);
#pragma unroll
        for (int i = 0; i < 8; ++i) o[i] = silu_mul(g[i], u[i]);
        const u32x4 w = {pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]), pack_bf16x2(o[4], o[5]), pack_bf16x2(o[6], o[7])};
        const unsigned int m = row16_max_bits(granule_amax_bits<Bf16>(w));
        const GroupScale gs = group_scale(as_f32(m), pow2);
        if (lane16 == 0) s[row * ssr + (kb0 + t) * ssk] = gs.s;
        float v[8];
        widen<Bf16>(w, v);
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = v[i] * gs.r;
        if (ok[t]) {
            const int64_t col = (kb0 + t) * 128 + lane16 * 8;
            u32x2 c = {cvt4_e4m3(v[0], v[1], v[2], v[3]), cvt4_e4m3(v[4], v[5], v[6], v[7])};
            st_nt(q + row * ldq + col, c);
        }
    }
}

// =============================================================================
// RMSNorm fused with the 1x128 quantizer of the following Linear's input: one
// workgroup per row.  The row (at most 8192 BF16 elements) stays in registers
// between the sum of squares and the cast; each of the 16 DPP rows of the
// workgroup then handles every sixteenth 1x128 tile exactly as the stand-alone
// quantizer does.  The normalised activation is rounded to BF16 first (it is a
// BF16 tensor for every other consumer) and optionally written out.
// =============================================================================
constexpr int kNormMaxGranules = 4;               // 16-byte granules per lane: rows of up to 4 * 2048 elements

__global__ __launch_bounds__(256) void rmsnorm_quant_1x128_kernel(
    const uint8_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx_bytes, const float* __restrict__ gamma,
    float eps, uint8_t* __restrict__ y, int64_t ldy_bytes, uint8_t* __restrict__ q, int64_t ldq,
    float* __restrict__ s, int64_t ssr, int64_t ssk, int pow2) {
    __shared__ float red[2][4];
    const int lane16 = threadIdx.x & 15, t16 = threadIdx.x >> 4;

    // granule i of this lane: tile 16*i + t16, elements [lane16*8, +8) of it; the gains stay in registers
    // for all the rows this workgroup walks
    f32x4 gm[kNormMaxGranules][2];
    bool ok[kNormMaxGranules];
#pragma unroll
    for (int i = 0; i < kNormMaxGranules; ++i) {
        const int64_t col = ((int64_t)(16 * i + t16) << 7) + lane16 * 8;
        ok[i] = col < cols;
        gm[i][0] = gm[i][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (ok[i]) {
            gm[i][0] = *reinterpret_cast<const f32x4*>(gamma + col);
            gm[i][1] = *reinterpret_cast<const f32x4*>(gamma + col + 4);
        }
    }
    auto load_row = [&](int64_t row, u32x4* g) {
#pragma unroll
        for (int i = 0; i < kNormMaxGranules; ++i) {
            const int64_t col = ((int64_t)(16 * i + t16) << 7) + lane16 * 8;
            g[i] = u32x4{0u, 0u, 0u, 0u};
            if (ok[i] && row < rows) g[i] = ld_stream(x + row * ldx_bytes + col * 2);
        }
    };

    u32x4 g[kNormMaxGranules], gn[kNormMaxGranules];
    int64_t row = blockIdx.x;
    load_row(row, g);
    for (int it = 0; row < rows; row += gridDim.x, ++it) {
        load_row(row + gridDim.x, gn);            // the next row travels while this one is worked on
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < kNormMaxGranules; ++i) {
            float v[8];
            widen<Bf16>(g[i], v);
#pragma unroll
            for (int e = 0; e < 8; ++e) ss = __builtin_fmaf(v[e], v[e], ss);
        }
        // sum over the workgroup: butterflies inside the 16-lane rows, across the wave's four rows, then LDS
        ss += as_f32(dpp_u32<0xB1>(as_u32(ss)));
        ss += as_f32(dpp_u32<0x4E>(as_u32(ss)));
        ss += as_f32(dpp_u32<0x141>(as_u32(ss)));
        ss += as_f32(dpp_u32<0x140>(as_u32(ss)));
        ss += __shfl_xor(ss, 16);
        ss += __shfl_xor(ss, 32);
        if ((threadIdx.x & 63) == 0) red[it & 1][threadIdx.x >> 6] = ss;
        __syncthreads();                          // the two halves of `red` alternate: one barrier per row suffices
        ss = (red[it & 1][0] + red[it & 1][1]) + (red[it & 1][2] + red[it & 1][3]);
        const float rstd = 1.0f / sqrtf(ss / (float)cols + eps);

#pragma unroll
        for (int i = 0; i < kNormMaxGranules; ++i) {
            const int64_t kb = 16 * i + t16;
            const int64_t col = (kb << 7) + lane16 * 8;
            if ((kb << 7) < cols) {               // a whole DPP row decides together
                float v[8];
                widen<Bf16>(g[i], v);
                const float gmv[8] = {gm[i][0].x, gm[i][0].y, gm[i][0].z, gm[i][0].w, gm[i][1].x, gm[i][1].y, gm[i][1].z, gm[i][1].w};
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = v[e] * rstd * gmv[e];
                const u32x4 w = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])};
                if (y != nullptr && ok[i]) st_nt(y + row * ldy_bytes + col * 2, w);
                const unsigned int m = row16_max_bits(granule_amax_bits<Bf16>(w));
                const GroupScale gs = group_scale(as_f32(m), pow2);
                if (lane16 == 0) s[row * ssr + kb * ssk] = gs.s;
                float r[8];
                widen<Bf16>(w, r);
#pragma unroll
                for (int e = 0; e < 8; ++e) r[e] = r[e] * gs.r;
                if (ok[i]) st_nt(q + row * ldq + col, u32x2{cvt4_e4m3(r[0], r[1], r[2], r[3]), cvt4_e4m3(r[4], r[5], r[6], r[7])});
            }
        }
#pragma unroll
        for (int i = 0; i < kNormMaxGranules; ++i) g[i] = gn[i];
    }
}

// =============================================================================
// E5M6 activation cache (Section 3.3.3 (1)): 1x128 tiles with power-of-two scales,
// two 12-bit codes per three bytes.  One 16-lane DPP row per tile as in the E4M3
// quantizer; a lane's eight codes are 12 contiguous bytes, a tile 192.
// =============================================================================
template <int TPG>
__global__ __launch_bounds__(256) void quant_act_1x128_e5m6_kernel(
    const uint8_t* __restrict__ x, int64_t rows, int64_t cols, int64_t ldx_bytes,
    uint8_t* __restrict__ q, int64_t ldq, float* __restrict__ s, int64_t ssr, int64_t ssk, int ngroups) {
    const int lane16 = threadIdx.x & 15;
    const int64_t row = (int64_t)(blockIdx.x / (unsigned)ngroups) * 16 + (threadIdx.x >> 4);
    if (row >= rows) return;
    const int64_t kb0 = (int64_t)(blockIdx.x % (unsigned)ngroups) * TPG;
    const int64_t nkb = (cols + 127) >> 7;
    const uint8_t* xr = x + row * ldx_bytes;
    u32x4 g[TPG];
    bool ok[TPG];
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
        const int64_t col = (kb0 + t) * 128 + lane16 * 8;
        ok[t] = col < cols;
        g[t] = u32x4{0u, 0u, 0u, 0u};
        if (ok[t]) g[t] = ld_stream(xr + col * 2);
    }
#pragma unroll
    for (int t = 0; t < TPG; ++t) {
        if (kb0 + t >= nkb) break;
        const unsigned int m = row16_max_bits(granule_amax_bits<Bf16>(g[t]));
        const GroupScale gs = group_scale_e5m6(as_f32(m));
        if (lane16 == 0) s[row * ssr + (kb0 + t) * ssk] = gs.s;
        float v[8];
        widen<Bf16>(g[t], v);
        unsigned int c[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) c[i] = e5m6_rne(v[i] * gs.r);
        if (ok[t]) {
            // 8 codes of 12 bits -> 3 words, code i at bit 12*i
            const int64_t col = (kb0 + t) * 128 + lane16 * 8;
            unsigned int* dst = reinterpret_cast<unsigned int*>(q + row * ldq + col * 3 / 2);   // 4-byte aligned, 12 bytes
            dst[0] = c[0] | (c[1] << 12) | (c[2] << 24);
            dst[1] = (c[2] >> 8) | (c[3] << 4) | (c[4] << 16) | (c[5] << 28);
            dst[2] = (c[5] >> 4) | (c[6] << 8) | (c[7] << 20);
        }
    }
}

// packed E5M6 codes + scales -> BF16 (exact: 7 significant bits times a power of two)
__global__ __launch_bounds__(256) void dequant_e5m6_kernel(const uint8_t* __restrict__ q, int64_t rows, int64_t cols, int64_t ldq,
                                                           const float* __restrict__ s, int64_t ssr, int64_t ssk,
                                                           uint8_t* __restrict__ y, int64_t ldy_bytes) {
    const int64_t gpr = cols >> 3;                                   // 8-element granules per row
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= rows * gpr) return;
    const int64_t row = idx / gpr, gi = idx - row * gpr;
    const unsigned int* src = reinterpret_cast<const unsigned int*>(q + row * ldq + gi * 12);   // 4-byte aligned, 12 bytes
    const unsigned int w0 = src[0], w1 = src[1], w2 = src[2];
    const float sc = s[row * ssr + (gi >> 4) * ssk];
    const unsigned int c[8] = {w0 & 0xfffu, (w0 >> 12) & 0xfffu, ((w0 >> 24) | (w1 << 8)) & 0xfffu, (w1 >> 4) & 0xfffu,
                               (w1 >> 16) & 0xfffu, ((w1 >> 28) | (w2 << 4)) & 0xfffu, (w2 >> 8) & 0xfffu, w2 >> 20};
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = e5m6_decode(c[i]) * sc;
    st_stream(y + row * ldy_bytes + gi * 16,
              u32x4{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7])});
}

// =============================================================================
// AdamW step with BF16 first and second moments, FP32 master weights and FP32
// gradients (Section 3.3.3, Low-Precision Optimizer States).  One pass over the
// parameters: 8 per thread, 16-byte accesses.  The moments are updated in FP32
// from their BF16 values and rounded back to BF16 (nearest even) for storage;
// the update itself uses the unrounded FP32 moments.
// =============================================================================
struct AdamwArgs { float lr, beta1, beta2, eps, wd, rbc1, rbc2; };   // rbc = 1 / (1 - beta^t)

__global__ __launch_bounds__(256) void adamw_bf16_states_kernel(int64_t n8, float* __restrict__ w, const float* __restrict__ g,
                                                                uint8_t* __restrict__ m, uint8_t* __restrict__ v,
                                                                uint8_t* __restrict__ wb, AdamwArgs a) {
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n8) return;
    const u32x4 g0 = ld_stream(reinterpret_cast<const uint8_t*>(g) + i * 32);
    const u32x4 g1 = ld_stream(reinterpret_cast<const uint8_t*>(g) + i * 32 + 16);
    const u32x4 w0 = ld_stream(reinterpret_cast<const uint8_t*>(w) + i * 32);
    const u32x4 w1 = ld_stream(reinterpret_cast<const uint8_t*>(w) + i * 32 + 16);
    const u32x4 mm = ld_stream(m + i * 16);
    const u32x4 vv = ld_stream(v + i * 16);
    float gf[8] = {as_f32(g0.x), as_f32(g0.y), as_f32(g0.z), as_f32(g0.w), as_f32(g1.x), as_f32(g1.y), as_f32(g1.z), as_f32(g1.w)};
    float wf[8] = {as_f32(w0.x), as_f32(w0.y), as_f32(w0.z), as_f32(w0.w), as_f32(w1.x), as_f32(w1.y), as_f32(w1.z), as_f32(w1.w)};
    float mf[8], vf[8];
    widen<Bf16>(mm, mf);
    widen<Bf16>(vv, vf);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        mf[e] = a.beta1 * mf[e] + (1.0f - a.beta1) * gf[e];
        vf[e] = a.beta2 * vf[e] + (1.0f - a.beta2) * (gf[e] * gf[e]);
        const float mhat = mf[e] * a.rbc1, vhat = vf[e] * a.rbc2;
        wf[e] = wf[e] - a.lr * (mhat / (sqrtf(vhat) + a.eps) + a.wd * wf[e]);
    }
    st_nt(reinterpret_cast<uint8_t*>(w) + i * 32, u32x4{as_u32(wf[0]), as_u32(wf[1]), as_u32(wf[2]), as_u32(wf[3])});
    st_nt(reinterpret_cast<uint8_t*>(w) + i * 32 + 16, u32x4{as_u32(wf[4]), as_u32(wf[5]), as_u32(wf[6]), as_u32(wf[7])});
    st_nt(m + i * 16, u32x4{pack_bf16x2(mf[0], mf[1]), pack_bf16x2(mf[2], mf[3]), pack_bf16x2(mf[4], mf[5]), pack_bf16x2(mf[6], mf[7])});
    st_nt(v + i * 16, u32x4{pack_bf16x2(vf[0], vf[1]), pack_bf16x2(vf[2], vf[3]), pack_bf16x2(vf[4], vf[5]), pack_bf16x2(vf[6], vf[7])});
    if (wb != nullptr)
        st_nt(wb + i * 16, u32x4{pack_bf16x2(wf[0], wf[1]), pack_bf16x2(wf[2], wf[3]), pack_bf16x2(wf[4], wf[5]), pack_bf16x2(wf[6], wf[7])});
}

// ----- host launchers -----------------------------------------------------------
// (every launcher first drops a stale error of earlier, unrelated work: it is not this launch's)
static ds3_status launch_status() { return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH; }
static void drop_stale_error() { (void)hipGetLastError(); }

// One-dimensional grid of the 1x128-shaped kernels: bands of 16 rows times groups of TPG tiles, the
// groups of a band consecutive.  0 if the grid would not fit 31 bits.
static unsigned grid_1x128(int64_t rows, int64_t nkb, int tpg, int* ngroups) {
    const int64_t ng = (nkb + tpg - 1) / tpg, n = ((rows + 15) / 16) * ng;
    *ngroups = (int)ng;
    return n > 0x7fffffffll || ng > 0x7fffffffll ? 0u : (unsigned)n;
}

// Two tiles per lane group: fastest on the large tensors (75% of HBM peak on 4096 x 18432,
// 70% on 8192 x 7168) and within 3% of the best choice on the small ones.
constexpr int kTilesPerGroup = 2;

ds3_status launch_quant_act_1x128(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q,
                                  int64_t ldq, float* s, int64_t ssr, int64_t ssk, int pow2, hipStream_t st) {
    constexpr int TPG = kTilesPerGroup;
    int ngroups = 0;
    const unsigned grid = grid_1x128(rows, (cols + 127) / 128, TPG, &ngroups);
    if (grid == 0) return DS3_ERR_UNSUPPORTED;
    drop_stale_error();
    if (xt == DS3_BF16)
        quant_act_1x128_kernel<Bf16, TPG><<<dim3(grid), 256, 0, st>>>((const uint8_t*)x, rows, cols, ldx * 2, q, ldq, s, ssr, ssk, pow2, ngroups);
    else
        quant_act_1x128_kernel<F32, TPG><<<dim3(grid), 256, 0, st>>>((const uint8_t*)x, rows, cols, ldx * 4, q, ldq, s, ssr, ssk, pow2, ngroups);
    return launch_status();
}

ds3_status launch_quant_w_128x128(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                  int64_t ldq, float* s, int pow2, hipStream_t st) {
    drop_stale_error();
    const int64_t nkb = (k + 127) / 128, nnb = (n + 127) / 128;
    dim3 grid((unsigned)nkb, (unsigned)nnb);
    if (wt == DS3_BF16)
        quant_w_128x128_kernel<Bf16><<<grid, 256, 0, st>>>((const uint8_t*)w, n, k, ldw * 2, q, ldq, s, nkb, pow2);
    else
        quant_w_128x128_kernel<F32><<<grid, 256, 0, st>>>((const uint8_t*)w, n, k, ldw * 4, q, ldq, s, nkb, pow2);
    return launch_status();
}

ds3_status launch_quant_w_128x128_dual(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                       int64_t ldq, float* s, uint8_t* qt, int64_t ldqt, float* s_t, int pow2,
                                       hipStream_t st) {
    drop_stale_error();
    const int64_t nkb = (k + 127) / 128, nnb = (n + 127) / 128;
    dim3 grid((unsigned)nkb, (unsigned)nnb);
    if (wt == DS3_BF16)
        quant_w_128x128_dual_kernel<Bf16><<<grid, 256, 0, st>>>((const uint8_t*)w, n, k, ldw * 2, q, ldq, s, qt, ldqt, s_t,
                                                                 nkb, nnb, pow2);
    else
        quant_w_128x128_dual_kernel<F32><<<grid, 256, 0, st>>>((const uint8_t*)w, n, k, ldw * 4, q, ldq, s, qt, ldqt, s_t,
                                                                nkb, nnb, pow2);
    return launch_status();
}

ds3_status launch_quant_act_128x1(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* qt,
                                  int64_t ldq, float* s_t, int64_t ssc, int64_t sst, int pow2, hipStream_t st) {
    drop_stale_error();
    dim3 grid((unsigned)((cols + 127) / 128), (unsigned)((rows + 127) / 128));
    if (xt == DS3_BF16)
        quant_act_128x1_kernel<Bf16><<<grid, 256, 0, st>>>((const uint8_t*)x, rows, cols, ldx * 2, qt, ldq, s_t, ssc, sst, pow2);
    else
        quant_act_128x1_kernel<F32><<<grid, 256, 0, st>>>((const uint8_t*)x, rows, cols, ldx * 4, qt, ldq, s_t, ssc, sst, pow2);
    return launch_status();
}

ds3_status launch_swiglu(const void* h, int64_t rows, int64_t inter, int64_t ldh, void* out, int64_t ldo,
                         hipStream_t st) {
    drop_stale_error();
    const int64_t n = rows * (inter / 8);
    swiglu_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>((const uint8_t*)h, rows, inter, ldh * 2,
                                                                     (uint8_t*)out, ldo * 2);
    return launch_status();
}

ds3_status launch_retile_1x128_to_128x1(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s,
                                        int64_t ssr, int64_t ssk, uint8_t* qt, int64_t ldqt, float* s_t, int64_t ssc,
                                        int64_t sst, int pow2, hipStream_t st) {
    drop_stale_error();
    dim3 grid((unsigned)((cols + 127) / 128), (unsigned)((rows + 127) / 128));
    retile_1x128_to_128x1_kernel<<<grid, 256, 0, st>>>(q, rows, cols, ldq, s, ssr, ssk, qt, ldqt, s_t, ssc, sst, pow2);
    return launch_status();
}

ds3_status launch_quant_act_1x128_e5m6(const void* x, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q, int64_t ldq,
                                       float* s, int64_t ssr, int64_t ssk, hipStream_t st) {
    constexpr int TPG = kTilesPerGroup;
    int ngroups = 0;
    const unsigned grid = grid_1x128(rows, (cols + 127) / 128, TPG, &ngroups);
    if (grid == 0) return DS3_ERR_UNSUPPORTED;
    drop_stale_error();
    quant_act_1x128_e5m6_kernel<TPG><<<dim3(grid), 256, 0, st>>>((const uint8_t*)x, rows, cols, ldx * 2, q, ldq, s, ssr, ssk, ngroups);
    return launch_status();
}

ds3_status launch_dequant_e5m6(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s, int64_t ssr,
                               int64_t ssk, void* y, int64_t ldy, hipStream_t st) {
    drop_stale_error();
    const int64_t n = rows * (cols / 8);
    dequant_e5m6_kernel<<<dim3((unsigned)((n + 255) / 256)), 256, 0, st>>>(q, rows, cols, ldq, s, ssr, ssk, (uint8_t*)y, ldy * 2);
    return launch_status();
}

ds3_status launch_adamw_bf16_states(int64_t n, float* w, const float* g, void* m, void* v, void* wb, float lr, float beta1,
                                    float beta2, float eps, float wd, float rbc1, float rbc2, hipStream_t st) {
    drop_stale_error();
    const int64_t n8 = n / 8;
    AdamwArgs a{lr, beta1, beta2, eps, wd, rbc1, rbc2};
    adamw_bf16_states_kernel<<<dim3((unsigned)((n8 + 255) / 256)), 256, 0, st>>>(n8, w, g, (uint8_t*)m, (uint8_t*)v, (uint8_t*)wb, a);
    return launch_status();
}

ds3_status launch_rmsnorm_quant_1x128(const void* x, int64_t rows, int64_t cols, int64_t ldx, const float* gamma, float eps,
                                      void* y, int64_t ldy, uint8_t* q, int64_t ldq, float* s, int64_t ssr, int64_t ssk,
                                      int pow2, hipStream_t st) {
    drop_stale_error();
    if (cols > (int64_t)kNormMaxGranules * 2048) return DS3_ERR_UNSUPPORTED;
    // four workgroups per compute unit (all resident at once), each walking rows a grid apart
    const int64_t grid = rows < 1024 ? rows : 1024;
    rmsnorm_quant_1x128_kernel<<<dim3((unsigned)grid), 256, 0, st>>>(
        (const uint8_t*)x, rows, cols, ldx * 2, gamma, eps, (uint8_t*)y, ldy * 2, q, ldq, s, ssr, ssk, pow2);
    return launch_status();
}

ds3_status launch_swiglu_quant_1x128(const void* h, int64_t rows, int64_t inter, int64_t ldh, uint8_t* q, int64_t ldq,
                                     float* s, int64_t ssr, int64_t ssk, int pow2, hipStream_t st) {
    constexpr int TPG = kTilesPerGroup;
    int ngroups = 0;
    const unsigned grid = grid_1x128(rows, (inter + 127) / 128, TPG, &ngroups);
    if (grid == 0) return DS3_ERR_UNSUPPORTED;
    drop_stale_error();
    swiglu_quant_1x128_kernel<TPG><<<dim3(grid), 256, 0, st>>>((const uint8_t*)h, rows, inter, ldh * 2, q, ldq, s, ssr, ssk, pow2, ngroups);
    return launch_status();
}

}  // namespace ds3
