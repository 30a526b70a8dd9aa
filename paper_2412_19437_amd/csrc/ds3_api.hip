// The C ABI of libds3: argument checking on the host, then a kernel launch.
// No entry point allocates, synchronises or touches device data on the host.
#include <cmath>

#include "ds3_internal.h"

namespace ds3 { int gemm_num_variants(); }
using namespace ds3;

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int64_t esize(ds3_dtype t) { return t == DS3_BF16 ? 2 : 4; }
inline bool dtype_ok(ds3_dtype t) { return t == DS3_BF16 || t == DS3_F32; }
constexpr int64_t kMaxDim = (1ll << 31) - 1;
// internal marker: "use the library's own statically allocated workspace" (16-byte aligned, never a device address)
void* const kStaticScratch = reinterpret_cast<void*>(static_cast<uintptr_t>(16));

ds3_status check_quant(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, const void* q,
                       int64_t ldq_min, int64_t ldq, const void* s) {
    if (!dtype_ok(xt)) return DS3_ERR_DTYPE;
    if (rows < 0 || cols < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DS3_OK;
    if (!x || !q || !s) return DS3_ERR_NULL;
    if (ldx < cols || ldq < ldq_min) return DS3_ERR_SHAPE;
    if (rows > kMaxDim || cols > kMaxDim) return DS3_ERR_UNSUPPORTED;
    const int64_t es = esize(xt);
    if (!aligned16(x) || !aligned16(q) || (ldx * es) % 16 || ldq % 16 || (cols * es) % 16) return DS3_ERR_ALIGN;
    return DS3_OK;
}

ds3_status gemm_common(bool pow2, int variant, int32_t G, const int32_t* offs, int64_t M, int64_t N, int64_t K, const uint8_t* a,
                       int64_t lda, const float* sa, int64_t sar, int64_t sak, const uint8_t* b, int64_t ldb,
                       const float* sb, int64_t sbr, int64_t sbk, ds3_bscale mode, void* c, ds3_dtype ct, int64_t ldc,
                       int accumulate, void* workspace, size_t workspace_bytes, void* stream) {
    if (!dtype_ok(ct)) return DS3_ERR_DTYPE;
    if (mode != DS3_BSCALE_128x128 && mode != DS3_BSCALE_PER_ROW) return DS3_ERR_DTYPE;
    if (accumulate && ct != DS3_F32) return DS3_ERR_DTYPE;
    if (M < 0 || N < 0 || K < 0 || G < 0) return DS3_ERR_SHAPE;
    if (K % 128) return DS3_ERR_SHAPE;
    if (variant < -1 || variant >= gemm_num_variants()) return DS3_ERR_UNSUPPORTED;
    if (M == 0 || N == 0) return DS3_OK;
    if (!c) return DS3_ERR_NULL;
    if (ldc < N) return DS3_ERR_SHAPE;
    if (!aligned16(c) || ldc % 4) return DS3_ERR_ALIGN;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim || G > 1023) return DS3_ERR_UNSUPPORTED;
    if (K == 0)                                               // an empty sum: C += 0, or C = 0
        return accumulate ? DS3_OK : launch_zero_fill(c, ct, M, N, ldc, static_cast<hipStream_t>(stream));
    if (!a || !b || !sa || !sb) return DS3_ERR_NULL;
    if (G > 0 && !offs) return DS3_ERR_NULL;
    if (lda < K || ldb < K) return DS3_ERR_SHAPE;
    if (workspace && !aligned16(workspace)) return DS3_ERR_ALIGN;
    if (!aligned16(a) || !aligned16(b) || lda % 16 || ldb % 16) return DS3_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(sa) & 3u) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return DS3_ERR_ALIGN;
    // the kernel addresses the scales with 31-bit byte offsets from sa / sb and non-negative strides
    {
        const int64_t kbm = K / 128, nb = mode == DS3_BSCALE_PER_ROW ? N : (N + 127) / 128, groups = G > 0 ? G : 1;
        if (sar < 0 || sak < 0 || sbr < 0 || sbk < 0) return DS3_ERR_UNSUPPORTED;
        const int64_t lim = (1ll << 29) - 1;       // elements
        if ((M - 1) > lim / (sar > 0 ? sar : 1) || (kbm - 1) > lim / (sak > 0 ? sak : 1) ||
            (M - 1) * sar + (kbm - 1) * sak > lim)
            return DS3_ERR_UNSUPPORTED;
        if ((nb - 1) > lim / (sbr > 0 ? sbr : 1) || (kbm - 1) > lim / (sbk > 0 ? sbk : 1) ||
            (groups - 1) * ((N + 127) / 128) * kbm + (nb - 1) * sbr + (kbm - 1) * sbk > lim)
            return DS3_ERR_UNSUPPORTED;
    }
    GemmParams p{};
    p.a = a; p.b = b; p.sa = sa; p.sb = sb; p.c = c;
    p.lda = lda; p.ldb = ldb; p.ldc = ldc;
    p.sar = sar; p.sak = sak; p.sbr = sbr; p.sbk = sbk;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.G = G;
    p.group_offsets = offs;
    p.b_group_stride = N * ldb;
    p.sb_group_stride = ((N + 127) / 128) * (K / 128);
    p.accumulate = accumulate;
    if (workspace == kStaticScratch) return launch_gemm_static_scratch(p, ct, mode, variant, pow2, static_cast<hipStream_t>(stream));
    return launch_gemm(p, ct, mode, variant, pow2, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

ds3_status grouped_common(bool pow2, int variant, int32_t G, const int32_t* group_offsets, int64_t total_rows, int64_t N,
                          int64_t K, const uint8_t* a, int64_t lda, const float* sa, int64_t sar, int64_t sak,
                          const uint8_t* b, int64_t ldb, const float* sb, void* c, ds3_dtype ct, int64_t ldc,
                          void* workspace, size_t workspace_bytes, void* stream) {
    if (G < 0) return DS3_ERR_SHAPE;
    if (G == 0) return DS3_OK;
    if (N > 0 && K > 0 && (int64_t)G * N * ldb >= (1ll << 40)) return DS3_ERR_UNSUPPORTED;
    return gemm_common(pow2, variant, G, group_offsets, total_rows, N, K, a, lda, sa, sar, sak, b, ldb, sb, K / 128, 1,
                       DS3_BSCALE_128x128, c, ct, ldc, 0, workspace, workspace_bytes, stream);
}

}  // namespace

extern "C" {

static ds3_status quant_1x128(int pow2, const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q,
                              int64_t ldq, float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    const ds3_status st = check_quant(x, xt, rows, cols, ldx, q, cols, ldq, s);
    if (st != DS3_OK || rows == 0 || cols == 0) return st;
    return launch_quant_act_1x128(x, xt, rows, cols, ldx, q, ldq, s, s_stride_row, s_stride_kb, pow2,
                                  static_cast<hipStream_t>(stream));
}

static ds3_status quant_128x1(int pow2, const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx,
                              uint8_t* q_t, int64_t ldq, float* s_t, int64_t s_stride_col, int64_t s_stride_tb,
                              void* stream) {
    const ds3_status st = check_quant(x, xt, rows, cols, ldx, q_t, rows, ldq, s_t);
    if (st != DS3_OK || rows == 0 || cols == 0) return st;
    if ((rows + 127) / 128 > 65535) return DS3_ERR_UNSUPPORTED;
    return launch_quant_act_128x1(x, xt, rows, cols, ldx, q_t, ldq, s_t, s_stride_col, s_stride_tb, pow2,
                                  static_cast<hipStream_t>(stream));
}

static ds3_status quant_128x128(int pow2, const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                int64_t ldq, float* s, void* stream) {
    const ds3_status st = check_quant(w, wt, n, k, ldw, q, k, ldq, s);
    if (st != DS3_OK || n == 0 || k == 0) return st;
    if ((n + 127) / 128 > 65535) return DS3_ERR_UNSUPPORTED;
    return launch_quant_w_128x128(w, wt, n, k, ldw, q, ldq, s, pow2, static_cast<hipStream_t>(stream));
}

ds3_status ds3_quant_act_1x128(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q,
                               int64_t ldq, float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    return quant_1x128(0, x, xt, rows, cols, ldx, q, ldq, s, s_stride_row, s_stride_kb, stream);
}
ds3_status ds3_quant_act_1x128_pow2(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q,
                                    int64_t ldq, float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    return quant_1x128(1, x, xt, rows, cols, ldx, q, ldq, s, s_stride_row, s_stride_kb, stream);
}

ds3_status ds3_quant_act_128x1(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q_t,
                               int64_t ldq, float* s_t, int64_t s_stride_col, int64_t s_stride_tb, void* stream) {
    return quant_128x1(0, x, xt, rows, cols, ldx, q_t, ldq, s_t, s_stride_col, s_stride_tb, stream);
}
ds3_status ds3_quant_act_128x1_pow2(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q_t,
                                    int64_t ldq, float* s_t, int64_t s_stride_col, int64_t s_stride_tb, void* stream) {
    return quant_128x1(1, x, xt, rows, cols, ldx, q_t, ldq, s_t, s_stride_col, s_stride_tb, stream);
}

ds3_status ds3_quant_w_128x128(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q, int64_t ldq,
                               float* s, void* stream) {
    return quant_128x128(0, w, wt, n, k, ldw, q, ldq, s, stream);
}
ds3_status ds3_quant_w_128x128_pow2(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                    int64_t ldq, float* s, void* stream) {
    return quant_128x128(1, w, wt, n, k, ldw, q, ldq, s, stream);
}

ds3_status ds3_gemm_fp8_bs_v(int variant, int64_t M, int64_t N, int64_t K, const uint8_t* a, int64_t lda,
                             const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b,
                             int64_t ldb, const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb,
                             ds3_bscale sb_mode, void* c, ds3_dtype ct, int64_t ldc, int accumulate, void* workspace,
                             size_t workspace_bytes, void* stream) {
    return gemm_common(false, variant, 0, nullptr, M, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb, sb,
                       sb_stride_row, sb_stride_kb, sb_mode, c, ct, ldc, accumulate, workspace, workspace_bytes, stream);
}

ds3_status ds3_gemm_fp8_bs_pow2(int variant, int64_t M, int64_t N, int64_t K, const uint8_t* a, int64_t lda,
                                const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b,
                                int64_t ldb, const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb,
                                ds3_bscale sb_mode, void* c, ds3_dtype ct, int64_t ldc, int accumulate, void* workspace,
                                size_t workspace_bytes, void* stream) {
    return gemm_common(true, variant, 0, nullptr, M, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb, sb,
                       sb_stride_row, sb_stride_kb, sb_mode, c, ct, ldc, accumulate, workspace, workspace_bytes, stream);
}

ds3_status ds3_gemm_fp8_bs(int64_t M, int64_t N, int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                           int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b, int64_t ldb,
                           const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode, void* c,
                           ds3_dtype ct, int64_t ldc, int accumulate, void* workspace, size_t workspace_bytes,
                           void* stream) {
    return ds3_gemm_fp8_bs_v(-1, M, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb, sb, sb_stride_row,
                             sb_stride_kb, sb_mode, c, ct, ldc, accumulate, workspace, workspace_bytes, stream);
}

ds3_status ds3_gemm_fp8_bs_noalloc(int64_t M, int64_t N, int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                                   int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b, int64_t ldb,
                                   const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode, void* c,
                                   ds3_dtype ct, int64_t ldc, int accumulate, void* stream) {
    return gemm_common(false, -1, 0, nullptr, M, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb, sb, sb_stride_row,
                       sb_stride_kb, sb_mode, c, ct, ldc, accumulate, kStaticScratch, 0, stream);
}

size_t ds3_gemm_noalloc_scratch_bytes(void) { return gemm_static_scratch_bytes(); }

ds3_status ds3_grouped_gemm_fp8_bs_v(int variant, int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                     int64_t N, int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                                     int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b, int64_t ldb,
                                     const float* sb, void* c, ds3_dtype ct, int64_t ldc, void* workspace,
                                     size_t workspace_bytes, void* stream) {
    return grouped_common(false, variant, G, group_offsets, total_rows, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b,
                          ldb, sb, c, ct, ldc, workspace, workspace_bytes, stream);
}

ds3_status ds3_grouped_gemm_fp8_bs_pow2(int variant, int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                        int64_t N, int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                                        int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b, int64_t ldb,
                                        const float* sb, void* c, ds3_dtype ct, int64_t ldc, void* workspace,
                                        size_t workspace_bytes, void* stream) {
    return grouped_common(true, variant, G, group_offsets, total_rows, N, K, a, lda, sa, sa_stride_row, sa_stride_kb, b,
                          ldb, sb, c, ct, ldc, workspace, workspace_bytes, stream);
}

ds3_status ds3_grouped_gemm_fp8_bs(int32_t G, const int32_t* group_offsets, int64_t total_rows, int64_t N, int64_t K,
                                   const uint8_t* a, int64_t lda, const float* sa, int64_t sa_stride_row,
                                   int64_t sa_stride_kb, const uint8_t* b, int64_t ldb, const float* sb, void* c,
                                   ds3_dtype ct, int64_t ldc, void* workspace, size_t workspace_bytes, void* stream) {
    return ds3_grouped_gemm_fp8_bs_v(-1, G, group_offsets, total_rows, N, K, a, lda, sa, sa_stride_row, sa_stride_kb,
                                     b, ldb, sb, c, ct, ldc, workspace, workspace_bytes, stream);
}

static ds3_status grouped_swiglu_quant(bool pow2, int32_t G, const int32_t* offs, int64_t M, int64_t inter, int64_t K,
                                       const uint8_t* a, int64_t lda, const float* sa, int64_t sar, int64_t sak,
                                       const uint8_t* b, int64_t ldb, const float* sb, uint8_t* q, int64_t ldq, float* s,
                                       int64_t sor, int64_t sok, void* workspace, size_t workspace_bytes, void* stream) {
    if (G < 0 || M < 0 || inter < 0 || K < 0) return DS3_ERR_SHAPE;
    if (K % 128 || inter % 128) return DS3_ERR_SHAPE;
    if (G == 0 || M == 0 || inter == 0) return DS3_OK;
    if (!q || !s) return DS3_ERR_NULL;
    if (ldq < inter) return DS3_ERR_SHAPE;
    if (!aligned16(q) || ldq % 16 || (reinterpret_cast<uintptr_t>(s) & 3u)) return DS3_ERR_ALIGN;
    const int64_t N = 2 * inter;
    if (M > kMaxDim || N > kMaxDim || K > kMaxDim || G > 1023) return DS3_ERR_UNSUPPORTED;
    if (K == 0) return DS3_ERR_SHAPE;                    // the quantised activation of an empty product is not offered
    if (!a || !b || !sa || !sb || !offs) return DS3_ERR_NULL;
    if (lda < K || ldb < K) return DS3_ERR_SHAPE;
    if (!aligned16(a) || !aligned16(b) || lda % 16 || ldb % 16) return DS3_ERR_ALIGN;
    if (workspace && !aligned16(workspace)) return DS3_ERR_ALIGN;
    if ((reinterpret_cast<uintptr_t>(sa) & 3u) || (reinterpret_cast<uintptr_t>(sb) & 3u)) return DS3_ERR_ALIGN;
    if ((int64_t)G * N * ldb >= (1ll << 40)) return DS3_ERR_UNSUPPORTED;
    {
        const int64_t kbm = K / 128, lim = (1ll << 29) - 1;
        if (sar < 0 || sak < 0) return DS3_ERR_UNSUPPORTED;
        if ((M - 1) > lim / (sar > 0 ? sar : 1) || (kbm - 1) > lim / (sak > 0 ? sak : 1) ||
            (M - 1) * sar + (kbm - 1) * sak > lim)
            return DS3_ERR_UNSUPPORTED;
        if ((int64_t)G * (N / 128) * kbm > lim) return DS3_ERR_UNSUPPORTED;
    }
    GemmParams p{};
    p.a = a; p.b = b; p.sa = sa; p.sb = sb; p.c = nullptr;
    p.lda = lda; p.ldb = ldb; p.ldc = 0;
    p.sar = sar; p.sak = sak; p.sbr = K / 128; p.sbk = 1;
    p.M = (int)M; p.N = (int)N; p.K = (int)K; p.G = G;
    p.group_offsets = offs;
    p.b_group_stride = N * ldb;
    p.sb_group_stride = (N / 128) * (K / 128);
    p.q_out = q; p.s_out = s; p.ldq = ldq; p.sor = sor; p.sok = sok; p.q_pow2 = pow2 ? 1 : 0;
    return launch_gemm_swiglu_quant(p, pow2, workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

ds3_status ds3_grouped_gemm_swiglu_quant_fp8_bs(int32_t G, const int32_t* group_offsets, int64_t total_rows, int64_t inter,
                                                int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                                                int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b, int64_t ldb,
                                                const float* sb, uint8_t* q, int64_t ldq, float* s, int64_t s_stride_row,
                                                int64_t s_stride_kb, void* workspace, size_t workspace_bytes, void* stream) {
    return grouped_swiglu_quant(false, G, group_offsets, total_rows, inter, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb,
                                sb, q, ldq, s, s_stride_row, s_stride_kb, workspace, workspace_bytes, stream);
}

ds3_status ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2(int32_t G, const int32_t* group_offsets, int64_t total_rows, int64_t inter,
                                                     int64_t K, const uint8_t* a, int64_t lda, const float* sa,
                                                     int64_t sa_stride_row, int64_t sa_stride_kb, const uint8_t* b,
                                                     int64_t ldb, const float* sb, uint8_t* q, int64_t ldq, float* s,
                                                     int64_t s_stride_row, int64_t s_stride_kb, void* workspace,
                                                     size_t workspace_bytes, void* stream) {
    return grouped_swiglu_quant(true, G, group_offsets, total_rows, inter, K, a, lda, sa, sa_stride_row, sa_stride_kb, b, ldb,
                                sb, q, ldq, s, s_stride_row, s_stride_kb, workspace, workspace_bytes, stream);
}

size_t ds3_grouped_gemm_workspace_bytes(void) { return grouped_workspace_bytes(); }

int ds3_gemm_num_variants(void) { return gemm_num_variants(); }

size_t ds3_gemm_workspace_bytes_v(int variant, int64_t M, int64_t N, int64_t K, ds3_bscale sb_mode) {
    if (M <= 0 || N <= 0 || K <= 0 || K % 128 || M > kMaxDim || N > kMaxDim || K > kMaxDim) return 0;
    if (variant < -1 || variant >= gemm_num_variants()) return 0;
    if (sb_mode != DS3_BSCALE_128x128 && sb_mode != DS3_BSCALE_PER_ROW) return 0;
    GemmParams p{};
    p.M = (int)M; p.N = (int)N; p.K = (int)K;
    return gemm_workspace_bytes(p, sb_mode, variant);
}

ds3_status ds3_gemm_workspace_init(void* workspace, size_t workspace_bytes, void* stream) {
    if (workspace_bytes == 0) return DS3_OK;
    if (!workspace) return DS3_ERR_NULL;
    if (!aligned16(workspace)) return DS3_ERR_ALIGN;
    return launch_workspace_init(workspace, workspace_bytes, static_cast<hipStream_t>(stream));
}

int ds3_gemm_tail_share_steps(int tail_tiles, int k_steps, int workgroups) {
    return tail_share_steps(tail_tiles, k_steps, workgroups);
}

size_t ds3_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K) {
    const size_t blk = ds3_gemm_workspace_bytes_v(-1, M, N, K, DS3_BSCALE_128x128);
    const size_t row = ds3_gemm_workspace_bytes_v(-1, M, N, K, DS3_BSCALE_PER_ROW);
    return blk > row ? blk : row;
}

ds3_status ds3_swiglu(const void* h, int64_t rows, int64_t inter, int64_t ldh, void* out, int64_t ldo, void* stream) {
    if (rows < 0 || inter < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || inter == 0) return DS3_OK;
    if (!h || !out) return DS3_ERR_NULL;
    if (ldh < 2 * inter || ldo < inter) return DS3_ERR_SHAPE;
    if (!aligned16(h) || !aligned16(out) || inter % 8 || ldh % 8 || ldo % 8) return DS3_ERR_ALIGN;
    if (rows > kMaxDim || inter > kMaxDim) return DS3_ERR_UNSUPPORTED;
    return launch_swiglu(h, rows, inter, ldh, out, ldo, static_cast<hipStream_t>(stream));
}

static ds3_status quant_dual(int pow2, const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                             int64_t ldq, float* s, uint8_t* q_t, int64_t ldqt, float* s_t, void* stream) {
    const ds3_status st = check_quant(w, wt, n, k, ldw, q, k, ldq, s);
    if (st != DS3_OK || n == 0 || k == 0) return st;
    if (!q_t || !s_t) return DS3_ERR_NULL;
    if (ldqt < n) return DS3_ERR_SHAPE;
    if (!aligned16(q_t) || ldqt % 16) return DS3_ERR_ALIGN;
    if ((n + 127) / 128 > 65535) return DS3_ERR_UNSUPPORTED;
    return launch_quant_w_128x128_dual(w, wt, n, k, ldw, q, ldq, s, q_t, ldqt, s_t, pow2, static_cast<hipStream_t>(stream));
}

ds3_status ds3_quant_w_128x128_dual(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q, int64_t ldq,
                                    float* s, uint8_t* q_t, int64_t ldqt, float* s_t, void* stream) {
    return quant_dual(0, w, wt, n, k, ldw, q, ldq, s, q_t, ldqt, s_t, stream);
}
ds3_status ds3_quant_w_128x128_dual_pow2(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                         int64_t ldq, float* s, uint8_t* q_t, int64_t ldqt, float* s_t, void* stream) {
    return quant_dual(1, w, wt, n, k, ldw, q, ldq, s, q_t, ldqt, s_t, stream);
}

static ds3_status retile(int pow2, const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s, int64_t ssr,
                         int64_t ssk, uint8_t* q_t, int64_t ldqt, float* s_t, int64_t ssc, int64_t sst, void* stream) {
    if (rows < 0 || cols < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DS3_OK;
    if (!q || !s || !q_t || !s_t) return DS3_ERR_NULL;
    if (ldq < cols || ldqt < rows) return DS3_ERR_SHAPE;
    if (!aligned16(q) || !aligned16(q_t) || cols % 16 || ldq % 16 || ldqt % 16) return DS3_ERR_ALIGN;
    if (rows > kMaxDim || cols > kMaxDim || (rows + 127) / 128 > 65535) return DS3_ERR_UNSUPPORTED;
    return launch_retile_1x128_to_128x1(q, rows, cols, ldq, s, ssr, ssk, q_t, ldqt, s_t, ssc, sst, pow2,
                                        static_cast<hipStream_t>(stream));
}

ds3_status ds3_retile_1x128_to_128x1(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s,
                                     int64_t s_stride_row, int64_t s_stride_kb, uint8_t* q_t, int64_t ldqt, float* s_t,
                                     int64_t st_stride_col, int64_t st_stride_tb, void* stream) {
    return retile(0, q, rows, cols, ldq, s, s_stride_row, s_stride_kb, q_t, ldqt, s_t, st_stride_col, st_stride_tb, stream);
}
ds3_status ds3_retile_1x128_to_128x1_pow2(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s,
                                          int64_t s_stride_row, int64_t s_stride_kb, uint8_t* q_t, int64_t ldqt,
                                          float* s_t, int64_t st_stride_col, int64_t st_stride_tb, void* stream) {
    return retile(1, q, rows, cols, ldq, s, s_stride_row, s_stride_kb, q_t, ldqt, s_t, st_stride_col, st_stride_tb, stream);
}

ds3_status ds3_quant_act_1x128_e5m6(const void* x, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q, int64_t ldq, float* s,
                                    int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    if (rows < 0 || cols < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DS3_OK;
    if (!x || !q || !s) return DS3_ERR_NULL;
    if (ldx < cols || ldq < cols * 3 / 2) return DS3_ERR_SHAPE;
    if (!aligned16(x) || (reinterpret_cast<uintptr_t>(q) & 3u) || cols % 8 || ldx % 8 || ldq % 4) return DS3_ERR_ALIGN;
    if (rows > kMaxDim || cols > kMaxDim) return DS3_ERR_UNSUPPORTED;
    return launch_quant_act_1x128_e5m6(x, rows, cols, ldx, q, ldq, s, s_stride_row, s_stride_kb,
                                       static_cast<hipStream_t>(stream));
}

ds3_status ds3_dequant_e5m6(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s, int64_t s_stride_row,
                            int64_t s_stride_kb, void* y, int64_t ldy, void* stream) {
    if (rows < 0 || cols < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DS3_OK;
    if (!q || !s || !y) return DS3_ERR_NULL;
    if (ldy < cols || ldq < cols * 3 / 2) return DS3_ERR_SHAPE;
    if (!aligned16(y) || (reinterpret_cast<uintptr_t>(q) & 3u) || cols % 8 || ldy % 8 || ldq % 4) return DS3_ERR_ALIGN;
    if (rows > kMaxDim || cols > kMaxDim) return DS3_ERR_UNSUPPORTED;
    return launch_dequant_e5m6(q, rows, cols, ldq, s, s_stride_row, s_stride_kb, y, ldy, static_cast<hipStream_t>(stream));
}

ds3_status ds3_adamw_bf16_states(int64_t n, float* master_w, const float* grad, void* m, void* v, void* w_bf16, float lr,
                                 float beta1, float beta2, float eps, float weight_decay, int64_t step, void* stream) {
    if (n < 0 || step < 1) return DS3_ERR_SHAPE;
    if (n == 0) return DS3_OK;
    if (!master_w || !grad || !m || !v) return DS3_ERR_NULL;
    if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f && eps >= 0.f)) return DS3_ERR_SHAPE;
    if (n % 8 || !aligned16(master_w) || !aligned16(grad) || !aligned16(m) || !aligned16(v) || (w_bf16 && !aligned16(w_bf16)))
        return DS3_ERR_ALIGN;
    if (n / 8 > kMaxDim * 256ll) return DS3_ERR_UNSUPPORTED;
    // bias corrections in double on the host, handed over as FP32 reciprocals
    const float rbc1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)step)));
    const float rbc2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)step)));
    return launch_adamw_bf16_states(n, master_w, grad, m, v, w_bf16, lr, beta1, beta2, eps, weight_decay, rbc1, rbc2,
                                    static_cast<hipStream_t>(stream));
}

static ds3_status rmsnorm_quant(int pow2, const void* x, int64_t rows, int64_t cols, int64_t ldx, const float* gamma,
                                float eps, void* y, int64_t ldy, uint8_t* q, int64_t ldq, float* s, int64_t ssr,
                                int64_t ssk, void* stream) {
    if (rows < 0 || cols < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || cols == 0) return DS3_OK;
    if (!x || !gamma || !q || !s) return DS3_ERR_NULL;
    if (ldx < cols || ldq < cols || (y && ldy < cols)) return DS3_ERR_SHAPE;
    if (!(eps >= 0.0f)) return DS3_ERR_SHAPE;
    if (!aligned16(x) || !aligned16(q) || !aligned16(gamma) || (y && !aligned16(y)) || cols % 8 || ldx % 8 || ldq % 16 ||
        (y && ldy % 8))
        return DS3_ERR_ALIGN;
    if (rows > kMaxDim || cols > 8192) return DS3_ERR_UNSUPPORTED;
    return launch_rmsnorm_quant_1x128(x, rows, cols, ldx, gamma, eps, y, ldy, q, ldq, s, ssr, ssk, pow2,
                                      static_cast<hipStream_t>(stream));
}

ds3_status ds3_rmsnorm_quant_1x128(const void* x, int64_t rows, int64_t cols, int64_t ldx, const float* gamma, float eps,
                                   void* y, int64_t ldy, uint8_t* q, int64_t ldq, float* s, int64_t s_stride_row,
                                   int64_t s_stride_kb, void* stream) {
    return rmsnorm_quant(0, x, rows, cols, ldx, gamma, eps, y, ldy, q, ldq, s, s_stride_row, s_stride_kb, stream);
}
ds3_status ds3_rmsnorm_quant_1x128_pow2(const void* x, int64_t rows, int64_t cols, int64_t ldx, const float* gamma,
                                        float eps, void* y, int64_t ldy, uint8_t* q, int64_t ldq, float* s,
                                        int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    return rmsnorm_quant(1, x, rows, cols, ldx, gamma, eps, y, ldy, q, ldq, s, s_stride_row, s_stride_kb, stream);
}

static ds3_status swiglu_quant(int pow2, const void* h, int64_t rows, int64_t inter, int64_t ldh, uint8_t* q, int64_t ldq,
                               float* s, int64_t ssr, int64_t ssk, void* stream) {
    if (rows < 0 || inter < 0) return DS3_ERR_SHAPE;
    if (rows == 0 || inter == 0) return DS3_OK;
    if (!h || !q || !s) return DS3_ERR_NULL;
    if (ldh < 2 * inter || ldq < inter) return DS3_ERR_SHAPE;
    if (!aligned16(h) || !aligned16(q) || inter % 8 || ldh % 8 || ldq % 16) return DS3_ERR_ALIGN;
    if (rows > kMaxDim || inter > kMaxDim) return DS3_ERR_UNSUPPORTED;
    return launch_swiglu_quant_1x128(h, rows, inter, ldh, q, ldq, s, ssr, ssk, pow2, static_cast<hipStream_t>(stream));
}

ds3_status ds3_swiglu_quant_1x128(const void* h, int64_t rows, int64_t inter, int64_t ldh, uint8_t* q, int64_t ldq,
                                  float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    return swiglu_quant(0, h, rows, inter, ldh, q, ldq, s, s_stride_row, s_stride_kb, stream);
}
ds3_status ds3_swiglu_quant_1x128_pow2(const void* h, int64_t rows, int64_t inter, int64_t ldh, uint8_t* q, int64_t ldq,
                                       float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream) {
    return swiglu_quant(1, h, rows, inter, ldh, q, ldq, s, s_stride_row, s_stride_kb, stream);
}

ds3_status ds3_probe_mfma_fp8(int iters, int workgroups, float* out, void* stream) {
    if (iters < 0 || workgroups < 0) return DS3_ERR_SHAPE;
    if (iters == 0 || workgroups == 0) return DS3_OK;
    if (!out) return DS3_ERR_NULL;
    if (iters > (1 << 24) || workgroups > (1 << 20)) return DS3_ERR_UNSUPPORTED;
    return launch_probe_mfma(iters, out, workgroups, static_cast<hipStream_t>(stream));
}

ds3_status ds3_probe_lds_feed(const void* src, size_t window_bytes, int64_t row_stride, int iters, int workgroups,
                              uint32_t* out, void* stream) {
    if (iters < 0 || workgroups < 0 || row_stride < 128 || row_stride % 128) return DS3_ERR_SHAPE;
    if (iters == 0 || workgroups == 0) return DS3_OK;
    if (!src || !out) return DS3_ERR_NULL;
    if (!aligned16(src)) return DS3_ERR_ALIGN;
    // the kernel addresses 8 panels of 512 rows with 32-bit offsets below the out-of-range marker
    if (window_bytes >= (1ull << 31) || (uint64_t)row_stride * 4096 > window_bytes) return DS3_ERR_UNSUPPORTED;
    if (iters > (1 << 24) || workgroups > (1 << 20)) return DS3_ERR_UNSUPPORTED;
    return launch_probe_feed(src, (unsigned)window_bytes, (int)row_stride, iters, out, workgroups,
                             static_cast<hipStream_t>(stream));
}

const char* ds3_status_string(ds3_status st) {
    switch (st) {
        case DS3_OK: return "ok";
        case DS3_ERR_NULL: return "null pointer";
        case DS3_ERR_SHAPE: return "bad shape or leading dimension";
        case DS3_ERR_ALIGN: return "pointer, leading dimension or column count not 16-byte aligned";
        case DS3_ERR_DTYPE: return "bad dtype / mode";
        case DS3_ERR_UNSUPPORTED: return "size or variant not supported";
        case DS3_ERR_LAUNCH: return "kernel launch failed";
        case DS3_ERR_WORKSPACE: return "workspace smaller than ds3_gemm_workspace_bytes asks for";
    }
    return "unknown status";
}

}  // extern "C"
