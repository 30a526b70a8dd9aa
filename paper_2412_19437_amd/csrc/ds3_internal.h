// Host-side declarations shared by the translation units of libds3.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/ds3.h"

namespace ds3 {

ds3_status launch_quant_act_1x128(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q,
                                  int64_t ldq, float* s, int64_t ssr, int64_t ssk, int pow2, hipStream_t st);
ds3_status launch_quant_act_128x1(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx, uint8_t* qt,
                                  int64_t ldq, float* s_t, int64_t ssc, int64_t sst, int pow2, hipStream_t st);
ds3_status launch_quant_w_128x128(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                  int64_t ldq, float* s, int pow2, hipStream_t st);
ds3_status launch_quant_w_128x128_dual(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw, uint8_t* q,
                                       int64_t ldq, float* s, uint8_t* qt, int64_t ldqt, float* s_t, int pow2,
                                       hipStream_t st);
ds3_status launch_swiglu(const void* h, int64_t rows, int64_t inter, int64_t ldh, void* out, int64_t ldo,
                         hipStream_t st);

ds3_status launch_retile_1x128_to_128x1(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s,
                                        int64_t ssr, int64_t ssk, uint8_t* qt, int64_t ldqt, float* s_t, int64_t ssc,
                                        int64_t sst, int pow2, hipStream_t st);
ds3_status launch_quant_act_1x128_e5m6(const void* x, int64_t rows, int64_t cols, int64_t ldx, uint8_t* q, int64_t ldq,
                                       float* s, int64_t ssr, int64_t ssk, hipStream_t st);
ds3_status launch_dequant_e5m6(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq, const float* s, int64_t ssr,
                               int64_t ssk, void* y, int64_t ldy, hipStream_t st);
ds3_status launch_adamw_bf16_states(int64_t n, float* w, const float* g, void* m, void* v, void* wb, float lr, float beta1,
                                    float beta2, float eps, float wd, float rbc1, float rbc2, hipStream_t st);
ds3_status launch_rmsnorm_quant_1x128(const void* x, int64_t rows, int64_t cols, int64_t ldx, const float* gamma, float eps,
                                      void* y, int64_t ldy, uint8_t* q, int64_t ldq, float* s, int64_t ssr, int64_t ssk,
                                      int pow2, hipStream_t st);
ds3_status launch_swiglu_quant_1x128(const void* h, int64_t rows, int64_t inter, int64_t ldh, uint8_t* q, int64_t ldq,
                                     float* s, int64_t ssr, int64_t ssk, int pow2, hipStream_t st);
ds3_status launch_probe_mfma(int iters, float* out, int blocks, hipStream_t st);
ds3_status launch_probe_feed(const void* src, unsigned window, int row_stride, int iters, unsigned* out, int blocks,
                             hipStream_t st);

// One description for the dense and the grouped GEMM.  Dense: G == 0.
struct GemmParams {
    const uint8_t* a;      // [M][lda] activation-side codes
    const uint8_t* b;      // [N][ldb] weight-side codes (grouped: [G][N][ldb])
    const float* sa;
    const float* sb;
    void* c;
    int64_t lda, ldb, ldc;
    int64_t sar, sak;      // sa strides: row, K-block
    int64_t sbr, sbk;      // sb strides: row (block row or row), K-block
    int64_t b_group_stride;   // bytes between experts in b
    int64_t sb_group_stride;  // floats between experts in sb
    const int32_t* group_offsets;
    int M, N, K;           // grouped: M = total rows
    int G;
    int tiles_m, tiles_n;  // grouped: tiles_m is the upper bound ceil(M/BM) + G
    int accumulate;
    int* ws_cnt;           // arrival counters of the tiles shared along K (nullptr: no sharing)
    float* ws_part;        // partial tiles [XCD][share_tail_max][2]
    int share_tail_max;    // most shared tiles any XCD has
    int share_steps, share_steps_last;   // K-steps per workgroup in a shared tail (XCDs with a full chunk / the last one)
    int share_skew;        // K-steps moved from the odd workgroups' runs to the even ones'
    // SwiGLU + 1x128 quantisation in the epilogue (grouped gate|up projection only; c is unused then)
    uint8_t* q_out;        // [M][ldq] codes of the activation
    float* s_out;          // scales, element (row, 1x128 tile t) at s_out[row * sor + t * sok]
    int64_t ldq, sor, sok;
    int q_pow2;            // scales of the activation rounded up to powers of two
};

// variant: which tile configuration to run (see ds3_gemm.hip); -1 = choose by shape.
// pow2: every scale is a power of two (the matrix instruction applies them).
// ws / ws_bytes: device workspace for sharing tail tiles along K (nullptr: never share).
ds3_status launch_gemm(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, bool pow2, void* ws, size_t ws_bytes,
                       hipStream_t st);
// As launch_gemm with the library's own statically allocated workspace (one per device).
ds3_status launch_gemm_static_scratch(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, bool pow2, hipStream_t st);
size_t gemm_static_scratch_bytes();
// Grouped GEMM over a gate|up weight interleaved in blocks of 128 rows, with SwiGLU and the 1x128
// quantiser of the following Linear's input applied to each tile before it leaves the chip.
ds3_status launch_gemm_swiglu_quant(const GemmParams& p, bool pow2, void* ws, size_t ws_bytes, hipStream_t st);
// Bytes of workspace with which the grouped GEMMs hand their tiles out through a queue (its counters).
size_t grouped_workspace_bytes();
// Bytes of workspace with which launch_gemm shares tail tiles for this shape (0: it would not).
size_t gemm_workspace_bytes(const GemmParams& p, ds3_bscale mode, int variant);
// K-steps per workgroup for a shared tail (see ds3_gemm.hip); host logic, exported for its test.
int tail_share_steps(int tail, int kb, int nslots);
// Sets the arrival counters at the head of a GEMM workspace to zero.
ds3_status launch_workspace_init(void* ws, size_t ws_bytes, hipStream_t st);
// C[M][N] = 0 (the product over an empty inner dimension).
ds3_status launch_zero_fill(void* c, ds3_dtype ct, int64_t M, int64_t N, int64_t ldc, hipStream_t st);

}  // namespace ds3
