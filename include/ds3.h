/*
 * ds3.h -- C ABI of the fine-grained FP8 linear layer for AMD MI355X (gfx950).
 *
 * The operations are those of Section 3.3 of the DeepSeek-V3 technical report
 * (arXiv 2412.19437):
 *   - Section 3.3.2 "Fine-Grained Quantization" / "Online Quantization":
 *     activations are grouped 1x128 (per token, per 128 channels), weights
 *     128x128; the max-abs of each group is mapped to the largest E4M3 value.
 *   - Section 3.3.3 "Low-Precision Activation" (1): in the backward pass the
 *     group of 128 runs along tokens (128x1 tiles).
 *   - Section 3.3.2 "Increasing Accumulation Precision": the GEMM multiplies
 *     the per-group scales in along the inner dimension at every N_C = 128
 *     interval and accumulates in FP32.
 *   - Section 3.3.1: Fprop, Dgrad and Wgrad take FP8 inputs and produce BF16
 *     or FP32 outputs.
 * The five core calls (ds3_quant_act_1x128, ds3_quant_act_128x1,
 * ds3_quant_w_128x128, ds3_gemm_fp8_bs, ds3_grouped_gemm_fp8_bs) come first;
 * after them the pieces of Section 3.3.3 / 3.5.2 around the layer: SwiGLU,
 * power-of-two scaling factors with the scales applied by the matrix
 * instruction, the weight quantizer that also writes the transposed codes,
 * re-tiling of the FP8 activation cache, SwiGLU and RMSNorm fused with their
 * quantizer, the E5M6 cache format, the AdamW step with BF16 moments, and two
 * machine probes for the benchmark.
 *
 * Common rules
 *   - Every data pointer is DEVICE memory owned by the caller.  The library
 *     allocates nothing, keeps no state between calls and retains no pointer.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls enqueue work and return; they never synchronise and never read
 *     device data on the host.
 *   - Argument errors are found on the host before anything is launched and
 *     reported as a status code; no kernel runs in that case.  Problems of
 *     size zero (no rows, no columns, an empty expert) are DS3_OK no-ops.
 *   - Leading dimensions (ld*) are in ELEMENTS of the array they belong to.
 *   - FP8 codes are OCP E4M3 bytes (bias 7, max 448, no infinities).
 *   - Quantisation of one group G (arithmetic in FP32, bit-exact contract):
 *         amax = max |x_i| over G
 *         s    = amax / 448          (stored de-quantisation scale; 1 if amax == 0)
 *         r    = 448 / amax          (0 if amax == 0)
 *         q_i  = E4M3_round_to_nearest_even(x_i * r)   (sign always copied)
 *     Both divisions are correctly rounded.  Inputs must be finite and nonzero
 *     magnitudes must lie in [2^-100, 2^100]; otherwise codes and scales are
 *     unspecified (but nothing faults).  A ragged trailing group is simply
 *     smaller.
 */
#ifndef DS3_H
#define DS3_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DS3_OK = 0,
    DS3_ERR_NULL = 1,        /* a required pointer is NULL                       */
    DS3_ERR_SHAPE = 2,       /* negative size, ld smaller than the row, K % 128  */
    DS3_ERR_ALIGN = 3,       /* pointer / ld / column count not vector aligned   */
    DS3_ERR_DTYPE = 4,       /* unknown dtype, or accumulate into a BF16 output  */
    DS3_ERR_UNSUPPORTED = 5, /* a size beyond what the kernels index (2^31 bytes per operand row span etc.) */
    DS3_ERR_LAUNCH = 6,      /* the HIP runtime refused the launch               */
    DS3_ERR_WORKSPACE = 7    /* a workspace was passed that is smaller than ds3_gemm_workspace_bytes asks for */
} ds3_status;

typedef enum { DS3_F32 = 0, DS3_BF16 = 1 } ds3_dtype;

/* How the scales of the second GEMM operand are indexed. */
typedef enum {
    DS3_BSCALE_128x128 = 0, /* sb[(n / 128) * sb_stride_row + kb * sb_stride_kb]: weight blocks (Fprop, Dgrad) */
    DS3_BSCALE_PER_ROW = 1  /* sb[ n        * sb_stride_row + kb * sb_stride_kb]: 128x1 tiles (Wgrad)          */
} ds3_bscale;

/*
 * 1x128 activation quantizer (Section 3.3.2, Fine-Grained Quantization (1)).
 *   x  [rows][ldx]  FP32 or BF16 (xt), `cols` valid columns per row.
 *   q  [rows][ldq]  E4M3 codes, same logical shape as x.
 *   s  scale of tile (row, kb) is s[row * s_stride_row + kb * s_stride_kb],
 *      kb = column / 128, kb < ceil(cols / 128).  Any two strides that do not
 *      make tiles overlap are accepted; (1, rows) gives the K-block-major
 *      layout the GEMM reads fastest.
 * Alignment: x, q 16-byte aligned; ldx * sizeof(element), ldq and
 * cols * sizeof(element) multiples of 16 bytes (cols % 8 == 0 for BF16,
 * cols % 4 == 0 for FP32).
 */
ds3_status ds3_quant_act_1x128(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx,
                               uint8_t* q, int64_t ldq,
                               float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);

/*
 * 128x1 activation quantizer (Section 3.3.3, Low-Precision Activation (1)):
 * the group of 128 runs along rows (tokens), one column (channel) wide.  The
 * results are written TRANSPOSED so that the token axis, which the
 * weight-gradient GEMM contracts over, is contiguous.
 *   x    [rows][ldx]  FP32 or BF16, rows = tokens, cols = channels.
 *   q_t  [cols][ldq]  code of (token t, channel c) at q_t[c * ldq + t].
 *   s_t  scale of (channel c, token block tb) at s_t[c * s_stride_col + tb * s_stride_tb],
 *        tb < ceil(rows / 128).
 * Alignment: x 16-byte aligned, ldx and cols as for the 1x128 call; q_t
 * 16-byte aligned and ldq % 16 == 0.  `rows` is arbitrary.
 */
ds3_status ds3_quant_act_128x1(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx,
                               uint8_t* q_t, int64_t ldq,
                               float* s_t, int64_t s_stride_col, int64_t s_stride_tb, void* stream);

/*
 * 128x128 weight quantizer (Section 3.3.2, Fine-Grained Quantization (2)).
 *   w  [n][ldw]  FP32 or BF16, `k` valid columns.
 *   q  [n][ldq]  codes.
 *   s  [ceil(n/128)][ceil(k/128)] row-major, one scale per block.
 * Alignment as for the 1x128 call.  n and k may be ragged (partial blocks).
 */
ds3_status ds3_quant_w_128x128(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw,
                               uint8_t* q, int64_t ldq, float* s, void* stream);

/*
 * Block-scaled FP8 GEMM (Section 3.3.2, Increasing Accumulation Precision;
 * Section 3.3.1 for the three uses Fprop / Dgrad / Wgrad):
 *
 *   C[m][n] (+)= sum over kb of  sa(m,kb) * sb(n,kb) * sum_{k in block kb} dec(a[m][k]) * dec(b[n][k])
 *
 * with FP32 accumulation and the scale product applied to each 128-long
 * partial sum.  Both operands are K-contiguous.
 *   a  [M][lda] codes, sa(m,kb) = sa[m * sa_stride_row + kb * sa_stride_kb]
 *   b  [N][ldb] codes, sb(n,kb) per `sb_mode` (see ds3_bscale)
 *   c  [M][ldc] BF16 (round to nearest even) or FP32 (ct).
 *   accumulate != 0: C += result; FP32 output only (gradient accumulation,
 *   Section 3.3.3 keeps gradients in FP32).
 * Requirements: K % 128 == 0; a, b 16-byte aligned and lda, ldb % 16 == 0;
 * c 16-byte aligned and ldc % 4 == 0.  M and N are arbitrary.
 * K == 0 is an empty sum: C is left as it is with `accumulate`, set to zero
 * without.
 * `workspace` (device memory, 16-byte aligned, owned by the caller, prepared
 * once with ds3_gemm_workspace_init, must not be shared by calls that may run
 * at the same time; every call leaves it ready for the next, whatever the shape): when
 * the output tiles do not divide evenly among the compute units, the tiles of
 * the last, partial round are shared along K -- every workgroup takes an
 * equal run of their K-steps, partial sums meet in the workspace and are added
 * in K order by whichever workgroup completes a tile (Section 3.3.2 leaves the
 * order of the FP32 additions open).  Pass ds3_gemm_workspace_bytes() bytes to
 * allow it, or NULL (with any size) to forbid it; a non-NULL workspace that is
 * too small is DS3_ERR_WORKSPACE.  Results are deterministic for a given shape
 * and workspace choice, but not bit-comparable across shapes or between a
 * call with and a call without workspace.
 */
ds3_status ds3_gemm_fp8_bs(int64_t M, int64_t N, int64_t K,
                           const uint8_t* a, int64_t lda,
                           const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                           const uint8_t* b, int64_t ldb,
                           const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode,
                           void* c, ds3_dtype ct, int64_t ldc, int accumulate,
                           void* workspace, size_t workspace_bytes, void* stream);

/*
 * ds3_gemm_fp8_bs for callers that cannot allocate device memory -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc -- and so cannot bring
 * a workspace: the same operation, arguments and results as ds3_gemm_fp8_bs with a
 * workspace of ds3_gemm_workspace_bytes() bytes, but the partial sums of shared tiles go
 * through a statically allocated device array of the library
 * (ds3_gemm_noalloc_scratch_bytes() = 76 MiB + 2.25 KiB, held by every GPU the library is
 * loaded on until the process ends).  The call allocates and frees nothing.  A shape that
 * would need more than the array holds is refused with DS3_ERR_WORKSPACE (no shape does on
 * a device of up to 256 compute units).  All calls on one GPU share the array: calls that
 * may run at the same time on one GPU race; calls on one stream, or ordered by events, are fine.
 */
ds3_status ds3_gemm_fp8_bs_noalloc(int64_t M, int64_t N, int64_t K,
                                   const uint8_t* a, int64_t lda,
                                   const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                   const uint8_t* b, int64_t ldb,
                                   const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode,
                                   void* c, ds3_dtype ct, int64_t ldc, int accumulate, void* stream);
size_t ds3_gemm_noalloc_scratch_bytes(void);

/*
 * Grouped block-scaled GEMM over MoE experts (Section 2.1.2: each routed
 * expert multiplies only the tokens routed to it; no token is dropped, so
 * groups are ragged and may be empty).  For expert g, rows
 * [group_offsets[g], group_offsets[g+1]) of `a` are multiplied by that
 * expert's weight b[g] with its 128x128 block scales:
 *   a   [total_rows][lda] codes, sa as in ds3_gemm_fp8_bs
 *   b   [G][N][ldb] codes (expert stride N * ldb)
 *   sb  [G][ceil(N/128)][K/128] row-major
 *   c   [total_rows][ldc] BF16 or FP32
 *   group_offsets  DEVICE array of G+1 int32, nondecreasing, [0] == 0 and
 *                  [G] <= total_rows; it is read on the device only.
 * Rows at or beyond group_offsets[G] are left untouched.  G <= 1023.
 */
ds3_status ds3_grouped_gemm_fp8_bs(int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                   int64_t N, int64_t K,
                                   const uint8_t* a, int64_t lda,
                                   const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                   const uint8_t* b, int64_t ldb, const float* sb,
                                   void* c, ds3_dtype ct, int64_t ldc,
                                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * Tuning hooks: the same two operations with the tile configuration chosen by
 * the caller instead of by shape.  `variant` in [0, ds3_gemm_num_variants());
 * -1 selects by shape exactly as the plain calls do.  Results of different
 * variants agree to FP32 summation-order differences only.
 */
int ds3_gemm_num_variants(void);
ds3_status ds3_gemm_fp8_bs_v(int variant, int64_t M, int64_t N, int64_t K,
                             const uint8_t* a, int64_t lda,
                             const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                             const uint8_t* b, int64_t ldb,
                             const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode,
                             void* c, ds3_dtype ct, int64_t ldc, int accumulate,
                             void* workspace, size_t workspace_bytes, void* stream);
ds3_status ds3_grouped_gemm_fp8_bs_v(int variant, int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                     int64_t N, int64_t K,
                                     const uint8_t* a, int64_t lda,
                                     const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                     const uint8_t* b, int64_t ldb, const float* sb,
                                     void* c, ds3_dtype ct, int64_t ldc,
                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * Power-of-two scaling factors (Section 3.3.3: the inputs of the Linear after
 * attention and the activations quantized before MoE dispatch use factors of
 * the form 2^e, e an integer).  The three quantizers with
 *         s = the smallest power of two >= amax / 448     (1 if amax == 0)
 *         r = 1 / s (exact),   q_i = E4M3_round_to_nearest_even(x_i * r)
 * in place of the rule at the top of this file; arguments, layouts and
 * alignment are those of the calls without the suffix.  Such a scale is an
 * E8M0 number, so a tile can be re-tiled or re-scaled by another power of two
 * without a second rounding of its significands.
 */
ds3_status ds3_quant_act_1x128_pow2(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx,
                                    uint8_t* q, int64_t ldq,
                                    float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);
ds3_status ds3_quant_act_128x1_pow2(const void* x, ds3_dtype xt, int64_t rows, int64_t cols, int64_t ldx,
                                    uint8_t* q_t, int64_t ldq,
                                    float* s_t, int64_t s_stride_col, int64_t s_stride_tb, void* stream);
ds3_status ds3_quant_w_128x128_pow2(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw,
                                    uint8_t* q, int64_t ldq, float* s, void* stream);

/*
 * The two GEMMs for operands whose scales are ALL powers of two in
 * [2^-126, 2^127] (both sa and sb; the outputs of the *_pow2 quantizers are).
 * Same result as ds3_gemm_fp8_bs / ds3_grouped_gemm_fp8_bs on the same
 * arguments, computed with the scales applied inside the matrix instruction
 * (gfx950 block-scaled MFMA, E8M0 scale per 32 elements along K) and the
 * partial sums chained in its FP32 accumulator, which removes the per-interval
 * rescale from the vector ALU.  Only the exponent field of each scale is read:
 * scales that are not powers of two give unspecified (finite-cost, fault-free)
 * results.  `variant` as in the tuning hooks above, -1 = choose by shape.
 */
ds3_status ds3_gemm_fp8_bs_pow2(int variant, int64_t M, int64_t N, int64_t K,
                                const uint8_t* a, int64_t lda,
                                const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                const uint8_t* b, int64_t ldb,
                                const float* sb, int64_t sb_stride_row, int64_t sb_stride_kb, ds3_bscale sb_mode,
                                void* c, ds3_dtype ct, int64_t ldc, int accumulate,
                                void* workspace, size_t workspace_bytes, void* stream);
ds3_status ds3_grouped_gemm_fp8_bs_pow2(int variant, int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                        int64_t N, int64_t K,
                                        const uint8_t* a, int64_t lda,
                                        const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                        const uint8_t* b, int64_t ldb, const float* sb,
                                        void* c, ds3_dtype ct, int64_t ldc,
                                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bytes of device workspace with which ds3_gemm_fp8_bs / _pow2 share tail tiles
 * along K for this shape (the larger of the two scale modes' needs; 0: the call
 * would not use a workspace).  The _v form answers for one tile configuration
 * and scale mode (variant -1: the default choice).
 * The grouped calls use a workspace of ds3_grouped_gemm_workspace_bytes() bytes
 * (a few counters, any shape): with it the tiles beyond each workgroup's first
 * are handed out through a queue, so workgroups that drew tiles with few valid
 * rows take more of them (the results do not depend on it, bit for bit); with
 * NULL the walk is static.  One workspace serves dense and grouped calls alike,
 * under the same rules (prepared once, not shared by overlapping calls).
 */
size_t ds3_gemm_workspace_bytes(int64_t M, int64_t N, int64_t K);
size_t ds3_gemm_workspace_bytes_v(int variant, int64_t M, int64_t N, int64_t K, ds3_bscale sb_mode);
size_t ds3_grouped_gemm_workspace_bytes(void);

/*
 * Prepares a freshly allocated workspace (enqueues a small kernel that zeroes
 * the arrival counters at its head; the rest needs no initialisation).  Once
 * per allocation: the GEMM calls leave the counters as they need them.
 * workspace_bytes == 0 is a no-op; a non-zero size below that of the counters
 * (ds3_grouped_gemm_workspace_bytes()) is DS3_ERR_WORKSPACE.
 */
ds3_status ds3_gemm_workspace_init(void* workspace, size_t workspace_bytes, void* stream);

/*
 * Host logic of the K-sharing, exported for its test (no GPU work): `tail_tiles`
 * tiles of `k_steps` K-steps each, laid end to end, are cut into one contiguous
 * run per workgroup, workgroup s taking steps [s*q, (s+1)*q).  Returns the
 * smallest q >= ceil(tail_tiles * k_steps / workgroups) with which no tile is
 * cut into more than two pieces, or 0 if only q = k_steps (no sharing) would do.
 */
int ds3_gemm_tail_share_steps(int tail_tiles, int k_steps, int workgroups);

/*
 * SwiGLU between the two expert GEMMs (Section 3.3.3, Low-Precision
 * Activation (2) names the operator): h is the BF16 output of the fused
 * gate|up projection, [rows][ldh] with 2*inter valid columns, gate in
 * columns [0, inter), up in [inter, 2*inter);
 *   out[r][j] = bf16( silu(h[r][j]) * h[r][inter + j] ),  silu(g) = g / (1 + exp(-g)),
 * computed in FP32.  inter % 8 == 0, pointers 16-byte aligned, ldh, ldo % 8 == 0.
 */
ds3_status ds3_swiglu(const void* h, int64_t rows, int64_t inter, int64_t ldh,
                      void* out, int64_t ldo, void* stream);

/*
 * 128x128 weight quantizer that also writes the transposed codes, the weight
 * operand of Dgrad (Section 3.3.1: dX = dY W contracts over W's rows; the
 * 128x128 blocks and their scales are transpose-invariant, so W^T needs no
 * second quantization -- Appendix B.2 makes the same point for block-wise
 * tiles).  One read of W, two layouts:
 *   q    [n][ldq]   and  s    [ceil(n/128)][ceil(k/128)]   as ds3_quant_w_128x128
 *   q_t  [k][ldqt]  and  s_t  [ceil(k/128)][ceil(n/128)]:  q_t[c][r] = q[r][c], s_t[j][i] = s[i][j]
 * Alignment as ds3_quant_w_128x128, plus q_t 16-byte aligned and ldqt % 16 == 0.
 */
ds3_status ds3_quant_w_128x128_dual(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw,
                                    uint8_t* q, int64_t ldq, float* s,
                                    uint8_t* q_t, int64_t ldqt, float* s_t, void* stream);
ds3_status ds3_quant_w_128x128_dual_pow2(const void* w, ds3_dtype wt, int64_t n, int64_t k, int64_t ldw,
                                         uint8_t* q, int64_t ldq, float* s,
                                         uint8_t* q_t, int64_t ldqt, float* s_t, void* stream);

/*
 * Re-tiling of a cached FP8 activation for the weight-gradient GEMM (Section
 * 3.5.2, Support for Transposed GEMM Operations: the activation kept from the
 * forward pass in 1x128 tiles is read back, dequantized, transposed and
 * re-quantized into 128x1 tiles; Section 3.3.3 (1)).  Per element
 *     v = fl32(dec(q[t][c]) * s(t, c / 128))
 * and then exactly ds3_quant_act_128x1 (or its _pow2 form) applied to v:
 *   q    [rows][ldq]  codes of the 1x128-quantized matrix, rows = tokens
 *   s    scale of (token t, block kb) at s[t * s_stride_row + kb * s_stride_kb]
 *   q_t  [cols][ldqt] code of (token t, channel c) at q_t[c * ldqt + t]
 *   s_t  scale of (channel c, token block tb) at s_t[c * st_stride_col + tb * st_stride_tb]
 * One byte read and one written per element (the BF16 source costs two to read).
 * With power-of-two scales on both sides the significands are not rounded a
 * second time unless a value falls below the new tile's normal range.
 * cols % 16 == 0, ldq % 16 == 0, ldqt % 16 == 0, q and q_t 16-byte aligned.
 */
ds3_status ds3_retile_1x128_to_128x1(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq,
                                     const float* s, int64_t s_stride_row, int64_t s_stride_kb,
                                     uint8_t* q_t, int64_t ldqt,
                                     float* s_t, int64_t st_stride_col, int64_t st_stride_tb, void* stream);
ds3_status ds3_retile_1x128_to_128x1_pow2(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq,
                                          const float* s, int64_t s_stride_row, int64_t s_stride_kb,
                                          uint8_t* q_t, int64_t ldqt,
                                          float* s_t, int64_t st_stride_col, int64_t st_stride_tb, void* stream);

/*
 * SwiGLU fused with the 1x128 quantization of its output (Section 3.3.3,
 * Low-Precision Activation: the down projection takes the SwiGLU output
 * quantized to FP8; Section 3.5.2 asks for the cast to be fused with the
 * producer so that the activation is not written to and re-read from HBM).
 * Same result, bit for bit, as ds3_swiglu followed by ds3_quant_act_1x128
 * (or its _pow2 form) on the BF16 activation: the activation is rounded to
 * BF16 in registers before its max-abs is taken.
 *   h  as in ds3_swiglu;  q [rows][ldq] codes with `inter` valid columns;
 *   s  as in ds3_quant_act_1x128 with cols = inter.
 * inter % 8 == 0, h and q 16-byte aligned, ldh % 8 == 0, ldq % 16 == 0.
 */
ds3_status ds3_swiglu_quant_1x128(const void* h, int64_t rows, int64_t inter, int64_t ldh,
                                  uint8_t* q, int64_t ldq,
                                  float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);
ds3_status ds3_swiglu_quant_1x128_pow2(const void* h, int64_t rows, int64_t inter, int64_t ldh,
                                       uint8_t* q, int64_t ldq,
                                       float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);

/*
 * Grouped gate|up projection with SwiGLU and the 1x128 quantization of its
 * output done on each GEMM tile before it leaves the chip (Section 3.3.2,
 * Online Quantization, and Section 3.3.3, Low-Precision Activation: the input
 * of the down projection is the SwiGLU output in FP8; Section 3.5.2 asks for
 * the cast to be fused with its producer).  Neither the projection's output h
 * nor the BF16 activation reaches HBM.
 *   a, sa, group_offsets, total_rows, K   as in ds3_grouped_gemm_fp8_bs
 *   b   [G][2*inter][ldb] codes of the fused gate|up weight with its rows
 *       INTERLEAVED in blocks of 128: rows [256 t, 256 t + 128) are gate rows
 *       [128 t, 128 t + 128), rows [256 t + 128, 256 t + 256) the up rows of
 *       the same range, so that both halves of an output tile meet in one
 *       GEMM tile.  Whole 128x128 blocks move, so the codes and scales are
 *       those of the gate and up matrices quantized on their own.
 *   sb  [G][2*inter/128][K/128] in the same block-row order
 *   q   [total_rows][ldq] codes of silu(gate) * up, `inter` valid columns
 *   s   scales of q, element (row, tile t) at s[row * s_stride_row + t * s_stride_kb]
 * inter % 128 == 0, K > 0; q 16-byte aligned, ldq % 16 == 0, ldq >= inter.
 * Result: bit for bit that of ds3_grouped_gemm_fp8_bs (BF16 output) on the
 * same operands followed by ds3_swiglu_quant_1x128 on its de-interleaved
 * output.  The _pow2 form takes operands whose scales
 * are all powers of two and writes power-of-two scales.
 * Rows at or beyond group_offsets[G] are left untouched.  workspace as in
 * ds3_grouped_gemm_fp8_bs.
 */
ds3_status ds3_grouped_gemm_swiglu_quant_fp8_bs(int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                                int64_t inter, int64_t K,
                                                const uint8_t* a, int64_t lda,
                                                const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                                const uint8_t* b, int64_t ldb, const float* sb,
                                                uint8_t* q, int64_t ldq,
                                                float* s, int64_t s_stride_row, int64_t s_stride_kb,
                                                void* workspace, size_t workspace_bytes, void* stream);
ds3_status ds3_grouped_gemm_swiglu_quant_fp8_bs_pow2(int32_t G, const int32_t* group_offsets, int64_t total_rows,
                                                     int64_t inter, int64_t K,
                                                     const uint8_t* a, int64_t lda,
                                                     const float* sa, int64_t sa_stride_row, int64_t sa_stride_kb,
                                                     const uint8_t* b, int64_t ldb, const float* sb,
                                                     uint8_t* q, int64_t ldq,
                                                     float* s, int64_t s_stride_row, int64_t s_stride_kb,
                                                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * RMSNorm fused with the 1x128 quantization of its output, the input of the
 * Linear that follows the normalisation (Section 3.3: normalisation operators
 * keep their original precision; Section 3.5.2 asks for the FP8 cast to be fused
 * with its producer instead of a round trip through HBM).  Per row
 *     r = 1 / sqrt(mean_c(x[c]^2) + eps)          (FP32; x is BF16)
 *     a[c] = bf16(x[c] * r * gamma[c])            (round to nearest even)
 * and then exactly ds3_quant_act_1x128 (or its _pow2 form) applied to a.
 *   x      [rows][ldx] BF16, `cols` valid columns, cols <= 8192
 *   gamma  [cols] FP32, DEVICE
 *   y      [rows][ldy] BF16 or NULL: if given, a is also written there
 *   q, s   as in ds3_quant_act_1x128
 * cols % 8 == 0; x, y, q, gamma 16-byte aligned; ldx, ldy % 8 == 0; ldq % 16 == 0;
 * eps >= 0.  The order of the FP32 additions of the squares is unspecified.
 */
ds3_status ds3_rmsnorm_quant_1x128(const void* x, int64_t rows, int64_t cols, int64_t ldx,
                                   const float* gamma, float eps, void* y, int64_t ldy,
                                   uint8_t* q, int64_t ldq,
                                   float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);
ds3_status ds3_rmsnorm_quant_1x128_pow2(const void* x, int64_t rows, int64_t cols, int64_t ldx,
                                        const float* gamma, float eps, void* y, int64_t ldy,
                                        uint8_t* q, int64_t ldq,
                                        float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);

/*
 * E5M6 activation cache (Section 3.3.3, Low-Precision Activation (1): the inputs
 * of the Linear after the attention operator are cached in a customized 12-bit
 * E5M6 format with 1x128 tiles and power-of-two scaling factors).  The report
 * gives no bit layout; this library's encoding is: sign, 5 exponent bits with
 * bias 15, 6 mantissa bits -- the upper 12 bits of IEEE binary16 -- exponent
 * field 0 subnormal (mantissa * 2^-20), exponent field 31 never produced,
 * largest magnitude 65024; codes a (even column) and b (odd column) share three
 * bytes: a[7:0], a[11:8] | b[3:0] << 4, b[11:4].
 *   quantizer:   x [rows][ldx] BF16 -> q [rows][ldq] bytes (3 * cols / 2 valid per row),
 *                s as in ds3_quant_act_1x128 with  s = smallest power of two >= amax / 65024
 *                (1 for an all-zero tile), q_i = E5M6_round_to_nearest_even(x_i / s).
 *   dequantizer: y [rows][ldy] BF16 = decode(q) * s, exact (7 significant bits times a power of two).
 * cols % 8 == 0; x, y 16-byte aligned, ldx, ldy % 8 == 0; q 4-byte aligned, ldq % 4 == 0.
 */
ds3_status ds3_quant_act_1x128_e5m6(const void* x, int64_t rows, int64_t cols, int64_t ldx,
                                    uint8_t* q, int64_t ldq,
                                    float* s, int64_t s_stride_row, int64_t s_stride_kb, void* stream);
ds3_status ds3_dequant_e5m6(const uint8_t* q, int64_t rows, int64_t cols, int64_t ldq,
                            const float* s, int64_t s_stride_row, int64_t s_stride_kb,
                            void* y, int64_t ldy, void* stream);

/*
 * AdamW step with low-precision optimizer states (Section 3.3.3: the first and
 * second moments are kept in BF16, master weights and gradients in FP32;
 * Section 4.2 gives beta1 = 0.9, beta2 = 0.95, weight_decay = 0.1).  For every
 * parameter, in FP32:
 *     m   = beta1 * m + (1 - beta1) * g            v = beta2 * v + (1 - beta2) * g * g
 *     w   = w - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * w )
 * and m, v are rounded to BF16 (nearest even) when stored; the update uses the
 * unrounded values.  The two bias corrections are formed in double on the host.
 *   master_w [n] FP32 in/out, grad [n] FP32, m, v [n] BF16 in/out,
 *   w_bf16   [n] BF16 out or NULL: the BF16 copy of the new weights the next
 *            forward pass quantizes from.   step = t >= 1.
 * n % 8 == 0, all pointers DEVICE and 16-byte aligned.  22 bytes of HBM traffic
 * per parameter (24 with FP32 moments, which would also need 8 more bytes resident).
 */
ds3_status ds3_adamw_bf16_states(int64_t n, float* master_w, const float* grad, void* m, void* v, void* w_bf16,
                                 float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step,
                                 void* stream);

/*
 * Machine probes for the benchmark (they compute nothing of the method; they
 * exist so that a roofline fraction can be read against what this chip
 * sustains, not only against the published peak).
 *
 * ds3_probe_mfma_fp8: `workgroups` workgroups of 8 waves, each wave issuing
 * iters * 32 FP8 16x16x128 MFMAs (65536 flop each) on register operands.
 * out: DEVICE, workgroups * 8 floats (checksums, ignored).
 *
 * ds3_probe_lds_feed: every workgroup moves iters * 64 KiB from `src` (DEVICE,
 * window_bytes < 2^31, rows of 128 bytes taken at `row_stride` bytes, a
 * multiple of 128, window_bytes >= 4096 * row_stride) into LDS with the
 * GEMM's load pattern, one step's loads queued behind the step it waits for.
 * out: DEVICE, `workgroups` words.
 */
ds3_status ds3_probe_mfma_fp8(int iters, int workgroups, float* out, void* stream);
ds3_status ds3_probe_lds_feed(const void* src, size_t window_bytes, int64_t row_stride, int iters, int workgroups,
                              uint32_t* out, void* stream);

/* Static, never NULL. */
const char* ds3_status_string(ds3_status st);

#ifdef __cplusplus
}
#endif
#endif /* DS3_H */
