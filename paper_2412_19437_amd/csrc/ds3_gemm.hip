// Block-scaled FP8 GEMM for gfx950, dense and grouped over MoE experts --
// Section 3.3.2 "Increasing Accumulation Precision" of the DeepSeek-V3 report:
// per-group scales along K are multiplied into every 128-long partial sum and
// the sums are accumulated in FP32.
//
// Design (not the report's Hopper scheme): one v_mfma_f32_16x16x128_f8f6f4
// spans exactly one N_C = 128 interval, so each MFMA is issued with a zero
// accumulator and its four results per lane are folded into the FP32
// accumulators with one v_fma each.  The weight tile is the MFMA row operand
// and the activation tile the column operand: a lane then owns ONE activation
// row and four consecutive weight rows, so the scale product
// sa(m,kb) * sb(n/128,kb) is a single per-lane value per activation fragment.
//
// Data path: 128-byte K-rows of both operands go global -> LDS directly
// (buffer loads with the LDS bit, 16 bytes per lane, no staging registers),
// two LDS stages.  LDS rows are 128 bytes with the eight 16-byte chunks
// XOR-swizzled by (row & 7) ^ (row>>3 & 1) so that the 16 rows x 2 chunks of a
// fragment read fall into distinct banks.  Workgroup ids are remapped so that
// each XCD (one L2 each; workgroups are dealt round-robin to the 8 XCDs) walks
// a compact panel of output tiles.
//
// Pipeline of one K-step (per wave): all sub-tiles but those of the last
// activation fragment are computed from registers / the current stage; then
// ONE workgroup barrier (next stage complete, current stage free); then, in
// the shadow of the last fragment's MFMAs, the loads for K-step kb+2 are
// issued into the freed stage and the first fragments and scales of K-step
// kb+1 are read from LDS, so the matrix pipe never waits for LDS at the start
// of a K-step.
#include <type_traits>

#include "ds3_dev.h"
#include "ds3_internal.h"

namespace ds3 {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kMaxGroups = 1023;                       // experts per grouped call (prefix table in LDS)

template <int BN_, int BM_, int WN_, int WM_, int NS_>
struct Cfg {
    static constexpr int BN = BN_, BM = BM_, WN = WN_, WM = WM_;
    static constexpr int NS = NS_;                     // LDS stages: loads run NS-1 K-steps ahead of the MFMAs
    static constexpr int NT = 64 * WN * WM;
    static constexpr int TN = BN / WN, TM = BM / WM;   // wave tile
    static constexpr int FN = TN / 16, FM = TM / 16;   // 16-row fragments per wave
    static constexpr int NSUB = FN * FM;               // 16x16 sub-tiles (= MFMAs per K-step) per wave
    static constexpr int ROWS = BN + BM;
    static constexpr int STAGE = ROWS * 128;           // bytes of codes per K-step
    static constexpr int RPI = NT / 8;                 // tile rows one load instruction of the workgroup covers
    static constexpr int LPT = ROWS / RPI;             // 16-byte loads per thread per K-step
#ifndef DS3_TAIL_LOADS
#define DS3_TAIL_LOADS (LPT < FN ? LPT : FN)
#endif
    // loads of a K-step that are issued right behind the barrier that frees their stage (the
    // rest go out at the head of the next K-step)
    static constexpr int TAILN = (DS3_TAIL_LOADS) < LPT ? (DS3_TAIL_LOADS) : LPT;
    static constexpr int SCALE_BYTES = 2 * NS * NT * 4;        // [NS][NT] sa + [NS][NT] per-row sb
    static constexpr int LDS_BYTES = NS * STAGE + SCALE_BYTES + (kMaxGroups + 1) * 4;   // + row-tile prefix of the experts
    // workgroups that fit one compute unit: 160 KiB of LDS, and two waves per SIMD (the
    // kernels need more than 128 registers per lane)
    static constexpr int WG_PER_CU = (160 * 1024 / LDS_BYTES) < (512 / NT) ? (160 * 1024 / LDS_BYTES) : (512 / NT);
    static_assert(ROWS % RPI == 0 && BN % RPI == 0 && RPI % 16 == 0, "load mapping");
    static_assert(BM <= NT && BN <= NT, "scale staging uses one thread per row");
    static_assert(TN <= 128 && 128 % TN == 0, "one weight-scale block per wave");
    static_assert(FM % 2 == 0 && FM >= 2, "activation fragments are double-buffered");
    static_assert(LPT <= 2 * FN, "loads are interleaved with the last fragment's MFMAs");
    static_assert(NS == 2 || NS == 3, "stage ring");
    static_assert(LDS_BYTES <= 160 * 1024, "LDS");
};

// XOR key of a tile row: depends on the row's position inside its 16-row fragment only.
__device__ __forceinline__ int swz_key(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// Offset that is out of range for every descriptor this kernel builds (their
// sizes are below 2^31): a load with it moves no data.
constexpr unsigned kOobOffset = 0x80000000u;

// What a workgroup needs to know about one output tile (all wave-uniform
// except the two per-thread scale pointers).
struct TileCtx {
    int m0, n0, m_rows, n_rows;
    __amdgpu_buffer_rsrc_t rs_a, rs_b;
    const float* sb_blk;      // block mode: this wave's block row of scales; row mode: tile base
    const float* sa_thr;      // this thread's activation-scale row
    const float* sbrow_thr;   // this thread's weight-scale row (per-row mode)
};

//
// POW2 (power-of-two scales, Section 3.3.3): the scales are E8M0 numbers, whose
// code is the exponent field of the FP32 value, and the MFMA applies them itself
// (one scale per lane and operand: the weight row's and the activation row's);
// the accumulators then chain through the matrix pipe across K-steps and the
// vector ALU does no rescaling at all.
template <class C, bool ROWSB, bool OUT_BF16, bool GROUPED, bool POW2>
__global__ __launch_bounds__(C::NT) void gemm_fp8_bs_kernel(const GemmParams p) {
    constexpr int BN = C::BN, BM = C::BM, NT = C::NT, FN = C::FN, FM = C::FM, STAGE = C::STAGE, NSUB = C::NSUB;
    __shared__ __attribute__((aligned(1024))) uint8_t smem[C::LDS_BYTES];
    constexpr int NS = C::NS;
    float* const sa_s = reinterpret_cast<float*>(smem + NS * STAGE);           // [NS][NT], first BM used
    float* const sbrow_s = sa_s + NS * NT;                                     // [NS][NT], first BN used (per-row mode)

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wn = wave % C::WN, wm = wave / C::WN;
    const int l16 = lane & 15, g4 = lane >> 4;
    const int KB = p.K >> 7;

    // ---- persistent tile walk ------------------------------------------------------
    // Workgroup b runs on XCD b % 8.  The tile list is cut into 8 contiguous
    // chunks, one per XCD; the workgroups of an XCD take consecutive tiles of
    // their chunk, so the tiles in flight on one L2 form a compact panel.
    int tiles_m = p.tiles_m;
    int* const gpre = reinterpret_cast<int*>(smem + NS * STAGE + C::SCALE_BYTES);   // [G+1] row tiles before expert g
    if constexpr (GROUPED) {
        // the host only knows an upper bound on the row tiles; build their prefix over the experts
        if (tid == 0) {
            int cum = 0;
            for (int g = 0; g < p.G; ++g) {
                gpre[g] = cum;
                cum += (min(p.group_offsets[g + 1], p.M) - min(p.group_offsets[g], p.M) + BM - 1) / BM;
            }
            gpre[p.G] = cum;
        }
        __syncthreads();
        tiles_m = gpre[p.G];
    }
    const int ntiles = tiles_m * p.tiles_n;
    const int per_xcd = (ntiles + 7) >> 3;
    const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3), nslots = (int)(gridDim.x >> 3);
    // A last round that would occupy at most half of the XCD's workgroups is cut into
    // half tiles (the two M halves of a tile belong to different waves, and the waves
    // of the missing half skip their MFMAs), so that every workgroup gets one.
    const int tail = per_xcd % nslots;
    const bool split_tail = !GROUPED && C::WM == 2 && per_xcd > nslots && tail > 0 && 2 * tail <= nslots && p.M % BM == 0;
    const int n_full = split_tail ? per_xcd - tail : per_xcd;
    const int n_virtual = split_tail ? n_full + 2 * tail : per_xcd;

    auto setup_tile = [&](int local, TileCtx& c) -> bool {
        if (local >= n_virtual) return false;
        const int half = local < n_full ? -1 : ((local - n_full) & 1);
        const int t = xcd * per_xcd + (local < n_full ? local : n_full + ((local - n_full) >> 1));
        if (t >= ntiles) return false;
        int m0, m_end, n0, grp = 0;
        if constexpr (!GROUPED) {
            constexpr int PM = 4;                      // tiles of M per panel
            const int panel = PM * p.tiles_n;
            const int pi = t / panel, r = t - pi * panel;
            const int pm = min(PM, tiles_m - pi * PM);
            m0 = (pi * PM + r % pm) * BM;
            n0 = (r / pm) * BN;
            m_end = p.M;
            if (half >= 0) { m0 += half * (BM / 2); m_end = min(m_end, m0 + BM / 2); }
        } else {
            // Tiles are ordered expert by expert, then by column tile, the expert's row
            // tiles innermost: the workgroups of an XCD that run side by side share one
            // weight tile through the L2, and every expert's weights are streamed once.
            int lo = 0, hi = p.G;                      // largest g with gpre[g] * tiles_n <= t
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (gpre[mid] * p.tiles_n <= t) lo = mid; else hi = mid;
            }
            grp = lo;
            const int nt_g = gpre[grp + 1] - gpre[grp];
            const int r = t - gpre[grp] * p.tiles_n;
            n0 = (r / nt_g) * BN;
            const int row_lo = min(p.group_offsets[grp], p.M);
            m0 = row_lo + (r % nt_g) * BM;
            m_end = min(p.group_offsets[grp + 1], p.M);
        }
        c.m0 = m0; c.n0 = n0;
        c.m_rows = min(m_end - m0, BM);                // valid rows of this tile (>= 1)
        c.n_rows = min(p.N - n0, BN);
        const uint8_t* a_tile = p.a + (int64_t)m0 * p.lda;
        const uint8_t* b_tile = p.b + (int64_t)grp * p.b_group_stride + (int64_t)n0 * p.ldb;
        // Buffer descriptors bound to the valid bytes of the tile.  The whole byte
        // offset of a load goes into the per-lane offset operand, which the
        // hardware range-checks: rows past the end of the matrix (or of the
        // expert's group) read as zero and touch no memory.
        c.rs_a = __builtin_amdgcn_make_buffer_rsrc((void*)a_tile, 0, (int)((int64_t)(c.m_rows - 1) * p.lda + p.K), 0x00020000);
        c.rs_b = __builtin_amdgcn_make_buffer_rsrc((void*)b_tile, 0, (int)((int64_t)(c.n_rows - 1) * p.ldb + p.K), 0x00020000);
        if constexpr (ROWSB) {
            c.sb_blk = p.sb + (int64_t)n0 * p.sbr;
        } else {
            const int nblocks = (p.N + 127) >> 7;
            const int nb = min((n0 + wn * C::TN) >> 7, nblocks - 1);
            c.sb_blk = p.sb + (int64_t)grp * p.sb_group_stride + (int64_t)nb * p.sbr;
        }
        // Every thread stages one activation scale (and one per-row weight scale);
        // threads past the valid rows re-read the last valid row, whose partial
        // sums are zero because its codes were read as zero.
        c.sa_thr = p.sa + ((int64_t)m0 + min(tid, c.m_rows - 1)) * p.sar;
        c.sbrow_thr = ROWSB ? c.sb_blk + (int64_t)min(tid, c.n_rows - 1) * p.sbr : nullptr;
        return true;
    };

    // load mapping: this thread moves chunk position (tid & 7) of tile row i*RPI + (tid >> 3)
    const int lrow = tid >> 3;
    const int gchunk = (tid & 7) ^ swz_key(lrow);      // which 16 bytes of the K-row land there
    const unsigned voff_b = (unsigned)(lrow * (int)p.ldb + gchunk * 16);
    const unsigned voff_a = (unsigned)(lrow * (int)p.lda + gchunk * 16);
    const unsigned step_b = (unsigned)(C::RPI * (int)p.ldb), step_a = (unsigned)(C::RPI * (int)p.lda);

    // fragment read offsets inside a 16-row group: lane reads chunks 2*g4 and 2*g4+1 of row l16
    const int key = swz_key(l16);
    const int foff0 = l16 * 128 + (((2 * g4) ^ key) << 4);
    const int foff1 = l16 * 128 + (((2 * g4 + 1) ^ key) << 4);
    const int p_base = wn * C::TN * 128;               // weight fragments of this wave
    const int q_base = (BN + wm * C::TM) * 128;        // activation fragments of this wave

    float sa_reg = 0.f, sbrow_reg = 0.f;

    // i-th 16-byte load of this thread for the K-step at byte offset koff, into LDS stage `stage`
    auto issue_load = [&](const TileCtx& c, int i, int stage, unsigned koff) {
        const bool is_b = i * C::RPI < BN;
        const int ii = is_b ? i : i - BN / C::RPI;
        const unsigned voff = (is_b ? voff_b : voff_a) + (koff + (unsigned)ii * (is_b ? step_b : step_a));
        uint8_t* dst = smem + stage * STAGE + (i * NT + wave * 64) * 16;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(is_b ? c.rs_b : c.rs_a, (lds_ptr_t)dst, 16, (int)voff, 0, 0, 0);
    };
    // only the waves whose thread index is a tile row take part (wave-uniform conditions)
    auto load_scales = [&](const TileCtx& c, int kb) { // global -> registers
        if (tid < BM) sa_reg = c.sa_thr[(int64_t)kb * p.sak];
        if constexpr (ROWSB) { if (tid < BN) sbrow_reg = c.sbrow_thr[(int64_t)kb * p.sbk]; }
    };
    auto commit_scales = [&](int stage) {              // registers -> LDS
        if (tid < BM) sa_s[stage * NT + tid] = sa_reg;
        if constexpr (ROWSB) { if (tid < BN) sbrow_s[stage * NT + tid] = sbrow_reg; }
    };
    auto load_frag = [&](const uint8_t* base) -> i32x8 {
        const i32x4 lo = *reinterpret_cast<const i32x4*>(base + foff0);
        const i32x4 hi = *reinterpret_cast<const i32x4*>(base + foff1);
        return i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    auto read_tj = [&](int stage, float sbv, float* tj) {
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const float sav = sa_s[stage * NT + wm * C::TM + j * 16 + l16];
            tj[j] = (ROWSB || POW2) ? sav : sav * sbv;
        }
    };

    TileCtx cur;
    int local = slot;
    if (!setup_tile(local, cur)) return;
    // Workgroup barrier that lets the newest `pending` vector-memory operations of this
    // wave stay in flight (the loads that run more than one K-step ahead); LDS
    // operations are all complete when it returns.
    auto barrier_keep = [&](auto pending_tag) {
        constexpr int pending = decltype(pending_tag)::value;
        static_assert(pending >= 0 && pending < 16, "vmcnt immediate");
        asm volatile("" ::: "memory");                 // the compiler moves no memory access across
        __builtin_amdgcn_s_waitcnt(pending | 0x70);    // vmcnt(pending) lgkmcnt(0), expcnt untouched
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };
    // the first NS-1 K-steps of the first tile into stages 0 .. NS-2
    auto issue_first_steps = [&](const TileCtx& c) {
#pragma unroll
        for (int ks = 0; ks < NS - 1; ++ks)
#pragma unroll
            for (int i = 0; i < C::LPT; ++i) issue_load(c, i, ks, ks < KB ? (unsigned)ks << 7 : kOobOffset);
        load_scales(c, 0);
    };
    issue_first_steps(cur);

    for (;;) {
        // ---- entry: K-steps 0 .. NS-2 of `cur` are in flight into stages 0 .. NS-2, the scales of K-step 0 are in registers ----
        commit_scales(0);
        __syncthreads();
        // the part of K-step NS-1 that a previous K-step's barrier would have issued
#pragma unroll
        for (int i = 0; i < C::TAILN; ++i)
            issue_load(cur, i, NS - 1, NS - 1 < KB ? (unsigned)(NS - 1) << 7 : kOobOffset);
        float sb_n = ROWSB ? 1.f : cur.sb_blk[(int64_t)min(1, KB - 1) * p.sbk];   // block scale of the NEXT K-step
        float tj[FM];
        [[maybe_unused]] float sb_c = ROWSB ? 1.f : cur.sb_blk[0];                  // block scale of THIS K-step (POW2 only)
        read_tj(0, sb_c, tj);
        i32x8 pf[FN], qf[2];
#pragma unroll
        for (int i = 0; i < FN; ++i) pf[i] = load_frag(smem + p_base + i * 2048);
        qf[0] = load_frag(smem + q_base);
        f32x4 acc[FN][FM];
#pragma unroll
        for (int i = 0; i < FN; ++i)
#pragma unroll
            for (int j = 0; j < FM; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

        // One K-step from LDS stage S.  The instruction order is pinned by hand:
        // the MFMA of sub-tile s is issued, then the four FMAs that fold sub-tile
        // s-D into the accumulators, so the vector ALU works in the shadow of the
        // matrix pipe.  The empty asm statements only tie values to program points
        // (they emit nothing); without them the compiler gathers all MFMAs first
        // and all FMAs last.
        constexpr int D = 2;                               // MFMAs in flight ahead of their FMAs
        // The stage a barrier frees is refilled at once: the first TAILN loads of the
        // K-step NS steps ahead go out behind the barrier, one per sub-tile of the last
        // activation fragment, the rest at the head of the next K-step.
        constexpr int TAILN = C::TAILN;                    // loads issued right behind the barrier
        constexpr int HEADN = C::LPT - TAILN;              // loads issued at the head of the following K-step
        static_assert(HEADN <= NSUB - FN, "not enough sub-tiles before the barrier for the head loads");
        auto kstep = [&](int kb, auto stage_tag) {
            constexpr int S = decltype(stage_tag)::value;
            const uint8_t* st = smem + S * STAGE;
            constexpr int SN = (S + 1) % NS;                // stage of the next K-step
            constexpr int SL = (S + NS - 1) % NS;           // stage this K-step's loads fill (K-step kb+NS-1)
            const uint8_t* nst = smem + SN * STAGE;
            f32x4 un[FN];
            if constexpr (ROWSB) {
#pragma unroll
                for (int i = 0; i < FN; ++i)
                    un[i] = *reinterpret_cast<const f32x4*>(sbrow_s + S * NT + wn * C::TN + i * 16 + g4 * 4);
            }
            f32x4 part[D + 1];
#pragma unroll
            for (int d = 0; d <= D; ++d) part[d] = f32x4{0.f, 0.f, 0.f, 0.f};
            float tjn[FM];                                  // scale products of the next K-step
            const unsigned koff1 = kb + NS - 1 < KB ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;   // head loads
            const unsigned koff2 = kb + NS < KB ? (unsigned)(kb + NS) << 7 : kOobOffset;           // tail loads
            load_scales(cur, min(kb + 1, KB - 1));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < NSUB + D; ++s) {
                if (s == NSUB - FN) {
                    // Everything this wave reads from stage S is in registers.  After the
                    // barrier the next stage is complete and stage S may be overwritten.
                    commit_scales(SN);
                    barrier_keep(std::integral_constant<int, (NS == 2 ? 0 : C::LPT)>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (s < HEADN) issue_load(cur, TAILN + s, SL, koff1);
                if (s < NSUB) {
                    const int j = s / FN, i = s % FN;
                    if (i == 0 && j + 1 < FM) qf[(j + 1) & 1] = load_frag(st + q_base + (j + 1) * 2048);
                    part[s % (D + 1)] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(
                        pf[i], qf[j & 1], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
                    if (j == FM - 1) {
                        // last activation fragment: refill this weight fragment for the next K-step
                        pf[i] = load_frag(nst + p_base + i * 2048);
#pragma unroll
                        for (int l = i; l < TAILN; l += FN) issue_load(cur, l, S, koff2);
                        if (i == FN - 1) {
                            qf[0] = load_frag(nst + q_base);
                            read_tj(SN, sb_n, tjn);
                            if constexpr (!ROWSB) sb_n = cur.sb_blk[(int64_t)min(kb + 2, KB - 1) * p.sbk];
                        }
                    }
                }
                if (s >= D) {
                    const int ps = s - D, j = ps / FN, i = ps % FN;
                    // the MFMA just issued comes before the FMAs of sub-tile ps
                    if (s < NSUB) asm volatile("" : "+v"(part[s % (D + 1)]), "+v"(part[ps % (D + 1)]));
                    const f32x4 pr = part[ps % (D + 1)];
                    f32x4 a = acc[i][j];
                    if constexpr (ROWSB) {
                        a.x = __builtin_fmaf(pr.x, tj[j] * un[i].x, a.x);
                        a.y = __builtin_fmaf(pr.y, tj[j] * un[i].y, a.y);
                        a.z = __builtin_fmaf(pr.z, tj[j] * un[i].z, a.z);
                        a.w = __builtin_fmaf(pr.w, tj[j] * un[i].w, a.w);
                    } else {
                        a.x = __builtin_fmaf(pr.x, tj[j], a.x);
                        a.y = __builtin_fmaf(pr.y, tj[j], a.y);
                        a.z = __builtin_fmaf(pr.z, tj[j], a.z);
                        a.w = __builtin_fmaf(pr.w, tj[j], a.w);
                    }
                    asm volatile("" : "+v"(a));              // the four FMAs are done by here
                    acc[i][j] = a;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int j = 0; j < FM; ++j) tj[j] = tjn[j];
        };

        // Power-of-two scales: the MFMA scales both operands itself and accumulates in
        // place; the order of the memory operations is that of the general K-step.
        auto kstep_p2 = [&](int kb, auto stage_tag) {
            constexpr int S = decltype(stage_tag)::value;
            const uint8_t* st = smem + S * STAGE;
            constexpr int SN = (S + 1) % NS, SL = (S + NS - 1) % NS;
            const uint8_t* nst = smem + SN * STAGE;
            int ea[FN], eb[FM];                             // E8M0 codes = FP32 exponent fields
#pragma unroll
            for (int i = 0; i < FN; ++i)
                ea[i] = (int)(as_u32(ROWSB ? sbrow_s[S * NT + wn * C::TN + i * 16 + l16] : sb_c) >> 23);
#pragma unroll
            for (int j = 0; j < FM; ++j) eb[j] = (int)(as_u32(tj[j]) >> 23);
            float tjn[FM];
            float sb_cn = sb_c;
            const unsigned koff1 = kb + NS - 1 < KB ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;
            const unsigned koff2 = kb + NS < KB ? (unsigned)(kb + NS) << 7 : kOobOffset;
            load_scales(cur, min(kb + 1, KB - 1));
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < NSUB; ++s) {
                if (s == NSUB - FN) {
                    commit_scales(SN);
                    barrier_keep(std::integral_constant<int, (NS == 2 ? 0 : C::LPT)>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (s < HEADN) issue_load(cur, TAILN + s, SL, koff1);
                const int j = s / FN, i = s % FN;
                if (i == 0 && j + 1 < FM) qf[(j + 1) & 1] = load_frag(st + q_base + (j + 1) * 2048);
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(pf[i], qf[j & 1], acc[i][j], 0, 0, 0, ea[i],
                                                                             0, eb[j]);
                if (j == FM - 1) {
                    pf[i] = load_frag(nst + p_base + i * 2048);
#pragma unroll
                    for (int l = i; l < TAILN; l += FN) issue_load(cur, l, S, koff2);
                    if (i == FN - 1) {
                        qf[0] = load_frag(nst + q_base);
                        read_tj(SN, 1.f, tjn);
                        if constexpr (!ROWSB) {
                            sb_cn = sb_n;
                            sb_n = cur.sb_blk[(int64_t)min(kb + 2, KB - 1) * p.sbk];
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int j = 0; j < FM; ++j) tj[j] = tjn[j];
            sb_c = sb_cn;
        };

        // The same K-step for a wave whose activation rows all lie beyond the tile's valid
        // rows (ragged expert groups, half tiles): it moves its share of the data and
        // keeps the barriers, in the same order of memory operations, but computes nothing.
        auto kstep_idle = [&](int kb, auto stage_tag) {
            constexpr int S = decltype(stage_tag)::value;
            constexpr int SN = (S + 1) % NS, SL = (S + NS - 1) % NS;
            const unsigned koff1 = kb + NS - 1 < KB ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;
            const unsigned koff2 = kb + NS < KB ? (unsigned)(kb + NS) << 7 : kOobOffset;
            load_scales(cur, min(kb + 1, KB - 1));
#pragma unroll
            for (int i = 0; i < HEADN; ++i) issue_load(cur, TAILN + i, SL, koff1);
            commit_scales(SN);
            barrier_keep(std::integral_constant<int, (NS == 2 ? 0 : C::LPT)>{});
#pragma unroll
            for (int i = 0; i < TAILN; ++i) issue_load(cur, i, S, koff2);
        };

        using st0 = std::integral_constant<int, 0>;
        using st1 = std::integral_constant<int, 1>;
        using st2 = std::integral_constant<int, 2>;
        const bool active = wm * C::TM < cur.m_rows;    // wave-uniform
        auto kloop = [&](auto step) {
            int kb = 0;
            if constexpr (NS == 2) {
                for (; kb + 1 < KB; kb += 2) {
                    step(kb, st0{});
                    step(kb + 1, st1{});
                }
                if (kb < KB) step(kb, st0{});
            } else {
                for (; kb + 2 < KB; kb += 3) {
                    step(kb, st0{});
                    step(kb + 1, st1{});
                    step(kb + 2, st2{});
                }
                if (kb < KB) step(kb, st0{});
                if (kb + 1 < KB) step(kb + 1, st1{});
            }
        };
        if (!active) kloop(kstep_idle);
        else if constexpr (POW2) kloop(kstep_p2);
        else kloop(kstep);
        __syncthreads();                               // every wave is done with all code stages

        // ---- the next tile's first K-steps fly into stages 0 .. NS-2 during this tile's epilogue ----
        TileCtx nxt;
        local += nslots;
        const bool more = setup_tile(local, nxt);
        if (more) issue_first_steps(nxt);

        // ---- epilogue ------------------------------------------------------------------
        // A lane owns one activation row m and, per weight fragment, 4 consecutive n:
        // stored directly that would be 8-byte pieces scattered over 16 rows.  Each
        // wave instead transposes 16 rows x TN columns at a time through a private
        // LDS strip in the last stage and writes 16 bytes per lane, a full 128-byte (BF16)
        // or 256-byte (FP32) row segment per group of lanes.
        constexpr int ESZ = OUT_BF16 ? 2 : 4;
        constexpr int SEG = C::TN * ESZ;                   // bytes of one output row segment of this wave
        constexpr int ROWB = SEG + 16;                     // padded LDS row
        constexpr int CPR = SEG / 16;                      // 16-byte chunks per row segment
        constexpr int PASSES = 16 * CPR / 64;              // 64 lanes move 16 rows x CPR chunks
        static_assert(16 * CPR % 64 == 0, "epilogue mapping");
        static_assert((NT / 64) * 16 * ROWB <= STAGE, "epilogue strips fit in one code stage");
        // two strips per wave where they fit: the next row group is written while this one's reads return
        constexpr int NSTRIP = (NT / 64) * 16 * ROWB * 2 <= STAGE ? 2 : 1;
        uint8_t* strip0 = smem + (NS - 1) * STAGE + wave * (16 * ROWB * NSTRIP);
        uint8_t* c_base = reinterpret_cast<uint8_t*>(p.c);
        const int n_w0 = wn * C::TN;                       // first column of this wave inside the tile
        // Accumulating FP32 output: the old values of fragment row group j+1 are fetched
        // while group j is transposed and stored, so the read-modify-write does not
        // expose one memory latency per store.
        [[maybe_unused]] f32x4 oldv[2][PASSES];
        auto fetch_old = [&](int j, f32x4* dstv) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int idx = ps * 64 + lane;
                const int ml = wm * C::TM + j * 16 + idx / CPR;
                const int nl = n_w0 + (idx % CPR) * (16 / ESZ);
                dstv[ps] = f32x4{0.f, 0.f, 0.f, 0.f};
                if (ml < cur.m_rows && nl + 16 / ESZ <= cur.n_rows)
                    dstv[ps] = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(c_base + ((int64_t)(cur.m0 + ml) * p.ldc + cur.n0 + nl) * ESZ));
            }
        };
        const bool accum = !OUT_BF16 && p.accumulate;
        auto put_group = [&](int j) {                      // accumulators of row group j -> strip
            uint8_t* sp = strip0 + (NSTRIP == 2 ? (j & 1) * (16 * ROWB) : 0);
#pragma unroll
            for (int i = 0; i < FN; ++i) {
                const f32x4 v = acc[i][j];
                uint8_t* dst = sp + l16 * ROWB + (i * 16 + g4 * 4) * ESZ;
                if constexpr (OUT_BF16) *reinterpret_cast<u32x2*>(dst) = u32x2{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
                else *reinterpret_cast<f32x4*>(dst) = v;
            }
        };
        auto get_group = [&](int j, u32x4* wv) {           // strip -> 16-byte row chunks
            const uint8_t* sp = strip0 + (NSTRIP == 2 ? (j & 1) * (16 * ROWB) : 0);
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int idx = ps * 64 + lane;
                wv[ps] = *reinterpret_cast<const u32x4*>(sp + (idx / CPR) * ROWB + (idx % CPR) * 16);
            }
        };
        auto store_group = [&](int j, const u32x4* wv) {
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
                const int idx = ps * 64 + lane;
                const int r = idx / CPR, ch = idx % CPR;
                const int ml = wm * C::TM + j * 16 + r;
                const int nl = n_w0 + ch * (16 / ESZ);     // first column of this chunk inside the tile
                const u32x4 w = wv[ps];
                if (ml >= cur.m_rows || nl >= cur.n_rows) continue;
                uint8_t* gp = c_base + ((int64_t)(cur.m0 + ml) * p.ldc + cur.n0 + nl) * ESZ;
                if (nl + 16 / ESZ <= cur.n_rows) {
                    if constexpr (OUT_BF16) {
                        __builtin_nontemporal_store(w, reinterpret_cast<u32x4*>(gp));
                    } else {
                        f32x4 o = f32x4{as_f32(w.x), as_f32(w.y), as_f32(w.z), as_f32(w.w)};
                        if (accum) {
                            const f32x4 old = oldv[j & 1][ps];
                            o.x += old.x; o.y += old.y; o.z += old.z; o.w += old.w;
                        }
                        __builtin_nontemporal_store(o, reinterpret_cast<f32x4*>(gp));
                    }
                } else {
                    const unsigned int wd[4] = {w.x, w.y, w.z, w.w};
                    for (int q = 0; q < 16 / ESZ && nl + q < cur.n_rows; ++q) {
                        if constexpr (OUT_BF16) {
                            reinterpret_cast<uint16_t*>(gp)[q] = (uint16_t)(wd[q >> 1] >> (16 * (q & 1)));
                        } else {
                            float* d = reinterpret_cast<float*>(gp) + q;
                            *d = p.accumulate ? *d + as_f32(wd[q]) : as_f32(wd[q]);
                        }
                    }
                }
            }
        };
        if (active) {
            if constexpr (!OUT_BF16) { if (accum) fetch_old(0, oldv[0]); }
            put_group(0);
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                if constexpr (!OUT_BF16) { if (accum && j + 1 < FM) fetch_old(j + 1, oldv[(j + 1) & 1]); }
                __builtin_amdgcn_wave_barrier();           // same-wave LDS accesses complete in order
                u32x4 wv[PASSES];
                get_group(j, wv);
                if constexpr (NSTRIP == 2) { if (j + 1 < FM) put_group(j + 1); }
                store_group(j, wv);
                if constexpr (NSTRIP == 1) {
                    __builtin_amdgcn_wave_barrier();       // reads of the strip precede the next round of writes
                    if (j + 1 < FM) put_group(j + 1);
                }
            }
        }
        if (!more) break;
        cur = nxt;
    }
}

// ---- host side -------------------------------------------------------------------
// Compute units of the current device, rounded down to a multiple of 8 (cached per device).
static int num_cus_x8() {
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 8) n = 256;
        cached[dev] = n / 8 * 8;
    }
    return cached[dev];
}

template <class C, bool ROWSB, bool OUT_BF16, bool GROUPED, bool POW2>
static ds3_status launch_one(GemmParams p, hipStream_t st) {
    if (GROUPED) p.tiles_m = (p.M + C::BM - 1) / C::BM + p.G;
    else p.tiles_m = (p.M + C::BM - 1) / C::BM;
    p.tiles_n = (p.N + C::BN - 1) / C::BN;
    const int64_t ntiles = (int64_t)p.tiles_m * p.tiles_n;
    if (ntiles <= 0) return DS3_OK;
    if (ntiles > (1 << 28)) return DS3_ERR_UNSUPPORTED;
    // 32-bit byte offsets inside one tile's rows, all below the out-of-range marker
    if ((int64_t)(C::BN + 1) * p.ldb + p.K >= (1ll << 31) || (int64_t)(C::BM + 1) * p.lda + p.K >= (1ll << 31))
        return DS3_ERR_UNSUPPORTED;
    // Persistent launch: as many workgroups as fit the chip at once (fewer if there
    // are fewer tiles), a multiple of 8 so that every XCD gets the same number.
    const int64_t want = ((ntiles + 7) / 8) * 8;
    const int64_t slots = (int64_t)num_cus_x8() * C::WG_PER_CU;
    const unsigned grid = (unsigned)(want < slots ? want : slots);
    gemm_fp8_bs_kernel<C, ROWSB, OUT_BF16, GROUPED, POW2><<<dim3(grid), dim3(C::NT), 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

template <class C, bool POW2>
static ds3_status launch_cfg(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, hipStream_t st) {
    const bool bf16 = ct == DS3_BF16;
    if (p.G > 0)
        return bf16 ? launch_one<C, false, true, true, POW2>(p, st) : launch_one<C, false, false, true, POW2>(p, st);
    if (mode == DS3_BSCALE_PER_ROW)
        return bf16 ? launch_one<C, true, true, false, POW2>(p, st) : launch_one<C, true, false, false, POW2>(p, st);
    return bf16 ? launch_one<C, false, true, false, POW2>(p, st) : launch_one<C, false, false, false, POW2>(p, st);
}

int gemm_num_variants() { return 3; }

template <bool POW2>
static ds3_status launch_variant(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, hipStream_t st) {
    switch (variant) {
        case 0: return launch_cfg<Cfg<256, 256, 4, 2, 2>, POW2>(p, ct, mode, st);
        case 1: return launch_cfg<Cfg<256, 128, 4, 2, 3>, POW2>(p, ct, mode, st);
        case 2: return launch_cfg<Cfg<128, 128, 2, 2, 2>, POW2>(p, ct, mode, st);
        default: return DS3_ERR_UNSUPPORTED;
    }
}

ds3_status launch_gemm(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, bool pow2, hipStream_t st) {
    if (variant < 0) {
        // default choice: the 256x256 tile (also the fastest for the ragged expert groups);
        // the per-row-scale form (more live registers) takes the narrower M tile; problems with
        // too few large tiles to fill the chip take 128x128 tiles, two workgroups per CU
        variant = (mode == DS3_BSCALE_PER_ROW) ? 1 : 0;
        const int64_t big = (int64_t)((p.M + 255) / 256) * ((p.N + 255) / 256);
        if (p.G == 0 && big * 8 < 5 * (int64_t)num_cus_x8()) variant = 2;
    }
    return pow2 ? launch_variant<true>(p, ct, mode, variant, st) : launch_variant<false>(p, ct, mode, variant, st);
}

}  // namespace ds3
