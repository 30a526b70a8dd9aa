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
#include <mutex>
#include <type_traits>

#include "ds3_dev.h"
#include "ds3_internal.h"

namespace ds3 {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

constexpr int kMaxGroups = 1023;                       // experts per grouped call (prefix table in LDS)
constexpr int kShareSkew = 6;                          // K-steps by which the two pieces of a halved tile differ, each way
constexpr int kAuxDevice = 16;                         // cache policy of a buffer access: sc1, coherent across the device
constexpr int kTailCounters = 64;                      // arrival counters per XCD (tail tiles < workgroups per XCD <= 64)
constexpr int kQueueInts = 64;                         // the grouped walk's tile queue: [XCD] {next ticket, workgroups done}
constexpr size_t kCounterBytes = (8 * kTailCounters + kQueueInts) * sizeof(int);

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
    // loads of a K-step that are issued right behind the barrier that frees their stage (the
    // rest go out at the head of the next K-step)
    static constexpr int TAILN = LPT < FN ? LPT : FN;
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

// Whether `tail` tiles left over after `rounds` full rounds on `nslots` workgroups are shared
// along K.  Sharing costs about a sixth of a tile's time (partial sums through memory), so it
// pays when the workgroups would otherwise idle for much longer: few tiles in all (no full
// round: up to 0.6 tiles per workgroup), or a small remainder (up to a third; up to a half the
// half-tile split does as well without a workspace).  Host and kernel use the same rule.
__host__ __device__ inline bool tail_worth_sharing(int rounds, int tail, int nslots) {
    if (tail <= 0) return false;
    return rounds == 0 ? 5 * tail <= 3 * nslots : 3 * tail <= nslots;
}

// XOR key of a tile row: depends on the row's position inside its 16-row fragment only.
__device__ __forceinline__ int swz_key(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// Offset that is out of range for every descriptor this kernel builds (their
// sizes are below 2^31): a load with it moves no data.
constexpr unsigned kOobOffset = 0x80000000u;

// What a workgroup needs to know about one output tile (all wave-uniform
// except the two per-thread scale pointers).
struct TileCtx {
    int m0, n0, m_rows, n_rows;
    int kb0, kb1;             // K-steps [kb0, kb1) of the tile that this unit of work covers
    __amdgpu_buffer_rsrc_t rs_a, rs_b;
    unsigned sc_off;          // byte offset of the row of scales this thread fetches one value of per K-step (see `scale_role`)
};

//
// POW2 (power-of-two scales, Section 3.3.3): the scales are E8M0 numbers, whose
// code is the exponent field of the FP32 value, and the MFMA applies them itself
// (one scale per lane and operand: the weight row's and the activation row's);
// the accumulators then chain through the matrix pipe across K-steps and the
// vector ALU does no rescaling at all.
template <class C, bool ROWSB, bool OUT_BF16, bool GROUPED, bool POW2, bool SWIQ = false>
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
    // Grouped walk with a workspace: the tiles of an XCD's chunk beyond the first round are handed
    // out through a ticket counter, so a workgroup that drew cheap tiles (few valid rows) takes
    // more of them.  Which workgroup computes a tile does not change its result.  A ticket is
    // drawn when a tile starts and read after its K-loop; the last workgroup of the XCD to run
    // out of work puts both counters back to zero for the next call.
    [[maybe_unused]] const bool dyn = GROUPED && p.ws_cnt != nullptr;
    [[maybe_unused]] int* const queue = p.ws_cnt + 8 * kTailCounters + xcd * 2;
    [[maybe_unused]] int* const ticket_s = reinterpret_cast<int*>(sbrow_s);   // (per-row scale staging is unused here)
    [[maybe_unused]] int dyn_local = slot;
    [[maybe_unused]] const int cnt_xcd = max(0, min(per_xcd, ntiles - xcd * per_xcd));
    auto leave_queue = [&]() {
        if constexpr (GROUPED) {
            if (dyn && tid == 0) {
                const int d = __hip_atomic_fetch_add(queue + 1, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if (d == nslots - 1) {
                    __hip_atomic_store(queue, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(queue + 1, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
        }
    };
    // The XCD's tiles are taken in rounds of one tile per workgroup.  What is left
    // after the last full round (`tail` tiles, fewer than workgroups) is either
    //  * shared along K: the tail's K-steps, tile after tile, are cut into equal
    //    contiguous ranges, one per workgroup; a workgroup's range touches at most two
    //    tiles (its pieces), every piece's partial sums meet in the workspace and the
    //    workgroup that finishes a tile's last piece adds them up in piece order and
    //    writes the output -- nobody ever waits for another workgroup; or
    //  * (no workspace) cut into half tiles when at most half of the workgroups would
    //    get one: the two M halves of a tile belong to different waves, and the waves
    //    of the missing half skip their MFMAs.
    // The walk's geometry is needed only between tiles; the dense kernels keep it in LDS
    // rather than in scalar registers across the K-loop.
    struct Walk { int rounds, tail, mode, q, ra, rb, pt0, pt1, n_units, tail_steps; };
    enum { kWhole = 0, kShareK = 1, kHalfTiles = 2 };
    auto compute_walk = [&]() -> Walk {
        Walk w;
        const int cnt_x = max(0, min(per_xcd, ntiles - xcd * per_xcd));
        w.rounds = cnt_x / nslots;
        w.tail = cnt_x - w.rounds * nslots;
        const bool share_k = !GROUPED && p.ws_cnt != nullptr && tail_worth_sharing(w.rounds, w.tail, nslots) &&
                             (cnt_x == per_xcd ? p.share_steps : p.share_steps_last) > 0;
        const bool halves = !share_k && !GROUPED && C::WM == 2 && w.rounds > 0 && w.tail > 0 && 2 * w.tail <= nslots && p.M % BM == 0;
        w.mode = share_k ? kShareK : (halves ? kHalfTiles : kWhole);
        w.tail_steps = w.tail * KB;
        // K-steps per workgroup: the host's choice (an equal share, raised until no tile is cut
        // into more than two pieces); the last XCD's chunk may be shorter and has its own
        w.q = share_k ? (cnt_x == per_xcd ? p.share_steps : p.share_steps_last) : 1;
        // (p.share_skew lengthens the even runs and shortens the odd ones when every tile is cut
        // exactly in the middle: the shorter piece is then stored while the longer one still
        // computes, and only one of the two is ever written)
        const int skew = p.share_skew;
        w.ra = share_k ? min(slot * w.q + ((slot & 1) ? skew : 0), w.tail_steps) : 0;
        w.rb = share_k ? min((slot + 1) * w.q + ((slot & 1) ? 0 : skew), w.tail_steps) : 0;
        w.pt0 = w.ra / KB;                                   // tail tile of the first piece
        w.pt1 = w.rb > w.ra ? (w.rb - 1) / KB : w.pt0;       // tail tile of the last piece
        const int n_tail_units = share_k ? (w.rb > w.ra ? 1 + (w.pt1 > w.pt0 ? 1 : 0) : 0)
                                         : (halves ? (slot < 2 * w.tail ? 1 : 0) : (slot < w.tail ? 1 : 0));
        w.n_units = w.rounds + n_tail_units;
        return w;
    };
    // Dense kernels keep the three numbers every unit needs in registers and the geometry of a
    // shared tail in LDS (the prefix table's space is free there), read when a tail unit comes up.
    int* const walk_s = gpre + 4;
    int w_rounds, w_mode, w_units;
    {
        const Walk w = compute_walk();
        w_rounds = w.rounds; w_mode = w.mode; w_units = w.n_units;
        if constexpr (!GROUPED) {
            if (tid == 0) {
                walk_s[0] = w.q; walk_s[1] = w.ra; walk_s[2] = w.rb; walk_s[3] = w.pt0; walk_s[4] = w.pt1; walk_s[5] = w.tail_steps;
            }
            __syncthreads();
        }
    }
    struct Tail { int q, ra, rb, pt0, pt1, tail_steps; };
    auto load_tail = [&]() -> Tail {
        Tail w;
        asm volatile("" ::: "memory");
        auto rd = [&](int i) { return __builtin_amdgcn_readfirstlane(walk_s[i]); };
        w.q = rd(0); w.ra = rd(1); w.rb = rd(2); w.pt0 = rd(3); w.pt1 = rd(4); w.tail_steps = rd(5);
        return w;
    };

    auto setup_unit = [&](int u, TileCtx& c) -> bool {
        int half = -1, local;                          // local: index of the tile inside the XCD's chunk
        c.kb0 = 0; c.kb1 = KB;
        if (GROUPED && dyn) {
            if (dyn_local >= cnt_xcd) return false;
            local = dyn_local;
        } else if (u >= w_units) return false;
        else if (u < w_rounds) local = u * nslots + slot;
        else if (!GROUPED && w_mode == kShareK) {
            const Tail w = load_tail();
            const int tt = u == w_rounds ? w.pt0 : w.pt1;   // first / second piece of this workgroup
            local = w_rounds * nslots + tt;
            c.kb0 = max(w.ra - tt * KB, 0);
            c.kb1 = min(w.rb - tt * KB, KB);
        } else if (w_mode == kHalfTiles) { half = slot & 1; local = w_rounds * nslots + (slot >> 1); }
        else local = w_rounds * nslots + slot;
        const int t = xcd * per_xcd + local;
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
            // The same for every lane, but read through vector registers (LDS, an indexed global
            // load): said to be uniform here, the tile's buffer descriptors live in scalar registers.
            // Left in vector registers, every load of the K-loop would sit in a loop of its own that
            // picks the descriptor lane by lane, cutting the K-step's instruction schedule to pieces.
            grp = __builtin_amdgcn_readfirstlane(grp);
            n0 = __builtin_amdgcn_readfirstlane(n0);
            m0 = __builtin_amdgcn_readfirstlane(m0);
            m_end = __builtin_amdgcn_readfirstlane(m_end);
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
        // Every K-step a thread fetches at most one scale, straight into LDS: the first BM
        // threads their activation row's; in block mode the lanes of the next wave the
        // weight-block scale of wave column min(lane, WN - 1); in per-row mode the last BN
        // threads their weight row's.  Rows past the valid ones repeat the last valid row,
        // whose partial sums are zero because its codes were read as zero.
        // (offsets from p.sa / p.sb in bytes; the host has checked that they fit 31 bits)
        if (tid < BM) c.sc_off = (unsigned)((m0 + min(tid, c.m_rows - 1)) * (int)p.sar) * 4u;
        else if constexpr (ROWSB) c.sc_off = (unsigned)((n0 + min(max(tid - (NT - BN), 0), c.n_rows - 1)) * (int)p.sbr) * 4u;
        else {
            const int nblocks = (p.N + 127) >> 7;
            const int nb = min((n0 + min(lane, C::WN - 1) * C::TN) >> 7, nblocks - 1);
            c.sc_off = (unsigned)(grp * (int)p.sb_group_stride + nb * (int)p.sbr) * 4u;
        }
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

    // which scale this wave fetches (wave-uniform): 0 none, 1 activation rows, 2 weight scales
    const int scale_role = wave * 64 < BM ? 1 : ((ROWSB ? wave * 64 >= NT - BN : wave * 64 == BM) ? 2 : 0);
    static_assert(ROWSB ? BM + BN <= NT : BM + 64 <= NT, "one scale per thread and K-step");
    // Bytes between the scales of consecutive K-steps in the row this thread fetches from.  Kept
    // in a vector register: as a scalar it would be re-read from the kernel arguments inside the
    // K-loop, and a scalar load in flight turns every counted wait for LDS data into a full one.
    unsigned sc_kstride = (unsigned)(scale_role == 1 ? (int)p.sak : (int)p.sbk) * 4u;
    asm volatile("" : "+v"(sc_kstride));
    // one descriptor over the activation or the weight scales, whichever this wave fetches (every
    // offset it is used with is valid; the range check is not relied on)
    const __amdgpu_buffer_rsrc_t rs_sc =
        __builtin_amdgcn_make_buffer_rsrc((void*)(scale_role == 1 ? p.sa : p.sb), 0, 0x7ffffffc, 0x00020000);

    // i-th 16-byte load of this thread for the K-step at byte offset koff, into LDS stage `stage`
    auto issue_load = [&](const TileCtx& c, int i, int stage, unsigned koff) {
        const bool is_b = i * C::RPI < BN;
        const int ii = is_b ? i : i - BN / C::RPI;
        // the wave-uniform part of the offset is summed in a scalar register and added last (tied to
        // a scalar register here so that it is not folded into eight per-load vector registers)
        unsigned uoff = koff + (unsigned)ii * (is_b ? step_b : step_a);
        asm volatile("" : "+s"(uoff));
        const unsigned voff = (is_b ? voff_b : voff_a) + uoff;
        uint8_t* dst = smem + stage * STAGE + (i * NT + wave * 64) * 16;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(is_b ? c.rs_b : c.rs_a, (lds_ptr_t)dst, 16, (int)voff, 0, 0, 0);
    };
    // The scales of K-step kb (clamped to the unit's last) go global -> LDS like the codes, into
    // staging slot `stage`: activation scales at sa_s[stage][row], block scales behind them at
    // sa_s[stage][BM + wave column], per-row weight scales at sbrow_s[stage][row].
    auto issue_scale = [&](const TileCtx& c, int kb, int stage) {
        if (scale_role == 0) return;
        const int kc = min(kb, c.kb1 - 1);
        float* dst = (ROWSB && scale_role == 2) ? sbrow_s + stage * NT + (wave * 64 - (NT - BN)) : sa_s + stage * NT + wave * 64;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_sc, (lds_ptr_t)dst, 4, (int)(c.sc_off + (unsigned)kc * sc_kstride), 0, 0, 0);
    };
    auto load_frag = [&](const uint8_t* base) -> i32x8 {
        const i32x4 lo = *reinterpret_cast<const i32x4*>(base + foff0);
        const i32x4 hi = *reinterpret_cast<const i32x4*>(base + foff1);
        return i32x8{lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
    };
    auto read_sb = [&](int stage) -> float {           // this wave's weight-block scale (block mode)
        return sa_s[stage * NT + BM + wn];
    };
    auto read_tj = [&](int stage, float* tj) {
        [[maybe_unused]] const float sbv = (ROWSB || POW2) ? 1.f : read_sb(stage);
#pragma unroll
        for (int j = 0; j < FM; ++j) {
            const float sav = sa_s[stage * NT + wm * C::TM + j * 16 + l16];
            tj[j] = (ROWSB || POW2) ? sav : sav * sbv;
        }
    };

    TileCtx cur;
    int unit = 0;
    if (!setup_unit(unit, cur)) { leave_queue(); return; }
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
    // The barrier of a K-step: the loads issued since the previous one -- LPT of codes, and one
    // of scales in the waves that fetch any -- run a K-step further ahead when there are three
    // stages and may stay in flight.
    auto kstep_barrier = [&]() {
        if constexpr (NS == 2) barrier_keep(std::integral_constant<int, 0>{});
        else if (scale_role != 0) barrier_keep(std::integral_constant<int, C::LPT + 1>{});
        else barrier_keep(std::integral_constant<int, C::LPT>{});
    };
    // the first NS-1 K-steps of the first tile into stages 0 .. NS-2
    auto issue_first_steps = [&](const TileCtx& c) {
#pragma unroll
        for (int ks = 0; ks < NS - 1; ++ks) {
#pragma unroll
            for (int i = 0; i < C::LPT; ++i) issue_load(c, i, ks, c.kb0 + ks < c.kb1 ? (unsigned)(c.kb0 + ks) << 7 : kOobOffset);
            issue_scale(c, c.kb0 + ks, ks);
        }
    };
    issue_first_steps(cur);

    for (;;) {
        // ---- entry: K-steps 0 .. NS-2 of `cur` (codes and scales) are in flight into stages 0 .. NS-2 ----
        __syncthreads();
        [[maybe_unused]] int ticket = 0;
        if constexpr (GROUPED) {
            if (dyn && tid == 0) ticket = __hip_atomic_fetch_add(queue, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        // the part of K-step NS-1 that a previous K-step's barrier would have issued
#pragma unroll
        for (int i = 0; i < C::TAILN; ++i)
            issue_load(cur, i, NS - 1, cur.kb0 + NS - 1 < cur.kb1 ? (unsigned)(cur.kb0 + NS - 1) << 7 : kOobOffset);
        issue_scale(cur, cur.kb0 + NS - 1, NS - 1);
        const int KE = cur.kb1;                            // end of this unit's K-steps
        float tj[FM];
        [[maybe_unused]] float sb_c = (POW2 && !ROWSB) ? read_sb(0) : 1.f;   // block scale of THIS K-step (POW2 only)
        read_tj(0, tj);
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
            const unsigned koff1 = kb + NS - 1 < KE ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;   // head loads
            const unsigned koff2 = kb + NS < KE ? (unsigned)(kb + NS) << 7 : kOobOffset;           // tail loads
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < NSUB + D; ++s) {
                if (s == NSUB - FN) {
                    // Everything this wave reads from stage S is in registers.  After the
                    // barrier the next stage is complete and stage S may be overwritten.
                    kstep_barrier();
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
                        if (i == 0) issue_scale(cur, kb + NS, S);
                        if (i == FN - 1) {
                            qf[0] = load_frag(nst + q_base);
                            read_tj(SN, tjn);
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
            const unsigned koff1 = kb + NS - 1 < KE ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;
            const unsigned koff2 = kb + NS < KE ? (unsigned)(kb + NS) << 7 : kOobOffset;
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int s = 0; s < NSUB; ++s) {
                if (s == NSUB - FN) {
                    kstep_barrier();
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (s < HEADN) issue_load(cur, TAILN + s, SL, koff1);
                const int j = s / FN, i = s % FN;
                if (i == 0 && j + 1 < FM) qf[(j + 1) & 1] = load_frag(st + q_base + (j + 1) * 2048);
                acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(pf[i], qf[j & 1], acc[i][j], 0, 0, 0, ea[i],
                                                                             0, eb[j]);
                asm volatile("" : "+v"(acc[i][j]));        // ties the MFMA to this point of the K-step
                if (j == FM - 1) {
                    pf[i] = load_frag(nst + p_base + i * 2048);
#pragma unroll
                    for (int l = i; l < TAILN; l += FN) issue_load(cur, l, S, koff2);
                    if (i == 0) issue_scale(cur, kb + NS, S);
                    if (i == FN - 1) {
                        qf[0] = load_frag(nst + q_base);
                        read_tj(SN, tjn);
                        if constexpr (!ROWSB) sb_cn = read_sb(SN);
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
            const unsigned koff1 = kb + NS - 1 < KE ? (unsigned)(kb + NS - 1) << 7 : kOobOffset;
            const unsigned koff2 = kb + NS < KE ? (unsigned)(kb + NS) << 7 : kOobOffset;
#pragma unroll
            for (int i = 0; i < HEADN; ++i) issue_load(cur, TAILN + i, SL, koff1);
            kstep_barrier();
#pragma unroll
            for (int i = 0; i < TAILN; ++i) issue_load(cur, i, S, koff2);
            issue_scale(cur, kb + NS, S);
        };

        using st0 = std::integral_constant<int, 0>;
        using st1 = std::integral_constant<int, 1>;
        using st2 = std::integral_constant<int, 2>;
        const bool active = wm * C::TM < cur.m_rows;    // wave-uniform
        auto kloop = [&](auto step) {
            int kb = cur.kb0;
            if constexpr (NS == 2) {
                for (; kb + 1 < KE; kb += 2) {
                    step(kb, st0{});
                    step(kb + 1, st1{});
                }
                if (kb < KE) step(kb, st0{});
            } else {
                for (; kb + 2 < KE; kb += 3) {
                    step(kb, st0{});
                    step(kb + 1, st1{});
                    step(kb + 2, st2{});
                }
                if (kb < KE) step(kb, st0{});
                if (kb + 1 < KE) step(kb + 1, st1{});
            }
        };
        if (!active) kloop(kstep_idle);
        else if constexpr (POW2) kloop(kstep_p2);
        else kloop(kstep);
        if constexpr (GROUPED) {
            if (dyn && tid == 0) ticket_s[0] = ticket;
        }
        __syncthreads();                               // every wave is done with all code stages
        if constexpr (GROUPED) {
            if (dyn) dyn_local = nslots + __builtin_amdgcn_readfirstlane(ticket_s[0]);
        }

        // ---- the next tile's first K-steps fly into stages 0 .. NS-2 during this tile's epilogue ----
        // (what is read from LDS here is read before those loads are issued: the compiler makes an
        // LDS read that follows LDS-bound loads wait for them)
        [[maybe_unused]] int pieces = 1, my_part = 0, tail_tile = 0, first_slot = 0, share_q = 1, tail_steps = 0;
        if constexpr (!GROUPED) {
            if (w_mode == kShareK && unit >= w_rounds) {
                const Tail w = load_tail();
                share_q = w.q; tail_steps = w.tail_steps;
                my_part = unit - w_rounds;                 // 0 / 1: first / second piece of this workgroup
                tail_tile = my_part == 0 ? w.pt0 : w.pt1;
                first_slot = (tail_tile * KB) / share_q;   // workgroup slot of the tile's first piece
                pieces = ((tail_tile + 1) * KB - 1) / share_q - first_slot + 1;
            }
        }
        TileCtx nxt;
        ++unit;
        const bool more = setup_unit(unit, nxt);
        if (more) issue_first_steps(nxt);

        // ---- a piece of a tile that is shared along K -----------------------------------
        // A shared tile has exactly two pieces.  The workgroup that finishes first stores its
        // partial sums in the workspace, lane by lane; the one whose arrival completes the
        // tile adds them to its own (a + b = b + a: the result does not depend on who is last)
        // and goes on to the epilogue.
        // Coherence without cache-wide operations: the partial sums are written and read
        // with device-scope accesses (sc1: written through, read past this XCD's L2), the
        // arrival counter is a device-scope atomic, and the order "sums before arrival" /
        // "arrival before sums" is kept by waiting for the stores and by the barriers.  A
        // device-scope fence would write back and invalidate the whole L2 under the
        // workgroups that are still computing.
        [[maybe_unused]] bool reduce = false;              // this unit completes a tile whose other piece waits in the workspace
        [[maybe_unused]] __amdgpu_buffer_rsrc_t rs_other = cur.rs_a;
        [[maybe_unused]] const int toff = tid * 16;
        if constexpr (!GROUPED) {
            if (pieces > 1) {
                constexpr int TILE_F = BN * BM;            // floats of one partial tile
                int* const cnt = p.ws_cnt + xcd * kTailCounters + tail_tile;
                // A partial tile is stored lane by lane: accumulator (i, j) of thread t at float
                // ((i * FM + j) * NT + t) * 4.  Buffer addressing keeps the per-thread part of
                // every address in one register (the accumulators leave few to spare).
                // two partial tiles per shared tile, one per piece (both pieces may store when they
                // finish together): [XCD][tail tile][piece]
                auto part_of = [&](int k) {                // partial tile of the tile's k-th piece, k = 0, 1 in K order
                    float* base = p.ws_part + (int64_t)((xcd * p.share_tail_max + tail_tile) * 2 + k) * TILE_F;
                    return __builtin_amdgcn_make_buffer_rsrc((void*)base, 0, TILE_F * 4, 0x00020000);
                };
                const int me = slot - first_slot;          // 0: this workgroup holds the tile's first piece, 1: its second
                auto store_mine = [&]() {
                    const __amdgpu_buffer_rsrc_t rs = part_of(me);
#pragma unroll
                    for (int i = 0; i < FN; ++i)
#pragma unroll
                        for (int j = 0; j < FM; ++j) {
                            const f32x4 v = acc[i][j];
                            __builtin_amdgcn_raw_buffer_store_b128(u32x4{as_u32(v.x), as_u32(v.y), as_u32(v.z), as_u32(v.w)}, rs, toff,
                                                                   (i * FM + j) * NT * 16, kAuxDevice);
                        }
                };
                // has the other piece arrived already?  then this one need not be stored
                if (tid == 0) gpre[0] = __hip_atomic_load(cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                const bool others_done = (gpre[0] & 1) != 0;
                __syncthreads();
                if (!others_done) store_mine();
                __builtin_amdgcn_s_waitcnt(0x0070);        // vmcnt(0): my partial sums have been written through
                __syncthreads();                           // ... and everybody else's of this workgroup
                if (tid == 0) gpre[0] = __hip_atomic_fetch_add(cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                __syncthreads();
                const bool last = (gpre[0] & 1) != 0;      // a tile's two arrivals take its counter from even to odd to even
                __syncthreads();
                if (!last) {
                    if (!more) break;
                    cur = nxt;
                    continue;
                }
                reduce = true;                             // the epilogue adds the other piece in on its way out
                rs_other = part_of(1 - me);
            }
        }

        // ---- epilogue ------------------------------------------------------------------
        // A lane owns one activation row m and, per weight fragment, 4 consecutive n:
        // stored directly that would be 8-byte pieces scattered over 16 rows.  Each
        // wave instead transposes 16 rows x TN columns at a time through a private
        // LDS strip in the last stage and writes 16 bytes per lane, a full 128-byte (BF16)
        // or 256-byte (FP32) row segment per group of lanes.
        // Every address of the epilogue derives from this copy of the thread index, which the
        // compiler cannot see through: none of them is computed before the K-loop and kept in a
        // register across it (the loop has none to spare).
        int tid_e = threadIdx.x;
        asm volatile("" : "+v"(tid_e));
        const int lane = tid_e & 63, l16 = tid_e & 15, g4 = (tid_e >> 4) & 3;
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
        // The other piece's partial sums of row group j (a shared tile's second arrival only),
        // fetched one group ahead of their use.
        [[maybe_unused]] u32x4 otherv[2][FN];
        auto fetch_other = [&](int j) {
#pragma unroll
            for (int i = 0; i < FN; ++i)
                otherv[j & 1][i] = __builtin_amdgcn_raw_buffer_load_b128(rs_other, toff, (i * FM + j) * NT * 16, kAuxDevice);
        };
        // RED (compile time): this is the second arrival at a shared tile, the other piece is added in
        auto put_group = [&](int j, auto red_tag) {        // accumulators of row group j -> strip
            constexpr bool RED = decltype(red_tag)::value;
            uint8_t* sp = strip0 + (NSTRIP == 2 ? (j & 1) * (16 * ROWB) : 0);
            if constexpr (RED) { if (j + 1 < FM) fetch_other(j + 1); }
#pragma unroll
            for (int i = 0; i < FN; ++i) {
                f32x4 v = acc[i][j];
                if constexpr (RED) {
                    const u32x4 o = otherv[j & 1][i];
                    v.x += as_f32(o.x); v.y += as_f32(o.y); v.z += as_f32(o.z); v.w += as_f32(o.w);
                }
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
        auto write_out = [&](auto red_tag) {
            if constexpr (!OUT_BF16) { if (accum) fetch_old(0, oldv[0]); }
            if constexpr (decltype(red_tag)::value) fetch_other(0);
            put_group(0, red_tag);
#pragma unroll
            for (int j = 0; j < FM; ++j) {
                if constexpr (!OUT_BF16) { if (accum && j + 1 < FM) fetch_old(j + 1, oldv[(j + 1) & 1]); }
                __builtin_amdgcn_wave_barrier();           // same-wave LDS accesses complete in order
                u32x4 wv[PASSES];
                get_group(j, wv);
                if constexpr (NSTRIP == 2) { if (j + 1 < FM) put_group(j + 1, red_tag); }
                store_group(j, wv);
                if constexpr (NSTRIP == 1) {
                    __builtin_amdgcn_wave_barrier();       // reads of the strip precede the next round of writes
                    if (j + 1 < FM) put_group(j + 1, red_tag);
                }
            }
        };
        // SwiGLU and the 1x128 quantiser of the following Linear's input on the tile itself
        // (Section 3.3.2 fuses the cast with the activation; here both ride on the GEMM that
        // produces their input).  The weight is stored with gate and up rows interleaved in
        // blocks of 128, so the 256 columns of a tile are the gate (first 128) and the up
        // projection (last 128) of the same 128 output columns: one 1x128 tile per row.
        // The accumulators are rounded to BF16 exactly as the unfused GEMM would store them
        // and pass through the last code stage, 128 rows at a time; then 16 lanes take one
        // row (8 columns each), as the stand-alone fused kernel does, with the same
        // expressions, so the two paths agree bit for bit.
        auto swiglu_quant_out = [&]() {
            static_assert(!SWIQ || (C::BN == 256 && C::WM == 2 && NT == 512 && C::TM * 512 <= STAGE), "SwiGLU epilogue shape");
            uint8_t* hs = smem + (NS - 1) * STAGE;         // [TM rows][256 BF16], 16-byte chunks XOR-swizzled by row
            const int64_t ob = cur.n0 >> 8;                // this tile's 1x128 tile of the output
            const int tid = tid_e, lane16 = l16;
            const int npass = cur.m_rows > C::TM ? 2 : 1;
            auto lds_barrier = [&]() {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F);        // lgkmcnt(0) only: the next tile's first loads stay in flight
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            };
            for (int ps = 0; ps < npass; ++ps) {
                if (wm == ps) {
#pragma unroll
                    for (int j = 0; j < FM; ++j) {
#pragma unroll
                        for (int i = 0; i < FN; ++i) {
                            const f32x4 v = acc[i][j];
                            const int col = wn * C::TN + i * 16 + g4 * 4;
                            uint8_t* dst = hs + (j * 16 + l16) * 512 + (((col >> 3) ^ l16) << 4) + (col & 7) * 2;
                            *reinterpret_cast<u32x2*>(dst) = u32x2{pack_bf16x2(v.x, v.y), pack_bf16x2(v.z, v.w)};
                        }
                    }
                }
                lds_barrier();
#pragma unroll
                for (int it = 0; it < C::TM / 32; ++it) {
                    const int row = it * 32 + (tid >> 4);
                    const uint8_t* hr = hs + row * 512;
                    const u32x4 gg = *reinterpret_cast<const u32x4*>(hr + ((lane16 ^ (row & 15)) << 4));
                    const u32x4 uu = *reinterpret_cast<const u32x4*>(hr + (((16 + lane16) ^ (row & 15)) << 4));
                    const unsigned int gw[4] = {gg.x, gg.y, gg.z, gg.w}, uw[4] = {uu.x, uu.y, uu.z, uu.w};
                    unsigned int w[4], m = 0;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        w[e] = pack_bf16x2(silu_mul(bf16_lo(gw[e]), bf16_lo(uw[e])), silu_mul(bf16_hi(gw[e]), bf16_hi(uw[e])));
                        m = umax(m, umax(w[e] & 0x7fff0000u, (w[e] << 16) & 0x7fff0000u));
                    }
                    m = row16_max_bits(m);
                    const GroupScale gs = group_scale(as_f32(m), p.q_pow2);
                    const int ml = ps * C::TM + row;
                    if (ml < cur.m_rows) {
                        const int64_t grow = cur.m0 + ml;
                        const u32x2 cw = {cvt4_e4m3(bf16_lo(w[0]) * gs.r, bf16_hi(w[0]) * gs.r, bf16_lo(w[1]) * gs.r, bf16_hi(w[1]) * gs.r),
                                          cvt4_e4m3(bf16_lo(w[2]) * gs.r, bf16_hi(w[2]) * gs.r, bf16_lo(w[3]) * gs.r, bf16_hi(w[3]) * gs.r)};
                        __builtin_nontemporal_store(cw, reinterpret_cast<u32x2*>(p.q_out + grow * p.ldq + ob * 128 + lane16 * 8));
                        if (lane16 == 0) p.s_out[grow * p.sor + ob * p.sok] = gs.s;
                    }
                }
                if (ps + 1 < npass) lds_barrier();         // the second half's rows replace the first's
            }
        };
        if constexpr (SWIQ) swiglu_quant_out();
        else if (active) {
            if constexpr (GROUPED) write_out(std::false_type{});
            else if (reduce) write_out(std::true_type{});
            else write_out(std::false_type{});
        }
        if (!more) break;
        cur = nxt;
    }
    leave_queue();
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

__global__ void clear_counters_kernel(int* cnt) { cnt[threadIdx.x] = 0; }     // one thread per counter
static_assert(kCounterBytes / sizeof(int) <= 1024, "one workgroup clears the counters");

// K-steps per workgroup when `tail` tiles of `kb` K-steps each are shared among `nslots`
// workgroups as contiguous runs (workgroup s takes steps [s*q, (s+1)*q) of the tiles laid end
// to end): the smallest q not below an equal share with which no tile is cut into more than
// two pieces; 0 if only whole tiles qualify (then nothing is shared).
int tail_share_steps(int tail, int kb, int nslots) {
    if (tail <= 0 || kb <= 1 || nslots <= tail) return 0;
    const int64_t total = (int64_t)tail * kb;
    for (int q = (int)((total + nslots - 1) / nslots); q < kb; ++q) {
        bool ok = true;
        for (int t = 0; t < tail && ok; ++t) {
            const int64_t first = (int64_t)t * kb / q, last = ((int64_t)(t + 1) * kb - 1) / q;
            ok = last - first <= 1;
        }
        if (ok) return q;
    }
    return 0;
}

// Bytes of workspace with which a dense launch of configuration C shares its tail tiles
// along K (0: the tile count leaves no tail worth sharing).  Mirrors the kernel's rule.
template <class C>
static size_t share_bytes(int64_t ntiles, int64_t slots, int kb, int* q_main, int* q_last, int* tail_max) {
    const int64_t nslots = slots / 8, per_xcd = (ntiles + 7) / 8;
    *q_main = *q_last = *tail_max = 0;
    for (int x = 0; x < 8; ++x) {
        int64_t cnt = ntiles - x * per_xcd;
        cnt = cnt < 0 ? 0 : (cnt > per_xcd ? per_xcd : cnt);
        const int64_t tail = cnt % nslots;
        if (!tail_worth_sharing((int)(cnt / nslots), (int)tail, (int)nslots)) continue;
        const int q = tail_share_steps((int)tail, kb, (int)nslots);
        if (cnt == per_xcd) *q_main = q; else *q_last = q;
        if (q > 0 && tail > *tail_max) *tail_max = (int)tail;
    }
    // arrival counters, then two partial tiles for every tile that may be shared
    return *tail_max ? kCounterBytes + (size_t)8 * *tail_max * 2 * C::BN * C::BM * sizeof(float) : 0;
}

template <class C, bool ROWSB, bool OUT_BF16, bool GROUPED, bool POW2, bool SWIQ = false>
static ds3_status launch_one(GemmParams p, void* ws, size_t ws_bytes, size_t* ws_need, hipStream_t st) {
    if (GROUPED) p.tiles_m = (p.M + C::BM - 1) / C::BM + p.G;
    else p.tiles_m = (p.M + C::BM - 1) / C::BM;
    p.tiles_n = (p.N + C::BN - 1) / C::BN;
    const int64_t ntiles = (int64_t)p.tiles_m * p.tiles_n;
    const int64_t slots = (int64_t)num_cus_x8() * C::WG_PER_CU;
    int q_main = 0, q_last = 0, tail_max = 0;
    // (the grouped walk needs the counters only: its tile queue)
    const size_t need = ntiles <= 0 ? 0 : GROUPED ? kCounterBytes
                                                  : share_bytes<C>(ntiles, slots, p.K / 128, &q_main, &q_last, &tail_max);
    if (ws_need) { *ws_need = need; return DS3_OK; }    // size query only
    if (ntiles <= 0) return DS3_OK;
    if (ntiles > (1 << 28)) return DS3_ERR_UNSUPPORTED;
    // 32-bit byte offsets inside one tile's rows, all below the out-of-range marker
    if ((int64_t)(C::BN + 1) * p.ldb + p.K >= (1ll << 31) || (int64_t)(C::BM + 1) * p.lda + p.K >= (1ll << 31))
        return DS3_ERR_UNSUPPORTED;
    const bool share = ws != nullptr && need > 0;
    if (share && ws_bytes < need) return DS3_ERR_WORKSPACE;
    // Persistent launch: as many workgroups as fit the chip at once (fewer if there
    // are fewer tiles and no tile is shared along K), a multiple of 8 so that every
    // XCD gets the same number.
    const int64_t want = ((ntiles + 7) / 8) * 8;
    const unsigned grid = (unsigned)(share || want > slots ? slots : want);
    (void)hipGetLastError();                            // a stale error of earlier, unrelated work is not this launch's
    if (share && GROUPED) p.ws_cnt = static_cast<int*>(ws);
    else if (share) {
        p.ws_cnt = static_cast<int*>(ws);
        p.ws_part = reinterpret_cast<float*>(static_cast<char*>(ws) + kCounterBytes);
        p.share_steps = q_main;
        p.share_steps_last = q_last;
        p.share_tail_max = tail_max;
        const int kb = p.K / 128;
        p.share_skew = (2 * q_main == kb && (q_last == 0 || q_last == q_main) && q_main > kShareSkew + 2) ? kShareSkew : 0;
    }
    gemm_fp8_bs_kernel<C, ROWSB, OUT_BF16, GROUPED, POW2, SWIQ><<<dim3(grid), dim3(C::NT), 0, st>>>(p);
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

template <class C, bool POW2>
static ds3_status launch_cfg(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, void* ws, size_t wsb, size_t* need, hipStream_t st) {
    const bool bf16 = ct == DS3_BF16;
    if (p.G > 0)
        return bf16 ? launch_one<C, false, true, true, POW2>(p, ws, wsb, need, st) : launch_one<C, false, false, true, POW2>(p, ws, wsb, need, st);
    if (mode == DS3_BSCALE_PER_ROW)
        return bf16 ? launch_one<C, true, true, false, POW2>(p, ws, wsb, need, st) : launch_one<C, true, false, false, POW2>(p, ws, wsb, need, st);
    return bf16 ? launch_one<C, false, true, false, POW2>(p, ws, wsb, need, st) : launch_one<C, false, false, false, POW2>(p, ws, wsb, need, st);
}

int gemm_num_variants() { return 3; }

template <bool POW2>
static ds3_status launch_variant(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, void* ws, size_t wsb, size_t* need,
                                 hipStream_t st) {
    switch (variant) {
        case 0: return launch_cfg<Cfg<256, 256, 4, 2, 2>, POW2>(p, ct, mode, ws, wsb, need, st);
        case 1: return launch_cfg<Cfg<256, 128, 4, 2, 3>, POW2>(p, ct, mode, ws, wsb, need, st);
        case 2: return launch_cfg<Cfg<128, 128, 2, 2, 2>, POW2>(p, ct, mode, ws, wsb, need, st);
        default: return DS3_ERR_UNSUPPORTED;
    }
}

// The tile configuration a shape runs with when the caller does not name one.
static int default_variant(const GemmParams& p, ds3_bscale mode) {
    // the 256x256 tile; the ragged expert groups take 256x128 tiles in three stages (their
    // weights come from HBM, not from the L2, and want the deeper prefetch; 128-row tiles
    // also pad less); problems with too few large tiles to fill the chip take 128x128 tiles,
    // two workgroups per CU
    (void)mode;
    int variant = p.G > 0 ? 1 : 0;
    const int64_t big = (int64_t)((p.M + 255) / 256) * ((p.N + 255) / 256);
    if (p.G == 0 && big * 8 < 5 * (int64_t)num_cus_x8()) variant = 2;
    return variant;
}

ds3_status launch_gemm(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, bool pow2, void* ws, size_t ws_bytes,
                       hipStream_t st) {
    if (variant < 0) variant = default_variant(p, mode);
    return pow2 ? launch_variant<true>(p, ct, mode, variant, ws, ws_bytes, nullptr, st)
                : launch_variant<false>(p, ct, mode, variant, ws, ws_bytes, nullptr, st);
}

size_t grouped_workspace_bytes() { return kCounterBytes; }

ds3_status launch_gemm_swiglu_quant(const GemmParams& p, bool pow2, void* ws, size_t ws_bytes, hipStream_t st) {
    // 256 weight rows per tile: the gate and the up half of one 1x128 output tile; 128 activation
    // rows and three stages, as the plain grouped GEMM runs by default
    using C = Cfg<256, 128, 4, 2, 3>;
    if (p.G <= 0 || p.N % 256) return DS3_ERR_SHAPE;
    return pow2 ? launch_one<C, false, true, true, true, true>(p, ws, ws_bytes, nullptr, st)
                : launch_one<C, false, true, true, false, true>(p, ws, ws_bytes, nullptr, st);
}

__global__ void zero_fill_kernel(uint8_t* c, int64_t row_bytes, int64_t ld_bytes, int64_t rows) {
    // 16-byte pieces of the rows' valid part, then the bytes of a row that are left
    const int64_t chunks = row_bytes / 16;
    for (int64_t r = blockIdx.y; r < rows; r += gridDim.y) {
        uint8_t* row = c + r * ld_bytes;
        for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < chunks; i += (int64_t)gridDim.x * blockDim.x)
            reinterpret_cast<u32x4*>(row)[i] = u32x4{0u, 0u, 0u, 0u};
        if (blockIdx.x == 0 && threadIdx.x < row_bytes - chunks * 16) row[chunks * 16 + threadIdx.x] = 0;
    }
}

ds3_status launch_zero_fill(void* c, ds3_dtype ct, int64_t M, int64_t N, int64_t ldc, hipStream_t st) {
    const int64_t es = ct == DS3_BF16 ? 2 : 4;
    const int64_t chunks = N * es / 16;
    const unsigned gx = (unsigned)(chunks / 256 + 1 > 64 ? 64 : chunks / 256 + 1), gy = (unsigned)(M > 1024 ? 1024 : M);
    (void)hipGetLastError();
    zero_fill_kernel<<<dim3(gx, gy), dim3(256), 0, st>>>(static_cast<uint8_t*>(c), N * es, ldc * es, M);
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

// ---- a workspace of the library's own, for callers that cannot allocate -----------------
// Large enough for every shape on a 256-CU device: at most 19 of an XCD's 32 workgroups' tiles
// are shared (the rule above), two partial tiles of 256 x 256 floats each, eight XCDs.  Each
// device the library runs on holds its own copy from the moment the code object is loaded
// (zero-filled then, which is what the arrival counters need; every call leaves them so).
constexpr size_t kScratchBytes = kCounterBytes + (size_t)8 * 19 * 2 * 256 * 256 * sizeof(float);
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

// The array's device address, per device (its name is only a host-side handle).
static ds3_status scratch_address(void** out, hipStream_t st) {
    static std::mutex mu;
    static void* addr[64] = {nullptr};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DS3_ERR_LAUNCH;
    std::lock_guard<std::mutex> lock(mu);
    if (addr[dev] == nullptr) {
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return DS3_ERR_LAUNCH;
        // the counters start even whatever ran before: once per device, in stream order before the first use
        (void)hipGetLastError();
        clear_counters_kernel<<<dim3(1), dim3(kCounterBytes / sizeof(int)), 0, st>>>(static_cast<int*>(ptr));
        if (hipGetLastError() != hipSuccess) return DS3_ERR_LAUNCH;
        addr[dev] = ptr;
    }
    *out = addr[dev];
    return DS3_OK;
}

ds3_status launch_gemm_static_scratch(const GemmParams& p, ds3_dtype ct, ds3_bscale mode, int variant, bool pow2, hipStream_t st) {
    void* ws = nullptr;
    const ds3_status rc = scratch_address(&ws, st);
    if (rc != DS3_OK) return rc;
    // (a shape that asked for more than the array holds would be refused with DS3_ERR_WORKSPACE)
    return launch_gemm(p, ct, mode, variant, pow2, ws, kScratchBytes, st);
}

size_t gemm_static_scratch_bytes() { return kScratchBytes; }

ds3_status launch_workspace_init(void* ws, size_t ws_bytes, hipStream_t st) {
    if (ws_bytes < kCounterBytes) return DS3_ERR_WORKSPACE;
    (void)hipGetLastError();
    // a small kernel, not a memset: callers may capture this call into a graph
    clear_counters_kernel<<<dim3(1), dim3(kCounterBytes / sizeof(int)), 0, st>>>(static_cast<int*>(ws));
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

size_t gemm_workspace_bytes(const GemmParams& p, ds3_bscale mode, int variant) {
    if (variant < 0) variant = default_variant(p, mode);
    size_t need = 0;
    // the requirement depends on the tile configuration only, not on the output type or the scale kind
    if (launch_variant<false>(p, DS3_BF16, mode, variant, nullptr, 0, &need, nullptr) != DS3_OK) return 0;
    return need;
}

}  // namespace ds3
