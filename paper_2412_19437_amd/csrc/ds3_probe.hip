// Two machine probes that put the GEMM's roofline figures in context: what the
// matrix pipe of THIS chip sustains with operands already in registers (its
// clock under full matrix load is well below the nominal one the published
// peak is quoted at), and how fast a compute unit can pull K-major operand
// rows from the L2 into LDS.  Neither touches the results of the library; the
// benchmark reports them next to the kernels it times.
#include "ds3_dev.h"
#include "ds3_internal.h"

namespace ds3 {

typedef __attribute__((address_space(3))) void* lds_ptr_t;

// 8 waves per compute unit, each chaining 32 independent FP8 16x16x128 MFMAs per
// iteration on fragments it loaded once: no LDS, no memory, no vector ALU work.
__global__ __launch_bounds__(512) void probe_mfma_kernel(float* out, int iters, unsigned seed) {
    const int lane = threadIdx.x & 63;
    i32x8 pf[4], qf[2];
    unsigned h = seed + threadIdx.x * 2654435761u;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) { h = h * 1664525u + 1013904223u; pf[i][e] = (int)(h & 0x7e7e7e7eu); }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) { h = h * 1664525u + 1013904223u; qf[i][e] = (int)(h & 0x7e7e7e7eu); }
    f32x4 acc[32];
#pragma unroll
    for (int i = 0; i < 32; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int s = 0; s < 32; ++s)
            acc[s] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(pf[s & 3], qf[(s >> 2) & 1], acc[s], 0, 0, 0, 0, 0, 0);
    }
    f32x4 t = acc[0];
#pragma unroll
    for (int i = 1; i < 32; ++i) { t.x += acc[i].x; t.y += acc[i].y; t.z += acc[i].z; t.w += acc[i].w; }
    if (lane == 0) out[(size_t)blockIdx.x * 8 + (threadIdx.x >> 6)] = t.x + t.y + t.z + t.w;
}

// Every workgroup (one per compute unit, 512 threads) streams 512 rows x 128 bytes per
// step -- the footprint of one K-step of a 256x256 tile -- from an L2-resident window
// into two alternating LDS stages with 16-byte LDS-direct loads, a barrier per step.  The
// loads of the next step are queued before the barrier waits for this step's (as the GEMM
// does): with nothing queued the figure is one L2 latency per step, not a feed rate.
__global__ __launch_bounds__(512) void probe_feed_kernel(const uint8_t* src, unsigned window, int row_stride, int iters,
                                                         unsigned* out) {
    __shared__ __attribute__((aligned(1024))) uint8_t smem[2 * 65536];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)src, 0, (int)window, 0x00020000);
    const unsigned panel = (blockIdx.x >> 3) & 7;                       // workgroups of an XCD share 8 row panels
    const unsigned voff0 = (panel * 512 + (tid >> 3)) * (unsigned)row_stride + (tid & 7) * 16;
    auto issue = [&](int it) {
        const unsigned kofs = ((unsigned)it * 128u) % (unsigned)row_stride;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            uint8_t* dst = smem + (it & 1) * 65536 + (i * 512 + wave * 64) * 16;
            // offsets beyond the window are range-checked by the descriptor and move no data
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_ptr_t)dst, 16, (int)(voff0 + i * 64 * row_stride + kofs), 0, 0, 0);
        }
    };
    issue(0);
    for (int it = 0; it < iters; ++it) {
        issue(it + 1);                                 // (one step more than asked for: it moves data nobody reads)
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(8 | 0x70);          // vmcnt(8): step `it` has landed, step it+1 stays in flight
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    }
    __builtin_amdgcn_s_waitcnt(0x70);                  // vmcnt(0)
    __syncthreads();
    const u32x4 v = *reinterpret_cast<const u32x4*>(smem + tid * 16);
    if (tid == 0) out[blockIdx.x] = v.x ^ v.y ^ v.z ^ v.w;
}

ds3_status launch_probe_mfma(int iters, float* out, int blocks, hipStream_t st) {
    (void)hipGetLastError();
    probe_mfma_kernel<<<dim3(blocks), dim3(512), 0, st>>>(out, iters, 12345u);
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

ds3_status launch_probe_feed(const void* src, unsigned window, int row_stride, int iters, unsigned* out, int blocks,
                             hipStream_t st) {
    (void)hipGetLastError();
    probe_feed_kernel<<<dim3(blocks), dim3(512), 0, st>>>((const uint8_t*)src, window, row_stride, iters, out);
    return hipGetLastError() == hipSuccess ? DS3_OK : DS3_ERR_LAUNCH;
}

}  // namespace ds3
