// Measurement aid, not part of the method: moves the bytes of one LM-head launch at no more than
// 128 rows -- the packed weight stream and, optionally, the logit tile read and written back
// unchanged -- with the persistent LM-head kernel's work split and access pattern but none of its
// arithmetic (no MFMA, no activation stage, no reduction).  What this takes is the floor the memory
// system sets for that kernel's traffic mix; bench.py --workload lm_traffic reports it beside the
// kernel itself.
#include "mrp_kernels.h"

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// mode 0: weights only; 1: + logit tile read; 2: + logit tile written back (same values)
template <int MODE>
__global__ __launch_bounds__(512) void lm_traffic_kernel(const u32x4 *__restrict__ Wp, float *__restrict__ z, int KB,
                                                         int n_rb, int M, int V, unsigned *__restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, ln = lane & 31, lh = lane >> 5;
    const int rb_begin = (int)(((long)n_rb * blockIdx.x) / gridDim.x);
    const int rb_end = (int)(((long)n_rb * (blockIdx.x + 1)) / gridDim.x);
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int rb = rb_begin + wave; rb < rb_end; rb += 8) {
        float4 zt[16];
        if (MODE >= 1) {
#pragma unroll
            for (int it = 0; it < 4; ++it)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    int i = it * 32 + ln, v = rb * 32 + 8 * q + 4 * lh;
                    i = i < M ? i : M - 1;
                    v = v < V - 4 ? v : V - 4;
                    zt[it * 4 + q] = *reinterpret_cast<const float4 *>(z + (size_t)i * V + v);
                }
        }
        const u32x4 *wp = Wp + (size_t)rb * KB * 64 + lane;     // the block's weights: KB contiguous 1 KiB fragments
#pragma unroll 1
        for (int g = 0; g + 16 <= KB; g += 16) {
            u32x4 w[16];
#pragma unroll
            for (int j = 0; j < 16; ++j) w[j] = wp[(size_t)(g + j) * 64];
#pragma unroll
            for (int j = 0; j < 16; ++j) acc ^= w[j];
        }
        if (MODE >= 1) {
#pragma unroll
            for (int k = 0; k < 16; ++k) acc[0] ^= __float_as_uint(zt[k].y);
            if (MODE >= 2) {
#pragma unroll
                for (int it = 0; it < 4; ++it)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int i = it * 32 + ln, v = rb * 32 + 8 * q + 4 * lh;
                        if (i < M && v < V) *reinterpret_cast<float4 *>(z + (size_t)i * V + v) = zt[it * 4 + q];
                    }
            }
        }
    }
    if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x9E3779B9u) sink[0] = 1u;   // keeps the loads alive
}

}  // namespace

hipError_t launch_lm_traffic(int mode, const uint4 *Wp, float *z, int KB, int n_rb, int M, int V, int nWG,
                             unsigned *sink, hipStream_t st) {
    const u32x4 *w = reinterpret_cast<const u32x4 *>(Wp);
    if (mode == 0) hipLaunchKernelGGL(lm_traffic_kernel<0>, dim3(nWG), dim3(512), 0, st, w, z, KB, n_rb, M, V, sink);
    else if (mode == 1) hipLaunchKernelGGL(lm_traffic_kernel<1>, dim3(nWG), dim3(512), 0, st, w, z, KB, n_rb, M, V, sink);
    else hipLaunchKernelGGL(lm_traffic_kernel<2>, dim3(nWG), dim3(512), 0, st, w, z, KB, n_rb, M, V, sink);
    return hipGetLastError();
}

}  // namespace mrp
