// Small per-row kernels around the stream GEMM: weight packing, activation
// packing (with the two-term fp16 split of fp32 activations), the SiLU
// between the head's two linear layers, and the RMSNorm that produces the bf16
// LM-head operand together with the hidden-state carry h <- h + Delta
// (paper Algorithm 2, inner loop).
#include "mrp_kernels.h"

namespace mrp {

namespace {

__global__ __launch_bounds__(256) void pack_weight_kernel(const uint16_t *__restrict__ src, int rows, int cols,
                                                          uint4 *__restrict__ dst, size_t nchunks, bool to_f16) {
    const size_t ci = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (ci >= nchunks) return;
    const int KB = cols >> 4;
    const int lane = (int)(ci & 63);
    const size_t blk = ci >> 6;
    const int kb = (int)(blk % KB);
    const int rb = (int)(blk / KB);
    const int row = rb * 32 + (lane & 31);
    const int col = kb * 16 + 8 * (lane >> 5);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row < rows) v = *reinterpret_cast<const uint4 *>(src + (size_t)row * cols + col);
    dst[ci] = to_f16 ? bf16x8_to_f16x8(v) : v;
}

// from_h: hrun <- fp32(h), plane 0 <- fp16(h).  else: planes <- split2(hrun).
__global__ __launch_bounds__(256) void init_hidden_kernel(const uint16_t *__restrict__ h, float *__restrict__ hrun,
                                                          uint4 *__restrict__ xh, long plane_stride, int nIb, int M,
                                                          int d, bool from_h) {
    int i, c8;
    if (!plane_block_lane((size_t)blockIdx.x * 4 + (threadIdx.x >> 6), d >> 4, M, i, c8)) return;
    const size_t dst = act_chunk_index(i, c8, nIb);
    if (from_h) {
        const uint4 v = *reinterpret_cast<const uint4 *>(h + (size_t)i * d + 8 * c8);
        float x[8];
        unpack_bf16x8(v, x);
        float4 *hp = reinterpret_cast<float4 *>(hrun + (size_t)i * d + 8 * c8);
        hp[0] = make_float4(x[0], x[1], x[2], x[3]);
        hp[1] = make_float4(x[4], x[5], x[6], x[7]);
        xh[dst] = bf16x8_to_f16x8(v);
    } else {
        const float4 *hp = reinterpret_cast<const float4 *>(hrun + (size_t)i * d + 8 * c8);
        const float4 a = hp[0], b = hp[1];
        const float x[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
        split_store(x, xh, dst, plane_stride);
    }
}

__global__ __launch_bounds__(256) void gather_e_kernel(const uint16_t *__restrict__ E,
                                                       const int32_t *__restrict__ cond_tok, uint4 *__restrict__ xe,
                                                       int nIb, int L, int d, int V, int *err_flag) {
    const int b = blockIdx.x;
    const int C8 = d >> 3;
    int tokc = cond_tok[b];  // caller contract: 0 <= cond_tok < V; a bad value is clamped and reported
    if ((tokc < 0 || tokc >= V) && threadIdx.x == 0 && err_flag) atomicOr(err_flag, ERR_COND_TOK);
    tokc = tokc < 0 ? 0 : (tokc >= V ? V - 1 : tokc);
    const uint4 *erow = reinterpret_cast<const uint4 *>(E + (size_t)tokc * d);
    for (int c8 = threadIdx.x; c8 < C8; c8 += 256) {
        const uint4 v = bf16x8_to_f16x8(erow[c8]);
        for (int p = 0; p < L; ++p) xe[act_chunk_index(b * L + p, c8, nIb)] = v;
    }
}

__global__ __launch_bounds__(256) void silu_split_kernel(const float *__restrict__ part, int nKs,
                                                         uint4 *__restrict__ s_planes, long plane_stride, int nIb,
                                                         int M, int d) {
    int i, c8;
    if (!plane_block_lane((size_t)blockIdx.x * 4 + (threadIdx.x >> 6), d >> 4, M, i, c8)) return;
    float x[8];
    sum_partials(part, (size_t)M * d, nKs, (size_t)i * d + 8 * c8, x);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = x[e] / (1.0f + expf(-x[e]));  // SiLU
    split_store(x, s_planes, act_chunk_index(i, c8, nIb), plane_stride);
}

constexpr int NORM_MAX_CHUNKS = 4;  // per thread: d <= 8 * 256 * 4 = 8192

// One workgroup per row: u = sum of k-split partials, RMSNorm -> bf16 y (packed),
// h_run += u and the split planes of the new h_run for the next head.
__global__ __launch_bounds__(256) void norm_kernel(const float *__restrict__ part, int nKs,
                                                   const float *__restrict__ resid,
                                                   const uint16_t *__restrict__ gamma, float eps,
                                                   float *__restrict__ hrun, bool carry, uint4 *__restrict__ y,
                                                   uint4 *__restrict__ xh, long plane_stride, int nIb, int M, int d) {
    __shared__ float wsum[4];
    const int i = xcd_row_of(blockIdx.x);
    if (i >= M) return;   // (uniform over the workgroup)
    const int C8 = d >> 3;
    float u[NORM_MAX_CHUNKS][8];
    float4 hv[NORM_MAX_CHUNKS][2];   // the row of h_run, requested with u (one round trip instead of two)
    float ss = 0.f;
#pragma unroll
    for (int n = 0; n < NORM_MAX_CHUNKS; ++n) {
        const int c8 = threadIdx.x + 256 * n;
#pragma unroll
        for (int e = 0; e < 8; ++e) u[n][e] = 0.f;
        hv[n][0] = hv[n][1] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (c8 < C8) {
            if (carry) {
                const float4 *hp = reinterpret_cast<const float4 *>(hrun + (size_t)i * d + 8 * c8);
                hv[n][0] = hp[0];
                hv[n][1] = hp[1];
            }
            sum_partials(part, (size_t)M * d, nKs, (size_t)i * d + 8 * c8, u[n]);
            if (resid) {   // transformer body: u = residual stream + last projection
                const float4 *rp = reinterpret_cast<const float4 *>(resid + (size_t)i * d + 8 * c8);
                const float4 a = rp[0], b = rp[1];
                u[n][0] += a.x; u[n][1] += a.y; u[n][2] += a.z; u[n][3] += a.w;
                u[n][4] += b.x; u[n][5] += b.y; u[n][6] += b.z; u[n][7] += b.w;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += u[n][e] * u[n][e];
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = ss;
    __syncthreads();
    ss = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]);
    const float inv = 1.0f / sqrtf(ss / (float)d + eps);
#pragma unroll
    for (int n = 0; n < NORM_MAX_CHUNKS; ++n) {
        const int c8 = threadIdx.x + 256 * n;
        if (c8 < C8) {
            float g[8];
            unpack_bf16x8(*reinterpret_cast<const uint4 *>(gamma + 8 * c8), g);
            uint16_t yb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) yb[e] = f32_to_bf16_rne(u[n][e] * inv * g[e]);
            const size_t dst = act_chunk_index(i, c8, nIb);
            y[dst] = make_uint4(pack2(yb[0], yb[1]), pack2(yb[2], yb[3]), pack2(yb[4], yb[5]), pack2(yb[6], yb[7]));
            if (carry) {
                float4 *hp = reinterpret_cast<float4 *>(hrun + (size_t)i * d + 8 * c8);
                const float4 a = hv[n][0], b = hv[n][1];
                const float x[8] = {a.x + u[n][0], a.y + u[n][1], a.z + u[n][2], a.w + u[n][3],
                                    b.x + u[n][4], b.y + u[n][5], b.z + u[n][6], b.w + u[n][7]};
                hp[0] = make_float4(x[0], x[1], x[2], x[3]);
                hp[1] = make_float4(x[4], x[5], x[6], x[7]);
                split_store(x, xh, dst, plane_stride);
            }
        }
    }
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }
// workgroups of 4 waves, one (k block, row block) unit per wave
inline unsigned plane_blocks(int M, int cols) { return (unsigned)(((size_t)((M + 31) / 32) * (cols / 16) + 3) / 4); }
// one workgroup per row, rows padded to whole XCD rounds of 32-row blocks
inline unsigned xcd_row_blocks(int M) { return (unsigned)((M + 255) / 256 * 256); }

}  // namespace

hipError_t launch_pack_weight(const uint16_t *src, int rows, int cols, uint4 *dst, bool to_f16, hipStream_t st) {
    const size_t rpad = ((size_t)rows + 31) / 32 * 32;
    const size_t nchunks = rpad * cols / 8;
    hipLaunchKernelGGL(pack_weight_kernel, dim3(blocks_for(nchunks)), dim3(256), 0, st, src, rows, cols, dst,
                       nchunks, to_f16);
    return hipGetLastError();
}

hipError_t launch_init_hidden(const uint16_t *h, float *hrun, uint4 *xh, long plane_stride, int nIb, int M,
                              int d, bool from_h, hipStream_t st) {
    hipLaunchKernelGGL(init_hidden_kernel, dim3(plane_blocks(M, d)), dim3(256), 0, st, h, hrun, xh,
                       plane_stride, nIb, M, d, from_h);
    return hipGetLastError();
}

hipError_t launch_gather_e(const uint16_t *E, const int32_t *cond_tok, uint4 *xe, int nIb, int B, int L, int d,
                           int V, int *err_flag, hipStream_t st) {
    hipLaunchKernelGGL(gather_e_kernel, dim3(B), dim3(256), 0, st, E, cond_tok, xe, nIb, L, d, V, err_flag);
    return hipGetLastError();
}

hipError_t launch_silu_split(const float *part, int nKs, uint4 *s_planes, long plane_stride, int nIb, int M,
                             int d, hipStream_t st) {
    hipLaunchKernelGGL(silu_split_kernel, dim3(plane_blocks(M, d)), dim3(256), 0, st, part, nKs,
                       s_planes, plane_stride, nIb, M, d);
    return hipGetLastError();
}

hipError_t launch_norm(const float *part, int nKs, const float *resid, const uint16_t *gamma, float eps, float *hrun,
                       bool carry, uint4 *y, uint4 *xh, long plane_stride, int nIb, int M, int d, hipStream_t st) {
    hipLaunchKernelGGL(norm_kernel, dim3(xcd_row_blocks(M)), dim3(256), 0, st, part, nKs, resid, gamma, eps, hrun, carry, y, xh,
                       plane_stride, nIb, M, d);
    return hipGetLastError();
}

}  // namespace mrp
