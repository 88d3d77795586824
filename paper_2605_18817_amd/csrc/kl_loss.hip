// Training-side loss of the MRP head (paper Section 3.3, Equation 3): per masked row
//     L_i = KL( softmax(l_{t-1}[i]) || softmax(l_t[i] + delta_t[i]) )
// and its gradient with respect to the student logits (hence to delta_t),
//     dL_i / ds[i][v] = softmax(s[i])[v] - softmax(l_{t-1}[i])[v],
// with teacher T = l_{t-1} and student S = l_t + delta_t given as fp32 [M][V].
//
// Like the chain's reductions it is a pure HBM stream.  Forward: one pass over both
// tensors; every (row, 8192-wide vocabulary tile) keeps the online partial
//     (m_T, s_T = sum e^{T - m_T}, a_T = sum e^{T - m_T} (T - S),  m_S, s_S = sum e^{S - m_S})
// and a second tiny kernel merges a row's partials in a fixed order:
//     L_i = a_T / s_T - (m_T + log s_T) + (m_S + log s_S).
// No softmax is written.  Backward: one more pass that reads both tensors and writes the
// gradient from the two row log-sum-exps.  Algorithmic bytes: 8 M V forward,
// 8 M V + 4 M V backward.
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int KT = 8192;   // vocabulary entries per workgroup

struct KlPart {
    float mT, sT, aT, mS, sS;
};

__device__ __forceinline__ KlPart kl_identity() { return {-INFINITY, 0.f, 0.f, -INFINITY, 0.f}; }

__device__ __forceinline__ KlPart kl_merge(const KlPart &x, const KlPart &y) {
    KlPart r;
    r.mT = fmaxf(x.mT, y.mT);
    const float fx = (x.mT == -INFINITY) ? 0.f : __expf(x.mT - r.mT);
    const float fy = (y.mT == -INFINITY) ? 0.f : __expf(y.mT - r.mT);
    r.sT = x.sT * fx + y.sT * fy;
    r.aT = x.aT * fx + y.aT * fy;
    r.mS = fmaxf(x.mS, y.mS);
    const float gx = (x.mS == -INFINITY) ? 0.f : __expf(x.mS - r.mS);
    const float gy = (y.mS == -INFINITY) ? 0.f : __expf(y.mS - r.mS);
    r.sS = x.sS * gx + y.sS * gy;
    return r;
}

__device__ __forceinline__ KlPart kl_shfl_xor(const KlPart &p, int off) {
    return {__shfl_xor(p.mT, off), __shfl_xor(p.sT, off), __shfl_xor(p.aT, off), __shfl_xor(p.mS, off),
            __shfl_xor(p.sS, off)};
}

// partial of one KT-wide tile of one row; partial (t, i) of array a lives at a[i * nT + t]
template <bool VEC4>
__global__ __launch_bounds__(256) void kl_partial_kernel(const float *__restrict__ T, const float *__restrict__ S,
                                                         const uint8_t *__restrict__ mask, int V,
                                                         float *__restrict__ part, size_t stride) {
    __shared__ KlPart sw[4];
    const int t = blockIdx.x, i = blockIdx.y;
    if (mask && !mask[i]) return;   // (uniform over the workgroup)
    const float *tr = T + (size_t)i * V, *sr = S + (size_t)i * V;
    const int v0 = t * KT;
    float xt[32], xs[32];
    if constexpr (VEC4) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int v = v0 + 4 * (threadIdx.x + 256 * n);
            float4 a = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY), b = a;
            if (v < V) {
                a = *reinterpret_cast<const float4 *>(tr + v);
                b = *reinterpret_cast<const float4 *>(sr + v);
            }
            xt[4 * n] = a.x; xt[4 * n + 1] = a.y; xt[4 * n + 2] = a.z; xt[4 * n + 3] = a.w;
            xs[4 * n] = b.x; xs[4 * n + 1] = b.y; xs[4 * n + 2] = b.z; xs[4 * n + 3] = b.w;
        }
    } else {
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            const int v = v0 + threadIdx.x + 256 * n;
            xt[n] = (v < V) ? tr[v] : -INFINITY;
            xs[n] = (v < V) ? sr[v] : -INFINITY;
        }
    }
    KlPart p = kl_identity();
#pragma unroll
    for (int n = 0; n < 32; ++n) { p.mT = fmaxf(p.mT, xt[n]); p.mS = fmaxf(p.mS, xs[n]); }
    if (p.mT > -INFINITY) {
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            if (xt[n] > -INFINITY) {   // (padding past V is -inf in both tensors: skip, T - S would be NaN)
                const float e = __expf(xt[n] - p.mT);
                p.sT += e;
                p.aT += e * (xt[n] - xs[n]);
                p.sS += __expf(xs[n] - p.mS);
            }
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) p = kl_merge(p, kl_shfl_xor(p, off));
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) sw[wave] = p;
    __syncthreads();
    if (threadIdx.x == 0) {
        p = sw[0];
        for (int w = 1; w < 4; ++w) p = kl_merge(p, sw[w]);
        const size_t o = (size_t)i * gridDim.x + t;
        part[o] = p.mT; part[stride + o] = p.sT; part[2 * stride + o] = p.aT;
        part[3 * stride + o] = p.mS; part[4 * stride + o] = p.sS;
    }
}

// one thread per row: merge the row's partials in tile order
__global__ __launch_bounds__(256) void kl_finish_kernel(const float *__restrict__ part, size_t stride, int nT, int M,
                                                        const uint8_t *__restrict__ mask, float scale,
                                                        float *__restrict__ loss_rows, float *__restrict__ lse) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= M) return;
    if (mask && !mask[i]) {
        loss_rows[i] = 0.f;
        lse[i] = 0.f; lse[M + i] = 0.f;
        return;
    }
    KlPart p = kl_identity();
    for (int t = 0; t < nT; ++t) {
        const size_t o = (size_t)i * nT + t;
        p = kl_merge(p, KlPart{part[o], part[stride + o], part[2 * stride + o], part[3 * stride + o],
                               part[4 * stride + o]});
    }
    const float lseT = p.mT + logf(p.sT), lseS = p.mS + logf(p.sS);
    loss_rows[i] = scale * (p.aT / p.sT - lseT + lseS);
    lse[i] = lseT; lse[M + i] = lseS;
}

template <bool VEC4>
__global__ __launch_bounds__(256) void kl_grad_kernel(const float *__restrict__ T, const float *__restrict__ S,
                                                      const uint8_t *__restrict__ mask, int V, int M,
                                                      const float *__restrict__ lse, float scale,
                                                      float *__restrict__ grad) {
    const int t = blockIdx.x, i = blockIdx.y;
    const bool on = !mask || mask[i];
    const float lT = lse[i], lS = lse[M + i];
    const size_t ro = (size_t)i * V;
    const int v0 = t * KT;
    if constexpr (VEC4) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int v = v0 + 4 * (threadIdx.x + 256 * n);
            if (v < V) {
                float4 g = make_float4(0.f, 0.f, 0.f, 0.f);
                if (on) {
                    const float4 a = *reinterpret_cast<const float4 *>(T + ro + v);
                    const float4 b = *reinterpret_cast<const float4 *>(S + ro + v);
                    g.x = scale * (__expf(b.x - lS) - __expf(a.x - lT));
                    g.y = scale * (__expf(b.y - lS) - __expf(a.y - lT));
                    g.z = scale * (__expf(b.z - lS) - __expf(a.z - lT));
                    g.w = scale * (__expf(b.w - lS) - __expf(a.w - lT));
                }
                *reinterpret_cast<float4 *>(grad + ro + v) = g;
            }
        }
    } else {
#pragma unroll 4
        for (int n = 0; n < 32; ++n) {
            const int v = v0 + threadIdx.x + 256 * n;
            if (v < V) grad[ro + v] = on ? scale * (__expf(S[ro + v] - lS) - __expf(T[ro + v] - lT)) : 0.f;
        }
    }
}

}  // namespace

int kl_tiles(int V) { return (V + KT - 1) / KT; }

hipError_t launch_kl_loss(int M, int V, const float *teacher, const float *student, const uint8_t *mask, float scale,
                          float *part, size_t part_stride, float *lse, float *loss_rows, float *grad,
                          hipStream_t st) {
    const int nT = kl_tiles(V);
    if (V % 4 == 0)
        hipLaunchKernelGGL(kl_partial_kernel<true>, dim3(nT, M), dim3(256), 0, st, teacher, student, mask, V, part,
                           part_stride);
    else
        hipLaunchKernelGGL(kl_partial_kernel<false>, dim3(nT, M), dim3(256), 0, st, teacher, student, mask, V, part,
                           part_stride);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kl_finish_kernel, dim3((M + 255) / 256), dim3(256), 0, st, part, part_stride, nT, M, mask,
                       scale, loss_rows, lse);
    e = hipGetLastError();
    if (e != hipSuccess || !grad) return e;
    if (V % 4 == 0)
        hipLaunchKernelGGL(kl_grad_kernel<true>, dim3(nT, M), dim3(256), 0, st, teacher, student, mask, V, M, lse,
                           scale, grad);
    else
        hipLaunchKernelGGL(kl_grad_kernel<false>, dim3(nT, M), dim3(256), 0, st, teacher, student, mask, V, M, lse,
                           scale, grad);
    return hipGetLastError();
}

}  // namespace mrp
