// Residual-magnitude measurement (paper Appendix B, the protocol behind Figure 2): for every
// decoded block the S = block + 1 states X^(0..S-1) of a backbone tensor (logits or hidden
// states of the block's positions, N entries each) give
//     ||X^(u) - X^(t)||_RMS for every t < u   (the residual delta_{t,r}, r = u - t)
//     ||X^(s)||_RMS                            (the reference magnitude)
// with ||Y||_RMS = sqrt(sum_i Y_i^2 / N), accumulated in fp64 as the paper prescribes, and then
// the mean over blocks and offsets t for every r.
//
// All S (S + 1) / 2 sums come out of ONE pass over the states: a workgroup stages a 512-entry
// tile of all S states in LDS (HBM traffic = every state once), every lane turns its entries of
// the S states to fp64 in registers, and the four waves split the jobs (job p goes to wave p mod
// 4), so a wave carries at most 39 fp64 accumulators.  Workgroup partials are summed in
// workgroup order by a second kernel: the result does not depend on timing.
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int RT = 512;            // entries of one state per tile
constexpr int RMS_MAX_PART = 4096; // workgroup partials the context's buffer holds (all blocks together)

// job (r, t): r = 0 is the plain magnitude of state t, r > 0 the pair (t, t + r)
__host__ __device__ constexpr int job_index(int S, int r, int t) { return r * S - r * (r - 1) / 2 + t; }

template <int S, int W>
__device__ __forceinline__ void accumulate(const double (&x)[S][2], double (&acc)[(S * (S + 1) / 2 + 3) / 4]) {
#pragma unroll
    for (int r = 0; r < S; ++r)
#pragma unroll
        for (int t = 0; t + r < S; ++t) {
            const int p = job_index(S, r, t);
            if ((p & 3) == W) {
                const double d0 = r == 0 ? x[t][0] : x[t + r][0] - x[t][0];
                const double d1 = r == 0 ? x[t][1] : x[t + r][1] - x[t][1];
                acc[p >> 2] = fma(d0, d0, acc[p >> 2]);
                acc[p >> 2] = fma(d1, d1, acc[p >> 2]);
            }
        }
}

__device__ __forceinline__ float bf16_val(uint32_t bits16) { return __uint_as_float(bits16 << 16); }

// X: [n_blocks][S][N]; part: [n_blocks][J][nwg] sums of squares
template <int S, bool BF16, bool VEC>
__global__ __launch_bounds__(256) void rms_partial_kernel(const void *__restrict__ X, long N, int nwg,
                                                          double *__restrict__ part) {
    constexpr int J = S * (S + 1) / 2, JA = (J + 3) / 4;
    __shared__ float tile[S][RT];
    const int blk = blockIdx.y, wg = blockIdx.x, tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const size_t base = (size_t)blk * S * N;
    double acc[JA];
#pragma unroll
    for (int j = 0; j < JA; ++j) acc[j] = 0.0;
    const long ntiles = (N + RT - 1) / RT;
    // the tile's items of 4 entries (VEC) or single entries, held in registers between the request
    // and the LDS store so that the next tile's requests are in flight while this one is computed
    constexpr int NV = VEC ? (S * (RT / 4) + 255) / 256 : (S * RT + 255) / 256;
    float4 rv[VEC ? NV : 1];
    float rs[VEC ? 1 : NV];
    auto request = [&](long tl) {
        const long e0 = tl * RT;
        if constexpr (VEC) {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const int idx = tid + 256 * n;
                const int s = idx / (RT / 4), c = idx % (RT / 4);
                const long e = e0 + 4 * c;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (idx < S * (RT / 4) && e < N) {   // (N % 4 == 0 here: an item is inside or outside as a whole)
                    if constexpr (BF16) {
                        const uint2 b = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(X) + base +
                                                                         (size_t)s * N + e);
                        v = make_float4(bf16_val(b.x & 0xFFFFu), bf16_val(b.x >> 16), bf16_val(b.y & 0xFFFFu),
                                        bf16_val(b.y >> 16));
                    } else {
                        v = *reinterpret_cast<const float4 *>(static_cast<const float *>(X) + base + (size_t)s * N + e);
                    }
                }
                rv[n] = v;
            }
        } else {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const int idx = tid + 256 * n;
                const int s = idx / RT, c = idx % RT;
                const long e = e0 + c;
                float v = 0.f;
                if (idx < S * RT && e < N) {
                    if constexpr (BF16) v = bf16_val(static_cast<const uint16_t *>(X)[base + (size_t)s * N + e]);
                    else v = static_cast<const float *>(X)[base + (size_t)s * N + e];
                }
                rs[n] = v;
            }
        }
    };
    auto stage = [&]() {
        if constexpr (VEC) {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const int idx = tid + 256 * n;
                if (idx < S * (RT / 4)) *reinterpret_cast<float4 *>(&tile[idx / (RT / 4)][4 * (idx % (RT / 4))]) = rv[n];
            }
        } else {
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const int idx = tid + 256 * n;
                if (idx < S * RT) tile[idx / RT][idx % RT] = rs[n];
            }
        }
    };
    if (wg < ntiles) request(wg);
    for (long tl = wg; tl < ntiles; tl += nwg) {
        stage();
        __syncthreads();
        if (tl + nwg < ntiles) request(tl + nwg);
#pragma unroll 1
        for (int it = 0; it < RT / 128; ++it) {
            const int c2 = (it * 64 + lane) * 2;
            double x[S][2];
#pragma unroll
            for (int s = 0; s < S; ++s) {
                const float2 v = *reinterpret_cast<const float2 *>(&tile[s][c2]);
                x[s][0] = (double)v.x;
                x[s][1] = (double)v.y;
            }
            // entries past N were staged as zeros in every state: they add nothing to any job
            switch (wave) {   // (uniform over the wave)
                case 0: accumulate<S, 0>(x, acc); break;
                case 1: accumulate<S, 1>(x, acc); break;
                case 2: accumulate<S, 2>(x, acc); break;
                default: accumulate<S, 3>(x, acc); break;
            }
        }
        __syncthreads();
    }
    // Sum over the 64 lanes of all JA accumulators at once: in the step with stride h a lane keeps
    // the half of its values selected by its lane bit h and hands the other half to its partner,
    // so after the six steps lane l holds the wave's total of accumulator l (63 exchanges in place
    // of 6 JA; a fixed tree).
    static_assert(JA <= 64, "one accumulator per lane at the end");
    double v[64];
#pragma unroll
    for (int j = 0; j < 64; ++j) v[j] = j < JA ? acc[j] : 0.0;
#pragma unroll
    for (int h = 32; h >= 1; h >>= 1) {
        const bool up = (lane & h) != 0;
#pragma unroll
        for (int j = 0; j < h; ++j) {
            const double keep = up ? v[h + j] : v[j];
            const double send = up ? v[j] : v[h + j];
            v[j] = keep + __shfl_xor(send, h);
        }
    }
    const int p = 4 * lane + wave;
    if (lane < JA && p < J) part[((size_t)blk * J + p) * nwg + wg] = v[0];
}

// fixed-order sum of n values by one wave: lane l adds entries l, l + 64, ... in order, then a
// butterfly over the lanes (the same tree whatever the timing)
template <typename F>
__device__ __forceinline__ double wave_sum(int n, F &&get) {
    const int lane = threadIdx.x & 63;
    double v = 0.0;
    int i = lane;
    for (; i + 3 * 64 < n; i += 4 * 64) {   // four loads in flight, added in index order
        const double a = get(i), b = get(i + 64), c = get(i + 128), d = get(i + 192);
        v += a; v += b; v += c; v += d;
    }
    for (; i < n; i += 64) v += get(i);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    return v;
}

// one wave per (block, job): workgroup (x = block, y) holds jobs 4 y .. 4 y + 3
__global__ __launch_bounds__(256) void rms_finish_kernel(const double *__restrict__ part, int S, long N, int nwg,
                                                         double *__restrict__ rms_pair) {
    const int blk = blockIdx.x, J = S * (S + 1) / 2, wave = threadIdx.x >> 6;
    double *out = rms_pair + (size_t)blk * S * S;
    if (blockIdx.y == 0)
        for (int i = threadIdx.x; i < S * S; i += 256)
            if (i / S > i % S) out[i] = 0.0;   // below the diagonal
    const int p = 4 * blockIdx.y + wave;
    if (p >= J) return;
    int r = 0, first = 0;   // job p = (r, t): jobs of offset r start at first
    while (p >= first + (S - r)) { first += S - r; ++r; }
    const int t = p - first;
    const double *src = part + ((size_t)blk * J + p) * nwg;
    const double sum = wave_sum(nwg, [&](int w) { return src[w]; });
    if ((threadIdx.x & 63) == 0) out[t * S + t + r] = sqrt(sum / (double)N);
}

// wave r: mean over blocks and offsets
__global__ __launch_bounds__(64) void rms_mean_kernel(const double *__restrict__ rms_pair, int n_blocks, int S,
                                                      double *__restrict__ rms_delta) {
    const int r = blockIdx.x;
    const int t0 = (r == 0) ? 1 : 0, nt = S - r - t0;   // offsets per block
    const int cnt = n_blocks * nt;
    const double sum = wave_sum(cnt, [&](int i) {
        const int b = i / nt, t = t0 + i % nt;
        return rms_pair[((size_t)b * S + t) * S + t + r];
    });
    if (threadIdx.x == 0) rms_delta[r] = cnt ? sum / (double)cnt : 0.0;
}

template <int S>
hipError_t launch_s(int n_blocks, long N, const void *X, bool bf16, bool vec, int nwg, double *part,
                    hipStream_t st) {
    const dim3 grid(nwg, n_blocks), block(256);
    if (bf16) {
        if (vec) hipLaunchKernelGGL((rms_partial_kernel<S, true, true>), grid, block, 0, st, X, N, nwg, part);
        else hipLaunchKernelGGL((rms_partial_kernel<S, true, false>), grid, block, 0, st, X, N, nwg, part);
    } else {
        if (vec) hipLaunchKernelGGL((rms_partial_kernel<S, false, true>), grid, block, 0, st, X, N, nwg, part);
        else hipLaunchKernelGGL((rms_partial_kernel<S, false, false>), grid, block, 0, st, X, N, nwg, part);
    }
    return hipGetLastError();
}

}  // namespace

size_t residual_rms_part_bytes() { return (size_t)RMS_MAX_PART * (17 * 18 / 2) * sizeof(double); }
int residual_rms_max_blocks() { return RMS_MAX_PART; }
bool residual_rms_supported(int S) { return S == 3 || S == 5 || S == 9 || S == 17; }

hipError_t launch_residual_rms(int n_blocks, int S, long N, const void *X, bool bf16, double *part,
                               double *rms_pair, double *rms_delta, hipStream_t st) {
    const long ntiles = (N + RT - 1) / RT;
    long nwg = RMS_MAX_PART / n_blocks;
    if (nwg > ntiles) nwg = ntiles;
    if (nwg < 1) nwg = 1;
    const uintptr_t a = reinterpret_cast<uintptr_t>(X);
    const bool vec = (N % 4 == 0) && (a % (bf16 ? 8 : 16) == 0);
    hipError_t e;
    switch (S) {
        case 3: e = launch_s<3>(n_blocks, N, X, bf16, vec, (int)nwg, part, st); break;
        case 5: e = launch_s<5>(n_blocks, N, X, bf16, vec, (int)nwg, part, st); break;
        case 9: e = launch_s<9>(n_blocks, N, X, bf16, vec, (int)nwg, part, st); break;
        case 17: e = launch_s<17>(n_blocks, N, X, bf16, vec, (int)nwg, part, st); break;
        default: return hipErrorInvalidValue;
    }
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rms_finish_kernel, dim3(n_blocks, (S * (S + 1) / 2 + 3) / 4), dim3(256), 0, st, part, S, N,
                       (int)nwg, rms_pair);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(rms_mean_kernel, dim3(S), dim3(64), 0, st, rms_pair, n_blocks, S, rms_delta);
    return hipGetLastError();
}

}  // namespace mrp
