// The MLP body of an MRP head at a small number of activation rows (below 768) (paper Section 3.2 and
// Algorithm 2, inner loop: u = W2 SiLU(W1 [h ; e])) as two launches with no
// partial sums in memory: each GEMM reduces its k split inside the workgroup
// through LDS, the first reads the conditioning embedding straight from the
// embedding table and applies the SiLU in its epilogue, the second writes u.
// The second kernel is a plain small-row GEMM and also serves the projections
// of the transformer head body (Section 4.5).
//
// A workgroup of 8 wavefronts owns one output tile of 32 activation rows x 32
// features (64 features when there are more 32-feature tiles than CUs: a
// workgroup's activation fragments then serve two weight row blocks); wave w
// takes the 16-wide k blocks kb = w, w + 8, ... of the tile's weight rows, which
// it streams from HBM fragment by fragment (1 KiB each, used once), together
// with the matching activation fragments from L2.  The grid is
// (d / tile features) x ceil(M / 32) workgroups.
#include "mrp_kernels.h"

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int HF_WAVES = 8;
constexpr int HF_THREADS = 64 * HF_WAVES;
constexpr int HF_CH = 4;    // k blocks per chunk
constexpr int HF_PAD = 4;    // floats of padding per row of a wave's partial tile in LDS (conflict-free float4 rows)

__device__ __forceinline__ f32x16 mma16(const u32x4 &w, const u32x4 &x, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
}

// Sum of the 8 waves' partial tiles for (row, 8-feature chunk c), in wave order.  LD: floats per tile row.
template <int LD>
__device__ __forceinline__ void reduce_chunk(const float (*tile)[32][LD], int row, int c, float (&x)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = 0.f;
#pragma unroll
    for (int w = 0; w < HF_WAVES; ++w) {
        const float4 a = *reinterpret_cast<const float4 *>(&tile[w][row][8 * c]);
        const float4 b = *reinterpret_cast<const float4 *>(&tile[w][row][8 * c + 4]);
        x[0] += a.x; x[1] += a.y; x[2] += a.z; x[3] += a.w;
        x[4] += b.x; x[5] += b.y; x[6] += b.z; x[7] += b.w;
    }
}

// A wave's accumulators of feature block f (lane = activation row ln, features 8q + 4lh + e) -> its partial tile in LDS
template <int LD>
__device__ __forceinline__ void spill_tile(float (*t)[LD], const f32x16 &acc, int f, int ln, int lh) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
        *reinterpret_cast<float4 *>(&t[ln][32 * f + 8 * q + 4 * lh]) =
            make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
}

// acc[f] += sum over this wave's k blocks kb = wave + 8 j (j < nj) of  Wfrag_f(kb0 + kb) * (sum of the
// activation planes' fragments of k block kb), for the NF weight row blocks of the tile.  wrow: the
// tile's first packed weight row block + lane, wstride: u32x4 between row blocks; x0: plane 0 + row block
// offset + lane; k block kb of plane p is at x0 + p * pstride + kb * kstride.  The k blocks come in
// chunks of HF_CH, one chunk fetched while the previous one is multiplied (weight fragments from HBM,
// activation fragments from L2).
template <int NF, int NP>
__device__ __forceinline__ void wave_gemm_planes(f32x16 (&acc)[NF], const u32x4 *wrow, size_t wstride, int kb0,
                                                 const u32x4 *x0, long pstride, size_t kstride, int nj, int wave) {
    u32x4 w[2][HF_CH][NF], x[2][HF_CH][NP];
    auto fetch = [&](int buf, int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u) {
            const int j = j0 + u < nj ? j0 + u : nj - 1;
            const int kb = wave + HF_WAVES * j;
#pragma unroll
            for (int f = 0; f < NF; ++f) w[buf][u][f] = wrow[f * wstride + (size_t)(kb0 + kb) * 64];
#pragma unroll
            for (int p = 0; p < NP; ++p) x[buf][u][p] = x0[(size_t)p * pstride + (size_t)kb * kstride];
        }
    };
    auto compute = [&](int buf, int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u)
            if (j0 + u < nj) {
#pragma unroll
                for (int p = 0; p < NP; ++p)
#pragma unroll
                    for (int f = 0; f < NF; ++f) acc[f] = mma16(w[buf][u][f], x[buf][u][p], acc[f]);
            }
    };
    auto compute_whole = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u)
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[f] = mma16(w[buf][u][f], x[buf][u][p], acc[f]);
    };
    // Whole pairs of chunks run without a condition on the fetches (past the end the last k block is fetched
    // again and not used): a fetch under a condition makes the compiler wait for every load at the loop's end,
    // and the scheduling barriers keep it from sinking the fetches below the MFMAs that hide them.
    fetch(0, 0);
    int j0 = 0;
    for (; j0 + 2 * HF_CH <= nj; j0 += 2 * HF_CH) {
        fetch(1, j0 + HF_CH);
        __builtin_amdgcn_sched_barrier(0);
        compute_whole(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(0, j0 + 2 * HF_CH);
        __builtin_amdgcn_sched_barrier(0);
        compute_whole(1);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (j0 < nj) {     // fewer than two chunks left; set 0 holds the first of them
        if (j0 + HF_CH < nj) fetch(1, j0 + HF_CH);
        compute(0, j0);
        if (j0 + HF_CH < nj) compute(1, j0 + HF_CH);
    }
}
// The conditioning half: the activation fragment of row i, k block kb is 16 bytes of the embedding
// row of the token that conditions row i's sequence (bf16 in the table, converted to the fp16 the head
// body's matrix cores take).  erow: that embedding row + this lane's 8-column half.
template <int NF>
__device__ __forceinline__ void wave_gemm_embed(f32x16 (&acc)[NF], const u32x4 *wrow, size_t wstride, int kb0,
                                                const uint4 *erow, int nj, int wave) {
    u32x4 w[2][HF_CH][NF];
    uint4 x[2][HF_CH];
    auto fetch = [&](int buf, int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u) {
            const int j = j0 + u < nj ? j0 + u : nj - 1;
            const int kb = wave + HF_WAVES * j;
#pragma unroll
            for (int f = 0; f < NF; ++f) w[buf][u][f] = wrow[f * wstride + (size_t)(kb0 + kb) * 64];
            x[buf][u] = erow[2 * kb];
        }
    };
    auto compute = [&](int buf, int j0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u)
            if (j0 + u < nj) {
                const uint4 fx = bf16x8_to_f16x8(x[buf][u]);
#pragma unroll
                for (int f = 0; f < NF; ++f) acc[f] = mma16(w[buf][u][f], __builtin_bit_cast(u32x4, fx), acc[f]);
            }
    };
    auto compute_whole = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < HF_CH; ++u) {
            const uint4 fx = bf16x8_to_f16x8(x[buf][u]);
#pragma unroll
            for (int f = 0; f < NF; ++f) acc[f] = mma16(w[buf][u][f], __builtin_bit_cast(u32x4, fx), acc[f]);
        }
    };
    // Whole pairs of chunks run without a condition on the fetches (past the end the last k block is fetched
    // again and not used): a fetch under a condition makes the compiler wait for every load at the loop's end,
    // and the scheduling barriers keep it from sinking the fetches below the MFMAs that hide them.
    fetch(0, 0);
    int j0 = 0;
    for (; j0 + 2 * HF_CH <= nj; j0 += 2 * HF_CH) {
        fetch(1, j0 + HF_CH);
        __builtin_amdgcn_sched_barrier(0);
        compute_whole(0);
        __builtin_amdgcn_sched_barrier(0);
        fetch(0, j0 + 2 * HF_CH);
        __builtin_amdgcn_sched_barrier(0);
        compute_whole(1);
        __builtin_amdgcn_sched_barrier(0);
    }
    if (j0 < nj) {     // fewer than two chunks left; set 0 holds the first of them
        if (j0 + HF_CH < nj) fetch(1, j0 + HF_CH);
        compute(0, j0);
        if (j0 + HF_CH < nj) compute(1, j0 + HF_CH);
    }
}

// workgroup -> tile: consecutive ids go to different XCDs (8, each with its own L2); the row tiles of
// one feature tile share its weight rows, so they sit on one XCD
__device__ __forceinline__ bool tile_of(int nct, int nrt, int &rt, int &ct) {
    const int nWG = nct * nrt;
    const int per = (nWG + 7) >> 3;
    const int w_id = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    rt = w_id % nrt;
    ct = w_id / nrt;
    return w_id < nWG;
}

// s = SiLU(W1 [h ; e]) as fp16 planes; nct = d / (32 NF) feature tiles
template <int NF>
__device__ __forceinline__ void head_gemm1_body(const HeadFusedArgs &a) {
    constexpr int LD = 32 * NF + HF_PAD;
    __shared__ float tile[HF_WAVES][32][LD];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, lh = lane >> 5;
    int rt, ct;
    if (!tile_of(a.nct, a.nrt, rt, ct)) return;
    const int KBd = a.d >> 4;          // k blocks per d columns
    const int nj = KBd / HF_WAVES;     // k blocks per wave per d columns (d % 128 == 0)
    const size_t kstride = (size_t)a.nIb * 64;
    {
        f32x16 acc[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][r] = 0.f;
        const size_t wstride = (size_t)(2 * KBd) * 64;
        const u32x4 *wrow = reinterpret_cast<const u32x4 *>(a.W1p) + (size_t)ct * NF * wstride + lane;
        const u32x4 *xh = reinterpret_cast<const u32x4 *>(a.XH) + (size_t)rt * 64 + lane;
        // the sequence of this lane's row, its conditioning token (a bad one is clamped and reported)
        int i = rt * 32 + ln;
        i = i < a.M ? i : a.M - 1;
        int tok = a.cond_tok[i / a.L];
        if ((tok < 0 || tok >= a.V) && ct == 0 && a.err_flag) atomicOr(a.err_flag, ERR_COND_TOK);
        tok = tok < 0 ? 0 : (tok >= a.V ? a.V - 1 : tok);
        const uint4 *erow = reinterpret_cast<const uint4 *>(a.E + (size_t)tok * a.d) + lh;
        if (a.np_h == 2) wave_gemm_planes<NF, 2>(acc, wrow, wstride, 0, xh, a.plane, kstride, nj, wave);
        else wave_gemm_planes<NF, 1>(acc, wrow, wstride, 0, xh, a.plane, kstride, nj, wave);
        wave_gemm_embed<NF>(acc, wrow, wstride, KBd, erow, nj, wave);
#pragma unroll
        for (int f = 0; f < NF; ++f) spill_tile<LD>(tile[wave], acc[f], f, ln, lh);
    }
    __syncthreads();
    if (tid < 128 * NF) {
        const int row = tid & 31, c = tid >> 5;    // 8-feature chunk c of the tile
        const int i = rt * 32 + row;
        float x[8];
        reduce_chunk<LD>(tile, row, c, x);
        if (i < a.M) {
#pragma unroll
            for (int e = 0; e < 8; ++e) x[e] = x[e] / (1.0f + expf(-x[e]));
            split_store(x, a.S, act_chunk_index(i, ct * 4 * NF + c, a.nIb), a.plane);
        }
    }
}

__global__ __launch_bounds__(HF_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void head_gemm1_kernel(
    const HeadFusedArgs a) {
    head_gemm1_body<1>(a);
}
__global__ __launch_bounds__(HF_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void head_gemm1_kernel_64(
    const HeadFusedArgs a) {
    head_gemm1_body<2>(a);
}

// out [M][R] fp32 = X W^T for packed fp16 weights [R / 32][Kc / 16][64] and an activation of one or two
// fp16 planes (the head's second GEMM u = W2 s, and the projections of the transformer body);
// nct = R / (32 NF) feature tiles
template <int NF>
__device__ __forceinline__ void small_gemm_body(const SmallGemmArgs &a) {
    constexpr int LD = 32 * NF + HF_PAD;
    __shared__ float tile[HF_WAVES][32][LD];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, lh = lane >> 5;
    int rt, ct;
    if (!tile_of(a.nct, a.nrt, rt, ct)) return;
    const int KB = a.Kc >> 4;
    const int nj = KB / HF_WAVES;   // (Kc % 128 == 0)
    const size_t kstride = (size_t)a.nIb * 64;
    {
        f32x16 acc[NF];
#pragma unroll
        for (int f = 0; f < NF; ++f)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[f][r] = 0.f;
        const size_t wstride = (size_t)KB * 64;
        const u32x4 *wrow = reinterpret_cast<const u32x4 *>(a.Wp) + (size_t)ct * NF * wstride + lane;
        const u32x4 *xs = reinterpret_cast<const u32x4 *>(a.X) + (size_t)rt * 64 + lane;
        if (a.nplanes == 2) wave_gemm_planes<NF, 2>(acc, wrow, wstride, 0, xs, a.plane, kstride, nj, wave);
        else wave_gemm_planes<NF, 1>(acc, wrow, wstride, 0, xs, a.plane, kstride, nj, wave);
#pragma unroll
        for (int f = 0; f < NF; ++f) spill_tile<LD>(tile[wave], acc[f], f, ln, lh);
    }
    __syncthreads();
    if (tid < 128 * NF) {
        const int row = tid & 31, c = tid >> 5;
        const int i = rt * 32 + row;
        float u[8];
        reduce_chunk<LD>(tile, row, c, u);
        if (i < a.M) {
            float4 *up = reinterpret_cast<float4 *>(a.out + (size_t)i * a.R + 32 * NF * ct + 8 * c);
            up[0] = make_float4(u[0], u[1], u[2], u[3]);
            up[1] = make_float4(u[4], u[5], u[6], u[7]);
        }
    }
}

__global__ __launch_bounds__(HF_THREADS) __attribute__((amdgpu_waves_per_eu(4, 4))) void small_gemm_kernel(
    const SmallGemmArgs a) {
    small_gemm_body<1>(a);
}
__global__ __launch_bounds__(HF_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void small_gemm_kernel_64(
    const SmallGemmArgs a) {
    small_gemm_body<2>(a);
}

}  // namespace

// 64-feature tiles (a.nf = 2) once there are more 32-feature tiles than CUs; a.nct counts tiles of 32 a.nf features
hipError_t launch_small_gemm(const SmallGemmArgs &a, hipStream_t st) {
    const int per = (a.nct * a.nrt + 7) / 8;
    if (a.nf == 2) hipLaunchKernelGGL(small_gemm_kernel_64, dim3(per * 8), dim3(HF_THREADS), 0, st, a);
    else hipLaunchKernelGGL(small_gemm_kernel, dim3(per * 8), dim3(HF_THREADS), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_head_fused(const HeadFusedArgs &a, hipStream_t st) {
    const int per = (a.nct * a.nrt + 7) / 8;
    if (a.nf == 2) hipLaunchKernelGGL(head_gemm1_kernel_64, dim3(per * 8), dim3(HF_THREADS), 0, st, a);
    else hipLaunchKernelGGL(head_gemm1_kernel, dim3(per * 8), dim3(HF_THREADS), 0, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    SmallGemmArgs g;
    g.Wp = a.W2p; g.X = a.S; g.plane = a.plane; g.nplanes = NSPLIT; g.out = a.U;
    g.nIb = a.nIb; g.M = a.M; g.R = a.d; g.Kc = a.d; g.nct = a.nct; g.nrt = a.nrt; g.nf = a.nf;
    return launch_small_gemm(g, st);
}

}  // namespace mrp
