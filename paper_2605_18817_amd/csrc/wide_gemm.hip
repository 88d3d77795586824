// Partial-sum GEMM for 65 .. 512 activation rows with wide tiles:  out[ks][i][r] = sum over k part ks of
// W[r][k] X[i][k]  (the projections of the transformer head body, paper Section 3.2, at the row counts of a
// draft step).
//
// With 32 x 32 tiles every workgroup re-reads its rows' activation planes (fp32 activations are two fp16
// planes, so 4 bytes per element against the weights' 2), and what the CUs pull out of the L2s is several times
// the weight bytes.  Here a workgroup owns 64 features (128 for wide outputs) x 128 rows, so a weight fragment
// meets all four row tiles and both planes (16 MFMAs per 16 k) and an activation fragment two (four) feature
// blocks; operand bytes entering the CU per MFMA fall from 1.5 KiB to 0.625 (0.375) KiB.  Its four wavefronts
// (one per SIMD, 128 or 256 accumulator registers and two sets of 8 / nf k blocks of operands each) split the k
// range of the workgroup and add their tiles up through LDS in wave order.  Few tiles do not fill the CUs, so k
// is also split over workgroups (at most 8 parts, one XCD per part where that fits, so that a part's activation
// slice stays in one L2); the parts are written as partial sums, which the consumers add in part order.
// (Measured at 128 rows, d = 2048: 9 to 24 us per projection against 7 to 39 us on the 32 x 32 tiles.  A CU's
// vector-memory path takes about 75 GB/s of 1 KiB wave loads; the bytes a workgroup pulls in set its time.)
#include "mrp_kernels.h"

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int WD_RT = 4;         // 32-row tiles per workgroup
constexpr int WD_WAVES = 4;

__device__ __forceinline__ f32x16 mma_h(const u32x4 &w, const u32x4 &x, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
}

// tile sums of the four waves: [wave][feature block][row tile][accumulator element][lane]
__shared__ float wd_red[WD_WAVES * 2 * WD_RT * 16 * 64];

template <int NP, int WD_NF>
__global__ __launch_bounds__(64 * WD_WAVES) __attribute__((amdgpu_waves_per_eu(1, 1))) void wide_gemm_kernel(
    const WideGemmArgs a) {
    constexpr int WD_CH = 8 / WD_NF;      // k blocks per operand set
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, lh = lane >> 5;

    // workgroup -> (k part, tile): the XCD (blockIdx % 8) fixes the k part when there are at most 8
    const int x = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int per = 8 / a.nKs;                       // XCDs per k part (nKs is 1, 2, 4 or 8)
    const int ks = x / per;
    const int t = j * per + (x % per);
    if (t >= a.nft * a.nrg) return;
    const int ft = t % a.nft, rg = t / a.nft;

    const int KB = a.Kc >> 4;
    const int nkb = KB / a.nKs / WD_WAVES;           // k blocks of this wave (a multiple of WD_CH)
    const int kb0 = ks * (KB / a.nKs) + wave * nkb;
    const u32x4 *wp = reinterpret_cast<const u32x4 *>(a.Wp) + ((size_t)(ft * WD_NF) * KB + kb0) * 64 + lane;
    const size_t wstride = (size_t)KB * 64;          // to the next 32-feature block
    // activation fragments of the four row tiles (tiles past the last one re-read it; their rows are not stored)
    const u32x4 *xp[WD_RT];
#pragma unroll
    for (int r = 0; r < WD_RT; ++r) {
        int ib = rg * WD_RT + r;
        ib = ib < a.nIb ? ib : a.nIb - 1;
        xp[r] = reinterpret_cast<const u32x4 *>(a.X) + ((size_t)kb0 * a.nIb + ib) * 64 + lane;
    }
    const size_t kstride = (size_t)a.nIb * 64;       // to the next k block of a plane

    f32x16 acc[WD_NF][WD_RT];
#pragma unroll
    for (int f = 0; f < WD_NF; ++f)
#pragma unroll
        for (int r = 0; r < WD_RT; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[f][r][e] = 0.f;

    u32x4 wb[2][WD_CH][WD_NF], xb[2][WD_CH][NP][WD_RT];
    auto request = [&](int set, int c) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < WD_CH; ++k) {
            const size_t kb = (size_t)c * WD_CH + k;
#pragma unroll
            for (int f = 0; f < WD_NF; ++f) wb[set][k][f] = wp[f * wstride + kb * 64];
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int r = 0; r < WD_RT; ++r) xb[set][k][p][r] = xp[r][p * a.plane + kb * kstride];
        }
    };
    auto compute = [&](int set) __attribute__((always_inline)) {
#pragma unroll
        for (int k = 0; k < WD_CH; ++k)
#pragma unroll
            for (int p = 0; p < NP; ++p)
#pragma unroll
                for (int r = 0; r < WD_RT; ++r)
#pragma unroll
                    for (int f = 0; f < WD_NF; ++f) acc[f][r] = mma_h(wb[set][k][f], xb[set][k][p][r], acc[f][r]);
    };
    // Two chunks per trip, so that the register sets keep fixed names.  Every trip issues both requests (past the
    // end the last chunk is fetched again and not used): with a request under a condition the compiler drains
    // all loads at the loop's end.
    const int nch = nkb / WD_CH, last = nch - 1;
    request(0, 0);
    // Within a trip the requests of the next set are dealt between the MFMAs of the current one (5 requests, then
    // 8 MFMAs, eight times): a request takes the CU's address unit 16 cycles or more, and a wave that issues its
    // 40 requests in one burst keeps its SIMD's matrix core idle meanwhile.
    constexpr int NLD = WD_CH * (WD_NF + NP * WD_RT), NMMA = WD_CH * NP * WD_RT * WD_NF, NGRP = 8;
    for (int c = 0; c + 2 <= nch; c += 2) {
        request(1, c + 1);
        compute(0);
#pragma unroll
        for (int g = 0; g < NGRP; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x020, NLD / NGRP, 0);     // VMEM reads
            __builtin_amdgcn_sched_group_barrier(0x008, NMMA / NGRP, 0);    // MFMAs
        }
        __builtin_amdgcn_sched_barrier(0);
        request(0, c + 2 <= last ? c + 2 : last);
        compute(1);
#pragma unroll
        for (int g = 0; g < NGRP; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x020, NLD / NGRP, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, NMMA / NGRP, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (nch & 1) compute(0);

    // ---- add the four waves' tiles in wave order, two feature blocks at a time; wave w finishes feature block
    // w / 2 of the pair, row tiles 2 (w % 2) ..
#pragma unroll
    for (int fp = 0; fp < WD_NF / 2; ++fp) {
        if (fp > 0) __syncthreads();
#pragma unroll
        for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int r = 0; r < WD_RT; ++r)
#pragma unroll
                for (int e = 0; e < 16; ++e) wd_red[(((wave * 2 + f) * WD_RT + r) * 16 + e) * 64 + lane] = acc[2 * fp + f][r][e];
        __syncthreads();
        const int f = wave >> 1;
#pragma unroll
        for (int r2 = 0; r2 < 2; ++r2) {
            const int r = 2 * (wave & 1) + r2;
            float s[16];
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                float v = wd_red[(((0 * 2 + f) * WD_RT + r) * 16 + e) * 64 + lane];
#pragma unroll
                for (int w = 1; w < WD_WAVES; ++w) v += wd_red[(((w * 2 + f) * WD_RT + r) * 16 + e) * 64 + lane];
                s[e] = v;
            }
            // a lane's 16 sums: activation row ln of the tile, features 8 q + 4 lh + (0 .. 3) of the block
            const int i = (rg * WD_RT + r) * 32 + ln;
            if (i < a.M) {
                float *o = a.out + ((size_t)ks * a.M + i) * a.R + (size_t)(ft * WD_NF + 2 * fp + f) * 32 + 4 * lh;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    *reinterpret_cast<float4 *>(o + 8 * q) = make_float4(s[4 * q], s[4 * q + 1], s[4 * q + 2], s[4 * q + 3]);
            }
        }
    }
}

}  // namespace

// k parts for `tiles` tiles over kbs k blocks: a power of two up to 8 that brings tiles x parts to one workgroup per
// CU at most, leaves every wave whole operand sets (kbs / parts / 4 a multiple of 8 / nf) and fits the partial-sum
// buffer of cap_rows rows; 0 when the kernel does not apply.
int wide_gemm_ksplit(int tiles, int kbs, int nCU, size_t cap_rows, int M, int nf) {
    const int unit = WD_WAVES * (8 / nf);
    if (kbs % unit != 0 || (size_t)M > cap_rows) return 0;
    int ks = 1;
    while (ks < 8 && tiles * ks * 2 <= nCU && kbs % (ks * 2 * unit) == 0 && (size_t)(ks * 2) * M <= cap_rows) ks *= 2;
    return ks;
}

hipError_t launch_wide_gemm(const WideGemmArgs &a, hipStream_t st) {
    const int nf = a.nf, ch = 8 / (nf > 0 ? nf : 2);
    if ((nf != 2 && nf != 4) || a.nplanes < 1 || a.nplanes > 2 || a.R % (32 * nf) != 0 || a.nKs < 1 || a.nKs > 8 ||
        (a.nKs & (a.nKs - 1)) || (a.Kc >> 4) % (a.nKs * WD_WAVES * ch) != 0 || a.nft != a.R / (32 * nf) ||
        a.nrg != (a.M + 32 * WD_RT - 1) / (32 * WD_RT))
        return hipErrorInvalidValue;
    const int per = 8 / a.nKs;
    const dim3 grid((a.nft * a.nrg + per - 1) / per * 8), block(64 * WD_WAVES);
    if (nf == 4) {
        if (a.nplanes == 2) hipLaunchKernelGGL((wide_gemm_kernel<2, 4>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((wide_gemm_kernel<1, 4>), grid, block, 0, st, a);
    } else {
        if (a.nplanes == 2) hipLaunchKernelGGL((wide_gemm_kernel<2, 2>), grid, block, 0, st, a);
        else hipLaunchKernelGGL((wide_gemm_kernel<1, 2>), grid, block, 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace mrp
