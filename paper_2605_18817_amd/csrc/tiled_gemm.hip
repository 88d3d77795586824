// Tiled bf16 MFMA GEMM for many activation rows (the MFMA-bound regime of the MRP
// chain):  out[i][r] (+)= sum_k W[r][k] * X[i][k]  with 256 x 256 output tiles.
//
// A workgroup of four wavefronts (2 x 2) computes a tile of 256 weight rows x 256
// activation rows; each wave owns 128 x 128 of it as 4 x 4 MFMA 32x32x16 tiles (256
// fp32 accumulators).  The weight fragments go from the packed layout straight into
// MFMA operand registers (one contiguous 1 KiB read per 32 rows x 16 k, fetched one k
// step ahead); only the activation operand passes through LDS (double-buffered 32 KiB
// stages, read back conflict-free one block per ds_read_b128).  Keeping the weights out
// of LDS matters because LDS would otherwise be as busy as the matrix cores: at one
// wave per SIMD, 64 KiB of ds_write_b128 (about 60 B/clk) plus 128 KiB of ds_read_b128
// (128 B/clk) per k step take as long as the step's 64 MFMAs.  As in the streaming
// kernels the weight fragment is the MFMA "A" operand, so a lane's accumulators of a
// sub-tile are 16 outputs of one activation row.
//
// Workgroups are ordered so that the 32 CUs of one XCD work at the same time on a
// block of 4 (activation) x 8 (weight) tiles and share its operand slices in that
// XCD's L2.
//
// Epilogues: EPI_PARTIAL (fp32 tile to out[i][r]) and EPI_LM (the tile is added to the
// logit state, which is stored back, and the per-row (max, sum-exp, argmax) partial of
// the tile's 256 vocabulary entries is written; paper Section 3.2 / Algorithm 2
// l <- l + delta).
#include "mrp_kernels.h"

#include <type_traits>

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8 as_frag(const u32x4 &u) { return __builtin_bit_cast(bf16x8, u); }

constexpr int TG_KB = 4;                    // 16-wide k blocks per step (64 k)
constexpr int TG_B = TG_KB * 8 * 64;        // u32x4 of an activation stage (256 rows x 64 k)
constexpr int TG_STAGE = TG_B;              // 32 KiB
constexpr int TG_NLD = TG_B / 256;          // u32x4 per thread per step (8)

template <int EPI>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void tiled_gemm_kernel(
    const TiledGemmArgs a) {
    extern __shared__ u32x4 smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wv = wave >> 1, wi = wave & 1;   // weight-row half, activation-row half
    const int ln = lane & 31, lh = lane >> 5;

    // ---- workgroup -> tile (XCD-aware) ----
    const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
    const int sb = (s >> 5) * 8 + x, t = s & 31;
    const int nMgrp = (a.nMt + 3) >> 2;
    const int mgrp = sb % nMgrp, vchunk = sb / nMgrp;
    const int mt = mgrp * 4 + (t & 3), vt = vchunk * 8 + (t >> 2);
    if (mt >= a.nMt || vt >= a.nVt) return;

    const int rb0 = vt * 8, ib0 = mt * 8;
    const u32x4 *Wp = reinterpret_cast<const u32x4 *>(a.Wp);

    // this wave's four weight row blocks (rows past the padded matrix re-read the last block)
    const u32x4 *asrc[4];
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4) {
        int rb = rb0 + wv * 4 + v4;
        rb = rb < a.n_rb ? rb : a.n_rb - 1;
        asrc[v4] = Wp + (size_t)rb * a.KBw * 64 + lane;
    }

    // k-step sequence: segments x (k quads) x planes
    const int seg0_steps = a.seg[0].nkq * a.seg[0].nplanes;
    const int nsteps = seg0_steps + (a.nseg > 1 ? a.seg[1].nkq * a.seg[1].nplanes : 0);
    auto step_src = [&](int st, int &kbw, const u32x4 *&bptr) {
        const bool s1 = st >= seg0_steps;
        const int l = s1 ? st - seg0_steps : st;
        const int np = s1 ? a.seg[1].nplanes : a.seg[0].nplanes;
        const int kq = l / np, p = l - kq * np;
        const int kq0 = s1 ? a.seg[0].nkq : 0;
        kbw = (kq0 + kq) * TG_KB;
        const uint4 *base = s1 ? a.seg[1].base : a.seg[0].base;
        const long pstr = s1 ? a.seg[1].plane_stride : a.seg[0].plane_stride;
        bptr = reinterpret_cast<const u32x4 *>(base) + (size_t)p * pstr + ((size_t)(kq * TG_KB) * a.nIb + ib0) * 64;
    };

    // Operands of the next step are fetched while this one computes: first the activation
    // chunk (to staging registers, then LDS), then the weight fragments (kept in registers),
    // so that waiting for the older activation loads leaves the weight loads in flight.
    u32x4 areg[2][4][TG_KB];   // [step parity][row block][k block]
    u32x4 bst[TG_NLD];
#define TG_LOAD(st, set)                                                                   \
    {                                                                                      \
        int kbw_;                                                                          \
        const u32x4 *bp_;                                                                  \
        step_src((st) < nsteps ? (st) : nsteps - 1, kbw_, bp_);                            \
        _Pragma("unroll") for (int n = 0; n < TG_NLD; ++n)                                 \
            bst[n] = bp_[(size_t)(n >> 1) * a.nIb * 64 + tid + 256 * (n & 1)];              \
        _Pragma("unroll") for (int v4 = 0; v4 < 4; ++v4)                                   \
            _Pragma("unroll") for (int kb = 0; kb < TG_KB; ++kb)                           \
                areg[set][v4][kb] = asrc[v4][(size_t)(kbw_ + kb) * 64];                    \
    }
#define TG_STORE(buf)                                                                      \
    {                                                                                      \
        u32x4 *db_ = smem + (buf) * TG_STAGE;                                              \
        _Pragma("unroll") for (int n = 0; n < TG_NLD; ++n) db_[tid + 256 * n] = bst[n];    \
    }

    TG_LOAD(0, 0)

    f32x16 acc[4][4];
#pragma unroll
    for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
        for (int it = 0; it < 4; ++it)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[v4][it][r] = 0.f;
    TG_STORE(0)
    __syncthreads();

    // activation fragments are double-buffered: the LDS reads of the next k block are issued
    // before the MFMAs of the current one (one wave per SIMD: nothing else hides them)
    bf16x8 bf[2][4];
#define TG_FRAGS(buf, kb, set)                                                             \
    {                                                                                      \
        const u32x4 *B_ = smem + (buf) * TG_STAGE;                                         \
        _Pragma("unroll") for (int it = 0; it < 4; ++it)                                   \
            bf[set][it] = as_frag(B_[((kb) * 8 + wi * 4 + it) * 64 + lane]);               \
    }
#define TG_MFMA(par, kb, set)                                                              \
    _Pragma("unroll") for (int v4 = 0; v4 < 4; ++v4)                                       \
        _Pragma("unroll") for (int it = 0; it < 4; ++it)                                   \
            acc[v4][it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(areg[par][v4][kb]), bf[set][it], acc[v4][it], 0, 0, 0);

    TG_FRAGS(0, 0, 0)
    auto step = [&](auto par_c, int st) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_c)::value;   // st & 1: LDS buffer and weight register set
        TG_LOAD(st + 1, PAR ^ 1)                       // (past the end: re-fetches the last step, never used)
        __builtin_amdgcn_sched_barrier(0);             // keep the fetches at the top of the step
        TG_FRAGS(PAR, 1, 1)
        TG_MFMA(PAR, 0, 0)
        TG_FRAGS(PAR, 2, 0)
        TG_MFMA(PAR, 1, 1)
        TG_FRAGS(PAR, 3, 1)
        TG_MFMA(PAR, 2, 0)
        // every read of this step's buffer is done; hand over the next step's activations
        TG_STORE(PAR ^ 1)
        __syncthreads();
        TG_FRAGS(PAR ^ 1, 0, 0)
        TG_MFMA(PAR, 3, 1)
    };
    // (the step count is even: every segment has d / 64 k steps per plane and d % 128 == 0)
    for (int st = 0; st < nsteps; st += 2) {
        step(std::integral_constant<int, 0>{}, st);
        step(std::integral_constant<int, 1>{}, st + 1);
    }
#undef TG_LOAD
#undef TG_STORE
#undef TG_FRAGS
#undef TG_MFMA

    // ---- epilogue ----
    // (an opaque zero keeps the compiler from sharing the prologue's 64 tile addresses with
    // the epilogue, which would hold them in registers across the whole k loop)
    int opq = 0;
    asm volatile("" : "+v"(opq));
    const int lne = ln + opq;
    if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
            for (int it = 0; it < 4; ++it) {
                const int i = (ib0 + wi * 4 + it) * 32 + lne;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int r = (rb0 + wv * 4 + v4) * 32 + 8 * q + 4 * lh;
                    if (i < a.M && r < a.R)
                        *reinterpret_cast<float4 *>(a.out + (size_t)i * a.R + r) = make_float4(
                            acc[v4][it][4 * q], acc[v4][it][4 * q + 1], acc[v4][it][4 * q + 2], acc[v4][it][4 * q + 3]);
                }
            }
    } else {
        // per wave: 128 activation rows x 128 vocabulary entries.  The logit tile is added here,
        // one 32-row slice (64 registers) at a time, the next slice's loads in flight meanwhile;
        // the row reduction over v runs in registers.
        float *red_m = reinterpret_cast<float *>(smem);            // [2 (wv)][256 rows] (LDS stages are dead)
        float *red_s = red_m + 512;
        int *red_i = reinterpret_cast<int *>(red_s + 512);
        float4 zc[2][16];
        auto zfetch = [&](int it, float4 (&dst)[16]) __attribute__((always_inline)) {
            const int i = (ib0 + wi * 4 + it) * 32 + lne;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int v = (rb0 + wv * 4 + v4) * 32 + 8 * q + 4 * lh;
                    dst[v4 * 4 + q] = make_float4(0.f, 0.f, 0.f, 0.f);
                    if (i < a.M && v < a.R) dst[v4 * 4 + q] = *reinterpret_cast<const float4 *>(a.z + (size_t)i * a.R + v);
                }
        };
        zfetch(0, zc[0]);
        zfetch(1, zc[1]);
#pragma unroll
        for (int it = 0; it < 4; ++it) {
            const int i = (ib0 + wi * 4 + it) * 32 + lne;
            Part pt = part_identity();
            float xs[4][16];
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int v = (rb0 + wv * 4 + v4) * 32 + 8 * q + 4 * lh;
                    const float4 zz = zc[it & 1][v4 * 4 + q];
                    xs[v4][4 * q + 0] = acc[v4][it][4 * q + 0] + zz.x;
                    xs[v4][4 * q + 1] = acc[v4][it][4 * q + 1] + zz.y;
                    xs[v4][4 * q + 2] = acc[v4][it][4 * q + 2] + zz.z;
                    xs[v4][4 * q + 3] = acc[v4][it][4 * q + 3] + zz.w;
                    if (i < a.M && v < a.R)
                        *reinterpret_cast<float4 *>(a.z + (size_t)i * a.R + v) =
                            make_float4(xs[v4][4 * q], xs[v4][4 * q + 1], xs[v4][4 * q + 2], xs[v4][4 * q + 3]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float xx = xs[v4][4 * q + e];
                        if (v < a.R && xx > pt.m) { pt.m = xx; pt.i = v + e; }
                    }
                }
            if (it + 2 < 4) zfetch(it + 2, zc[it & 1]);
            float sum = 0.f;
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool ok = (rb0 + wv * 4 + v4) * 32 + 8 * q + 4 * lh < a.R;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (ok) sum += __expf(xs[v4][4 * q + e] - pt.m);
                }
            pt.s = sum;
            Part other;
            other.m = __shfl_xor(pt.m, 32);
            other.s = __shfl_xor(pt.s, 32);
            other.i = __shfl_xor(pt.i, 32);
            pt = part_merge(pt, other);
            if (lh == 0) {
                const int row = (wi * 4 + it) * 32 + lne;
                red_m[wv * 256 + row] = pt.m;
                red_s[wv * 256 + row] = pt.s;
                red_i[wv * 256 + row] = pt.i;
            }
        }
        __syncthreads();
        {
            const Part pt = part_merge(Part{red_m[tid], red_s[tid], red_i[tid]},
                                       Part{red_m[256 + tid], red_s[256 + tid], red_i[256 + tid]});
            const int i = ib0 * 32 + tid;
            if (i < a.M) {
                a.pm[(size_t)vt * a.M + i] = pt.m;
                a.ps[(size_t)vt * a.M + i] = pt.s;
                a.pi[(size_t)vt * a.M + i] = pt.i;
            }
        }
    }
}

template <int EPI>
hipError_t launch_inst(const TiledGemmArgs &a, hipStream_t st) {
    static bool attr_set = false;
    const size_t lds = (size_t)2 * TG_STAGE * 16;   // 64 KiB (the reduction scratch of EPI_LM reuses it)
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(tiled_gemm_kernel<EPI>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int nMgrp = (a.nMt + 3) / 4, nVch = (a.nVt + 7) / 8;
    const int nsb = nMgrp * nVch;
    const int per_xcd = (nsb + 7) / 8;          // super-blocks per XCD
    const int grid = per_xcd * 32 * 8;
    hipLaunchKernelGGL(tiled_gemm_kernel<EPI>, dim3(grid), dim3(256), lds, st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_tiled_gemm(const TiledGemmArgs &a, int epi, hipStream_t st) {
    return epi == EPI_LM ? launch_inst<EPI_LM>(a, st) : launch_inst<EPI_PARTIAL>(a, st);
}

}  // namespace mrp
