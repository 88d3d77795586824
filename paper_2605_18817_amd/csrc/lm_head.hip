// Persistent LM-head kernel for up to 256 activation rows (the HBM-bound case of
// the MRP chain): z <- z + y W_lm^T fused with the split-vocabulary
// (max, sum-exp, argmax) partials (paper Section 3.2: the head reuses the
// backbone's LM head; Algorithm 2: l <- l + delta; Section 2: confidence is the
// top-1 softmax probability, so only the partials are kept, never a softmax).
//
// One workgroup of 8 wavefronts per CU owns a contiguous, balanced range of
// 32-row vocabulary blocks and walks it in passes of up to 8 blocks (one per
// wave).  The weight stream never stops at a pass boundary: every wave keeps
// a ring of three k ranges (24 KiB) of packed weight fragments in flight,
// refilled right after each use, also across passes.  The bf16 activation y is
// re-read per pass from L2 and shared by the 8 waves through a double-buffered
// LDS stage.  The logit tile is the MFMA accumulator's initial value and is
// stored back from the accumulators; its loads for the next pass are issued
// before the next weight refills so that a wait for them leaves the younger
// weight loads in flight.
#include "mrp_kernels.h"

#include <type_traits>

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ bf16x8 as_frag(const u32x4 &u) { return __builtin_bit_cast(bf16x8, u); }

constexpr int LM_WAVES = 8;
constexpr int LM_THREADS = 64 * LM_WAVES;
#ifndef MRP_LM_RING
#define MRP_LM_RING 3
#endif
constexpr int LM_RING = MRP_LM_RING;           // k ranges of weight fragments held per wave (2 or 3)
static_assert(LM_RING == 2 || LM_RING == 3, "ring depth");

// LM_IT: 32-row blocks of activation rows that are computed (1, 2 or 4: a launch with at most 32 or 64 rows
// skips the matrix-core and LDS work of the empty blocks, which the 128-row form only just hides behind its
// memory time)
// KS: 16-wide k blocks per activation stage and weight ring slot (8; 4 in the 256-row form, whose 128
// accumulators leave room for half the ring)
template <int LM_IT, int KS>
__device__ __forceinline__ void lm_persist_body(const LmPersistArgs &a) {
    constexpr int LM_ROWS = 32 * LM_IT;
    constexpr int LM_STAGE = KS * LM_IT * 64;      // u32x4 per activation stage (32 KiB)
    constexpr int LM_NLD = LM_STAGE / LM_THREADS;  // u32x4 per thread per stage
    extern __shared__ u32x4 smem[];
    // reduction scratch, one copy per pass parity (a pass may end one iteration after the last)
    float *red_base = reinterpret_cast<float *>(smem + 2 * LM_STAGE);
    constexpr int RED_SET = 3 * LM_WAVES * LM_ROWS;  // floats per copy

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps the control flow scalar
    const int ln = lane & 31, lh = lane >> 5;
    const int wg = blockIdx.x;

    // this workgroup's vocabulary blocks, spread evenly over P passes
    const int rb_begin = (int)(((long)a.n_rb * wg) / a.nWG);
    const int rb_end = (int)(((long)a.n_rb * (wg + 1)) / a.nWG);
    const int cnt = rb_end - rb_begin;
    const int P = (cnt + LM_WAVES - 1) / LM_WAVES;
    const int n_lo = P ? cnt / P : 0, n_rem = P ? cnt % P : 0;
    // (reverse: the passes walk the workgroup's range from its end, so that a launch starts on the
    //  part of W_lm and z that the previous launch, walking forward, touched last)
    auto pass_rb = [&](int p, bool &active) -> int {
        const int q = (a.reverse && p < P) ? P - 1 - p : p;
        const int o = q * n_lo + (q < n_rem ? q : n_rem);
        const int n = n_lo + (q < n_rem ? 1 : 0);
        active = (p < P) && (wave < n);
        return rb_begin + o + wave;
    };
    const int nkr = a.KB / KS;
    const int T = P * nkr;
    const int T3 = (T + LM_RING - 1) / LM_RING * LM_RING;  // padded: the tail iterations only re-load
    const u32x4 *Wp = reinterpret_cast<const u32x4 *>(a.Wp);
    const u32x4 *Yp = reinterpret_cast<const u32x4 *>(a.Y);

    // This workgroup's partial of every row: the passes' partials are merged in registers (thread i
    // holds row i) and stored once, to slot wg of the row's contiguous slot array.
    Part run_pt = part_identity();
    if (P == 0) {
        if (tid < a.M) {
            const size_t o = (size_t)tid * a.nWG + wg;
            a.pm[o] = run_pt.m; a.ps[o] = run_pt.s; a.pi[o] = run_pt.i;
        }
        return;
    }

    // ---- weight prefetch cursor, flattened over passes.  Every load is unconditional: a wave
    // without a block in the cursor's pass re-reads block 0 (cache hits, no HBM traffic), so the
    // loop body is straight-line code and outstanding loads can be counted exactly. ----
    int pw = 0, gw = 0;
    const u32x4 *wsrc = Wp + lane;
    int wmul = 0;  // 1: walk the block's k ranges, 0: stay on the dummy block
    auto wcursor_set = [&]() {
        bool act;
        const int rb = pass_rb(pw, act);
        wsrc = Wp + (act ? (size_t)rb * a.KB * 64 : (size_t)0) + lane;
        wmul = act ? 1 : 0;
    };
    u32x4 wreg[LM_RING][KS];
#define LM_WLOAD(slot)                                                                   \
    {                                                                                    \
        _Pragma("unroll") for (int j = 0; j < KS; ++j)                                \
            wreg[slot][j] = wsrc[(size_t)((gw * KS + j) * wmul) * 64];                 \
        if (++gw == nkr) { gw = 0; ++pw; wcursor_set(); }                                \
    }
    // activation stage g (the same in every pass)
    u32x4 st[LM_NLD];
#define LM_YLOAD(g)                                                                      \
    _Pragma("unroll") for (int n = 0; n < LM_NLD; ++n) {                                 \
        const int c = tid + LM_THREADS * n;                                              \
        const int j = c / (LM_IT * 64), rem = c % (LM_IT * 64);                          \
        st[n] = Yp[((size_t)((g) * KS + j) * a.nIb) * 64 + rem];                      \
    }

    f32x16 acc[LM_IT];
    auto zload = [&](int p) __attribute__((always_inline)) {
        bool act;
        const int rb = pass_rb(p, act);
#pragma unroll
        for (int it = 0; it < LM_IT; ++it) {
            const int i = it * 32 + ln;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int v = rb * 32 + 8 * q + 4 * lh;
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (act && i < a.M && v < a.V) x = *reinterpret_cast<const float4 *>(a.z + (size_t)i * a.V + v);
                acc[it][4 * q + 0] = x.x; acc[it][4 * q + 1] = x.y;
                acc[it][4 * q + 2] = x.z; acc[it][4 * q + 3] = x.w;
            }
        }
    };
    auto epilogue = [&](int p) __attribute__((always_inline)) {
        bool act;
        const int rb = pass_rb(p, act);
        float *red_m = red_base + (p & 1) * RED_SET;
        float *red_s = red_m + LM_WAVES * LM_ROWS;
        int *red_i = reinterpret_cast<int *>(red_s + LM_WAVES * LM_ROWS);
#pragma unroll
        for (int it = 0; it < LM_IT; ++it) {
            const int i = it * 32 + ln;
            Part pt = part_identity();
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int v = rb * 32 + 8 * q + 4 * lh;
                const bool ok = act && v < a.V;
                if (ok && i < a.M)
                    *reinterpret_cast<float4 *>(a.z + (size_t)i * a.V + v) =
                        make_float4(acc[it][4 * q], acc[it][4 * q + 1], acc[it][4 * q + 2], acc[it][4 * q + 3]);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = acc[it][4 * q + e];
                    if (ok && x > pt.m) { pt.m = x; pt.i = v + e; }
                }
            }
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool ok = act && rb * 32 + 8 * q + 4 * lh < a.V;
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (ok) s += __expf(acc[it][4 * q + e] - pt.m);
            }
            pt.s = s;
            Part other;
            other.m = __shfl_xor(pt.m, 32);
            other.s = __shfl_xor(pt.s, 32);
            other.i = __shfl_xor(pt.i, 32);
            pt = part_merge(pt, other);
            if (lh == 0) {
                red_m[wave * LM_ROWS + it * 32 + ln] = pt.m;
                red_s[wave * LM_ROWS + it * 32 + ln] = pt.s;
                red_i[wave * LM_ROWS + it * 32 + ln] = pt.i;
            }
        }
    };
    // after a barrier: merge the 8 waves' partials of pass p into the running partial
    auto write_partials = [&](int p) __attribute__((always_inline)) {
        const float *red_m = red_base + (p & 1) * RED_SET;
        const float *red_s = red_m + LM_WAVES * LM_ROWS;
        const int *red_i = reinterpret_cast<const int *>(red_s + LM_WAVES * LM_ROWS);
        if (tid < LM_ROWS) {
            Part pt = {red_m[tid], red_s[tid], red_i[tid]};
#pragma unroll
            for (int wv = 1; wv < LM_WAVES; ++wv)
                pt = part_merge(pt, Part{red_m[wv * LM_ROWS + tid], red_s[wv * LM_ROWS + tid], red_i[wv * LM_ROWS + tid]});
            run_pt = part_merge(run_pt, pt);
        }
    };

    // ---- prologue ----
    // (issue order as in the loop: an activation stage is always older than the weight
    // ranges that follow it, so waiting for it leaves those in flight)
    wcursor_set();
    LM_YLOAD(0)
#pragma unroll
    for (int n = 0; n < LM_NLD; ++n) smem[tid + LM_THREADS * n] = st[n];
    LM_YLOAD(1 % nkr)
    LM_WLOAD(0)
    zload(0);
    LM_WLOAD(1)
    if constexpr (LM_RING >= 3) LM_WLOAD(2)
    __syncthreads();

    int g = 0, p = 0, buf = 0;  // k range, pass, LDS buffer
    bool act_cur;
    (void)pass_rb(0, act_cur);

    auto iter = [&](auto slot_c) __attribute__((always_inline)) {
        constexpr int S = decltype(slot_c)::value;
        const u32x4 *cur = smem + buf * LM_STAGE;
        if (act_cur) {
#pragma unroll
            for (int j = 0; j < KS; ++j) {
                bf16x8 bfr[LM_IT];
#pragma unroll
                for (int it = 0; it < LM_IT; ++it) bfr[it] = as_frag(cur[(j * LM_IT + it) * 64 + lane]);
#pragma unroll
                for (int it = 0; it < LM_IT; ++it)
                    acc[it] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(wreg[S][j]), bfr[it], acc[it], 0, 0, 0);
            }
        }
        // hand the next stage (fetched one iteration ago, before the younger weight loads) to LDS
        {
            u32x4 *nxt = smem + (buf ^ 1) * LM_STAGE;
#pragma unroll
            for (int n = 0; n < LM_NLD; ++n) nxt[tid + LM_THREADS * n] = st[n];
        }
        const bool boundary = (p < P) && (g == nkr - 1);
        if (boundary) {
            epilogue(p);
            zload(p + 1);  // (all zeros, no loads, past the last pass)
        }
        // refill before the barrier, so that no wave's requests wait for the slowest wave:
        // first the activation stage after next, then this ring slot's next k range
        {
            int g2 = g + 2;
            g2 = g2 >= nkr ? g2 - nkr : g2;
            g2 = g2 >= nkr ? g2 - nkr : g2;
            LM_YLOAD(g2)
        }
        LM_WLOAD(S)
        __syncthreads();
        if (boundary) write_partials(p);
        if (++g == nkr) {
            g = 0;
            ++p;
            (void)pass_rb(p, act_cur);
        }
        buf ^= 1;
    };
    for (int t = 0; t < T3; t += LM_RING) {
        iter(std::integral_constant<int, 0>{});
        iter(std::integral_constant<int, 1>{});
        if constexpr (LM_RING >= 3) iter(std::integral_constant<int, 2>{});
    }
    if (tid < a.M) {
        const size_t o = (size_t)tid * a.nWG + wg;
        a.pm[o] = run_pt.m; a.ps[o] = run_pt.s; a.pi[o] = run_pt.i;
    }
#undef LM_WLOAD
#undef LM_YLOAD
}

__global__ __launch_bounds__(LM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lm_persist_kernel(
    const LmPersistArgs a) {
    lm_persist_body<4, 8>(a);
}
__global__ __launch_bounds__(LM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lm_persist_kernel_256rows(
    const LmPersistArgs a) {
    lm_persist_body<8, 4>(a);
}
__global__ __launch_bounds__(LM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lm_persist_kernel_64rows(
    const LmPersistArgs a) {
    lm_persist_body<2, 8>(a);
}
__global__ __launch_bounds__(LM_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2))) void lm_persist_kernel_32rows(
    const LmPersistArgs a) {
    lm_persist_body<1, 8>(a);
}

}  // namespace

// two 32 KiB activation stages + two copies of the reduction scratch (sized for the 256-row form; the
// smaller forms use less)
size_t lm_persist_lds_bytes() { return (size_t)2 * 32768 + (size_t)2 * LM_WAVES * 256 * 12; }

// Once per device (mrp_create): the kernels need more than the default 64 KiB of dynamic LDS.
hipError_t lm_persist_configure() {
    hipError_t e = hipSuccess;
    for (const void *k : {reinterpret_cast<const void *>(lm_persist_kernel),
                          reinterpret_cast<const void *>(lm_persist_kernel_256rows),
                          reinterpret_cast<const void *>(lm_persist_kernel_64rows),
                          reinterpret_cast<const void *>(lm_persist_kernel_32rows)})
        if (e == hipSuccess)
            e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lm_persist_lds_bytes());
    return e;
}

hipError_t launch_lm_persist(const LmPersistArgs &a, hipStream_t st) {
    if (a.M > 256) return hipErrorInvalidValue;
    auto k = a.M <= 32 ? lm_persist_kernel_32rows
                       : (a.M <= 64 ? lm_persist_kernel_64rows : (a.M <= 128 ? lm_persist_kernel : lm_persist_kernel_256rows));
    hipLaunchKernelGGL(k, dim3(a.nWG), dim3(LM_THREADS), lm_persist_lds_bytes(), st, a);
    return hipGetLastError();
}

}  // namespace mrp
