// Tiled MFMA GEMM (bf16 operands for the LM head, fp16 for the head body) for many activation rows (the MFMA-bound regime of the MRP
// chain):  out[i][r] (+)= sum_k W[r][k] * X[i][k]  with 256 x 256 output tiles.
//
// A workgroup of four wavefronts computes a tile of 256 weight rows x 256 activation rows;
// each wave owns 64 weight rows x all 256 activation rows as 2 x 8 MFMA 32x32x16 tiles (256
// fp32 accumulators).  The weight fragments go from the packed layout straight into MFMA
// operand registers (one contiguous 1 KiB read per 32 rows x 16 k); no two waves load the
// same fragment.  The activation operand arrives in LDS by LDS-direct loads (three 32 KiB
// stages) and every wave reads all of it.  What limits this kernel is how many memory
// requests the CU's address unit takes per k step next to the MFMAs of four single-wave
// SIMDs, so the layout is the one with the fewest request bytes (64 KiB per step), operands
// are requested two steps ahead, and the requests are spread between the MFMAs.  As in the
// streaming kernels the weight fragment is the MFMA "A" operand, so a lane's accumulators of
// a sub-tile are 16 outputs of one activation row.
//
// Workgroups are ordered so that the 32 CUs of one XCD work at the same time on a
// block of 4 (activation) x 8 (weight) tiles and share its operand slices in that
// XCD's L2.
//
// Epilogues: EPI_PARTIAL (fp32 tile to out[i][r]; part ks of a k split to out[ks][i][r]), EPI_SILU (SiLU of the
// tile as the two fp16 activation planes of the next GEMM; no k split) and EPI_LM (the tile is added to the
// logit state, which is stored back, and the per-row (max, sum-exp, argmax) partial of
// the tile's 256 vocabulary entries is written; paper Section 3.2 / Algorithm 2
// l <- l + delta).
#include "mrp_kernels.h"

#include <type_traits>

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));   // native vector: arrays of it stay in registers
// One 32x32x16 matrix multiply-accumulate on 16-byte operand fragments: the partial-sum GEMMs of the
// head body take fp16 operands (weights converted at pack time, activations as fp16 planes), the LM
// head bf16 ones.
template <int EPI>
__device__ __forceinline__ f32x16 mma_frag(const u32x4 &w, const u32x4 &x, const f32x16 &c) {
    if constexpr (EPI != EPI_LM)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), c, 0, 0, 0);
}

constexpr int TG_KB = 4;                    // 16-wide k blocks per step (64 k)
constexpr int TG_B = TG_KB * 8 * 64;        // u32x4 of an activation stage (256 rows x 64 k)
constexpr int TG_STAGE = TG_B;              // 32 KiB
constexpr int TG_NLD = TG_B / 256;          // 1 KiB chunks per wave per step (8)
constexpr int TG_DEPTH = 3;                 // operand sets: steps s, s + 1, s + 2

// One array per activation stage: the stage arrives by LDS-direct loads, and with separate
// arrays the compiler's wait before reading one stage does not cover the loads into the others.
__shared__ u32x4 tg_stage0[TG_STAGE];
__shared__ u32x4 tg_stage1[TG_STAGE];
__shared__ u32x4 tg_stage2[TG_STAGE];

typedef const __attribute__((address_space(1))) void *gas_ptr;
typedef __attribute__((address_space(3))) void *las_ptr;

// Workgroup barrier after this wave's LDS accesses have completed; no fence, so the loads in
// flight for later steps are not drained.
__device__ __forceinline__ void tg_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// REM = 2 + (k steps - 2) % 3: the k steps left for the straight-line tail after the unrolled loop
template <int EPI, int REM>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 1))) void tiled_gemm_kernel(
    const TiledGemmArgs a) {
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int ln = lane & 31, lh = lane >> 5;

    // ---- workgroup -> tile (XCD-aware) ----
    // (with a k split every (tile block, k part) pair is a block of its own, so that few tiles still spread
    //  over all XCDs)
    const int x = blockIdx.x & 7, s = blockIdx.x >> 3;
    const int sbk = (s >> 5) * 8 + x, t = s & 31;
    const int nMgrp = (a.nMt + 3) >> 2;
    const int nsb = nMgrp * ((a.nVt + 7) >> 3);
    const int sb = sbk % nsb, ks = sbk / nsb;
    if (ks >= a.nKs) return;
    const int mgrp = sb % nMgrp, vchunk = sb / nMgrp;
    const int mt = mgrp * 4 + (t & 3), vt = vchunk * 8 + (t >> 2);
    if (mt >= a.nMt || vt >= a.nVt) return;

    const int rb0 = vt * 8, ib0 = mt * 8;
    const u32x4 *Wp = reinterpret_cast<const u32x4 *>(a.Wp);

    // this wave's two weight row blocks (rows past the padded matrix re-read the last block)
    const u32x4 *asrc[2];
#pragma unroll
    for (int v2 = 0; v2 < 2; ++v2) {
        int rb = rb0 + wave * 2 + v2;
        rb = rb < a.n_rb ? rb : a.n_rb - 1;
        asrc[v2] = Wp + (size_t)rb * a.KBw * 64 + lane;
    }

    // k-step sequence: segments x (k quads) x planes
    const int seg0_steps = a.seg[0].nkq * a.seg[0].nplanes;
    const int nsteps_all = seg0_steps + (a.nseg > 1 ? a.seg[1].nkq * a.seg[1].nplanes : 0);
    const int nsteps = nsteps_all / a.nKs;          // this k part's steps (the host makes the split even)
    const int st_begin = ks * nsteps, st_end = st_begin + nsteps;
    // Cursor over the k steps (segment, k quad, plane), advanced one step at a time without
    // divisions; it stops on the last step, which the padded tail re-fetches.  The segment
    // descriptions are copied out of the kernel arguments once (and made opaque, so that they
    // are not re-read from memory in every step).
    long seg_base0 = (long)a.seg[0].base, seg_base1 = (long)a.seg[1].base;
    long seg_ps0 = a.seg[0].plane_stride, seg_ps1 = a.seg[1].plane_stride;
    int seg_np0 = a.seg[0].nplanes, seg_np1 = a.seg[1].nplanes;
    int seg_nkq0 = a.seg[0].nkq;
    asm volatile("" : "+s"(seg_base0), "+s"(seg_base1), "+s"(seg_ps0), "+s"(seg_ps1), "+s"(seg_np0), "+s"(seg_np1),
                 "+s"(seg_nkq0));
    const long kq_stride = (long)TG_KB * a.nIb * 64;   // u32x4 per k quad of a plane
    int cu_st = st_begin, cu_seg = 0, cu_kq = 0, cu_p = 0;
    if (st_begin > 0) {      // where this k part starts: steps run over (segment, k quad, plane)
        cu_seg = st_begin >= seg0_steps ? 1 : 0;
        const int sl = cu_seg ? st_begin - seg0_steps : st_begin, np = cu_seg ? seg_np1 : seg_np0;
        cu_kq = sl / np;
        cu_p = sl % np;
    }
    auto cursor_get = [&](int &kbw, const u32x4 *&bptr) __attribute__((always_inline)) {
        kbw = ((cu_seg ? seg_nkq0 : 0) + cu_kq) * TG_KB;
        const long base = cu_seg ? seg_base1 : seg_base0;
        const long ps = cu_seg ? seg_ps1 : seg_ps0;
        bptr = reinterpret_cast<const u32x4 *>(base) + (cu_p * ps + cu_kq * kq_stride + (long)ib0 * 64);
    };
    auto cursor_next = [&]() __attribute__((always_inline)) {
        if (cu_st + 1 < st_end) {
            ++cu_st;
            if (++cu_p == (cu_seg ? seg_np1 : seg_np0)) {
                cu_p = 0;
                if (++cu_kq == seg_nkq0 && cu_seg == 0) { cu_kq = 0; cu_seg = 1; }
            }
        }
    };

    // Operands are requested two steps ahead.  Per step and wave: 8 LDS-direct loads (this wave's
    // quarter of the 32 KiB activation stage) and 8 weight-fragment loads into the register set
    // of that step; requests complete in issue order.
    u32x4 areg[TG_DEPTH][2][TG_KB];   // [step % 3][row block][k block]
#define TG_LOAD(st, set, stage)                                                            \
    {                                                                                      \
        int kbw_;                                                                          \
        const u32x4 *bp_;                                                                  \
        cursor_get(kbw_, bp_);                                                             \
        cursor_next();                                                                     \
        _Pragma("unroll") for (int n = 0; n < TG_NLD; ++n) {                               \
            const int c = wave + 4 * n;            /* chunk: k block c / 8, row block c % 8 */ \
            __builtin_amdgcn_global_load_lds(                                              \
                (gas_ptr)(bp_ + ((size_t)(c >> 3) * a.nIb + (c & 7)) * 64 + lane),         \
                (las_ptr)((stage) + c * 64), 16, 0, 0);                                    \
        }                                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                 \
        _Pragma("unroll") for (int v2 = 0; v2 < 2; ++v2)                                   \
            _Pragma("unroll") for (int kb = 0; kb < TG_KB; ++kb)                           \
                areg[set][v2][kb] = asrc[v2][(size_t)(kbw_ + kb) * 64];                    \
    }
    // the group requested one step ago is complete when at most the youngest group (16) is pending
#define TG_WAIT_PREV() __builtin_amdgcn_s_waitcnt(0x4F70)   /* vmcnt(16) */

    TG_LOAD(0, 0, tg_stage0)
    TG_LOAD(1, 1, tg_stage1)

    f32x16 acc[2][8];
#pragma unroll
    for (int v2 = 0; v2 < 2; ++v2)
#pragma unroll
        for (int ib = 0; ib < 8; ++ib)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[v2][ib][r] = 0.f;
    TG_WAIT_PREV();
    tg_barrier();

    // activation fragments are double-buffered: the LDS reads of the next k block are issued
    // among the MFMAs of the current one (one wave per SIMD: nothing else hides them)
    u32x4 bf[2][8];

    // Logit tile of the epilogue (EPI_LM): 8 slices of 32 activation rows x this wave's 64 vocabulary
    // entries, 8 16-byte pieces per lane each.  A piece is always fetched (addresses clamped into
    // the matrix; what lies outside is never used), so the number of requests per step is fixed.
    // The first two slices are requested during the last two k steps, in place of the operand
    // requests those steps no longer need (more would not fit the registers next to the k loop's).
    constexpr int ZD = 6;                       // slice buffers: five slices in flight ahead of the one added
    f32x4 zc[ZD][8];
    const int zv_lane = (rb0 + wave * 2) * 32 + 4 * lh;     // + 32 v2 + 8 q
    auto zpiece = [&](int ib, int pc) __attribute__((always_inline)) -> f32x4 {
        int i = (ib0 + ib) * 32 + ln;
        int v = zv_lane + 32 * (pc >> 2) + 8 * (pc & 3);
        i = i < a.M ? i : a.M - 1;
        v = v < a.R - 4 ? v : a.R - 4;          // (R % 4 == 0 on this path)
        return *reinterpret_cast<const f32x4 *>(a.z + (size_t)i * a.R + v);
    };

    // One k step.  A wave issues in order, and a memory request that finds the request queue full
    // holds up the MFMAs behind it, so the step's 16 requests are spread between its 64 MFMAs
    // (one ahead of every group of four but the first) instead of being issued in a burst.
    int kbw_n;
    const u32x4 *bp_n;
    auto step = [&](auto par_c, auto role_c, const u32x4 *cur, u32x4 *after) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_c)::value;   // st % 3: activation stage and weight register set
        constexpr int NS = (PAR + 2) % TG_DEPTH;      // set and stage (`after`) of step st + 2
        // 0: the operands of the step after next are still to request, 1: second to last step,
        // 2: last step
        constexpr int role = decltype(role_c)::value;
        // (`after` was last read one step ago and every wave has passed the barrier since;
        //  past the end the last step is re-fetched, never used)
        constexpr bool live = true;
        {
#pragma unroll
            for (int ib = 0; ib < 8; ++ib) bf[0][ib] = cur[ib * 64 + lane];
        }
#pragma unroll
        for (int kb = 0; kb < TG_KB; ++kb) {
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                const int c = kb * 4 + g4;             // group 0..15
                if (c >= 1) {                          // requests 0..14 (15 goes with group 15, too)
                    const int rq = c - 1;
                    if constexpr (role == 0) {
                        if (rq & 1) {
                            const int wl = rq >> 1;        // weight fragment 0..6 (7 below)
                            areg[NS][wl >> 2][wl & 3] = asrc[wl >> 2][(size_t)(kbw_n + (wl & 3)) * 64];
                        } else {
                            const int ch = wave + 4 * (rq >> 1);   // chunk: k block ch / 8, row block ch % 8
                            __builtin_amdgcn_global_load_lds(
                                (gas_ptr)(bp_n + ((size_t)(ch >> 3) * a.nIb + (ch & 7)) * 64 + lane),
                                (las_ptr)(after + ch * 64), 16, 0, 0);
                        }
                        if (c == 15) areg[NS][1][3] = asrc[1][(size_t)(kbw_n + 3) * 64];
                    } else if constexpr (EPI == EPI_LM) {
                        if (rq < 8) {                      // second to last step: slice 0; last step: slice 1
                            if constexpr (role == 1) zc[0][rq] = zpiece(0, rq);
                            else zc[1][rq] = zpiece(1, rq);
                        }
                    }
                }
                if (live) {
                    if (kb + 1 < TG_KB) {
                        bf[(kb + 1) & 1][2 * g4] = cur[((kb + 1) * 8 + 2 * g4) * 64 + lane];
                        bf[(kb + 1) & 1][2 * g4 + 1] = cur[((kb + 1) * 8 + 2 * g4 + 1) * 64 + lane];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    const int v2 = g4 >> 1, i0 = (g4 & 1) * 4;
#pragma unroll
                    for (int it = 0; it < 4; ++it)
                        acc[v2][i0 + it] = mma_frag<EPI>(areg[PAR][v2][kb], bf[kb & 1][i0 + it], acc[v2][i0 + it]);
                }
                if (c == 0 && role == 0) {   // behind the first MFMAs: where the operands of the step after next are
                    cursor_get(kbw_n, bp_n);
                    cursor_next();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the next step's operands (requested one step ago) are there once at most this step's 16
        // requests are pending; the second to last step requests 8 logit pieces (none in the partial-sum kernel)
        if constexpr (role == 1) __builtin_amdgcn_s_waitcnt(EPI == EPI_LM ? 0x0F78 : 0x0F70);   // vmcnt(8) / vmcnt(0)
        else if constexpr (role == 0) TG_WAIT_PREV();
        tg_barrier();
    };
    {
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        using P2 = std::integral_constant<int, 2>;
        for (int st = 0; st + TG_DEPTH <= nsteps - 2; st += TG_DEPTH) {
            step(P0{}, P0{}, tg_stage0, tg_stage2);
            step(P1{}, P0{}, tg_stage1, tg_stage0);
            step(P2{}, P0{}, tg_stage2, tg_stage1);
        }
        // the last REM steps (second template argument: 0 ordinary, 1 second to last, 2 last)
        if constexpr (REM == 2) {
            step(P0{}, P1{}, tg_stage0, tg_stage2);
            step(P1{}, P2{}, tg_stage1, tg_stage0);
        } else if constexpr (REM == 3) {
            step(P0{}, P0{}, tg_stage0, tg_stage2);
            step(P1{}, P1{}, tg_stage1, tg_stage0);
            step(P2{}, P2{}, tg_stage2, tg_stage1);
        } else {
            step(P0{}, P0{}, tg_stage0, tg_stage2);
            step(P1{}, P0{}, tg_stage1, tg_stage0);
            step(P2{}, P1{}, tg_stage2, tg_stage1);
            step(P0{}, P2{}, tg_stage0, tg_stage2);
        }
    }
#undef TG_LOAD
#undef TG_WAIT_PREV

    // ---- epilogue ----
    // (an opaque zero keeps the compiler from sharing the prologue's 64 tile addresses with
    // the epilogue, which would hold them in registers across the whole k loop)
    int opq = 0;
    asm volatile("" : "+v"(opq));
    const int lne = ln + opq;
    if constexpr (EPI == EPI_PARTIAL) {
#pragma unroll
        for (int v2 = 0; v2 < 2; ++v2)
#pragma unroll
            for (int ib = 0; ib < 8; ++ib) {
                const int i = (ib0 + ib) * 32 + lne;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int r = (rb0 + wave * 2 + v2) * 32 + 8 * q + 4 * lh;
                    if (i < a.M && r < a.R)
                        *reinterpret_cast<float4 *>(a.out + ((size_t)ks * a.M + i) * a.R + r) = make_float4(
                            acc[v2][ib][4 * q], acc[v2][ib][4 * q + 1], acc[v2][ib][4 * q + 2], acc[v2][ib][4 * q + 3]);
                }
            }
    } else if constexpr (EPI == EPI_SILU) {
        // s = SiLU(tile) written as the two fp16 planes of the next GEMM's activation: a lane holds 4 of the
        // 8 features of a 16-byte chunk (the lane ^ 32 holds the other 4), so it stores 8 bytes per plane;
        // the 64 lanes' pieces of one (v2, ib, q) are 512 contiguous bytes
        uint2 *planes = reinterpret_cast<uint2 *>(a.planes);
#pragma unroll
        for (int v2 = 0; v2 < 2; ++v2)
#pragma unroll
            for (int ib = 0; ib < 8; ++ib) {
                const int i = (ib0 + ib) * 32 + lne;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int c8 = (rb0 + wave * 2 + v2) * 4 + q;
                    if (i < a.M && c8 * 8 < a.R) {
                        uint16_t h[4], l[4];
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float x = acc[v2][ib][4 * q + e];
                            split2(x / (1.0f + expf(-x)), h[e], l[e]);
                        }
                        const size_t o = 2 * act_chunk_index(i, c8, a.nIb) + lh;
                        planes[o] = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
                        planes[o + 2 * a.plane_stride] = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
                    }
                }
            }
    } else {
        // per wave: 256 activation rows x 64 vocabulary entries.  The logit tile is added here, one
        // 32-row slice (32 registers) at a time; the row reduction over v runs in registers.
        float *red_m = reinterpret_cast<float *>(tg_stage0);       // [4 waves][256 rows] (the stages are dead)
        float *red_s = red_m + 1024;
        int *red_i = reinterpret_cast<int *>(red_s + 1024);
        // Slices 0 and 1 were requested during the last two k steps; five slices are kept in flight
        // ahead of the one being added; the sum is formed in place in the fetched registers.
        auto zfetch = [&](int ib, f32x4 (&dst)[8]) __attribute__((always_inline)) {
#pragma unroll
            for (int pc = 0; pc < 8; ++pc) dst[pc] = zpiece(ib, pc);
        };
        zfetch(2, zc[2]);
        zfetch(3, zc[3]);
        zfetch(4, zc[4]);
#pragma unroll
        for (int ib = 0; ib < 8; ++ib) {
            if (ib + ZD - 1 < 8) zfetch(ib + ZD - 1, zc[(ib + ZD - 1) % ZD]);
            const int i = (ib0 + ib) * 32 + lne;
            f32x4(&xs)[8] = zc[ib % ZD];
            Part pt = part_identity();
#pragma unroll
            for (int v2 = 0; v2 < 2; ++v2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int v = (rb0 + wave * 2 + v2) * 32 + 8 * q + 4 * lh;
                    f32x4 &x4 = xs[v2 * 4 + q];
                    x4[0] += acc[v2][ib][4 * q + 0];
                    x4[1] += acc[v2][ib][4 * q + 1];
                    x4[2] += acc[v2][ib][4 * q + 2];
                    x4[3] += acc[v2][ib][4 * q + 3];
                    if (i < a.M && v < a.R) *reinterpret_cast<f32x4 *>(a.z + (size_t)i * a.R + v) = x4;
                    if (v < a.R) {
                        if (x4[0] > pt.m) { pt.m = x4[0]; pt.i = v; }
                        if (x4[1] > pt.m) { pt.m = x4[1]; pt.i = v + 1; }
                        if (x4[2] > pt.m) { pt.m = x4[2]; pt.i = v + 2; }
                        if (x4[3] > pt.m) { pt.m = x4[3]; pt.i = v + 3; }
                    }
                }
            float sum = 0.f;
#pragma unroll
            for (int v2 = 0; v2 < 2; ++v2)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const bool ok = (rb0 + wave * 2 + v2) * 32 + 8 * q + 4 * lh < a.R;
                    const f32x4 x4 = xs[v2 * 4 + q];
                    if (ok) sum += (__expf(x4[0] - pt.m) + __expf(x4[1] - pt.m)) + (__expf(x4[2] - pt.m) + __expf(x4[3] - pt.m));
                }
            pt.s = sum;
            Part other;
            other.m = __shfl_xor(pt.m, 32);
            other.s = __shfl_xor(pt.s, 32);
            other.i = __shfl_xor(pt.i, 32);
            pt = part_merge(pt, other);
            if (lh == 0) {
                const int row = ib * 32 + lne;
                red_m[wave * 256 + row] = pt.m;
                red_s[wave * 256 + row] = pt.s;
                red_i[wave * 256 + row] = pt.i;
            }
        }
        __syncthreads();
        {
            Part pt = {red_m[tid], red_s[tid], red_i[tid]};
#pragma unroll
            for (int w = 1; w < 4; ++w) pt = part_merge(pt, Part{red_m[w * 256 + tid], red_s[w * 256 + tid], red_i[w * 256 + tid]});
            const int i = ib0 * 32 + tid;
            if (i < a.M) {
                a.pm[(size_t)vt * a.M + i] = pt.m;
                a.ps[(size_t)vt * a.M + i] = pt.s;
                a.pi[(size_t)vt * a.M + i] = pt.i;
            }
        }
    }
}

template <int EPI, int REM>
hipError_t launch_inst(const TiledGemmArgs &a, hipStream_t st) {
    const int nMgrp = (a.nMt + 3) / 4, nVch = (a.nVt + 7) / 8;
    const int nsb = nMgrp * nVch * a.nKs;
    const int per_xcd = (nsb + 7) / 8;          // super-blocks per XCD
    const int grid = per_xcd * 32 * 8;
    hipLaunchKernelGGL((tiled_gemm_kernel<EPI, REM>), dim3(grid), dim3(256), 0, st, a);
    return hipGetLastError();
}

template <int EPI>
hipError_t launch_epi(const TiledGemmArgs &a, hipStream_t st) {
    int nsteps = 0;
    for (int sg = 0; sg < a.nseg; ++sg) nsteps += a.seg[sg].nkq * a.seg[sg].nplanes;
    if (a.nKs < 1 || nsteps % a.nKs != 0 || nsteps / a.nKs < 2 || (EPI != EPI_PARTIAL && a.nKs != 1)) return hipErrorInvalidValue;
    nsteps /= a.nKs;
    const int rem = 2 + (nsteps - 2) % 3;       // (at least two k steps per part)
    if (rem == 2) return launch_inst<EPI, 2>(a, st);
    if (rem == 3) return launch_inst<EPI, 3>(a, st);
    return launch_inst<EPI, 4>(a, st);
}

}  // namespace

// Few output tiles (the head body's GEMMs at 1024 or 2048 rows have 64 or 128) leave most CUs idle: split k
// into up to 16 parts so that tiles x parts comes near the CU count; every part must have an equal number of at
// least MRP_TILED_MIN_STEPS k steps and its partial sums must fit the buffer.
#ifndef MRP_TILED_MIN_STEPS
#define MRP_TILED_MIN_STEPS 4
#endif
int tiled_ksplit(int tiles, int nsteps, int nCU, size_t cap_rows, int M) {
    int ks = 1;
    while (ks < 16 && tiles * ks * 2 <= nCU && nsteps % (ks * 2) == 0 && nsteps / (ks * 2) >= MRP_TILED_MIN_STEPS &&
           (size_t)(ks * 2) * M <= cap_rows)
        ks *= 2;
    return ks;
}

hipError_t launch_tiled_gemm(const TiledGemmArgs &a, int epi, hipStream_t st) {
    if (epi == EPI_SILU) return launch_epi<EPI_SILU>(a, st);
    return epi == EPI_LM ? launch_epi<EPI_LM>(a, st) : launch_epi<EPI_PARTIAL>(a, st);
}

}  // namespace mrp
