// Weight-streaming MFMA GEMM for gfx950 (bf16 operands for the LM head, fp16 for the head body):  out[i][r] (+)= sum_k W[r][k] * X[i][k].
//
// W is a packed weight matrix (32x16 fragment blocks, contiguous along k for a
// 32-row block), X a packed activation operand made of one or more 16-bit planes.
// Each wavefront owns 32 weight rows and streams their fragments straight from
// HBM into registers (one contiguous 1 KiB read per 16 k), never through LDS;
// the activation slice of the current k range is shared by the four waves of a
// workgroup through LDS.  The MFMA's "A" operand is the weight fragment, its
// "B" operand the activation fragment, so a lane's 16 accumulators of a 32x32
// tile are 16 outputs of ONE activation row: a row reduction over the outputs
// (the vocabulary, for the LM head) is done in registers plus one cross-lane
// exchange.
//
// Epilogues:
//   EPI_PARTIAL  store the fp32 tile to out[ks][i][r] (k-split partial sums)
//   EPI_LM       LM head of the MRP chain (paper Section 3.2: the head reuses
//                the backbone's LM head; Algorithm 2: l <- l + delta): the
//                accumulators start from the logit state z, the updated z is
//                stored back, and the tile's per-row (max, sum-exp, argmax)
//                partial is written for the split-vocabulary softmax reduction.
#include "mrp_kernels.h"

#include <type_traits>

namespace mrp {

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));  // native vector: stays in registers

// One 32x32x16 matrix multiply-accumulate on 16-byte operand fragments: the partial-sum GEMMs of the
// head body take fp16 operands (weights converted at pack time, activations as fp16 planes), the LM
// head bf16 ones.
template <int EPI>
__device__ __forceinline__ f32x16 mma_frag(const u32x4 &w, const u32x4 &x, const f32x16 &c) {
    if constexpr (EPI == EPI_PARTIAL)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, w), __builtin_bit_cast(f16x8, x), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w), __builtin_bit_cast(bf16x8, x), c, 0, 0, 0);
}

template <int IT, int EPI, bool VEC4>
__device__ __forceinline__ void stream_gemm_body(const StreamGemmArgs &a) {
    extern __shared__ u32x4 smem[];
    constexpr int STAGE = KSTEP * IT * 64;  // uint4 per activation stage
    constexpr int NLD = STAGE / 256;        // uint4 each thread moves per stage
    constexpr int ROWS = IT * 32;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 31, lh = lane >> 5;

    // workgroup -> (row group, weight tile, k split); consecutive slots of one
    // XCD (blockIdx % 8) share a weight tile across row groups
    const int nWG = a.nVt * a.nMg * a.nKs;
    const int per = (nWG + 7) >> 3;
    const int w = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if (w >= nWG) return;
    const int mg = w % a.nMg;
    const int t = w / a.nMg;
    const int vt = t % a.nVt;
    const int ks = t / a.nVt;

    const int rb = vt * WG_WAVES + wave;
    const bool rb_ok = rb < a.n_rb;
    const int rbc = rb_ok ? rb : a.n_rb - 1;
    const u32x4 *wptr = reinterpret_cast<const u32x4 *>(a.Wp) + (size_t)rbc * a.KBw * 64 + lane;

    const int ib0 = mg * IT;
    const int g_begin = (int)(((long)a.G * ks) / a.nKs);
    const int g_end = (int)(((long)a.G * (ks + 1)) / a.nKs);

    // (fields are picked with selects, not indexed, so the kernel arguments stay in SGPRs)
    const int seg0_nkr = a.seg[0].nkr;
    const bool two_seg = a.nseg > 1;
    auto in_seg1 = [&](int g) { return two_seg && g >= seg0_nkr; };
    auto planes_of = [&](int g) { return in_seg1(g) ? a.seg[1].nplanes : a.seg[0].nplanes; };
    auto act_ptr = [&](int g, int p) -> const u32x4 * {
        const bool s1 = in_seg1(g);
        const int krl = s1 ? g - seg0_nkr : g;
        const uint4 *base = s1 ? a.seg[1].base : a.seg[0].base;
        const long pstride = s1 ? a.seg[1].plane_stride : a.seg[0].plane_stride;
        return reinterpret_cast<const u32x4 *>(base) + (size_t)p * pstride +
               ((size_t)(krl * KSTEP) * a.nIb + ib0) * 64;
    };
    // thread's n-th 16-byte piece of a stage: k block j, offset rem inside the row group
#define MRP_LOAD_STAGE(ptr, st)                                           \
    _Pragma("unroll") for (int n = 0; n < NLD; ++n) {                     \
        const int c = tid + 256 * n;                                      \
        const int j = c / (IT * 64), rem = c % (IT * 64);                 \
        st[n] = (ptr)[(size_t)j * a.nIb * 64 + rem];                      \
    }

    // ---- prologue: weight fragments of the first two k ranges, first stage ----
    u32x4 wreg[2 * KSTEP];
#pragma unroll
    for (int j = 0; j < KSTEP; ++j) wreg[j] = wptr[(size_t)(g_begin * KSTEP + j) * 64];
    {
        const int g1 = (g_begin + 1 < g_end) ? g_begin + 1 : g_begin;
#pragma unroll
        for (int j = 0; j < KSTEP; ++j) wreg[KSTEP + j] = wptr[(size_t)(g1 * KSTEP + j) * 64];
    }
    {
        u32x4 st[NLD];
        const u32x4 *p0 = act_ptr(g_begin, 0);
        MRP_LOAD_STAGE(p0, st)
#pragma unroll
        for (int n = 0; n < NLD; ++n) smem[tid + 256 * n] = st[n];
    }

    f32x16 acc[IT];
    if constexpr (EPI == EPI_LM) {
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int i = (ib0 + it) * 32 + ln;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int v = rb * 32 + 8 * q + 4 * lh;
                float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
                if (rb_ok && i < a.M) {
                    const float *zp = a.z + (size_t)i * a.R + v;
                    if constexpr (VEC4) {
                        if (v < a.R) x = *reinterpret_cast<const float4 *>(zp);
                    } else {
                        if (v + 0 < a.R) x.x = zp[0];
                        if (v + 1 < a.R) x.y = zp[1];
                        if (v + 2 < a.R) x.z = zp[2];
                        if (v + 3 < a.R) x.w = zp[3];
                    }
                }
                acc[it][4 * q + 0] = x.x; acc[it][4 * q + 1] = x.y;
                acc[it][4 * q + 2] = x.z; acc[it][4 * q + 3] = x.w;
            }
        }
    } else {
#pragma unroll
        for (int it = 0; it < IT; ++it)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[it][r] = 0.f;
    }
    __syncthreads();

    // ---- main loop over (k range, plane) stages ----
    int buf = 0;
    int gn = g_begin, pn = 0;  // next stage to fetch
    auto advance = [&]() {
        if (++pn == planes_of(gn)) { pn = 0; ++gn; }
    };
    advance();

    auto krange = [&](auto par_c, int g) __attribute__((always_inline)) {
        constexpr int PAR = decltype(par_c)::value;
        const int np = planes_of(g);
        for (int p = 0; p < np; ++p) {
            // fetch the next stage (the last stage re-fetches itself: in bounds, never read)
            u32x4 st[NLD];
            const bool has_next = gn < g_end;
            const u32x4 *pnext = act_ptr(has_next ? gn : g, has_next ? pn : p);
            MRP_LOAD_STAGE(pnext, st)
            const u32x4 *cur = smem + buf * STAGE;
#pragma unroll
            for (int j = 0; j < KSTEP; ++j) {
                u32x4 bfr[IT];
#pragma unroll
                for (int it = 0; it < IT; ++it) bfr[it] = cur[(j * IT + it) * 64 + lane];
#pragma unroll
                for (int it = 0; it < IT; ++it) acc[it] = mma_frag<EPI>(wreg[PAR * KSTEP + j], bfr[it], acc[it]);
            }
            if (p == np - 1 && g + 2 < g_end) {
#pragma unroll
                for (int j = 0; j < KSTEP; ++j)
                    wreg[PAR * KSTEP + j] = wptr[(size_t)((g + 2) * KSTEP + j) * 64];
            }
            u32x4 *nxt = smem + (buf ^ 1) * STAGE;
#pragma unroll
            for (int n = 0; n < NLD; ++n) nxt[tid + 256 * n] = st[n];
            if (has_next) advance();
            __syncthreads();
            buf ^= 1;
        }
    };
    for (int g = g_begin; g < g_end; g += 2) {
        krange(std::integral_constant<int, 0>{}, g);
        if (g + 1 < g_end) krange(std::integral_constant<int, 1>{}, g + 1);
    }

#undef MRP_LOAD_STAGE
    // ---- epilogue ----
    if constexpr (EPI == EPI_PARTIAL) {
        if (rb_ok) {
#pragma unroll
            for (int it = 0; it < IT; ++it) {
                const int i = (ib0 + it) * 32 + ln;
                if (i < a.M) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const int r = rb * 32 + 8 * q + 4 * lh;
                        if (r < a.R)
                            *reinterpret_cast<float4 *>(a.out + ((size_t)ks * a.M + i) * a.R + r) =
                                make_float4(acc[it][4 * q], acc[it][4 * q + 1], acc[it][4 * q + 2],
                                            acc[it][4 * q + 3]);
                    }
                }
            }
        }
    } else {
        float *red_m = reinterpret_cast<float *>(smem + 2 * STAGE);
        float *red_s = red_m + WG_WAVES * ROWS;
        int *red_i = reinterpret_cast<int *>(red_s + WG_WAVES * ROWS);
#pragma unroll
        for (int it = 0; it < IT; ++it) {
            const int i = (ib0 + it) * 32 + ln;
            const bool row_ok = rb_ok && i < a.M;
            Part pt = part_identity();
            // store the updated logits and find this lane's maximum (ascending v)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int v = rb * 32 + 8 * q + 4 * lh;
                if (row_ok) {
                    float *zp = a.z + (size_t)i * a.R + v;
                    if constexpr (VEC4) {
                        if (v < a.R)
                            *reinterpret_cast<float4 *>(zp) = make_float4(
                                acc[it][4 * q], acc[it][4 * q + 1], acc[it][4 * q + 2], acc[it][4 * q + 3]);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (v + e < a.R) zp[e] = acc[it][4 * q + e];
                    }
                }
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float x = acc[it][4 * q + e];
                    if (rb_ok && v + e < a.R && x > pt.m) { pt.m = x; pt.i = v + e; }
                }
            }
            float s = 0.f;
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int v = rb * 32 + 8 * q + 4 * lh + e;
                    if (rb_ok && v < a.R) s += __expf(acc[it][4 * q + e] - pt.m);
                }
            pt.s = s;
            Part other;
            other.m = __shfl_xor(pt.m, 32);
            other.s = __shfl_xor(pt.s, 32);
            other.i = __shfl_xor(pt.i, 32);
            pt = part_merge(pt, other);
            if (lh == 0) {
                red_m[wave * ROWS + it * 32 + ln] = pt.m;
                red_s[wave * ROWS + it * 32 + ln] = pt.s;
                red_i[wave * ROWS + it * 32 + ln] = pt.i;
            }
        }
        __syncthreads();
        if (tid < ROWS) {
            Part pt = {red_m[tid], red_s[tid], red_i[tid]};
#pragma unroll
            for (int wv = 1; wv < WG_WAVES; ++wv)
                pt = part_merge(pt, Part{red_m[wv * ROWS + tid], red_s[wv * ROWS + tid], red_i[wv * ROWS + tid]});
            const int i = ib0 * 32 + tid;
            if (i < a.M) {
                a.pm[(size_t)vt * a.M + i] = pt.m;
                a.ps[(size_t)vt * a.M + i] = pt.s;
                a.pi[(size_t)vt * a.M + i] = pt.i;
            }
        }
    }
}

// IT = 4 (up to 128 activation rows per workgroup): two workgroups per CU, so the
// register budget is capped at 256 per lane.  IT = 8: one workgroup per CU.
template <int EPI, bool VEC4>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void stream_gemm_kernel4(
    const StreamGemmArgs a) {
    stream_gemm_body<4, EPI, VEC4>(a);
}
template <int EPI, bool VEC4>
__global__ __launch_bounds__(256) void stream_gemm_kernel8(const StreamGemmArgs a) {
    stream_gemm_body<8, EPI, VEC4>(a);
}

template <int IT>
constexpr size_t lds_bytes() {
    return (size_t)2 * KSTEP * IT * 64 * 16 + (size_t)WG_WAVES * IT * 32 * 12;
}

template <int IT, int EPI, bool VEC4>
auto kernel_of() -> void (*)(const StreamGemmArgs) {
    if constexpr (IT == 4) return stream_gemm_kernel4<EPI, VEC4>;
    else return stream_gemm_kernel8<EPI, VEC4>;
}

template <int IT, int EPI, bool VEC4>
hipError_t configure_inst() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(kernel_of<IT, EPI, VEC4>()),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes<IT>());
}

template <int IT, int EPI, bool VEC4>
hipError_t launch_inst(const StreamGemmArgs &a, hipStream_t st) {
    const int nWG = a.nVt * a.nMg * a.nKs;
    const int per = (nWG + 7) / 8;
    hipLaunchKernelGGL((kernel_of<IT, EPI, VEC4>()), dim3(per * 8), dim3(256), lds_bytes<IT>(), st, a);
    return hipGetLastError();
}

}  // namespace

// Once per device (mrp_create): the kernels need more than the default 64 KiB of dynamic LDS.
hipError_t stream_gemm_configure() {
    hipError_t e = configure_inst<4, EPI_PARTIAL, true>();
    if (e == hipSuccess) e = configure_inst<8, EPI_PARTIAL, true>();
    if (e == hipSuccess) e = configure_inst<4, EPI_LM, true>();
    if (e == hipSuccess) e = configure_inst<4, EPI_LM, false>();
    if (e == hipSuccess) e = configure_inst<8, EPI_LM, true>();
    if (e == hipSuccess) e = configure_inst<8, EPI_LM, false>();
    return e;
}

int stream_gemm_it(int M) { return M > 128 ? 8 : 4; }

size_t stream_gemm_lds_bytes(int it) { return it == 8 ? lds_bytes<8>() : lds_bytes<4>(); }

hipError_t launch_stream_gemm(const StreamGemmArgs &a, int epi, hipStream_t st) {
    const int it = stream_gemm_it(a.M);
    const bool vec4 = (a.R % 4) == 0;
    if (epi == EPI_PARTIAL) {
        return it == 8 ? launch_inst<8, EPI_PARTIAL, true>(a, st) : launch_inst<4, EPI_PARTIAL, true>(a, st);
    }
    if (it == 8)
        return vec4 ? launch_inst<8, EPI_LM, true>(a, st) : launch_inst<8, EPI_LM, false>(a, st);
    return vec4 ? launch_inst<4, EPI_LM, true>(a, st) : launch_inst<4, EPI_LM, false>(a, st);
}

}  // namespace mrp
