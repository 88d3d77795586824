// Transformer head body (paper Section 3.2: fuse projection -> D transformer layers -> shared LM
// head; D = 3 in Section 4.1).  The paper gives the outline only; the layer is the decoder layer of
// the backbone's model family:
//     n = RMSNorm(u) g1;  q, k, v = Wqkv n;  rotary embedding of q, k at position prefix_len + i
//     o = attention of every block row over the sequence's prefix cache (bf16 keys / values) and
//         the L rows of the block itself (no mask inside the block), grouped-query heads
//     a = u + Wo o;  m = RMSNorm(a) g2;  u' = a + Wdown( SiLU(Wgate m) * (Wup m) )
// The four projections run on the shared GEMM kernels (fp32 activations as two fp16 planes, fp32
// partial sums); this file holds what sits between them: the residual-stream update with RMSNorm,
// the gated activation, the rotary table and the attention kernel.  Everything here is fp32.
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int HD = 128;   // head dimension (fixed)
constexpr int TK = 128;   // prefix keys per tile
constexpr int LB = 16;    // largest block length the attention kernel stages
constexpr int KROW = HD + 8;   // padded key row in LDS (272 bytes)
constexpr int SROW = TK + 4;   // padded score row: queries a wave works on side by side fall on different banks

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

// cos / sin of pos * theta^(-2j/HD) for every row and j < HD/2, evaluated in fp64
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t *__restrict__ prefix_len, int B, int L,
                                                         int P_max, double theta, float2 *__restrict__ out) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)B * L * (HD / 2)) return;
    const int j = (int)(idx % (HD / 2));
    const int row = (int)(idx / (HD / 2));
    const int b = row / L, i = row % L;
    int P = prefix_len[b];
    P = P < 0 ? 0 : (P > P_max ? P_max : P);
    const double ang = (double)(P + i) * pow(theta, -2.0 * (double)j / (double)HD);
    out[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

constexpr int NORM_MAX_CHUNKS = 4;  // per thread: d <= 8 * 256 * 4 = 8192

// One workgroup per row: x = (resid ? resid : 0) + sum of partials; stream <- x;
// planes <- split2(RMSNorm(x) gain).
__global__ __launch_bounds__(256) void resid_norm_split_kernel(const float *__restrict__ part, int nKs,
                                                               const float *resid, float *stream,
                                                               const uint16_t *__restrict__ gain, float eps,
                                                               uint4 *__restrict__ planes, long plane_stride, int nIb,
                                                               int M, int d) {
    __shared__ float wsum[4];
    const int i = xcd_row_of(blockIdx.x);
    if (i >= M) return;   // (uniform over the workgroup)
    const int C8 = d >> 3;
    float x[NORM_MAX_CHUNKS][8];
    float ss = 0.f;
#pragma unroll
    for (int n = 0; n < NORM_MAX_CHUNKS; ++n) {
        const int c8 = threadIdx.x + 256 * n;
#pragma unroll
        for (int e = 0; e < 8; ++e) x[n][e] = 0.f;
        if (c8 < C8) {
            sum_partials(part, (size_t)M * d, nKs, (size_t)i * d + 8 * c8, x[n]);
            if (resid) {
                const float4 *rp = reinterpret_cast<const float4 *>(resid + (size_t)i * d + 8 * c8);
                const float4 a = rp[0], b = rp[1];
                x[n][0] += a.x; x[n][1] += a.y; x[n][2] += a.z; x[n][3] += a.w;
                x[n][4] += b.x; x[n][5] += b.y; x[n][6] += b.z; x[n][7] += b.w;
            }
            float4 *sp = reinterpret_cast<float4 *>(stream + (size_t)i * d + 8 * c8);
            sp[0] = make_float4(x[n][0], x[n][1], x[n][2], x[n][3]);
            sp[1] = make_float4(x[n][4], x[n][5], x[n][6], x[n][7]);
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += x[n][e] * x[n][e];
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
            float g[8], y[8];
            unpack_bf16x8(*reinterpret_cast<const uint4 *>(gain + 8 * c8), g);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = x[n][e] * inv * g[e];
            split_store(y, planes, act_chunk_index(i, c8, nIb), plane_stride);
        }
    }
}

// part: [nKs][M][2 ff] (gate columns, then up columns) -> planes of SiLU(gate) * up, ff columns
__global__ __launch_bounds__(256) void swiglu_split_kernel(const float *__restrict__ part, int nKs,
                                                           uint4 *__restrict__ planes, long plane_stride, int nIb,
                                                           int M, int ff) {
    int i, c8;
    if (!plane_block_lane((size_t)blockIdx.x * 4 + (threadIdx.x >> 6), ff >> 4, M, i, c8)) return;
    float g[8], u[8], x[8];
    sum_partials(part, (size_t)M * 2 * ff, nKs, (size_t)i * 2 * ff + 8 * c8, g);
    sum_partials(part, (size_t)M * 2 * ff, nKs, (size_t)i * 2 * ff + ff + 8 * c8, u);
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = g[e] / (1.0f + expf(-g[e])) * u[e];
    split_store(x, planes, act_chunk_index(i, c8, nIb), plane_stride);
}

// ------------------------------------------------------------------------------------------------
// Attention.  One workgroup per (kv head g, sequence b): its Q = (nh / nkv) * L query vectors
// (query qq = hrep * L + i: head g * rep + hrep, block row i) share the keys and values of head g.
// Keys arrive in tiles (TK prefix positions from the bf16 cache, then the block's own L rows in
// fp32); per tile: scores -> LDS, online softmax per query (running max / sum, rescale factor),
// then the value sum.
struct AttnArgs {
    const float *qkv;        // partial sums [nKs][M][ldq] of the q | k | v projection
    size_t split_stride;
    int nKs, ldq;
    const float2 *rope;      // [M][HD / 2]
    const uint16_t *kc, *vc; // [B][P_max][nkv][HD] bf16
    const int32_t *prefix_len;
    int P_max, nh, nkv, L;
    uint4 *o_planes;         // attention output, columns head * HD + e, as the activation planes of the next GEMM
    long plane_stride;
    int nIb;
};

// sum over the k splits of one projection output, in split order; eight loads in flight at a time
__device__ __forceinline__ float sum_col(const AttnArgs &a, size_t off) {
    float x = 0.f;
    for (int k0 = 0; k0 < a.nKs; k0 += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = (k0 + u < a.nKs) ? a.qkv[(size_t)(k0 + u) * a.split_stride + off] : 0.f;
#pragma unroll
        for (int u = 0; u < 8; ++u) x += v[u];
    }
    return x;
}

// softmax bookkeeping of one tile: S[qq][0 .. ncols) holds raw scores (-inf = no key) and is
// replaced by exp(score - new running max); 256 / NQ adjacent lanes share a query, lane `part`
// taking columns part, part + TPQ, ...
template <int NQ>
__device__ __forceinline__ void softmax_tile(float (*S)[SROW], float *run_m, float *run_l, float *rescale, int ncols) {
    constexpr int TPQ = 256 / NQ;   // 4 .. 32 lanes per query, inside one wave
    const int qq = threadIdx.x / TPQ, part = threadIdx.x % TPQ;
    float mx = -INFINITY;
    for (int c = part; c < ncols; c += TPQ) mx = fmaxf(mx, S[qq][c]);
#pragma unroll
    for (int off = TPQ / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float m_old = run_m[qq];
    const float m_new = fmaxf(m_old, mx);   // finite: every tile holds at least one key
    float sum = 0.f;
    for (int c = part; c < ncols; c += TPQ) {
        const float p = __expf(S[qq][c] - m_new);   // exp(-inf) = 0 for absent keys
        S[qq][c] = p;
        sum += p;
    }
#pragma unroll
    for (int off = TPQ / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (part == 0) {
        const float f = (m_old == -INFINITY) ? 0.f : __expf(m_old - m_new);
        rescale[qq] = f;
        run_m[qq] = m_new;
        run_l[qq] = run_l[qq] * f + sum;
    }
}

template <int QP>
__global__ __launch_bounds__(256) void attn_kernel(AttnArgs a) {
    constexpr int NQ = 8 * QP;   // query slots (Q <= NQ; unused slots hold zeros)
    extern __shared__ float smem[];
    float (*qs)[HD] = reinterpret_cast<float (*)[HD]>(smem);                       // [NQ][HD] rotated, scaled
    float (*kb)[HD] = reinterpret_cast<float (*)[HD]>(smem + NQ * HD);             // [LB][HD] rotated block keys
    float (*vb)[HD] = reinterpret_cast<float (*)[HD]>(smem + (NQ + LB) * HD);      // [LB][HD] block values
    float (*S)[SROW] = reinterpret_cast<float (*)[SROW]>(smem + (NQ + 2 * LB) * HD);   // [NQ][TK] (padded rows)
    float *run_m = smem + (NQ + 2 * LB) * HD + NQ * SROW;
    float *run_l = run_m + NQ;
    float *rescale = run_l + NQ;
    // the current prefix tile: keys with rows padded to KROW entries (a lane reading its own key row
    // 16 bytes at a time then hits every LDS bank once per 16 lanes), values unpadded
    uint16_t (*kt)[KROW] = reinterpret_cast<uint16_t (*)[KROW]>(rescale + NQ);
    uint16_t (*vt)[HD] = reinterpret_cast<uint16_t (*)[HD]>(reinterpret_cast<uint16_t *>(rescale + NQ) + TK * KROW);

    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int L = a.L, rep = a.nh / a.nkv, Q = rep * L;
    const int qd = a.nh * HD, kvd = a.nkv * HD;
    int P = a.prefix_len[b];
    P = P < 0 ? 0 : (P > a.P_max ? a.P_max : P);
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)

    // ---- prefix tiles: a tile's keys and values are requested (16 bytes per lane, whole cache rows)
    // while the previous tile is being worked on, then parked in LDS
    uint4 kreg[TK * HD / 8 / 256], vreg[TK * HD / 8 / 256];
    auto request = [&](int t0) {
#pragma unroll
        for (int n = 0; n < TK * HD / 8 / 256; ++n) {
            const int idx = tid + 256 * n, key = idx >> 4, c = idx & 15;
            const int t = t0 + key;
            kreg[n] = make_uint4(0, 0, 0, 0);
            vreg[n] = make_uint4(0, 0, 0, 0);
            if (t < P) {
                const size_t off = (((size_t)b * a.P_max + t) * a.nkv + g) * HD + 8 * c;
                kreg[n] = *reinterpret_cast<const uint4 *>(a.kc + off);
                vreg[n] = *reinterpret_cast<const uint4 *>(a.vc + off);
            }
        }
    };
    if (P > 0) request(0);

    // ---- prologue: the block's q (rotated, scaled), k (rotated) and v for this kv head
    for (int idx = tid; idx < NQ * (HD / 2); idx += 256) {
        const int qq = idx / (HD / 2), j = idx % (HD / 2);
        float r0 = 0.f, r1 = 0.f;
        if (qq < Q) {
            const int hrep = qq / L, i = qq % L, row = b * L + i;
            const size_t off = (size_t)row * a.ldq + (size_t)(g * rep + hrep) * HD;
            const float x0 = sum_col(a, off + j), x1 = sum_col(a, off + j + HD / 2);
            const float2 cs = a.rope[(size_t)row * (HD / 2) + j];
            r0 = (x0 * cs.x - x1 * cs.y) * scale;
            r1 = (x1 * cs.x + x0 * cs.y) * scale;
        }
        qs[qq][j] = r0;
        qs[qq][j + HD / 2] = r1;
    }
    for (int idx = tid; idx < L * (HD / 2); idx += 256) {
        const int i = idx / (HD / 2), j = idx % (HD / 2), row = b * L + i;
        const size_t off = (size_t)row * a.ldq + qd + (size_t)g * HD;
        const float x0 = sum_col(a, off + j), x1 = sum_col(a, off + j + HD / 2);
        const float2 cs = a.rope[(size_t)row * (HD / 2) + j];
        kb[i][j] = x0 * cs.x - x1 * cs.y;
        kb[i][j + HD / 2] = x1 * cs.x + x0 * cs.y;
    }
    for (int idx = tid; idx < L * HD; idx += 256) {
        const int i = idx / HD, e = idx % HD, row = b * L + i;
        vb[i][e] = sum_col(a, (size_t)row * a.ldq + qd + kvd + (size_t)g * HD + e);
    }
    if (tid < NQ) { run_m[tid] = -INFINITY; run_l[tid] = 0.f; rescale[tid] = 0.f; }
    __syncthreads();

    // register tiles: a thread works on 4 keys x QP queries (scores) and 4 dimensions x QP queries
    // (values), so that one LDS read feeds four multiply-adds per query
    const int lg = tid & 31, qg = tid >> 5;   // key group / dimension group, query group
    float o[QP][4];
#pragma unroll
    for (int q = 0; q < QP; ++q)
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) o[q][dd] = 0.f;

    for (int t0 = 0; t0 < P; t0 += TK) {
#pragma unroll
        for (int n = 0; n < TK * HD / 8 / 256; ++n) {
            const int idx = tid + 256 * n, key = idx >> 4, c = idx & 15;
            *reinterpret_cast<uint4 *>(&kt[key][8 * c]) = kreg[n];
            *reinterpret_cast<uint4 *>(&vt[key][8 * c]) = vreg[n];
        }
        __syncthreads();
        if (t0 + TK < P) request(t0 + TK);
        {   // scores of keys lg, lg + 32, lg + 64, lg + 96 of the tile
            float acc[QP][4];
#pragma unroll
            for (int q = 0; q < QP; ++q)
#pragma unroll
                for (int u = 0; u < 4; ++u) acc[q][u] = 0.f;
            if (t0 + lg < P) {
#pragma unroll 2
                for (int c = 0; c < HD / 8; ++c) {
                    float kf[4][8];
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        unpack_bf16x8(*reinterpret_cast<const uint4 *>(&kt[lg + 32 * u][8 * c]), kf[u]);
#pragma unroll
                    for (int q = 0; q < QP; ++q) {
                        const float4 q0 = *reinterpret_cast<const float4 *>(&qs[qg * QP + q][8 * c]);
                        const float4 q1 = *reinterpret_cast<const float4 *>(&qs[qg * QP + q][8 * c + 4]);
#pragma unroll
                        for (int u = 0; u < 4; ++u)
                            acc[q][u] += q0.x * kf[u][0] + q0.y * kf[u][1] + q0.z * kf[u][2] + q0.w * kf[u][3] +
                                         q1.x * kf[u][4] + q1.y * kf[u][5] + q1.z * kf[u][6] + q1.w * kf[u][7];
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < QP; ++q)
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    S[qg * QP + q][lg + 32 * u] = (t0 + lg + 32 * u < P) ? acc[q][u] : -INFINITY;
        }
        __syncthreads();
        softmax_tile<NQ>(S, run_m, run_l, rescale, TK);
        __syncthreads();
        {   // values: dimensions 4 lg .. 4 lg + 3
#pragma unroll
            for (int q = 0; q < QP; ++q) {
                const float f = rescale[qg * QP + q];
#pragma unroll
                for (int dd = 0; dd < 4; ++dd) o[q][dd] *= f;
            }
            const int nk = (P - t0 < TK) ? (P - t0) : TK;   // (absent keys: probability 0, value 0)
            for (int k4 = 0; k4 < nk; k4 += 4) {
                float v[4][4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const uint2 raw = *reinterpret_cast<const uint2 *>(&vt[k4 + u][4 * lg]);
                    v[u][0] = __uint_as_float(raw.x << 16); v[u][1] = __uint_as_float(raw.x & 0xFFFF0000u);
                    v[u][2] = __uint_as_float(raw.y << 16); v[u][3] = __uint_as_float(raw.y & 0xFFFF0000u);
                }
#pragma unroll
                for (int q = 0; q < QP; ++q) {
                    const float4 p = *reinterpret_cast<const float4 *>(&S[qg * QP + q][k4]);
#pragma unroll
                    for (int dd = 0; dd < 4; ++dd)
                        o[q][dd] += p.x * v[0][dd] + p.y * v[1][dd] + p.z * v[2][dd] + p.w * v[3][dd];
                }
            }
        }
        __syncthreads();
    }

    // ---- the block's own rows (fp32 keys and values from LDS); 16 score columns, absent keys -inf
    for (int qq = tid >> 4; qq < NQ; qq += 16) {
        const int key = tid & 15;
        float acc = -INFINITY;
        if (key < L) {
            acc = 0.f;
            for (int e = 0; e < HD; ++e) acc += qs[qq][e] * kb[key][e];
        }
        S[qq][key] = acc;
    }
    __syncthreads();
    softmax_tile<NQ>(S, run_m, run_l, rescale, 16);
    __syncthreads();
#pragma unroll
    for (int q = 0; q < QP; ++q) {
        const float f = rescale[qg * QP + q];
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) o[q][dd] *= f;
    }
    for (int k = 0; k < L; ++k) {
        const float4 v = *reinterpret_cast<const float4 *>(&vb[k][4 * lg]);
#pragma unroll
        for (int q = 0; q < QP; ++q) {
            const float pk = S[qg * QP + q][k];
            o[q][0] += pk * v.x; o[q][1] += pk * v.y; o[q][2] += pk * v.z; o[q][3] += pk * v.w;
        }
    }
    __syncthreads();

    // ---- normalise, stage as [query][dimension], write the activation planes
#pragma unroll
    for (int q = 0; q < QP; ++q) {
        const float inv_l = 1.0f / run_l[qg * QP + q];
        *reinterpret_cast<float4 *>(&S[qg * QP + q][4 * lg]) =
            make_float4(o[q][0] * inv_l, o[q][1] * inv_l, o[q][2] * inv_l, o[q][3] * inv_l);   // (TK == HD)
    }
    __syncthreads();
    for (int idx = tid; idx < Q * (HD / 8); idx += 256) {
        const int qq = idx / (HD / 8), c = idx % (HD / 8);
        const int hrep = qq / L, i = qq % L, row = b * L + i;
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = S[qq][8 * c + e];
        split_store(x, a.o_planes, act_chunk_index(row, (g * rep + hrep) * (HD / 8) + c, a.nIb), a.plane_stride);
    }
}

static_assert(TK == HD, "the score tile doubles as the output staging buffer");

template <int QP>
constexpr size_t attn_lds_bytes() {
    return sizeof(float) * ((size_t)(8 * QP + 2 * LB) * HD + (size_t)8 * QP * SROW + 3 * 8 * QP) +
           sizeof(uint16_t) * ((size_t)TK * KROW + (size_t)TK * HD);
}

template <int QP>
hipError_t attn_configure_one() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_kernel<QP>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)attn_lds_bytes<QP>());
}

template <int QP>
hipError_t attn_launch_one(const AttnArgs &a, int B, hipStream_t st) {
    hipLaunchKernelGGL(attn_kernel<QP>, dim3(a.nkv, B), dim3(256), attn_lds_bytes<QP>(), st, a);
    return hipGetLastError();
}

}  // namespace

hipError_t tbody_configure() {
    hipError_t e = attn_configure_one<1>();
    if (e == hipSuccess) e = attn_configure_one<2>();
    if (e == hipSuccess) e = attn_configure_one<4>();
    if (e == hipSuccess) e = attn_configure_one<8>();
    return e;
}

bool tbody_shape_ok(int nh, int nkv, int head_dim, int L) {
    return head_dim == HD && nkv >= 1 && nh >= nkv && nh % nkv == 0 && L >= 1 && L <= LB && (nh / nkv) * L <= 64;
}

hipError_t launch_rope_table(const int32_t *prefix_len, int B, int L, int P_max, double theta, float2 *out,
                             hipStream_t st) {
    hipLaunchKernelGGL(rope_table_kernel, dim3(blocks_for((size_t)B * L * (HD / 2))), dim3(256), 0, st, prefix_len,
                       B, L, P_max, theta, out);
    return hipGetLastError();
}

hipError_t launch_resid_norm_split(const float *part, int nKs, const float *resid, float *stream,
                                   const uint16_t *gain, float eps, uint4 *planes, long plane_stride, int nIb, int M,
                                   int d, hipStream_t st) {
    hipLaunchKernelGGL(resid_norm_split_kernel, dim3((M + 255) / 256 * 256), dim3(256), 0, st, part, nKs, resid, stream, gain, eps,
                       planes, plane_stride, nIb, M, d);
    return hipGetLastError();
}

hipError_t launch_swiglu_split(const float *part, int nKs, uint4 *planes, long plane_stride, int nIb, int M, int ff,
                               hipStream_t st) {
    hipLaunchKernelGGL(swiglu_split_kernel, dim3((unsigned)(((size_t)((M + 31) / 32) * (ff / 16) + 3) / 4)), dim3(256), 0, st, part, nKs,
                       planes, plane_stride, nIb, M, ff);
    return hipGetLastError();
}

hipError_t launch_attention(const float *qkv, int nKs, int M, int B, int L, int nh, int nkv, const float2 *rope,
                            const uint16_t *kc, const uint16_t *vc, const int32_t *prefix_len, int P_max,
                            uint4 *o_planes, long plane_stride, int nIb, hipStream_t st) {
    AttnArgs a;
    a.qkv = qkv;
    a.ldq = (nh + 2 * nkv) * HD;
    a.split_stride = (size_t)M * a.ldq;
    a.nKs = nKs;
    a.rope = rope;
    a.kc = kc; a.vc = vc;
    a.prefix_len = prefix_len;
    a.P_max = P_max; a.nh = nh; a.nkv = nkv; a.L = L;
    a.o_planes = o_planes; a.plane_stride = plane_stride; a.nIb = nIb;
    const int Q = (nh / nkv) * L;
    if (Q <= 8) return attn_launch_one<1>(a, B, st);
    if (Q <= 16) return attn_launch_one<2>(a, B, st);
    if (Q <= 32) return attn_launch_one<4>(a, B, st);
    return attn_launch_one<8>(a, B, st);
}

}  // namespace mrp
