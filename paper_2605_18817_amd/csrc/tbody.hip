// Transformer head body (paper Section 3.2: fuse projection -> D transformer layers -> shared LM
// head; D = 3 in Section 4.1).  The paper gives the outline only; the layer is the decoder layer of
// the backbone's model family:
//     n = RMSNorm(u) g1;  q, k, v = Wqkv n;  rotary embedding of q, k at position prefix_len + i
//     o = attention of every block row over the sequence's prefix cache (bf16 keys / values) and
//         the L rows of the block itself (no mask inside the block), grouped-query heads
//     a = u + Wo o;  m = RMSNorm(a) g2;  u' = a + Wdown( SiLU(Wgate m) * (Wup m) )
// The four projections run on the shared GEMM kernels (fp32 activations as two fp16 planes, fp32
// partial sums); this file holds what sits between them: the residual-stream update with RMSNorm,
// the gated activation, the rotary table and the attention kernel (fp32 on the vector ALU, and the
// matrix cores with three-term bf16 operands for the two contractions over the prefix cache).
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int HD = 128;   // head dimension (fixed)
constexpr int LB = 16;    // largest block length the attention kernel stages
constexpr int KROW = HD + 8;   // padded key row in LDS (272 bytes)
constexpr int ATTN_MAX_SPLIT = 4;       // workgroups that may share one (kv head, sequence) pair's prefix
constexpr int ATTN_SPLIT_PAIRS = 256;   // pairs x split stays within this (one workgroup per CU)

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

// cos / sin of pos * theta^(-2j/HD) for every row and j < HD/2, evaluated in fp64
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t *__restrict__ prefix_len, int B, int L,
                                                         int P_max, double theta, float2 *__restrict__ out,
                                                         int *err_flag) {
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)B * L * (HD / 2)) return;
    const int j = (int)(idx % (HD / 2));
    const int row = (int)(idx / (HD / 2));
    const int b = row / L, i = row % L;
    int P = prefix_len[b];
    if ((P < 0 || P > P_max) && i == 0 && j == 0 && err_flag) atomicOr(err_flag, ERR_PREFIX_LEN);   // clamped and reported
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
// Attention.  One workgroup (NW = 8 or 4 wavefronts) per (kv head g, sequence b), or several that share
// the pair's prefix: its Q = (nh / nkv) * L query
// vectors (query qq = hrep * L + i: head g * rep + hrep, block row i) share the keys and values of
// head g.
//   * The block's own L keys and values (fp32, from the projection) are handled by the whole
//     workgroup on the vector ALU.
//   * The prefix cache is walked in chunks of 32 positions, chunk c by wavefront c % NW, and each
//     wavefront runs its own online softmax over its chunks: no workgroup barrier inside the walk.
//     Both contractions run on the matrix cores on the cache's bf16 values as they are, with the fp32
//     operand of each (queries, probabilities) as three bf16 terms (x = a + b + c up to 2^-24 |x|):
//       scores  S^T[key][q]  = K[key][:] . (q_a + q_b + q_c)[q][:]          A = keys,      B = query planes
//       values  o^T[dim][q] += V^T[dim][key] (p_a + p_b + p_c)[q][key]      A = values^T,  B = probabilities
//     In both a lane's 16 accumulators belong to ONE query (column lane % 32), so the chunk's maximum
//     and sum per query need one exchange with lane ^ 32, and the lane's 16 probabilities are, as they
//     stand, its two B fragments of the value product.  Key fragments come straight from global memory;
//     a chunk's value rows are parked in LDS as they are and the transposed fragments (a lane = one
//     dimension, 8 positions) are read back with the transposing 64-bit LDS read, four positions at a time.
//   * At the end the partial results per query (block, the wavefronts) are merged in a fixed order.
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
    // Few (kv head, sequence) pairs leave most CUs idle: then `ns` workgroups share a pair's prefix (workgroup sp
    // of a pair walks chunks (j ns + sp) NW + wave; sp = 0 also takes the block's own rows), each writes its
    // partial (maximum, sum, value sum in units of P_SCALE relative to that maximum) and attn_merge_kernel
    // combines the ns partials in the order sp = 0, 1, ...
    int ns;
    float *po;               // [pairs][ns][NQ][HD]
    float *pml;              // [pairs][ns][NQ][2]
};

constexpr float P_SCALE = 1.f;         // unit of the value sums (bf16 terms need no scaling)
constexpr int NTERM = 3;               // bf16 terms of an fp32 operand
constexpr int VROW = HD + 16;          // padded value row in LDS (288 bytes: four consecutive rows fall into different banks)
constexpr int CK = 32;                 // prefix positions per chunk
constexpr int SCOLS = 20;              // score columns of the block phase (16 + padding)
constexpr int QROW = HD + 4;           // padded fp32 query / merged-output row in LDS: a wave's 32 rows at one column spread over the banks
constexpr int KBROW = HD + 4;          // padded fp32 block-key row in LDS: the 16 keys of a score pass fall into different banks

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

__device__ __forceinline__ f32x16 mma_bf16(const uint4 &x, const uint4 &y, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, x), __builtin_bit_cast(bf16x8, y), c, 0, 0, 0);
}

// x = t[0] + t[1] + t[2] up to 2^-24 |x|: three bf16 terms by truncation, each left as the fp32 bit pattern of the
// term (low 16 bits zero); every remainder is exact and has the sign of x
__device__ __forceinline__ void split3(float x, uint32_t (&t)[NTERM]) {
    t[0] = __float_as_uint(x) & 0xffff0000u;
    const float r1 = x - __uint_as_float(t[0]);
    t[1] = __float_as_uint(r1) & 0xffff0000u;
    const float r2 = r1 - __uint_as_float(t[1]);
    t[2] = __float_as_uint(r2) & 0xffff0000u;
}
// two such terms as a bf16 pair (first term in the low half)
__device__ __forceinline__ uint32_t pair_bf16(uint32_t first, uint32_t second) { return second | (first >> 16); }

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 *lds_s16x4_ptr;

// row of a 32 x 32 accumulator tile held in element r of a lane of half-wave `half`
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// LDS carve-up of the attention kernel (NQ query slots); offsets in bytes
template <int NQ, int NW>
struct AttnLds {
    static constexpr size_t qs = 0;                                                // float [NQ][HD] (later: merged output)
    static constexpr size_t kb = qs + sizeof(float) * NQ * QROW;                   // float [LB][KBROW]
    static constexpr size_t vb = kb + sizeof(float) * LB * KBROW;                  // float [LB][HD]
    static constexpr size_t S = vb + sizeof(float) * LB * HD;                      // float [NQ][SCOLS]
    static constexpr size_t stat = S + sizeof(float) * NQ * SCOLS;                 // float [4][NQ] block max / sum, merged sum / max
    static constexpr size_t wstat = stat + sizeof(float) * 4 * NQ;                 // float [2][NW][NQ] per-wave max / sum
    static constexpr size_t qp = wstat + sizeof(float) * 2 * NW * NQ;              // bf16 [NTERM][NQ][KROW]
    static constexpr size_t vch = qp + sizeof(uint16_t) * NTERM * NQ * KROW;       // bf16 [NW][CK][VROW] per-wave value chunk
    static constexpr size_t total = vch + sizeof(uint16_t) * NW * CK * VROW;
};

// softmax of the block phase: S[qq][0 .. 16) holds raw scores (-inf = no key) and is replaced by
// exp(score - max); 256 / NQ adjacent lanes share a query.
template <int NQ, int NT>
__device__ __forceinline__ void softmax_block(float (*S)[SCOLS], float *blk_m, float *blk_l) {
    constexpr int TPQ = NT / NQ;    // 4 .. 16 lanes per query, inside one wave
    const int qq = threadIdx.x / TPQ, part = threadIdx.x % TPQ;
    float mx = -INFINITY;
    for (int c = part; c < 16; c += TPQ) mx = fmaxf(mx, S[qq][c]);
#pragma unroll
    for (int off = TPQ / 2; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float sum = 0.f;
    for (int c = part; c < 16; c += TPQ) {
        const float pr = __expf(S[qq][c] - mx);   // exp(-inf) = 0 for absent keys; the block has at least one row
        S[qq][c] = pr;
        sum += pr;
    }
#pragma unroll
    for (int off = TPQ / 2; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
    if (part == 0) { blk_m[qq] = mx; blk_l[qq] = sum; }
}

// NQB: blocks of 32 query slots (1 or 2); NW: wavefronts (8 = two per SIMD, with the next chunk's
// requests left to the other wave to hide; 4 = one per SIMD, each requesting one chunk ahead)
template <int NQB, int NW>
__global__ __launch_bounds__(64 * NW) void attn_kernel(AttnArgs a) {
    constexpr int NQ = 32 * NQB, NT = 64 * NW;
    using Lds = AttnLds<NQ, NW>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float (*qs)[QROW] = reinterpret_cast<float (*)[QROW]>(smem_raw + Lds::qs);   // rotated, scaled queries (fp32)
    float (*kb)[KBROW] = reinterpret_cast<float (*)[KBROW]>(smem_raw + Lds::kb); // rotated block keys
    float (*vb)[HD] = reinterpret_cast<float (*)[HD]>(smem_raw + Lds::vb);       // block values
    float (*S)[SCOLS] = reinterpret_cast<float (*)[SCOLS]>(smem_raw + Lds::S);
    float *blk_m = reinterpret_cast<float *>(smem_raw + Lds::stat);
    float *blk_l = blk_m + NQ;
    float *tot_l = blk_l + NQ;
    float *tot_m = tot_l + NQ;
    float (*w_m)[NQ] = reinterpret_cast<float (*)[NQ]>(smem_raw + Lds::wstat);    // [NW] per-wave running max
    float (*w_l)[NQ] = w_m + NW;                                                  // [NW] per-wave running sum
    uint16_t (*qp)[NQ][KROW] = reinterpret_cast<uint16_t (*)[NQ][KROW]>(smem_raw + Lds::qp);   // [NTERM] query planes
    uint16_t (*vch)[CK][VROW] = reinterpret_cast<uint16_t (*)[CK][VROW]>(smem_raw + Lds::vch); // [NW] value chunks

    const int g = blockIdx.x, b = blockIdx.y, sp = blockIdx.z, ns = a.ns, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int L = a.L, rep = a.nh / a.nkv, Q = rep * L;
    const int qd = a.nh * HD, kvd = a.nkv * HD;
    int P = a.prefix_len[b];
    P = P < 0 ? 0 : (P > a.P_max ? a.P_max : P);
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    const int nchunks = (P + CK - 1) / CK;
    const int c_first = sp * NW, c_step = NW * ns;    // this workgroup's chunks: c_first + wave + j c_step
    float *po = a.po + ((size_t)(b * a.nkv + g) * ns + sp) * NQ * HD;
    float *pml = a.pml + ((size_t)(b * a.nkv + g) * ns + sp) * NQ * 2;
    if (sp > 0 && c_first >= nchunks) {     // nothing of the prefix falls to this workgroup: an empty partial
        for (int q = tid; q < NQ; q += NT) { pml[2 * q] = -INFINITY; pml[2 * q + 1] = 0.f; }
        return;
    }

    // A wave's next chunk is requested while it works on the current one.  Keys go straight into
    // matrix-core A fragments (lane = key row, 16 bytes per 16 dimensions); values are fetched as
    // whole rows (16 consecutive lanes per position) and parked in the wave's LDS chunk.  Only the
    // prefix's last chunk can hold absent positions: its value rows are zeroed (their probabilities
    // are zero, but what lies in the cache there need not be finite); its key rows are masked by
    // the scores.
    uint4 kreg[HD / 16], vreg[CK * HD / 8 / 64];
    auto request_k = [&](int c) __attribute__((always_inline)) {
        const int tk = c * CK + l32;
        const uint16_t *kp = a.kc + (((size_t)b * a.P_max + (tk < P ? tk : P - 1)) * a.nkv + g) * HD + 8 * half;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) kreg[ks] = *reinterpret_cast<const uint4 *>(kp + 16 * ks);
    };
    auto request_v = [&](int c) __attribute__((always_inline)) {
        const bool whole = (c + 1) * CK <= P;     // (uniform over the wave)
        const uint16_t *vp = a.vc + (((size_t)b * a.P_max + c * CK + (lane >> 4)) * a.nkv + g) * HD + 8 * (lane & 15);
        const size_t vstep = (size_t)4 * a.nkv * HD;     // four positions further
        if (whole) {
#pragma unroll
            for (int n = 0; n < CK * HD / 8 / 64; ++n) vreg[n] = *reinterpret_cast<const uint4 *>(vp + n * vstep);
        } else {
#pragma unroll
            for (int n = 0; n < CK * HD / 8 / 64; ++n) {
                vreg[n] = make_uint4(0, 0, 0, 0);
                if (c * CK + (lane >> 4) + 4 * n < P) vreg[n] = *reinterpret_cast<const uint4 *>(vp + n * vstep);
            }
        }
    };
    if (c_first + wave < nchunks) { request_k(c_first + wave); request_v(c_first + wave); }

    // ---- prologue: the block's q (rotated, scaled; fp32 and as two fp16 planes), k (rotated) and v
    for (int idx = tid; idx < NQ * (HD / 2); idx += NT) {
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
        uint32_t t0[NTERM], t1[NTERM];
        split3(r0, t0);
        split3(r1, t1);
#pragma unroll
        for (int t = 0; t < NTERM; ++t) {
            qp[t][qq][j] = (uint16_t)(t0[t] >> 16);
            qp[t][qq][j + HD / 2] = (uint16_t)(t1[t] >> 16);
        }
    }
    if (sp == 0) {    // (uniform over the workgroup) the block's own keys and values
        for (int idx = tid; idx < L * (HD / 2); idx += NT) {
            const int i = idx / (HD / 2), j = idx % (HD / 2), row = b * L + i;
            const size_t off = (size_t)row * a.ldq + qd + (size_t)g * HD;
            const float x0 = sum_col(a, off + j), x1 = sum_col(a, off + j + HD / 2);
            const float2 cs = a.rope[(size_t)row * (HD / 2) + j];
            kb[i][j] = x0 * cs.x - x1 * cs.y;
            kb[i][j + HD / 2] = x1 * cs.x + x0 * cs.y;
        }
        for (int idx = tid; idx < L * HD; idx += NT) {
            const int i = idx / HD, e = idx % HD, row = b * L + i;
            vb[i][e] = sum_col(a, (size_t)row * a.ldq + qd + kvd + (size_t)g * HD + e);
        }
    }
    __syncthreads();

    // ---- the block's own rows (fp32 keys and values, vector ALU); absent keys -inf.  The value sum is
    // held in accumulator layout: wave w owns dimensions 32 w .. 32 w + 31, element r of a lane is
    // o[query 32 qb + lane % 32][dimension 32 w + acc_row(r, half)], in units of P_SCALE.
    f32x16 o_blk[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_blk[qb][r] = 0.f;
    if (sp == 0) {
        for (int qq = tid >> 4; qq < NQ; qq += NT / 16) {
            const int key = tid & 15;
            float acc = -INFINITY;
            if (key < L) {
                float4 s4 = make_float4(0.f, 0.f, 0.f, 0.f);
                for (int e = 0; e < HD; e += 4) {
                    const float4 qv = *reinterpret_cast<const float4 *>(&qs[qq][e]);
                    const float4 kv = *reinterpret_cast<const float4 *>(&kb[key][e]);
                    s4.x += qv.x * kv.x; s4.y += qv.y * kv.y; s4.z += qv.z * kv.z; s4.w += qv.w * kv.w;
                }
                acc = (s4.x + s4.y) + (s4.z + s4.w);
            }
            S[qq][key] = acc;
        }
        __syncthreads();
        softmax_block<NQ, NT>(S, blk_m, blk_l);
        __syncthreads();
        for (int k = 0; k < L && wave < 4; ++k) {   // (waves 0 .. 3 own the 4 x 32 dimensions of the block's partial)
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb) {
                const float pk = S[32 * qb + l32][k] * P_SCALE;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float4 v = *reinterpret_cast<const float4 *>(&vb[k][32 * wave + 8 * j + 4 * half]);
                    o_blk[qb][4 * j + 0] += pk * v.x; o_blk[qb][4 * j + 1] += pk * v.y;
                    o_blk[qb][4 * j + 2] += pk * v.z; o_blk[qb][4 * j + 3] += pk * v.w;
                }
            }
        }
    } else {          // the block's rows belong to the pair's first workgroup
        for (int q = tid; q < NQ; q += NT) { blk_m[q] = -INFINITY; blk_l[q] = 0.f; }
    }

    // ---- this wave's chunks of the prefix: running max / sum per query (both half-waves hold the
    // same copy) and the value sum for ALL 128 dimensions (4 blocks of 32), in units of P_SCALE
    float run_m[NQB], run_l[NQB];
    f32x16 o_acc[NQB][4];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        run_m[qb] = -INFINITY;
        run_l[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) o_acc[qb][db][r] = 0.f;
    }
    // LDS addresses of this lane's transposing reads: the 16 lanes of a group fetch 4 rows x 16 dimensions
    // (lane s of the group: row s / 4, dimensions 4 (s % 4) ..) and lane L of the group receives the 4 rows'
    // values of dimension L.  Groups 0, 1 serve half-wave 0 (dimensions 0 .. 15 and 16 .. 31 of a block of 32),
    // groups 2, 3 half-wave 1, whose accumulator rows start 4 positions further.
    const int gq = lane >> 4, gs = lane & 15;
    const uint16_t *vt_base = &vch[wave][4 * half + (gs >> 2)][16 * (gq & 1) + 4 * (gs & 3)];
    for (int c = c_first + wave; c < nchunks; c += c_step) {
        __builtin_amdgcn_wave_barrier();   // (the previous chunk's value reads come before these writes)
#pragma unroll
        for (int n = 0; n < CK * HD / 8 / 64; ++n)
            *reinterpret_cast<uint4 *>(&vch[wave][(lane >> 4) + 4 * n][8 * (lane & 15)]) = vreg[n];
        __builtin_amdgcn_wave_barrier();
        if (c + c_step < nchunks) request_v(c + c_step);   // (the value registers are free again)

        uint4 pf[NQB][2][NTERM];          // probabilities: [k step of the value product][term]
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            // scores of the chunk's 32 keys for this lane's query
            f32x16 sc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < HD / 16; ++ks) {
                const int col = 16 * ks + 8 * half;
#pragma unroll
                for (int t = 0; t < NTERM; ++t)
                    sc = mma_bf16(kreg[ks], *reinterpret_cast<const uint4 *>(&qp[t][32 * qb + l32][col]), sc);
            }
            if (qb == NQB - 1 && c + c_step < nchunks) request_k(c + c_step);   // (the key registers are free again)
            float cmax = -INFINITY;
            if ((c + 1) * CK > P) {     // (uniform) the prefix's last chunk: absent positions score -inf
#pragma unroll
                for (int r = 0; r < 16; ++r) sc[r] = (c * CK + acc_row(r, half) < P) ? sc[r] : -INFINITY;
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) cmax = fmaxf(cmax, sc[r]);
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32));   // finite: a chunk holds at least one key
            const float m_new = fmaxf(run_m[qb], cmax);
            const float f = (run_m[qb] == -INFINITY) ? 0.f : __expf(run_m[qb] - m_new);
            float csum = 0.f;
            uint32_t pt[16][NTERM];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pr = __expf(sc[r] - m_new);   // exp(-inf) = 0 for absent keys
                csum += pr;
                split3(pr, pt[r]);
            }
            csum += __shfl_xor(csum, 32);
            run_l[qb] = run_l[qb] * f + csum;
            run_m[qb] = m_new;
            if (__any(f != 1.0f)) {   // (uniform over the wave: once the maxima have settled nothing is rescaled)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) o_acc[qb][db][r] *= f;
            }
            // the lane's 16 probabilities are its B fragments: k step s holds accumulator rows 8 s .. 8 s + 7
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int t = 0; t < NTERM; ++t)
                    pf[qb][s2][t] = make_uint4(pair_bf16(pt[8 * s2][t], pt[8 * s2 + 1][t]), pair_bf16(pt[8 * s2 + 2][t], pt[8 * s2 + 3][t]),
                                               pair_bf16(pt[8 * s2 + 4][t], pt[8 * s2 + 5][t]), pair_bf16(pt[8 * s2 + 6][t], pt[8 * s2 + 7][t]));
        }
        // values: V^T fragments in the same key order (k step s, element e <-> accumulator row 8 s + e =
        // chunk row 16 s + 8 (e / 4) + 4 half + e % 4): two transposing reads of four rows each
#pragma unroll
        for (int db = 0; db < 4; ++db) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                const s16x4 v0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt_base + (16 * s2) * VROW + 32 * db));
                const s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(vt_base + (16 * s2 + 8) * VROW + 32 * db));
                const uint2 w0 = __builtin_bit_cast(uint2, v0), w1 = __builtin_bit_cast(uint2, v1);
                const uint4 vf = make_uint4(w0.x, w0.y, w1.x, w1.y);
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                    for (int t = 0; t < NTERM; ++t) o_acc[qb][db] = mma_bf16(vf, pf[qb][s2][t], o_acc[qb][db]);
            }
        }
    }

    // ---- merge the partial results per query in a fixed order: block, then the waves
    if (half == 0) {
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) { w_m[wave][32 * qb + l32] = run_m[qb]; w_l[wave][32 * qb + l32] = run_l[qb]; }
    }
    __syncthreads();   // (also: every wave is done with the fp32 queries, whose buffer takes the merged output)
    float f_blk[NQB], f_own[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb) {
        const int q = 32 * qb + l32;
        float m_tot = blk_m[q];
#pragma unroll
        for (int w = 0; w < NW; ++w) m_tot = fmaxf(m_tot, w_m[w][q]);
        f_blk[qb] = (blk_m[q] == -INFINITY) ? 0.f : __expf(blk_m[q] - m_tot);   // (m_tot is finite: some wave had a chunk)
        float l_tot = blk_l[q] * f_blk[qb];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float fw = (w_m[w][q] == -INFINITY) ? 0.f : __expf(w_m[w][q] - m_tot);
            l_tot += w_l[w][q] * fw;
            if (w == wave) f_own[qb] = fw;
        }
        if (wave == 0 && half == 0) { tot_l[q] = l_tot; tot_m[q] = m_tot; }
        if (wave < 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j)   // the block's partial: this wave's 32 dimensions
                *reinterpret_cast<float4 *>(&qs[q][32 * wave + 8 * j + 4 * half]) =
                    make_float4(o_blk[qb][4 * j] * f_blk[qb], o_blk[qb][4 * j + 1] * f_blk[qb],
                                o_blk[qb][4 * j + 2] * f_blk[qb], o_blk[qb][4 * j + 3] * f_blk[qb]);
        }
    }
    __syncthreads();
    for (int w = 0; w < NW && c_first + w < nchunks; ++w) {   // (uniform over the workgroup)
        if (wave == w) {
#pragma unroll
            for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        float4 *dst = reinterpret_cast<float4 *>(&qs[32 * qb + l32][32 * db + 8 * j + 4 * half]);
                        float4 v = *dst;
                        v.x += o_acc[qb][db][4 * j] * f_own[qb]; v.y += o_acc[qb][db][4 * j + 1] * f_own[qb];
                        v.z += o_acc[qb][db][4 * j + 2] * f_own[qb]; v.w += o_acc[qb][db][4 * j + 3] * f_own[qb];
                        *dst = v;
                    }
        }
        __syncthreads();
    }

    if (ns > 1) {     // this workgroup's partial; attn_merge_kernel finishes
        for (int idx = tid; idx < Q * (HD / 4); idx += NT) {
            const int qq = idx / (HD / 4), c = idx % (HD / 4);
            *reinterpret_cast<float4 *>(po + (size_t)qq * HD + 4 * c) = *reinterpret_cast<const float4 *>(&qs[qq][4 * c]);
        }
        for (int q = tid; q < Q; q += NT) { pml[2 * q] = tot_m[q]; pml[2 * q + 1] = tot_l[q]; }
        return;
    }
    // ---- normalise and write the activation planes
    for (int idx = tid; idx < Q * (HD / 8); idx += NT) {
        const int qq = idx / (HD / 8), c = idx % (HD / 8);
        const int hrep = qq / L, i = qq % L, row = b * L + i;
        const float inv = 1.0f / (tot_l[qq] * P_SCALE);
        float x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = qs[qq][8 * c + e] * inv;
        split_store(x, a.o_planes, act_chunk_index(row, (g * rep + hrep) * (HD / 8) + c, a.nIb), a.plane_stride);
    }
}

// Combines the ns partials of every (kv head, sequence) pair in the order 0 .. ns - 1, normalises and writes the
// activation planes.  One thread per (query, 8 dimensions); NQ = the attention kernel's query slots.
__global__ __launch_bounds__(256) void attn_merge_kernel(AttnArgs a, int NQ) {
    const int g = blockIdx.x, b = blockIdx.y, ns = a.ns;
    const int L = a.L, rep = a.nh / a.nkv, Q = rep * L;
    const float *po = a.po + (size_t)(b * a.nkv + g) * ns * NQ * HD;
    const float *pml = a.pml + (size_t)(b * a.nkv + g) * ns * NQ * 2;
    for (int idx = threadIdx.x; idx < Q * (HD / 8); idx += 256) {
        const int qq = idx / (HD / 8), c = idx % (HD / 8);
        float m_tot = -INFINITY;
        for (int s = 0; s < ns; ++s) m_tot = fmaxf(m_tot, pml[((size_t)s * NQ + qq) * 2]);   // (partial 0 is never empty)
        float l_tot = 0.f, x[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] = 0.f;
        for (int s = 0; s < ns; ++s) {
            const float m = pml[((size_t)s * NQ + qq) * 2];
            if (m == -INFINITY) continue;
            const float f = __expf(m - m_tot);
            l_tot += pml[((size_t)s * NQ + qq) * 2 + 1] * f;
            const float4 *o = reinterpret_cast<const float4 *>(po + ((size_t)s * NQ + qq) * HD + 8 * c);
            const float4 o0 = o[0], o1 = o[1];
            x[0] += o0.x * f; x[1] += o0.y * f; x[2] += o0.z * f; x[3] += o0.w * f;
            x[4] += o1.x * f; x[5] += o1.y * f; x[6] += o1.z * f; x[7] += o1.w * f;
        }
        const float inv = 1.0f / (l_tot * P_SCALE);
#pragma unroll
        for (int e = 0; e < 8; ++e) x[e] *= inv;
        const int hrep = qq / L, i = qq % L, row = b * L + i;
        split_store(x, a.o_planes, act_chunk_index(row, (g * rep + hrep) * (HD / 8) + c, a.nIb), a.plane_stride);
    }
}

template <int NQB, int NW>
hipError_t attn_configure_one() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_kernel<NQB, NW>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)AttnLds<32 * NQB, NW>::total);
}

template <int NQB, int NW>
hipError_t attn_launch_one(const AttnArgs &a, int B, hipStream_t st) {
    constexpr size_t lds = AttnLds<32 * NQB, NW>::total;
    hipLaunchKernelGGL((attn_kernel<NQB, NW>), dim3(a.nkv, B, a.ns), dim3(64 * NW), lds, st, a);
    if (a.ns > 1) hipLaunchKernelGGL(attn_merge_kernel, dim3(a.nkv, B), dim3(256), 0, st, a, 32 * NQB);
    return hipGetLastError();
}

}  // namespace

hipError_t tbody_configure() {
    hipError_t e = attn_configure_one<1, 8>();
    if (e == hipSuccess) e = attn_configure_one<2, 4>();
    return e;
}

bool tbody_shape_ok(int nh, int nkv, int head_dim, int L) {
    return head_dim == HD && nkv >= 1 && nh >= nkv && nh % nkv == 0 && L >= 1 && L <= LB && (nh / nkv) * L <= 64;
}

hipError_t launch_rope_table(const int32_t *prefix_len, int B, int L, int P_max, double theta, float2 *out,
                             int *err_flag, hipStream_t st) {
    hipLaunchKernelGGL(rope_table_kernel, dim3(blocks_for((size_t)B * L * (HD / 2))), dim3(256), 0, st, prefix_len,
                       B, L, P_max, theta, out, err_flag);
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

// Workgroups per (kv head, sequence) pair: one when the pairs alone fill the CUs, else up to ATTN_MAX_SPLIT, no
// more than the longest prefix has rounds of chunks; pairs x split never exceeds ATTN_SPLIT_PAIRS.
int attention_split(int B, int nkv, int Q, int P_max) {
    const int pairs = B * nkv, nw = Q <= 32 ? 8 : 4;
    const int rounds = ((P_max + CK - 1) / CK + nw - 1) / nw;
    int ns = 1;
    while (ns * 2 <= ATTN_MAX_SPLIT && pairs * ns * 2 <= ATTN_SPLIT_PAIRS && ns * 2 <= rounds) ns *= 2;
    return ns;
}

size_t attention_scratch_floats() { return (size_t)ATTN_SPLIT_PAIRS * 64 * (HD + 2); }

hipError_t launch_attention(const float *qkv, int nKs, int M, int B, int L, int nh, int nkv, const float2 *rope,
                            const uint16_t *kc, const uint16_t *vc, const int32_t *prefix_len, int P_max,
                            uint4 *o_planes, long plane_stride, int nIb, float *scratch, hipStream_t st) {
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
    a.ns = attention_split(B, nkv, Q, P_max);
    a.po = scratch;
    a.pml = scratch + (size_t)ATTN_SPLIT_PAIRS * 64 * HD;
    if (Q <= 32) return attn_launch_one<1, 8>(a, B, st);
    return attn_launch_one<2, 4>(a, B, st);
}

}  // namespace mrp
