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
// matrix cores with two-term fp16 operands for the two contractions over the prefix cache).
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int HD = 128;   // head dimension (fixed)
constexpr int LB = 16;    // largest block length the attention kernel stages
constexpr int KROW = HD + 8;   // padded key row in LDS (272 bytes)

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
// Attention.  One workgroup (4 wavefronts) per (kv head g, sequence b): its Q = (nh / nkv) * L query
// vectors (query qq = hrep * L + i: head g * rep + hrep, block row i) share the keys and values of
// head g.
//   * The block's own L keys and values (fp32, from the projection) are handled by the whole
//     workgroup on the vector ALU.
//   * The prefix cache is walked in chunks of 32 positions, chunk c by wavefront c % 4, and each
//     wavefront runs its own online softmax over its chunks: no workgroup barrier inside the walk.
//     Both contractions run on the matrix cores with fp32-accurate operands (the same two-term fp16
//     split as the head body's GEMMs; the cache's bf16 values are converted to fp16):
//       scores  S^T[key][q]  = K[key][:] . (q_hi + q_lo)[q][:]        A = keys,      B = query planes
//       values  o^T[dim][q] += V^T[dim][key] (p_hi + p_lo)[q][key]    A = values^T,  B = probabilities
//     In both a lane's 16 accumulators belong to ONE query (column lane % 32), so the chunk's maximum
//     and sum per query need one exchange with lane ^ 32, and the lane's 16 probabilities are, as they
//     stand, its two B fragments of the value product (the key order inside a chunk is immaterial as
//     long as the value fragments are gathered in the same order).
//   * At the end the five partial results per query (block, four wavefronts) are merged in a fixed order.
// Queries are scaled by 2^6 / sqrt(HD) and probabilities by 2^14 before the split so that the low
// terms stay normal fp16 numbers; both powers of two are taken out again exactly.
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

constexpr float Q_SCALE = 64.f;        // 2^6
constexpr float P_SCALE = 16384.f;     // 2^14
constexpr int CK = 32;                 // prefix positions per chunk
constexpr int SCOLS = 20;              // score columns of the block phase (16 + padding)

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

__device__ __forceinline__ f32x16 mma_f16(const uint4 &x, const uint4 &y, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, x), __builtin_bit_cast(f16x8, y), c, 0, 0, 0);
}

// row of a 32 x 32 accumulator tile held in element r of a lane of half-wave `half`
__device__ __forceinline__ int acc_row(int r, int half) { return 8 * (r >> 2) + 4 * half + (r & 3); }

// LDS carve-up of the attention kernel (NQ query slots); offsets in bytes
template <int NQ, int NW>
struct AttnLds {
    static constexpr size_t qs = 0;                                                // float [NQ][HD] (later: merged output)
    static constexpr size_t kb = qs + sizeof(float) * NQ * HD;                     // float [LB][HD]
    static constexpr size_t vb = kb + sizeof(float) * LB * HD;                     // float [LB][HD]
    static constexpr size_t S = vb + sizeof(float) * LB * HD;                      // float [NQ][SCOLS]
    static constexpr size_t stat = S + sizeof(float) * NQ * SCOLS;                 // float [3][NQ] block max / sum / scratch
    static constexpr size_t wstat = stat + sizeof(float) * 3 * NQ;                 // float [2][NW][NQ] per-wave max / sum
    static constexpr size_t qp = wstat + sizeof(float) * 2 * NW * NQ;              // half [2][NQ][KROW]
    static constexpr size_t vch = qp + sizeof(uint16_t) * 2 * NQ * KROW;           // half [NW][CK][HD] per-wave value chunk
    static constexpr size_t total = vch + sizeof(uint16_t) * NW * CK * HD;
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
    constexpr bool AHEAD = NW == 4;
    using Lds = AttnLds<NQ, NW>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float (*qs)[HD] = reinterpret_cast<float (*)[HD]>(smem_raw + Lds::qs);       // rotated, scaled queries (fp32)
    float (*kb)[HD] = reinterpret_cast<float (*)[HD]>(smem_raw + Lds::kb);       // rotated block keys
    float (*vb)[HD] = reinterpret_cast<float (*)[HD]>(smem_raw + Lds::vb);       // block values
    float (*S)[SCOLS] = reinterpret_cast<float (*)[SCOLS]>(smem_raw + Lds::S);
    float *blk_m = reinterpret_cast<float *>(smem_raw + Lds::stat);
    float *blk_l = blk_m + NQ;
    float *tot_l = blk_l + NQ;
    float (*w_m)[NQ] = reinterpret_cast<float (*)[NQ]>(smem_raw + Lds::wstat);    // [NW] per-wave running max
    float (*w_l)[NQ] = w_m + NW;                                                  // [NW] per-wave running sum
    uint16_t (*qp)[NQ][KROW] = reinterpret_cast<uint16_t (*)[NQ][KROW]>(smem_raw + Lds::qp);   // [2] query planes
    uint16_t (*vch)[CK][HD] = reinterpret_cast<uint16_t (*)[CK][HD]>(smem_raw + Lds::vch);     // [NW] value chunks

    const int g = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int L = a.L, rep = a.nh / a.nkv, Q = rep * L;
    const int qd = a.nh * HD, kvd = a.nkv * HD;
    int P = a.prefix_len[b];
    P = P < 0 ? 0 : (P > a.P_max ? a.P_max : P);
    const float scale = 0.08838834764831845f;   // 1 / sqrt(128)
    const int nchunks = (P + CK - 1) / CK;

    // A wave's next chunk is requested while it works on the current one.  Keys go straight into
    // matrix-core A fragments (lane = key row, 16 bytes per 16 dimensions); values are fetched as
    // whole rows (16 consecutive lanes per position) and parked in the wave's LDS chunk.
    uint4 kreg[HD / 16], vreg[CK * HD / 8 / 64];
    auto request = [&](int c) {
        const int tk = c * CK + l32;
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) {
            kreg[ks] = make_uint4(0, 0, 0, 0);
            if (tk < P)
                kreg[ks] = *reinterpret_cast<const uint4 *>(a.kc + (((size_t)b * a.P_max + tk) * a.nkv + g) * HD +
                                                            16 * ks + 8 * half);
        }
#pragma unroll
        for (int n = 0; n < CK * HD / 8 / 64; ++n) {
            const int idx = lane + 64 * n, key = idx >> 4, c16 = idx & 15;
            const int tv = c * CK + key;
            vreg[n] = make_uint4(0, 0, 0, 0);
            if (tv < P)
                vreg[n] = *reinterpret_cast<const uint4 *>(a.vc + (((size_t)b * a.P_max + tv) * a.nkv + g) * HD + 8 * c16);
        }
    };
    if (AHEAD && wave < nchunks) request(wave);

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
        uint16_t hi, lo;
        split2(r0 * Q_SCALE, hi, lo);
        qp[0][qq][j] = hi; qp[1][qq][j] = lo;
        split2(r1 * Q_SCALE, hi, lo);
        qp[0][qq][j + HD / 2] = hi; qp[1][qq][j + HD / 2] = lo;
    }
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
    __syncthreads();

    // ---- the block's own rows (fp32 keys and values, vector ALU); absent keys -inf.  The value sum is
    // held in accumulator layout: wave w owns dimensions 32 w .. 32 w + 31, element r of a lane is
    // o[query 32 qb + lane % 32][dimension 32 w + acc_row(r, half)], in units of P_SCALE.
    for (int qq = tid >> 4; qq < NQ; qq += NT / 16) {
        const int key = tid & 15;
        float acc = -INFINITY;
        if (key < L) {
            acc = 0.f;
            for (int e = 0; e < HD; ++e) acc += qs[qq][e] * kb[key][e];
        }
        S[qq][key] = acc;
    }
    __syncthreads();
    softmax_block<NQ, NT>(S, blk_m, blk_l);
    __syncthreads();
    f32x16 o_blk[NQB];
#pragma unroll
    for (int qb = 0; qb < NQB; ++qb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o_blk[qb][r] = 0.f;
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
    for (int c = wave; c < nchunks; c += NW) {
        if (!AHEAD) request(c);
        uint4 kf[HD / 16];
#pragma unroll
        for (int ks = 0; ks < HD / 16; ++ks) kf[ks] = bf16x8_to_f16x8(kreg[ks]);
        __builtin_amdgcn_wave_barrier();   // (the previous chunk's value reads come before these writes)
#pragma unroll
        for (int n = 0; n < CK * HD / 8 / 64; ++n) {
            const int idx = lane + 64 * n, key = idx >> 4, c16 = idx & 15;
            *reinterpret_cast<uint4 *>(&vch[wave][key][8 * c16]) = bf16x8_to_f16x8(vreg[n]);
        }
        __builtin_amdgcn_wave_barrier();
        if (AHEAD && c + NW < nchunks) request(c + NW);

        uint4 p_hi[NQB][2], p_lo[NQB][2];
#pragma unroll
        for (int qb = 0; qb < NQB; ++qb) {
            // scores of the chunk's 32 keys for this lane's query
            f32x16 sc;
#pragma unroll
            for (int r = 0; r < 16; ++r) sc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < HD / 16; ++ks) {
                const int col = 16 * ks + 8 * half;
                const uint4 q_hi = *reinterpret_cast<const uint4 *>(&qp[0][32 * qb + l32][col]);
                const uint4 q_lo = *reinterpret_cast<const uint4 *>(&qp[1][32 * qb + l32][col]);
                sc = mma_f16(kf[ks], q_hi, sc);
                sc = mma_f16(kf[ks], q_lo, sc);
            }
            float cmax = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sc[r] = (c * CK + acc_row(r, half) < P) ? sc[r] * (1.0f / Q_SCALE) : -INFINITY;
                cmax = fmaxf(cmax, sc[r]);
            }
            cmax = fmaxf(cmax, __shfl_xor(cmax, 32));   // finite: a chunk holds at least one key
            const float m_new = fmaxf(run_m[qb], cmax);
            const float f = (run_m[qb] == -INFINITY) ? 0.f : __expf(run_m[qb] - m_new);
            float csum = 0.f;
            uint16_t hi[16], lo[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const float pr = __expf(sc[r] - m_new);   // exp(-inf) = 0 for absent keys
                csum += pr;
                split2(pr * P_SCALE, hi[r], lo[r]);
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
            for (int s2 = 0; s2 < 2; ++s2) {
                p_hi[qb][s2] = make_uint4(pack2(hi[8 * s2], hi[8 * s2 + 1]), pack2(hi[8 * s2 + 2], hi[8 * s2 + 3]),
                                          pack2(hi[8 * s2 + 4], hi[8 * s2 + 5]), pack2(hi[8 * s2 + 6], hi[8 * s2 + 7]));
                p_lo[qb][s2] = make_uint4(pack2(lo[8 * s2], lo[8 * s2 + 1]), pack2(lo[8 * s2 + 2], lo[8 * s2 + 3]),
                                          pack2(lo[8 * s2 + 4], lo[8 * s2 + 5]), pack2(lo[8 * s2 + 6], lo[8 * s2 + 7]));
            }
        }
        // values: V^T fragments gathered in the same key order (k step s, element e <-> accumulator row 8 s + e)
#pragma unroll
        for (int db = 0; db < 4; ++db) {
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2) {
                uint16_t vh[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) vh[e] = vch[wave][acc_row(8 * s2 + e, half)][32 * db + l32];
                const uint4 vf = make_uint4(pack2(vh[0], vh[1]), pack2(vh[2], vh[3]), pack2(vh[4], vh[5]), pack2(vh[6], vh[7]));
#pragma unroll
                for (int qb = 0; qb < NQB; ++qb) {
                    o_acc[qb][db] = mma_f16(vf, p_hi[qb][s2], o_acc[qb][db]);
                    o_acc[qb][db] = mma_f16(vf, p_lo[qb][s2], o_acc[qb][db]);
                }
            }
        }
    }

    // ---- merge the five partial results per query in a fixed order: block, waves 0 .. 3
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
        f_blk[qb] = __expf(blk_m[q] - m_tot);
        float l_tot = blk_l[q] * f_blk[qb];
#pragma unroll
        for (int w = 0; w < NW; ++w) {
            const float fw = (w_m[w][q] == -INFINITY) ? 0.f : __expf(w_m[w][q] - m_tot);
            l_tot += w_l[w][q] * fw;
            if (w == wave) f_own[qb] = fw;
        }
        if (wave == 0 && half == 0) tot_l[q] = l_tot;
        if (wave < 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j)   // the block's partial: this wave's 32 dimensions
                *reinterpret_cast<float4 *>(&qs[q][32 * wave + 8 * j + 4 * half]) =
                    make_float4(o_blk[qb][4 * j] * f_blk[qb], o_blk[qb][4 * j + 1] * f_blk[qb],
                                o_blk[qb][4 * j + 2] * f_blk[qb], o_blk[qb][4 * j + 3] * f_blk[qb]);
        }
    }
    __syncthreads();
    for (int w = 0; w < NW && w < nchunks; ++w) {   // (uniform over the workgroup)
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

template <int NQB, int NW>
hipError_t attn_configure_one() {
    return hipFuncSetAttribute(reinterpret_cast<const void *>(&attn_kernel<NQB, NW>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)AttnLds<32 * NQB, NW>::total);
}

template <int NQB, int NW>
hipError_t attn_launch_one(const AttnArgs &a, int B, hipStream_t st) {
    constexpr size_t lds = AttnLds<32 * NQB, NW>::total;
    hipLaunchKernelGGL((attn_kernel<NQB, NW>), dim3(a.nkv, B), dim3(64 * NW), lds, st, a);
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
    if (Q <= 32) return attn_launch_one<1, 8>(a, B, st);
    return attn_launch_one<2, 4>(a, B, st);
}

}  // namespace mrp
