// Internal declarations shared by the HIP translation units of libmrp.
// Nothing here is part of the C ABI (see include/mrp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mrp {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Number of fp16 terms an fp32 activation is split into before it enters an
// fp16 MFMA: hi + lo reproduces the fp32 value to 2^-22 relative (or 2^-25
// absolute where lo is subnormal; the matrix cores honour fp16 subnormals), so
// the head body is computed to fp32 accuracy although the matrix cores take
// 16-bit operands.  The head body's weights are converted from bf16 to fp16
// when they are packed (exact for 6.1e-5 <= |w| < 65504, within 3e-8 below);
// activations must stay below 65504 in magnitude.  The LM head itself runs on
// bf16 operands (its activation y is bf16 by definition).
constexpr int NSPLIT = 2;

constexpr int MAX_L = 64;         // largest block length (rows per sequence)
constexpr int KSTEP = 8;          // 16-wide k blocks per pipeline stage (128 k)
constexpr int WG_WAVES = 4;       // wavefronts per workgroup of the stream GEMM
constexpr int WG_ROWS = 32 * WG_WAVES;  // weight rows per workgroup tile

// One K segment of the activation operand of the stream GEMM.  The operand is
// the sum over `nplanes` packed 16-bit planes (fp16 for the head body, bf16 for the LM head); plane p of local k block kb, row
// block ib lives at base + p * plane_stride + (kb * nIb + ib) * 64 (uint4 units).
struct ActSeg {
    const uint4 *base;
    long plane_stride;
    int nkr;       // k ranges (of KSTEP blocks) in this segment
    int nplanes;
};

enum { EPI_PARTIAL = 0, EPI_LM = 1, EPI_SILU = 2 };

struct StreamGemmArgs {
    const uint4 *Wp;   // packed weights [n_rb][KBw][64] uint4
    int KBw;           // k blocks per weight row block
    int n_rb;          // weight row blocks (padded rows / 32)
    int nIb;           // activation row blocks per k block (allocation stride)
    int M;             // valid activation rows
    int R;             // valid weight rows (outputs per activation row)
    ActSeg seg[2];
    int nseg;
    int nVt, nMg, nKs; // grid decomposition: weight tiles, row groups, k splits
    int G;             // total k ranges = KBw / KSTEP
    // EPI_PARTIAL: out[ks][M][R] fp32
    float *out;
    // EPI_LM: z [M][R] fp32 in/out; partials [nVt][M]
    float *z;
    float *pm, *ps;
    int *pi;
};

// Persistent LM-head kernel (at most 128 activation rows, V % 4 == 0)
struct LmPersistArgs {
    const uint4 *Wp;   // packed W_lm [n_rb][KB][64]
    const uint4 *Y;    // packed bf16 activation plane [KB][nIb][64]
    int KB, n_rb, nIb;
    int M, V;
    int nWG;           // workgroups (one per CU)
    int reverse;       // 1: every workgroup walks its vocabulary range from the end
    float *z;          // [M][V] in/out
    float *pm, *ps;    // partials [M][nWG]: one slot per workgroup, a row's slots contiguous
    int *pi;
};

// LDS-tiled GEMM (256 x 256 tiles) for many activation rows
struct TiledSeg {
    const uint4 *base;   // activation planes of this K segment
    long plane_stride;
    int nkq;             // k steps of 64 in this segment
    int nplanes;
};
struct TiledGemmArgs {
    const uint4 *Wp;
    int KBw, n_rb, nIb, M, R;
    TiledSeg seg[2];
    int nseg;
    int nMt, nVt;        // tiles along activation rows / weight rows
    int nKs;             // k parts (EPI_PARTIAL only: part ks writes out[ks][M][R]; 1 for EPI_LM)
    float *out;          // EPI_PARTIAL: [nKs][M][R]
    uint4 *planes;       // EPI_SILU: the NSPLIT fp16 planes [R / 16][nIb][64] of SiLU(X W^T), plane_stride apart
    long plane_stride;
    float *z;            // EPI_LM: [M][R] in/out, partials [nVt][M]
    float *pm, *ps;
    int *pi;
};

// Bits of a context's device error word (the MRP_FLAG_* values of include/mrp.h): an index the caller
// passed in device memory was out of range; the kernel clamped or skipped it and reports it here.
enum { ERR_COND_TOK = 1, ERR_DRAFT_POS = 2, ERR_PREFIX_LEN = 4, ERR_X_TOK = 8 };

// MLP head body for fewer than 768 activation rows without partial sums in memory (head_fused.hip)
struct HeadFusedArgs {
    const uint4 *W1p;          // packed fp16 W1 [d / 32][2 d / 16][64]
    const uint4 *W2p;          // packed fp16 W2 [d / 32][d / 16][64]
    const uint4 *XH;           // planes of the running hidden state
    long plane;                // plane stride (uint4 units) of XH and S
    int np_h;                  // planes of XH to read (1: the state is an exact single term)
    const uint16_t *E;         // embedding table [V][d] bf16
    const int32_t *cond_tok;   // [B] conditioning token per sequence
    int L, V;
    uint4 *S;                  // planes of s = SiLU(a): written by the first launch, read by the second
    float *U;                  // [M][d] fp32 u = W2 s
    int nIb, M, d;
    int *err_flag;
    int nf;                    // weight row blocks per tile (1 or 2)
    int nct, nrt;              // feature tiles d / (32 nf), row tiles ceil(M / 32)
};

// row-reduction partial: running max, sum of exp(x - max), index of the max
struct Part {
    float m, s;
    int i;
};

__device__ __forceinline__ Part part_identity() { return {-INFINITY, 0.f, 0x7fffffff}; }

// Merge two partials; equal maxima keep the lower index.
__device__ __forceinline__ Part part_merge(Part a, Part b) {
    const bool b_wins = (b.m > a.m) || (b.m == a.m && b.i < a.i);
    const float mx = b_wins ? b.m : a.m;
    const float sa = (a.m == -INFINITY) ? 0.f : a.s * __expf(a.m - mx);
    const float sb = (b.m == -INFINITY) ? 0.f : b.s * __expf(b.m - mx);
    return {mx, sa + sb, b_wins ? b.i : a.i};
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ uint16_t f32_to_f16_bits(float x) {
    const _Float16 h = (_Float16)x;   // round to nearest even
    return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }

// hi/lo fp16 terms of an fp32 value (the remainder is exact in fp32)
__device__ __forceinline__ void split2(float x, uint16_t &hi, uint16_t &lo) {
    hi = f32_to_f16_bits(x);
    lo = f32_to_f16_bits(x - f16_bits_to_f32(hi));
}

// index (in uint4 units) of the 16-byte chunk holding X[row][8*c8 .. 8*c8+7]
// inside an activation plane laid out [kb][ib][64 lanes]
__device__ __forceinline__ size_t act_chunk_index(int row, int c8, int nIb) {
    const int kb = c8 >> 1, half = c8 & 1;
    return ((size_t)kb * nIb + (row >> 5)) * 64 + (row & 31) + 32 * half;
}

// Elementwise producers of activation planes: wave `unit` owns the 1 KiB block (k block kb, row
// block ib) of every plane, so that its 64 lanes store one contiguous block; the four waves of a
// workgroup take four consecutive k blocks of the same row block (256 contiguous input bytes per row).
// Returns false for a lane without a row.  c8: the lane's 8-column chunk.
__device__ __forceinline__ bool plane_block_lane(size_t unit, int KB, int M, int &row, int &c8) {
    const int lane = threadIdx.x & 63;
    const int kb = (int)(unit % KB), ib = (int)(unit / KB);
    row = ib * 32 + (lane & 31);
    c8 = 2 * kb + (lane >> 5);
    return row < M;
}

// Row handled by workgroup w of a one-row-per-workgroup kernel.  Consecutive workgroup ids go to
// different XCDs (8, each with its own L2); this mapping gives every XCD whole 32-row blocks, so
// the 16-byte pieces that 32 workgroups store into one 1 KiB plane block meet in one L2.
__device__ __forceinline__ int xcd_row_of(int w) {
    const int xcd = w & 7, slot = w >> 3;
    return ((slot >> 5) * 8 + xcd) * 32 + (slot & 31);
}

__device__ __forceinline__ uint32_t pack2(uint16_t lo, uint16_t hi) { return (uint32_t)lo | ((uint32_t)hi << 16); }

// 8 fp32 values -> the 16-byte chunks of the NSPLIT activation planes at index dst
__device__ __forceinline__ void split_store(const float (&x)[8], uint4 *planes, size_t dst, long plane_stride) {
    uint16_t h[8], l[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) split2(x[e], h[e], l[e]);
    planes[dst] = make_uint4(pack2(h[0], h[1]), pack2(h[2], h[3]), pack2(h[4], h[5]), pack2(h[6], h[7]));
    planes[dst + plane_stride] = make_uint4(pack2(l[0], l[1]), pack2(l[2], l[3]), pack2(l[4], l[5]), pack2(l[6], l[7]));
}

__device__ __forceinline__ void unpack_bf16x8(const uint4 &u, float (&x)[8]) {
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        x[2 * e] = bf16_to_f32((uint16_t)(w[e] & 0xFFFFu));
        x[2 * e + 1] = bf16_to_f32((uint16_t)(w[e] >> 16));
    }
}

// 8 bf16 values -> the same values as fp16 (one plane; exact inside fp16's normal range)
__device__ __forceinline__ uint4 bf16x8_to_f16x8(const uint4 &u) {
    float x[8];
    unpack_bf16x8(u, x);
    uint16_t h[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) h[e] = f32_to_f16_bits(x[e]);
    return make_uint4(pack2(h[0], h[1]), pack2(h[2], h[3]), pack2(h[4], h[5]), pack2(h[6], h[7]));
}

// Sum over the k-split partial buffers of the 8 floats at `off` (same order for any batching:
// ((p0 + p1) + p2) + ...).  Four splits are fetched at a time so their latencies overlap.
__device__ __forceinline__ void sum_partials(const float *__restrict__ part, size_t split_stride, int nKs, size_t off,
                                             float (&x)[8]) {
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = 0.f;
    int ks = 0;
    for (; ks + 4 <= nKs; ks += 4) {
        float4 a[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float4 *p = reinterpret_cast<const float4 *>(part + (size_t)(ks + u) * split_stride + off);
            a[u] = p[0]; b[u] = p[1];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            x[0] += a[u].x; x[1] += a[u].y; x[2] += a[u].z; x[3] += a[u].w;
            x[4] += b[u].x; x[5] += b[u].y; x[6] += b[u].z; x[7] += b[u].w;
        }
    }
    for (; ks < nKs; ++ks) {
        const float4 *p = reinterpret_cast<const float4 *>(part + (size_t)ks * split_stride + off);
        const float4 a = p[0], b = p[1];
        x[0] += a.x; x[1] += a.y; x[2] += a.z; x[3] += a.w;
        x[4] += b.x; x[5] += b.y; x[6] += b.z; x[7] += b.w;
    }
}

// ---- host-side launchers (defined in the .hip files) ----
hipError_t launch_stream_gemm(const StreamGemmArgs &a, int epi, hipStream_t st);
size_t stream_gemm_lds_bytes(int it);
hipError_t stream_gemm_configure();   // once per device
int stream_gemm_it(int M);   // activation row blocks per workgroup for M rows

hipError_t launch_tiled_gemm(const TiledGemmArgs &a, int epi, hipStream_t st);
// k parts for a partial-sum tile GEMM with `tiles` output tiles and `nsteps` k steps, writing at most `cap_rows` rows
int tiled_ksplit(int tiles, int nsteps, int nCU, size_t cap_rows, int M);
hipError_t launch_lm_persist(const LmPersistArgs &a, hipStream_t st);
size_t lm_persist_lds_bytes();
hipError_t lm_persist_configure();    // once per device

hipError_t launch_pack_weight(const uint16_t *src, int rows, int cols, uint4 *dst, bool to_f16, hipStream_t st);
hipError_t launch_init_hidden(const uint16_t *h, float *hrun, uint4 *xh, long plane_stride, int nIb,
                              int M, int d, bool from_h, hipStream_t st);
hipError_t launch_gather_e(const uint16_t *E, const int32_t *cond_tok, uint4 *xe, int nIb, int B, int L,
                           int d, int V, int *err_flag, hipStream_t st);
hipError_t launch_silu_split(const float *part, int nKs, uint4 *s_planes, long plane_stride, int nIb,
                             int M, int d, hipStream_t st);
// u = (resid ? resid : 0) + sum of partials; y = bf16(RMSNorm(u) gamma); carry: hrun += u and its planes
hipError_t launch_norm(const float *part, int nKs, const float *resid, const uint16_t *gamma, float eps,
                       float *hrun, bool carry, uint4 *y, uint4 *xh, long plane_stride, int nIb, int M, int d,
                       hipStream_t st);

struct SelectArgs {
    const float *pm, *ps;
    const int *pi;
    int nT;                 // partial tiles per row
    long slot_stride, row_stride;  // partial (t, i) lives at t * slot_stride + i * row_stride
    int M, B, L, d, V;
    int state;              // global state index recorded in revealed_at
    int do_reveal;          // apply the reveal rule at this state
    int fresh;              // treat every row as masked first (state 0 of a fresh block)
    int write_protect;      // record the top row in protect_pos (state 0)
    float tau;
    int r_min, max_accept;
    float tau_remask;       // < 0: no remask at this state
    int32_t *tok;
    float *conf, *lse;      // this state's slots [M]
    int8_t *revealed_at;
    uint8_t *masked;
    int32_t *cond_tok, *protect_pos;
    int32_t *draft_pos, *draft_tok;  // this state's column, stride draft_stride
    int draft_stride;
    uint8_t *remasked;      // this state's slot [M] or nullptr
    int32_t *x_tok;         // [M] token recorded at reveal, or nullptr
    int remask_mode;        // 1: remask on the probability of the recorded token (needs z, x_tok)
    const float *z;         // [M][V] updated logits (remask_mode 1)
    const uint16_t *E;      // embedding rows to gather for the next head (nullptr: skip)
    uint4 *xe;
    int nIb;
    int *err_flag;          // device error word (may be nullptr)
};
hipError_t launch_reduce_rows(const float *z, int M, int V, float *pm, float *ps, int *pi, int *nT_out,
                              hipStream_t st);
int reduce_rows_tiles(int V);
hipError_t launch_merge_select(const SelectArgs &a, hipStream_t st);
hipError_t launch_commit(int B, int L, const int32_t *x_tok, int8_t *revealed_at, const uint8_t *masked,
                         int32_t *x_out, int32_t *n_masked, hipStream_t st);
hipError_t launch_remask(int B, int L, int state, const float *conf, float tau_remask,
                         const int32_t *protect_pos, int8_t *revealed_at, uint8_t *masked,
                         uint8_t *remasked, hipStream_t st);
hipError_t launch_verify(int B, int L, int V, int K, int joint, const float *verify, const int32_t *draft_pos,
                         const int32_t *draft_tok, int draft_stride, float *wm, int *wi, uint8_t *match,
                         int32_t *accept_len, int32_t *correction_tok, int *err_flag, hipStream_t st);
hipError_t launch_build_candidates(int B, int L, int K, const int32_t *x_t, const uint8_t *masked_t,
                                   const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride,
                                   int32_t mask_token, int32_t *cand_tok, uint8_t *cand_masked, int *err_flag,
                                   hipStream_t st);
int verify_chunks(int V);
void *verify_static_scratch();   // current device's file-scope scratch of mrp_verify_accept_static (nullptr on failure)

// transformer head body (tbody.hip)
hipError_t tbody_configure();   // once per device
bool tbody_shape_ok(int nh, int nkv, int head_dim, int L);
hipError_t launch_rope_table(const int32_t *prefix_len, int B, int L, int P_max, double theta, float2 *out,
                             int *err_flag, hipStream_t st);
hipError_t launch_resid_norm_split(const float *part, int nKs, const float *resid, float *stream,
                                   const uint16_t *gain, float eps, uint4 *planes, long plane_stride, int nIb, int M,
                                   int d, hipStream_t st);
hipError_t launch_swiglu_split(const float *part, int nKs, uint4 *planes, long plane_stride, int nIb, int M, int ff,
                               hipStream_t st);
hipError_t launch_attention(const float *qkv, int nKs, int M, int B, int L, int nh, int nkv, const float2 *rope,
                            const uint16_t *kc, const uint16_t *vc, const int32_t *prefix_len, int P_max,
                            uint4 *o_planes, long plane_stride, int nIb, float *scratch, hipStream_t st);
size_t attention_scratch_floats();   // floats of `scratch` (partials of workgroups that share a prefix)

// out [nKs][M][R] fp32 partial sums of X W^T on 64-feature x 128-row tiles (wide_gemm.hip)
struct WideGemmArgs {
    const uint4 *Wp;           // packed fp16 weights [R / 32][Kc / 16][64]
    const uint4 *X;            // activation planes [Kc / 16][nIb][64]
    long plane;                // plane stride (uint4 units)
    int nplanes;               // 1 or 2
    float *out;                // [nKs][M][R]
    int nIb, M, R, Kc;
    int nKs;                   // k parts (1, 2, 4 or 8)
    int nft, nrg;              // R / (32 nf) feature tiles, ceil(M / 128) row groups
    int nf;                    // 32-feature blocks per workgroup: 2 or 4
};
int wide_gemm_ksplit(int tiles, int kbs, int nCU, size_t cap_rows, int M, int nf);   // 0: not applicable
hipError_t launch_wide_gemm(const WideGemmArgs &a, hipStream_t st);

// out [M][R] fp32 = X W^T, k split reduced inside the workgroup (R % 32 == 0, Kc % 128 == 0)
struct SmallGemmArgs {
    const uint4 *Wp;           // packed fp16 weights [R / 32][Kc / 16][64]
    const uint4 *X;            // activation planes [Kc / 16][nIb][64]
    long plane;                // plane stride (uint4 units)
    int nplanes;               // 1 or 2
    float *out;                // [M][R]
    int nIb, M, R, Kc;
    int nf;                    // weight row blocks per tile (1 or 2; R % (32 nf) == 0)
    int nct, nrt;              // feature tiles R / (32 nf), row tiles ceil(M / 32)
};
hipError_t launch_small_gemm(const SmallGemmArgs &a, hipStream_t st);
hipError_t launch_head_fused(const HeadFusedArgs &a, hipStream_t st);   // both GEMMs: S and U written

hipError_t launch_lm_traffic(int mode, const uint4 *Wp, float *z, int KB, int n_rb, int M, int V, int nWG,
                             unsigned *sink, hipStream_t st);

size_t residual_rms_part_bytes();
int residual_rms_max_blocks();
bool residual_rms_supported(int S);
hipError_t launch_residual_rms(int n_blocks, int S, long N, const void *X, bool bf16, double *part,
                               double *rms_pair, double *rms_delta, hipStream_t st);

int kl_tiles(int V);
hipError_t launch_kl_loss(int M, int V, const float *teacher, const float *student, const uint8_t *mask, float scale,
                          float *part, size_t part_stride, float *lse, float *loss_rows, float *grad,
                          hipStream_t st);

}  // namespace mrp
