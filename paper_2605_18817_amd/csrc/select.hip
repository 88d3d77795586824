// Vocabulary reductions and the per-sequence decision logic of the MRP chain:
//   reduce_rows    state 0: split-vocabulary (max, sum-exp, argmax) partials of z
//   merge_select   merge a row's partials into (token, confidence, log-sum-exp)
//                  — confidence is the top-1 softmax probability (paper
//                  Section 2) — then, one workgroup per sequence, apply the
//                  reveal rule (threshold with a forced minimum, Section 4.1;
//                  optional max-accept cap, Section 4.4), record the draft
//                  (Algorithm 3: most confident new reveal), optionally remask
//                  (Algorithm 4) and gather the embedding row that conditions
//                  the next head
//   remask         Algorithm 4's remask rule on its own
//   verify         Algorithm 3's accept test: argmax of the verifier's logits at
//                  the drafted positions, longest matching prefix
#include "mrp_kernels.h"

namespace mrp {

namespace {

constexpr int RT = 8192;  // vocabulary entries per workgroup in the plain row reductions

__device__ __forceinline__ Part wave_merge(Part p) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        Part o;
        o.m = __shfl_xor(p.m, off);
        o.s = __shfl_xor(p.s, off);
        o.i = __shfl_xor(p.i, off);
        p = part_merge(p, o);
    }
    return p;
}

// all 256 threads call; result valid in thread 0
__device__ __forceinline__ Part block_merge(Part p, float *sm, float *ss, int *si) {
    p = wave_merge(p);
    const int wave = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sm[wave] = p.m; ss[wave] = p.s; si[wave] = p.i; }
    __syncthreads();
    if (threadIdx.x == 0) {
        p = Part{sm[0], ss[0], si[0]};
        for (int w = 1; w < 4; ++w) p = part_merge(p, Part{sm[w], ss[w], si[w]});
    }
    return p;
}

template <bool VEC4>
__global__ __launch_bounds__(256) void reduce_rows_kernel(const float *__restrict__ z, int M, int V,
                                                          float *__restrict__ pm, float *__restrict__ ps,
                                                          int *__restrict__ pi) {
    __shared__ float sm[4], ss[4];
    __shared__ int si[4];
    const int t = blockIdx.x, i = blockIdx.y;
    const float *row = z + (size_t)i * V;
    const int v0 = t * RT;
    float x[32];
    if constexpr (VEC4) {
#pragma unroll
        for (int n = 0; n < 8; ++n) {
            const int v = v0 + 4 * (threadIdx.x + 256 * n);
            float4 q = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
            if (v < V) q = *reinterpret_cast<const float4 *>(row + v);
            x[4 * n] = q.x; x[4 * n + 1] = q.y; x[4 * n + 2] = q.z; x[4 * n + 3] = q.w;
        }
    } else {
#pragma unroll
        for (int n = 0; n < 32; ++n) {
            const int v = v0 + threadIdx.x + 256 * n;
            x[n] = (v < V) ? row[v] : -INFINITY;
        }
    }
    Part p = part_identity();
#pragma unroll
    for (int n = 0; n < 32; ++n) {
        const int v = VEC4 ? v0 + 4 * (threadIdx.x + 256 * (n >> 2)) + (n & 3) : v0 + threadIdx.x + 256 * n;
        if (x[n] > p.m) { p.m = x[n]; p.i = v; }
    }
    float s = 0.f;
    if (p.m > -INFINITY) {
#pragma unroll
        for (int n = 0; n < 32; ++n) s += __expf(x[n] - p.m);  // exp(-inf) = 0 for padding
    }
    p.s = s;
    p = block_merge(p, sm, ss, si);
    if (threadIdx.x == 0) {
        // a row's partials are contiguous, so that the merge reads them coalesced
        const size_t o = (size_t)i * gridDim.x + t;
        pm[o] = p.m;
        ps[o] = p.s;
        pi[o] = p.i;
    }
}

constexpr int MERGE_BATCH = 16;  // strides of 64 partial tiles fetched together (1024 tiles per round trip)

__device__ __forceinline__ bool more_confident(const float *conf, int a, int b) {
    if (conf[a] != conf[b]) return conf[a] > conf[b];
    return a < b;
}

__global__ __launch_bounds__(256) void merge_select_kernel(const SelectArgs a) {
    __shared__ float s_conf[MAX_L], s_lse[MAX_L];
    __shared__ int s_tok[MAX_L], s_xtok[MAX_L];
    __shared__ uint8_t s_mk[MAX_L];
    __shared__ int8_t s_ra[MAX_L];
    __shared__ int s_gather;
    const int b = blockIdx.x, L = a.L;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;

    // state of the sequence: fetched up front so that its latency hides behind the merge
    int in_cond = 0, in_prot = -1;
    if (threadIdx.x < L) {
        s_mk[threadIdx.x] = a.fresh ? (uint8_t)1 : a.masked[b * L + threadIdx.x];
        s_ra[threadIdx.x] = a.fresh ? (int8_t)-1 : a.revealed_at[b * L + threadIdx.x];
        s_xtok[threadIdx.x] = (a.x_tok && !a.fresh) ? a.x_tok[b * L + threadIdx.x] : -1;
    }
    if (threadIdx.x == 0) {
        in_cond = a.cond_tok[b];
        in_prot = a.write_protect ? -1 : a.protect_pos[b];
    }

    if (a.row_stride == 1 && a.slot_stride > 1) {
        // Layout [tile][row] (the GEMM kernels that own whole row tiles write it): the sequence's L
        // rows of one tile are contiguous.  Thread (row p, group grp) merges tiles grp, grp + NG, ...
        // in order, so a load instruction fetches whole 4 L-byte runs; the groups' results are then
        // merged per row in group order.
        __shared__ float g_m[256], g_s[256];
        __shared__ int g_i[256];
        int Lp = 1;
        while (Lp < L) Lp <<= 1;
        const int NG = 256 / Lp, p = threadIdx.x % Lp, grp = threadIdx.x / Lp;
        Part pt = part_identity();
        if (p < L) {
            const size_t i = (size_t)b * L + p;
            for (int t0 = grp; t0 < a.nT; t0 += NG * 8) {
                float m[8], sx[8];
                int ix[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) {   // eight tiles in flight
                    const int t = t0 + u * NG;
                    const bool ok = t < a.nT;
                    const size_t o = (size_t)(ok ? t : 0) * a.slot_stride + i;
                    m[u] = ok ? a.pm[o] : -INFINITY;
                    sx[u] = ok ? a.ps[o] : 0.f;
                    ix[u] = ok ? a.pi[o] : 0x7fffffff;
                }
#pragma unroll
                for (int u = 0; u < 8; ++u) pt = part_merge(pt, Part{m[u], sx[u], ix[u]});
            }
        }
        g_m[threadIdx.x] = pt.m; g_s[threadIdx.x] = pt.s; g_i[threadIdx.x] = pt.i;
        __syncthreads();
        if (threadIdx.x < L) {
            const int q = threadIdx.x;
            Part r = part_identity();
            for (int gq = 0; gq < NG; ++gq) r = part_merge(r, Part{g_m[gq * Lp + q], g_s[gq * Lp + q], g_i[gq * Lp + q]});
            const int i = b * L + q;
            const float conf = 1.0f / r.s;
            const float lse = r.m + logf(r.s);
            a.tok[i] = r.i; a.conf[i] = conf; a.lse[i] = lse;
            s_lse[q] = lse; s_conf[q] = conf; s_tok[q] = r.i;
        }
    } else {
    // one wavefront per row: merge the row's nT partials in a fixed order
    for (int p = wave; p < L; p += 4) {
        const int i = b * L + p;
        Part pt = part_identity();
        for (int t0 = 0; t0 < a.nT; t0 += 64 * MERGE_BATCH) {
            float m[MERGE_BATCH], sx[MERGE_BATCH];
            int ix[MERGE_BATCH];
#pragma unroll
            for (int u = 0; u < MERGE_BATCH; ++u) {  // issue every load of the batch before merging any
                const int t = t0 + u * 64 + lane;
                const bool ok = t < a.nT;
                const size_t o = (size_t)(ok ? t : 0) * a.slot_stride + (size_t)i * a.row_stride;
                m[u] = ok ? a.pm[o] : -INFINITY;
                sx[u] = ok ? a.ps[o] : 0.f;
                ix[u] = ok ? a.pi[o] : 0x7fffffff;
            }
#pragma unroll
            for (int u = 0; u < MERGE_BATCH; ++u) pt = part_merge(pt, Part{m[u], sx[u], ix[u]});
        }
        pt = wave_merge(pt);
        if (lane == 0) {
            const float conf = 1.0f / pt.s;
            a.tok[i] = pt.i;
            a.conf[i] = conf;
            const float lse = pt.m + logf(pt.s);
            a.lse[i] = lse;
            s_lse[p] = lse;
            s_conf[p] = conf;
            s_tok[p] = pt.i;
        }
    }
    }
    __syncthreads();

    // The decision of the state, one lane per position (L <= 64: the first wavefront).  A still-masked
    // position's rank is the number of still-masked positions that are more confident (ties: lower
    // position first), so "the ns most confident" are the positions of rank < ns; the number above the
    // threshold, the cap and the forced minimum are counted with ballots.  Same outcome as sorting the
    // candidates and walking the sorted list, without a serial part.
    if (wave == 0) {
        const int p = lane;
        const bool in = p < L;
        bool mk = in && s_mk[in ? p : 0] != 0;
        const float cf = in ? s_conf[p] : 0.f;
        int ra = in ? (int)s_ra[p] : -1;
        int xt = in ? s_xtok[p] : -1;
        in_cond = __shfl(in_cond, 0);
        in_prot = __shfl(in_prot, 0);
        int dpos = -1, dtok = -1, cond = in_cond, prot = in_prot;
        if (a.do_reveal) {
            int rank = 0;
            for (int q = 0; q < L; ++q) {
                const float cq = s_conf[q];
                if (s_mk[q] && (cq > cf || (cq == cf && q < p))) ++rank;
            }
            const int nc = __popcll(__ballot(mk));
            int ns = __popcll(__ballot(mk && cf > a.tau));
            if (a.max_accept) {
                int m = (7 * nc) / 10;
                if (m < 5) m = 5;
                if (m > L) m = L;
                if (ns > m) ns = m;
            }
            if (ns < a.r_min) ns = a.r_min < nc ? a.r_min : nc;
            const unsigned long long top = __ballot(mk && rank == 0);
            if (ns > 0) {
                dpos = __ffsll((long long)top) - 1;
                dtok = s_tok[dpos];
                cond = dtok;
                if (lane == 0) a.cond_tok[b] = dtok;
            }
            if (mk && rank < ns) { mk = false; ra = a.state; xt = s_tok[p]; }
            if (a.write_protect) {
                prot = dpos;
                if (lane == 0) a.protect_pos[b] = dpos;
            }
        }
        if (lane == 0) {
            a.draft_pos[(size_t)b * a.draft_stride] = dpos;
            a.draft_tok[(size_t)b * a.draft_stride] = dtok;
            s_gather = cond;
        }
        uint8_t rem = 0;
        if (in && a.tau_remask >= 0.f) {
            float cr = cf;
            if (a.remask_mode == 1 && ra >= 0 && ra <= a.state - 1) {
                // probability of the token that was revealed here under the updated logits
                int t = xt;
                if (t >= a.V && a.err_flag) atomicOr(a.err_flag, ERR_X_TOK);
                t = t < 0 ? 0 : (t >= a.V ? a.V - 1 : t);
                cr = (xt >= 0) ? expf(a.z[(size_t)(b * L + p) * a.V + t] - s_lse[p]) : 0.f;
            }
            if (ra >= 0 && ra <= a.state - 1 && p != prot && cr < a.tau_remask) {
                mk = true; ra = -1; rem = 1;
            }
        }
        if (in) {
            a.masked[b * L + p] = mk ? 1 : 0;
            a.revealed_at[b * L + p] = (int8_t)ra;
            if (a.remasked) a.remasked[b * L + p] = rem;
            if (a.x_tok) a.x_tok[b * L + p] = xt;
        }
    }
    __syncthreads();

    if (a.E != nullptr) {  // embedding row that conditions the next head
        const int C8 = a.d >> 3;
        int tokc = s_gather;  // caller contract: 0 <= cond_tok < V; a bad value is clamped and reported
        if ((tokc < 0 || tokc >= a.V) && threadIdx.x == 0 && a.err_flag) atomicOr(a.err_flag, ERR_COND_TOK);
        tokc = tokc < 0 ? 0 : (tokc >= a.V ? a.V - 1 : tokc);
        const uint4 *erow = reinterpret_cast<const uint4 *>(a.E + (size_t)tokc * a.d);
        for (int c8 = threadIdx.x; c8 < C8; c8 += 256) {
            const uint4 v = bf16x8_to_f16x8(erow[c8]);   // the head body's operands are fp16
            for (int p = 0; p < L; ++p) a.xe[act_chunk_index(b * L + p, c8, a.nIb)] = v;
        }
    }
}

// End of a denoising step: commit this step's reveals (one workgroup per sequence, one lane per row).
__global__ __launch_bounds__(64) void commit_kernel(int L, const int32_t *__restrict__ x_tok,
                                                    int8_t *__restrict__ revealed_at,
                                                    const uint8_t *__restrict__ masked, int32_t *__restrict__ x_out,
                                                    int32_t *__restrict__ n_masked) {
    const int b = blockIdx.x, p = threadIdx.x;
    int m = 0;
    if (p < L) {
        const int i = b * L + p;
        if (revealed_at[i] >= 0) {
            x_out[i] = x_tok[i];
            revealed_at[i] = -2;
        }
        m = masked[i] ? 1 : 0;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) m += __shfl_xor(m, off);
    if (p == 0) n_masked[b] = m;
}

__global__ __launch_bounds__(64) void remask_kernel(int B, int L, int state, const float *__restrict__ conf,
                                                    float tau_remask, const int32_t *__restrict__ protect_pos,
                                                    int8_t *__restrict__ revealed_at, uint8_t *__restrict__ masked,
                                                    uint8_t *__restrict__ remasked) {
    const int b = blockIdx.x, p = threadIdx.x;
    if (p >= L) return;
    const int i = b * L + p;
    const int prot = protect_pos ? protect_pos[b] : -1;
    const int r = revealed_at[i];
    uint8_t rem = 0;
    if (r >= 0 && r <= state - 1 && p != prot && conf[i] < tau_remask) {
        masked[i] = 1;
        revealed_at[i] = -1;
        rem = 1;
    }
    remasked[i] = rem;
}

// argmax partial of one RT-wide chunk of the verifier row of draft (b, j)
template <bool VEC4>
__global__ __launch_bounds__(256) void verify_argmax_kernel(int L, int V, int K, int joint,
                                                            const float *__restrict__ verify,
                                                            const int32_t *__restrict__ draft_pos, int draft_stride,
                                                            int nC, float *__restrict__ wm, int *__restrict__ wi,
                                                            int *err_flag) {
    __shared__ float sm[4], ss[4];
    __shared__ int si[4];
    const int c = blockIdx.x, bk = blockIdx.y;
    const int b = bk / K, j = bk % K;
    int pos = draft_pos[(size_t)b * draft_stride + j];
    if (pos >= L) {  // caller contract: pos < L; an invalid position counts as a missing draft and is reported
        if (threadIdx.x == 0 && c == 0 && err_flag) atomicOr(err_flag, ERR_DRAFT_POS);
        pos = -1;
    }
    Part p = part_identity();
    if (pos >= 0) {  // uniform over the workgroup
        // joint: [B][K+1][L][V], draft j reads candidate j; else one [B][L][V] tensor
        const size_t blk = joint ? (size_t)b * (K + 1) + j : (size_t)b;
        const float *row = verify + (blk * L + pos) * V;
        const int v0 = c * RT;
        if constexpr (VEC4) {
            float4 q[8];
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int v = v0 + 4 * (threadIdx.x + 256 * n);
                q[n] = make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
                if (v < V) q[n] = *reinterpret_cast<const float4 *>(row + v);
            }
#pragma unroll
            for (int n = 0; n < 8; ++n) {
                const int v = v0 + 4 * (threadIdx.x + 256 * n);
                if (q[n].x > p.m) { p.m = q[n].x; p.i = v; }
                if (q[n].y > p.m) { p.m = q[n].y; p.i = v + 1; }
                if (q[n].z > p.m) { p.m = q[n].z; p.i = v + 2; }
                if (q[n].w > p.m) { p.m = q[n].w; p.i = v + 3; }
            }
        } else {
            for (int n = 0; n < 32; ++n) {
                const int v = v0 + threadIdx.x + 256 * n;
                const float x = (v < V) ? row[v] : -INFINITY;
                if (x > p.m) { p.m = x; p.i = v; }
            }
        }
    }
    p = block_merge(p, sm, ss, si);
    if (threadIdx.x == 0) {
        wm[(size_t)bk * nC + c] = p.m;
        wi[(size_t)bk * nC + c] = (pos >= 0) ? p.i : -1;
    }
}

__global__ __launch_bounds__(256) void verify_accept_kernel(int B, int K, int nC, const float *__restrict__ wm,
                                                            const int *__restrict__ wi,
                                                            const int32_t *__restrict__ draft_tok, int draft_stride,
                                                            uint8_t *__restrict__ match, int32_t *__restrict__ accept_len,
                                                            int32_t *__restrict__ correction_tok) {
    const int b = blockIdx.x * 256 + threadIdx.x;
    if (b >= B) return;
    int alen = 0, corr = -1;
    bool open = true;
    for (int j = 0; j < K; ++j) {
        const size_t base = ((size_t)b * K + j) * nC;
        float m = wm[base];
        int vj = wi[base];
        for (int c = 1; c < nC; ++c)
            if (wm[base + c] > m) { m = wm[base + c]; vj = wi[base + c]; }
        const bool ok = vj >= 0 && vj == draft_tok[(size_t)b * draft_stride + j];
        match[(size_t)b * K + j] = ok ? 1 : 0;
        if (open) {
            if (ok) ++alen;
            else { open = false; corr = vj; }
        }
    }
    accept_len[b] = alen;
    correction_tok[b] = corr;
}

// Candidate blocks of the joint verification (paper Figure 1 (d)): candidate k of a sequence is its
// block x_t with the first k drafts written in.  One workgroup per sequence, one lane per position.
__global__ __launch_bounds__(64) void build_candidates_kernel(int L, int K, const int32_t *__restrict__ x_t,
                                                              const uint8_t *__restrict__ masked_t,
                                                              const int32_t *__restrict__ draft_pos,
                                                              const int32_t *__restrict__ draft_tok, int draft_stride,
                                                              int32_t mask_token, int32_t *__restrict__ cand_tok,
                                                              uint8_t *__restrict__ cand_masked, int *err_flag) {
    const int b = blockIdx.x, p = threadIdx.x;
    if (p >= L) return;
    const uint8_t m0 = masked_t[(size_t)b * L + p] ? 1 : 0;
    int32_t tok = m0 ? mask_token : x_t[(size_t)b * L + p];
    uint8_t m = m0;
    for (int k = 0; k <= K; ++k) {
        if (k > 0) {   // candidate k adds draft k - 1
            const int pos = draft_pos[(size_t)b * draft_stride + k - 1];
            if (pos >= L && p == 0 && err_flag) atomicOr(err_flag, ERR_DRAFT_POS);
            if (pos == p) { tok = draft_tok[(size_t)b * draft_stride + k - 1]; m = 0; }
        }
        const size_t o = ((size_t)b * (K + 1) + k) * L + p;
        cand_tok[o] = tok;
        cand_masked[o] = m;
    }
}

}  // namespace

hipError_t launch_build_candidates(int B, int L, int K, const int32_t *x_t, const uint8_t *masked_t,
                                   const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride,
                                   int32_t mask_token, int32_t *cand_tok, uint8_t *cand_masked, int *err_flag,
                                   hipStream_t st) {
    hipLaunchKernelGGL(build_candidates_kernel, dim3(B), dim3(64), 0, st, L, K, x_t, masked_t, draft_pos, draft_tok,
                       draft_stride, mask_token, cand_tok, cand_masked, err_flag);
    return hipGetLastError();
}

int reduce_rows_tiles(int V) { return (V + RT - 1) / RT; }
int verify_chunks(int V) { return (V + RT - 1) / RT; }

hipError_t launch_reduce_rows(const float *z, int M, int V, float *pm, float *ps, int *pi, int *nT_out,
                              hipStream_t st) {
    const int nT = reduce_rows_tiles(V);
    *nT_out = nT;
    if (V % 4 == 0)
        hipLaunchKernelGGL(reduce_rows_kernel<true>, dim3(nT, M), dim3(256), 0, st, z, M, V, pm, ps, pi);
    else
        hipLaunchKernelGGL(reduce_rows_kernel<false>, dim3(nT, M), dim3(256), 0, st, z, M, V, pm, ps, pi);
    return hipGetLastError();
}

hipError_t launch_merge_select(const SelectArgs &a, hipStream_t st) {
    hipLaunchKernelGGL(merge_select_kernel, dim3(a.B), dim3(256), 0, st, a);
    return hipGetLastError();
}

hipError_t launch_commit(int B, int L, const int32_t *x_tok, int8_t *revealed_at, const uint8_t *masked,
                         int32_t *x_out, int32_t *n_masked, hipStream_t st) {
    hipLaunchKernelGGL(commit_kernel, dim3(B), dim3(64), 0, st, L, x_tok, revealed_at, masked, x_out, n_masked);
    return hipGetLastError();
}

hipError_t launch_remask(int B, int L, int state, const float *conf, float tau_remask,
                         const int32_t *protect_pos, int8_t *revealed_at, uint8_t *masked, uint8_t *remasked,
                         hipStream_t st) {
    hipLaunchKernelGGL(remask_kernel, dim3(B), dim3(64), 0, st, B, L, state, conf, tau_remask, protect_pos,
                       revealed_at, masked, remasked);
    return hipGetLastError();
}

hipError_t launch_verify(int B, int L, int V, int K, int joint, const float *verify, const int32_t *draft_pos,
                         const int32_t *draft_tok, int draft_stride, float *wm, int *wi, uint8_t *match,
                         int32_t *accept_len, int32_t *correction_tok, int *err_flag, hipStream_t st) {
    const int nC = verify_chunks(V);
    if (V % 4 == 0)
        hipLaunchKernelGGL(verify_argmax_kernel<true>, dim3(nC, B * K), dim3(256), 0, st, L, V, K, joint, verify,
                           draft_pos, draft_stride, nC, wm, wi, err_flag);
    else
        hipLaunchKernelGGL(verify_argmax_kernel<false>, dim3(nC, B * K), dim3(256), 0, st, L, V, K, joint, verify,
                           draft_pos, draft_stride, nC, wm, wi, err_flag);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(verify_accept_kernel, dim3((B + 255) / 256), dim3(256), 0, st, B, K, nC, wm, wi,
                       draft_tok, draft_stride, match, accept_len, correction_tok);
    return hipGetLastError();
}

}  // namespace mrp
