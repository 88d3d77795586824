/*
 * mrp.h — C ABI of the MI355X (gfx950) Multi-token Residual Prediction chain step.
 *
 * One denoising step of a block-diffusion LM with MRP (paper Section 3.4,
 * Algorithms 2-4): after the backbone has produced hidden states h and logits z
 * for the B x L rows of the current blocks, a chain of K lightweight heads
 * repeatedly predicts a logit residual through the shared LM head, adds it to
 * the logit state, and reduces every row over the vocabulary (softmax
 * confidence = top-1 probability, argmax) to drive reveal, draft, remask and
 * speculative accept decisions.
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless it
 *     says "host".  The library allocates only the workspace inside mrp_ctx
 *     (at mrp_create) and never allocates or synchronises in the calls below.
 *   - `stream` is a hipStream_t passed as void*; all work is enqueued on it,
 *     in order, and the call returns without waiting.
 *   - Arguments are validated on the host before anything is launched; a
 *     failed validation returns a negative status and launches nothing.
 *   - Rows: M = B * L, row i belongs to sequence b = i / L, position p = i % L.
 *   - bf16 tensors are raw 16-bit patterns.  "packed" matrices are in the
 *     MFMA fragment order produced by mrp_pack_weight (the LM head) or
 *     mrp_pack_body_weight (every weight of a head body), see below.
 *   - Ties: an argmax over the vocabulary takes the lowest index; "most
 *     confident" ties take the lowest position.
 */
#ifndef MRP_H
#define MRP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MRP_OK 0
#define MRP_ERR_NULL (-1)      /* a required pointer is NULL                      */
#define MRP_ERR_SHAPE (-2)     /* a size is out of range or inconsistent          */
#define MRP_ERR_ALIGN (-3)     /* a pointer is not 16-byte aligned                */
#define MRP_ERR_WORKSPACE (-4) /* rows / sizes exceed what mrp_create reserved    */
#define MRP_ERR_HIP (-5)       /* a HIP runtime call failed (see mrp_last_error)  */

#define MRP_MAX_BLOCK_LEN 64
#define MRP_MAX_HEADS 16

typedef struct mrp_ctx mrp_ctx;

/* Problem sizes fixed for the life of a context.
 *   d          hidden size, multiple of 128 and at most 8192 (one k range of the
 *              GEMM kernels is 128 wide; not the multiple of 8 a plain GEMM
 *              would accept)
 *   V          vocabulary size, >= 1 (any value; multiples of 4 take the
 *              vectorised logit path)
 *   max_rows   largest M = B * L any call will use
 *   block_len  L, 1..MRP_MAX_BLOCK_LEN
 *   rms_eps    epsilon inside the RMSNorm square root */
typedef struct {
    int d, V, max_rows, block_len;
    float rms_eps;
} mrp_dims;

/* One head's weights (device).  W1: [d][2d], W2: [d][d], both packed with
 * mrp_pack_body_weight; gamma: bf16 [d], plain.  Every matrix a GEMM kernel
 * streams (the heads' weights, the transformer layers' projections and the
 * shared LM head) is taken in the packed layout only: a frozen weight is
 * packed once at load time (mrp_pack_weight / mrp_pack_body_weight read the
 * plain row-major bf16 matrix); the embedding table E, which is gathered by
 * row, stays plain [V][d].  Head body (benchmark layout
 * standing in for the transformer layers of Section 3.2):
 *   x = [h_run ; E[cond_tok]],  a = W1 x,  s = a * sigmoid(a),  u = W2 s,
 *   h_run += u (hidden residual, Algorithm 2 line "h <- h + Delta"),
 *   y = bf16(u / sqrt(mean(u^2) + eps) * gamma),  delta = W_lm y. */
typedef struct {
    const void *W1_packed, *W2_packed, *gamma;
} mrp_head;

/* Decision rules of one chain step.
 *   tau          reveal every still-masked row with confidence > tau (strict;
 *                Section 4.1 "Denoising Mode": dynamic denoising)
 *   r_min        forced minimum number of reveals per sequence and state
 *                (dynamic denoising reveals at least one position per step);
 *                static top-r decoding is tau >= 1 with r_min = r (Algorithm 2)
 *   max_accept   1: cap threshold reveals at min(max(floor(0.7 n), 5), L),
 *                n = masked rows of the sequence (Section 4.4)
 *   carry_hidden 1: h_run <- h_run + u between heads
 *   tau_remask   >= 0: after each head, rows revealed earlier in this chain
 *                step whose new confidence is < tau_remask (strict) are masked
 *                again, except the protected state-0 top row (Algorithm 4 with
 *                tau_remask = tau); < 0: off
 *   head_reveal  1: apply the reveal rule after every head (Algorithms 2, 3);
 *                0: only at state 0 (Algorithm 4)
 *   fresh_block  1: state 0 treats every row as masked and resets revealed_at
 *   state_offset index of the state that precedes the first head: the K heads
 *                run as states state_offset+1 .. state_offset+K (0 for a whole
 *                chain step; s to continue a step after its state s)
 *   run_state0   1: first reduce z and apply the reveal rule as state
 *                state_offset (the backbone's own reveal, Algorithm 2 line
 *                before the inner loop); 0: skip it and take cond_tok /
 *                protect_pos / masks as given
 *   remask_mode  which confidence the remask rule compares with tau_remask:
 *                0 the row's top-1 probability under the updated logits (the
 *                definition of confidence, Section 2); 1 the probability the
 *                updated logits give to the token that was revealed at that row
 *                (Section 3.4's requirement that a reveal keeps its confidence
 *                over two consecutive steps, read as a statement about the
 *                revealed token); needs x_tok */
typedef struct {
    float tau;
    int r_min;
    int max_accept;
    int carry_hidden;
    float tau_remask;
    int head_reveal;
    int fresh_block;
    int state_offset;
    int run_state0;
    int remask_mode;
} mrp_reveal_cfg;

/* Per-step state and outputs (device).  Slot k of tok/conf/lse is the local
 * state index: 0 = state 0 (untouched when run_state0 = 0), k = after head k.
 *   tok, conf, lse   [(K+1)][M]  argmax, top-1 probability, log-sum-exp; required
 *   revealed_at      [M] in/out  -1 masked, -2 committed in an earlier step,
 *                                else the state index that revealed the row
 *   masked           [M] in/out  1 = still [MASK]
 *   cond_tok         [B] in/out  token that conditions the next head: the token
 *                                of the most confident row revealed by the
 *                                previous state (kept if nothing was revealed)
 *   protect_pos      [B] in/out  position of the state-0 top row (-1 if none);
 *                                written at state 0, read by remask
 *   draft_pos/tok    [B][K+1]    most confident new reveal of each local state
 *                                (position in block, token), -1 if none
 *   remasked         [(K+1)][M]  1 where a row was remasked at that state; may
 *                                be NULL
 *   x_tok            [M] in/out  token recorded when a row is revealed (what
 *                                mrp_commit writes into the block); may be NULL
 *                                unless remask_mode = 1 */
typedef struct {
    int32_t *tok;
    float *conf;
    float *lse;
    int8_t *revealed_at;
    uint8_t *masked;
    int32_t *cond_tok;
    int32_t *protect_pos;
    int32_t *draft_pos, *draft_tok;
    uint8_t *remasked;
    int32_t *x_tok;
} mrp_step_io;

/* Create / destroy a context on the current device.  mrp_create allocates the
 * workspace (see mrp_workspace_bytes) with hipMalloc and zero-fills it. */
int mrp_create(mrp_ctx **out, const mrp_dims *dims);
int mrp_destroy(mrp_ctx *ctx);
size_t mrp_workspace_bytes(const mrp_dims *dims);
/* Message of the last error on this context (host string, never NULL). */
const char *mrp_last_error(const mrp_ctx *ctx);

/* Packed layout of a row-major bf16 matrix X[rows][cols] (cols % 16 == 0):
 * 1 KiB blocks of 32 rows x 16 columns ordered [row block][column block];
 * inside a block, lane l (0..63) owns the 8 consecutive values
 * X[32 rb + l % 32][16 cb + 8 (l / 32) .. + 7] — the operand order of the
 * 32x32x16 bf16 MFMA, so a wavefront's load of a block is one contiguous
 * 1 KiB read.  rows are padded to a multiple of 32 with zeros. */
size_t mrp_packed_bytes(int rows, int cols);
int mrp_pack_weight(void *stream, const void *src /* bf16 [rows][cols] */, int rows, int cols,
                    void *dst /* mrp_packed_bytes(rows, cols), 16-B aligned */);
/* The same layout with every value converted from bf16 to fp16 (round to
 * nearest even): the form the head bodies take their weights in (W1, W2 and
 * the transformer layers' projections).  The head body multiplies fp32
 * activations, split into two fp16 terms, by these weights on the fp16 matrix
 * cores with fp32 accumulation; the shared LM head keeps bf16 operands (its
 * activation is bf16 by definition, Section 3.2).  The conversion is exact for
 * 6.1e-5 <= |w| < 65504 and within 3e-8 for smaller magnitudes; activations of
 * the head body must stay below 65504 in magnitude. */
int mrp_pack_body_weight(void *stream, const void *src /* bf16 [rows][cols] */, int rows, int cols,
                         void *dst /* mrp_packed_bytes(rows, cols), 16-B aligned */);

/* One denoising step's chain (Algorithm 2 inner loop / Algorithm 3 drafting
 * loop / Algorithm 4 with tau_remask): state 0 = reduce z and reveal, then for
 * k = 1..K: head k, z += W_lm y (fused with the per-row online
 * max / sum-exp / argmax), reveal [, remask].
 *   h       bf16 [M][d] backbone hidden states, or NULL to continue from h_run
 *   h_run   fp32 [M][d] running hidden state: overwritten from h when h is
 *           given, otherwise read; updated in place when carry_hidden
 *   E       bf16 [V][d] token embedding, plain row-major
 *   W_lm_packed  the shared LM head [V][d], packed
 *   heads   HOST array of K entries (the same entry K times = weight sharing)
 *   z       fp32 [M][V] logit state, updated in place */
int mrp_chain_step(mrp_ctx *ctx, void *stream, int B, int K, const void *h, float *h_run,
                   const void *E, const void *W_lm_packed, const mrp_head *heads, float *z,
                   const mrp_reveal_cfg *cfg, const mrp_step_io *io);

/* Remask rule alone (Algorithm 4, last line of the loop body): rows with
 * revealed_at in [0, state-1], other than protect_pos[b] (NULL = none), whose
 * conf_new < tau_remask become masked again (masked = 1, revealed_at = -1).
 * remasked_out [M] receives 1 for those rows and 0 elsewhere. */
int mrp_remask(mrp_ctx *ctx, void *stream, int B, int state, const float *conf_new,
               float tau_remask, const int32_t *protect_pos, int8_t *revealed_at,
               uint8_t *masked, uint8_t *remasked_out);

/* End of a denoising step (Algorithm 2: "x_t <- reveal ..."; Algorithm 4 returns
 * the reveals that survived remasking): every row revealed in this step
 * (revealed_at >= 0) is committed -- its recorded token x_tok goes into the
 * block x_out, revealed_at becomes -2, and the row stays unmasked in later
 * steps.  n_masked[b] = rows of sequence b still masked (the decode loop of a
 * block ends when it is 0).  All pointers device; x_tok [M] in, revealed_at [M]
 * in/out, masked [M] in, x_out [M] in/out, n_masked [B] out. */
int mrp_commit(mrp_ctx *ctx, void *stream, int B, const int32_t *x_tok, int8_t *revealed_at,
               const uint8_t *masked, int32_t *x_out, int32_t *n_masked);

/* Speculative verification (Algorithm 3: a drafted position is rejected where the
 * verifier's argmax differs from the draft): for each sequence b and draft j < K,
 *   v_j = argmax_v verify[b][draft_pos[b][j]][v],  match[b][j] = (v_j == draft_tok[b][j]);
 *   accept_len[b] = length of the longest all-matching prefix of the K drafts;
 *   correction_tok[b] = v at the first non-matching draft (-1 if all matched or
 *   that draft is missing).  A draft with pos < 0 is a non-match.
 *   verify fp32 [B][L][V]; draft_pos/draft_tok int32 [B][K] with row stride
 *   draft_stride (>= K) elements. */
int mrp_verify_accept(mrp_ctx *ctx, void *stream, int B, int K, const float *verify,
                      const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride,
                      uint8_t *match /* [B][K] */, int32_t *accept_len /* [B] */,
                      int32_t *correction_tok /* [B] */);

/* Joint verification of the K + 1 draft candidates (Figure 1 (d): candidate k
 * embeds the first k drafts and all candidates are scored in one backbone
 * pass).  verify is fp32 [B][K+1][L][V]; draft j is checked against candidate
 * j's row at draft_pos[b][j].  Outputs as mrp_verify_accept; correction_tok[b]
 * is candidate accept_len[b]'s argmax at the first rejected draft's position. */
int mrp_verify_accept_joint(mrp_ctx *ctx, void *stream, int B, int K, const float *verify,
                            const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride,
                            uint8_t *match /* [B][K] */, int32_t *accept_len /* [B] */,
                            int32_t *correction_tok /* [B] */);

/* Candidate blocks of the joint verification (Figure 1 (d)): candidate k (k = 0 .. K) of a sequence is
 * its block x_t with the first k drafts written in and every other position as in x_t; the
 * backbone scores all K + 1 candidates in one pass and mrp_verify_accept_joint checks draft j on
 * candidate j, where draft j's position is still masked.
 *   x_t       int32 [B][L]  tokens of the block before the drafting (ignored where masked_t = 1)
 *   masked_t  uint8 [B][L]  1 = the position holds the mask token in x_t
 *   draft_pos/draft_tok  int32 [B][K] with row stride draft_stride (>= K): the chain step's drafts in
 *             draft order (columns 1..K of its draft arrays); pos < 0 = missing draft, adds nothing;
 *             pos >= L is skipped and reported (MRP_FLAG_DRAFT_POS)
 *   mask_token  token id written at masked positions
 *   cand_tok  int32 [B][K+1][L] out,  cand_masked  uint8 [B][K+1][L] out (1 = still masked).
 * K = 0 gives the block itself. */
int mrp_build_candidates(mrp_ctx *ctx, void *stream, int B, int K, const int32_t *x_t, const uint8_t *masked_t,
                         const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride, int32_t mask_token,
                         int32_t *cand_tok, uint8_t *cand_masked);

/* Device error word.  An index that lives in device memory cannot be validated on the host before a
 * launch; a kernel that meets one out of range clamps or skips it (so that nothing faults) and sets a
 * bit of the context's error word:
 *   MRP_FLAG_COND_TOK    cond_tok[b] outside [0, V): clamped into the embedding table
 *   MRP_FLAG_DRAFT_POS   a draft position >= L: taken as a missing draft
 *   MRP_FLAG_PREFIX_LEN  prefix_len[b] outside [0, max_prefix]: clamped
 *   MRP_FLAG_X_TOK       a recorded token >= V (remask_mode 1): clamped
 * mrp_poll_error waits for `stream` (hipStreamSynchronize: not for use under stream capture), returns the
 * bits set since the last poll (0 = none) and clears them, or a negative status; mrp_last_error then
 * names the conditions. */
#define MRP_FLAG_COND_TOK 1
#define MRP_FLAG_DRAFT_POS 2
#define MRP_FLAG_PREFIX_LEN 4
#define MRP_FLAG_X_TOK 8
int mrp_poll_error(mrp_ctx *ctx, void *stream);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): mrp_verify_accept without a context.  Same computation, arguments and
 * outputs, with L and V passed in; the kernels' partial (max, argmax) array lives in a device array
 * of fixed size inside the library (MRP_VERIFY_STATIC_MAX_ENTRIES entries of 8 bytes = 512 KiB on
 * every GPU the library runs on, held until the process ends) instead of a context's workspace.
 * The call allocates nothing and launches only kernels.  B * K * ceil(V / 8192) must not exceed
 * MRP_VERIFY_STATIC_MAX_ENTRIES: a larger problem is refused with MRP_ERR_WORKSPACE and nothing is
 * launched (config 3 of the benchmarks, B = 128, K = 3, V = 151936, needs 7296).  All calls on one GPU
 * share that GPU's array: calls that overlap in time on one GPU (different streams or threads) race
 * and must be serialised by the caller; calls on one stream are ordered and safe.  The array keeps the
 * last call's contents; every entry a call reads it has written itself.  The array's address is looked
 * up on a device's first call (or by mrp_create on that device): under stream capture make that first
 * call before capturing.  Returns MRP_OK or a negative status (no context, so no message). */
#define MRP_VERIFY_STATIC_MAX_ENTRIES 65536
size_t mrp_verify_accept_static_scratch_bytes(void);
int mrp_verify_accept_static(void *stream, int B, int L, int V, int K, const float *verify,
                             const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride,
                             uint8_t *match /* [B][K] */, int32_t *accept_len /* [B] */,
                             int32_t *correction_tok /* [B] */);

/* Transformer head body (Section 3.2 outlines the head as a learned projection
 * that fuses the hidden states with the token embeddings, a few transformer
 * layers, and the backbone's own LM head
 * on top; D = 3 in Section 4.1).  The layer is the decoder layer of the
 * backbone's model family:
 *   u_0 = W1 [h_run ; E[cond_tok]]                        (the head's W1 is the fuse projection)
 *   n = RMSNorm(u) g1;  q | k | v = Wqkv n;  rotary embedding (rotate-half,
 *       base rope_theta) of q and k at position prefix_len[b] + i
 *   o = softmax(q k^T / sqrt(head_dim)) v over the sequence's prefix cache
 *       (positions 0 .. prefix_len[b]-1, keys already rotated) and the L rows
 *       of the block itself, no mask inside the block, grouped-query heads
 *   a = u + Wo o;  m = RMSNorm(a) g2;  u' = a + Wdown (SiLU(Wgate m) * (Wup m))
 * after D layers: h_run += u_D, y = bf16(RMSNorm(u_D) gamma), delta = W_lm y
 * as for the MLP body.  All weights given as bf16 and packed with mrp_pack_body_weight:
 *   Wqkv [(n_heads + 2 n_kv_heads) * 128][d]  rows: query heads, key heads, value heads
 *   Wo   [d][n_heads * 128]      Wgu [2 d_ff][d]  rows: gate, then up      Wdown [d][d_ff]
 *   g1, g2: bf16 [d], plain;  k_cache, v_cache: bf16 [B][max_prefix][n_kv_heads][128]
 * (row b of a cache belongs to sequence b of the call; may be NULL when max_prefix = 0). */
#define MRP_MAX_TLAYERS 16
typedef struct {
    int D;                 /* layers per head, 1..MRP_MAX_TLAYERS */
    int n_heads, n_kv_heads, head_dim;   /* head_dim must be 128; (n_heads / n_kv_heads) * block_len <= 64 */
    int d_ff;              /* multiple of 128 */
    int max_prefix;        /* positions per sequence in every prefix cache */
    float rope_theta;
} mrp_tbody_dims;

typedef struct {
    const void *Wqkv_packed, *Wo_packed, *Wgu_packed, *Wdown_packed;
    const void *g1, *g2;
    const void *k_cache, *v_cache;
} mrp_tlayer;

/* Reserve the transformer body's workspace on the context's device (one
 * hipMalloc, freed by mrp_destroy); once per context, block_len <= 16. */
int mrp_tbody_create(mrp_ctx *ctx, const mrp_tbody_dims *dims);

/* mrp_chain_step with the transformer head body: layers holds K * D entries,
 * head k's layer l at [k * D + l] (one module applied K times repeats its
 * entries); heads[k].W2_packed is ignored; prefix_len: device int32 [B],
 * values clamped to [0, max_prefix].  Everything else as mrp_chain_step. */
int mrp_chain_step_tf(mrp_ctx *ctx, void *stream, int B, int K, const void *h, float *h_run, const void *E,
                      const void *W_lm_packed, const mrp_head *heads, const mrp_tlayer *layers,
                      const int32_t *prefix_len, float *z, const mrp_reveal_cfg *cfg, const mrp_step_io *io);

/* Training-side objective of the head (Section 3.3, Equation 3), forward and
 * gradient: for every row i with row_mask[i] != 0 (NULL = all rows),
 *   loss_rows[i] = scale * KL( softmax(teacher[i]) || softmax(student[i]) ),
 *   grad[i][v]   = scale * ( softmax(student[i])[v] - softmax(teacher[i])[v] )
 * (the derivative of loss_rows[i] with respect to student[i][v], i.e. to the
 * predicted residual delta), and 0 for the other rows.  teacher = l_{t-1},
 * student = l_t + delta_t, both fp32 [M][V] device; loss_rows fp32 [M];
 * grad fp32 [M][V] or NULL (forward only).  M <= max_rows.  No softmax is
 * materialised: one pass over both tensors for the loss, one more for grad. */
int mrp_kl_loss(mrp_ctx *ctx, void *stream, int M, const float *teacher, const float *student,
                const uint8_t *row_mask, float scale, float *loss_rows, float *grad);

/* Residual-magnitude measurement (Appendix B, the protocol behind Figure 2).
 * X: device, [n_blocks][S][N], fp32 (dtype MRP_DTYPE_F32) or bf16 (MRP_DTYPE_BF16):
 * for each decoded block the S = block length + 1 states of one backbone
 * tensor restricted to the block (logits: N = L*V; hidden states: N = L*d),
 * state s having s revealed positions.  With ||Y||_RMS = sqrt(sum Y_i^2 / N),
 * all sums in fp64:
 *   rms_pair  [n_blocks][S][S] (device, fp64):  [b][t][u] = ||X^(u) - X^(t)||_RMS
 *             for u > t, ||X^(s)||_RMS on the diagonal, 0 below it;
 *   rms_delta [S] (device, fp64): [r] for r >= 1 = mean of rms_pair[b][t][t+r]
 *             over all blocks and t = 0 .. S-1-r; [0] = the reference line, the
 *             mean of the diagonal over all blocks and s = 1 .. S-1.
 * S must be 3, 5, 9 or 17; n_blocks <= 4096; every state is read once. */
#define MRP_DTYPE_F32 0
#define MRP_DTYPE_BF16 1
int mrp_residual_rms(mrp_ctx *ctx, void *stream, int n_blocks, int S, long N, const void *X, int dtype,
                     double *rms_pair, double *rms_delta);

/* Timing of the dominant kernel.  With profiling on, every LM-head kernel
 * launched by mrp_chain_step is bracketed by a pair of HIP events on the call's
 * stream (up to 4096 pairs between reads); a chain step recorded while profiling
 * is on contains event records and is not meant for HIP graph capture: capture
 * with profiling off (the default).  mrp_profile_read waits for the
 * recorded events, stores up to `cap` elapsed times in milliseconds into the
 * HOST array ms_out, returns how many it stored, and clears the record. */
int mrp_profile_enable(mrp_ctx *ctx, int on);
int mrp_profile_read(mrp_ctx *ctx, float *ms_out, int cap);

/* Measurement aid (not part of the method): move the bytes of one LM-head launch at M <= 128 rows
 * with the persistent LM-head kernel's work split and access pattern and none of its arithmetic.
 *   mode 0  stream the packed W_lm once
 *   mode 1  ... and read the [M][V] logit tile
 *   mode 2  ... and write the logit tile back (the same values: z is unchanged)
 * Its time is the floor the memory system sets for that traffic mix; bench.py --workload lm_traffic
 * reports it next to the kernel.  Needs V % 4 == 0 and d % 256 == 0. */
int mrp_probe_lm_traffic(mrp_ctx *ctx, void *stream, int mode, int M, const void *W_lm_packed, float *z);

#ifdef __cplusplus
}
#endif
#endif /* MRP_H */
