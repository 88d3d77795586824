/*
 * CPU oracle for the MRP chain step.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 statement of what one denoising step's chain of K
 * Multi-token Residual Prediction heads computes.  It exists so that the GPU
 * library can be checked against something that is obviously right; only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or helper with the GPU path.
 *
 * What follows the paper and where:
 *   - confidence = top-1 softmax probability of a row of logits
 *       (Section 2, "Denoising Loop").
 *   - one MRP step: (Delta, delta) <- g(x, h); h <- h + Delta;
 *       l <- l + delta; then reveal / draft from softmax(l)
 *       (Section 3.4, Algorithm 2 inner loop; Algorithm 3 drafting loop).
 *   - the head reuses the backbone's LM head to turn its output into the
 *       residual logits (Section 3.2).
 *   - dynamic reveal: every masked position whose confidence exceeds tau,
 *       at least one per step (Section 4.1 "Denoising Mode"); static reveal
 *       of the r most confident is the same rule with tau >= 1, r_min = r.
 *   - max-accept cap m = min(max(floor(0.7 n), 5), L) (Section 4.4).
 *   - remask: positions revealed earlier in this step whose updated
 *       confidence is below the remask threshold (Section 3.4, Algorithm 4).
 *       Variant (remask_mode 1): the confidence compared is the probability
 *       the updated logits assign to the token that was revealed at that
 *       position (the requirement that a reveal keeps its confidence over two
 *       consecutive steps, read as a statement about that token),
 *       not the row's top-1 probability.
 *   - commit: at the end of a denoising step the revealed tokens are written
 *       into the block and those positions stay unmasked in later steps
 *       (Algorithm 2: x_t <- reveal; Algorithm 4 returns R after remasking).
 *   - joint verification: the K + 1 candidates C^0..C^K (candidate k holds the
 *       first k drafts) are scored in one backbone pass; draft j is checked
 *       against candidate j (Figure 1 (d)).
 *   - candidate blocks: candidate k is the block with the first k drafts written
 *       in and every other position as before the drafting (Figure 1 (d)).
 *   - verify: a draft is accepted where the verifier's argmax equals the
 *       drafted token (Algorithm 3); the accepted length is the longest
 *       all-matching prefix of the draft list.
 *
 *   - training objective: KL(softmax(l_{t-1}) || softmax(l_t + delta_t)) on
 *       masked rows and its gradient w.r.t. the residual (Section 3.3,
 *       Equation 3).
 *   - residual magnitudes: per-entry RMS of X^(t+r) - X^(t) over the states of
 *       a decoded block, in fp64, averaged per r (Appendix B).
 *   - the transformer head body: fuse projection, D transformer layers,
 *       shared LM head (Section 3.2; D = 3 in Section 4.1); the layer itself
 *       (pre-norm, rotary grouped-query attention over a prefix cache and the
 *       block, gated MLP) is a reading, the paper gives only the outline.
 *
 * The default head body is the benchmark's lightweight layout (not the paper's
 * transformer layers): x = [h ; E[cond_tok]], a = W1 x, s = SiLU(a),
 * u = W2 s, Delta = u, y = RMSNorm(u) * gamma, delta = W_lm y, all in fp64:
 * with round_y = 0 no intermediate is rounded -- this is the plain definition
 * l <- l + W_lm (RMSNorm(u) gamma) (Section 3.2, Algorithm 2), and the logit
 * tolerance of the parity rule is stated against it.  round_y = 1 rounds y --
 * and only y -- to bf16 before the LM-head projection: the arithmetic of an
 * implementation whose LM-head activation operand is bf16.  It is used to
 * compare discrete decisions bit for bit (both sides then take each decision
 * on logits that differ by fp32 round-off only); it is a variant, not the
 * definition.
 *
 * Ties: lowest vocabulary index wins an argmax; lowest position wins a
 * confidence tie.  Reveal compares strictly (conf > tau), remask compares
 * strictly (conf < tau_remask).
 *
 * Pins (tests -m "not gpu"): library logsumexp / matmul on random shapes,
 * closed forms (uniform row, one-hot-plus-a row), shift invariance,
 * permutation equivariance, sum of probabilities, zero-residual invariance,
 * the softmax half-Lipschitz bound, tau = 0 / tau >= 1 reveal sets, the cap
 * values, brute-force longest matching prefix, remask set inclusions; a chain
 * resumed head by head against the full run; the candidate blocks against a
 * by-hand example and their nesting invariants;
 * KL against scipy's softmax / rel_entr, a two-class closed form, finite
 * differences and the one-hot cross-entropy limit; residual magnitudes against
 * a hand-worked example, a linear ramp and numpy's norm; the transformer layer
 * against closed-form rotations, a numpy / scipy library version and the
 * identity / uniform-attention / single-key special cases.
 * Parity unpinned: the end-to-end numeric values of both head layouts (the
 * paper prints no worked example, and fixes the transformer layer only in
 * outline); they are pinned only through the library compositions and the
 * invariants above.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int d, V, B, L, K;
    double rms_eps;
    double tau;          /* reveal threshold, strict >                       */
    int r_min;           /* forced minimum number of reveals per state       */
    int max_accept;      /* 1: cap the number of threshold reveals           */
    int carry_hidden;    /* 1: h <- h + Delta between heads                  */
    double tau_remask;   /* < 0: no remask                                    */
    int head_reveal;     /* 1: reveal after every head (Alg. 2/3); 0: Alg. 4 */
    int fresh_block;     /* 1: state 0 starts from an all-masked block       */
    int state_offset;    /* heads run as states offset+1 .. offset+K          */
    int run_state0;      /* 1: reduce z and reveal (state 0) before the heads */
    int remask_mode;     /* 0: remask on the row's top-1 probability; 1: on the probability the updated
                            logits give to the token that was revealed there */
    int round_y;         /* 0: y stays fp64 (the definition); 1: y is rounded to bf16 before W_lm y */
} orc_cfg;

/* threads the parallel loops will use */
int orc_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* Nearest bf16 value (8 significant bits, ties to even), as a double.
 * Normal range only: |x| far from the fp32 exponent limits. */
double orc_bf16_round(double x) {
    if (x == 0.0 || !isfinite(x)) return x;
    int e;
    double m = frexp(x, &e);            /* |m| in [0.5, 1) */
    double q = nearbyint(m * 256.0);    /* default mode: ties to even */
    return ldexp(q / 256.0, e);
}

void orc_bf16_round_array(const double *x, double *out, long n) {
    for (long i = 0; i < n; ++i) out[i] = orc_bf16_round(x[i]);
}

/* Per row: m = max, s = sum exp(z - m), tok = lowest index attaining m,
 * conf = 1/s (top-1 probability), lse = m + log s.  gap (may be NULL) receives
 * the top-2 logit gap: m minus the largest entry at any other index. */
void orc_reduce_rows(const double *z, int M, int V, int32_t *tok, double *conf, double *lse,
                     double *gap) {
#pragma omp parallel for schedule(static)
    for (int i = 0; i < M; ++i) {
        const double *r = z + (size_t)i * V;
        double m = r[0];
        int am = 0;
        for (int v = 1; v < V; ++v)
            if (r[v] > m) { m = r[v]; am = v; }
        double s = 0.0;
        for (int v = 0; v < V; ++v) s += exp(r[v] - m);
        tok[i] = am;
        conf[i] = 1.0 / s;
        lse[i] = m + log(s);
        if (gap) {
            double second = -INFINITY;
            for (int v = 0; v < V; ++v)
                if (v != am && r[v] > second) second = r[v];
            gap[i] = m - second;
        }
    }
}

/* Head body for every row i of every sequence b = i / L.
 *   hrun [M][d] in/out (updated only if carry_hidden)
 *   u_out, y_out [M][d] (may be NULL): pre-norm output and normalised output
 *   (rounded to bf16 when round_y is set). */
void orc_head_mlp(const orc_cfg *c, const uint16_t *W1, const uint16_t *W2, const uint16_t *gamma,
                  const uint16_t *E, const int32_t *cond_tok, double *hrun, double *u_out,
                  double *y_out) {
    const int d = c->d, M = c->B * c->L;
#pragma omp parallel
    {
        double *x = (double *)malloc(sizeof(double) * 2 * d);
        double *s = (double *)malloc(sizeof(double) * d);
        double *u = (double *)malloc(sizeof(double) * d);
#pragma omp for schedule(static)
        for (int i = 0; i < M; ++i) {
            const int b = i / c->L;
            const uint16_t *e = E + (size_t)cond_tok[b] * d;
            for (int j = 0; j < d; ++j) x[j] = hrun[(size_t)i * d + j];
            for (int j = 0; j < d; ++j) x[d + j] = bf16_bits_to_double(e[j]);
            for (int j = 0; j < d; ++j) {
                const uint16_t *w = W1 + (size_t)j * 2 * d;
                double a = 0.0;
                for (int k = 0; k < 2 * d; ++k) a += bf16_bits_to_double(w[k]) * x[k];
                s[j] = a * (1.0 / (1.0 + exp(-a)));          /* SiLU */
            }
            double ss = 0.0;
            for (int j = 0; j < d; ++j) {
                const uint16_t *w = W2 + (size_t)j * d;
                double acc = 0.0;
                for (int k = 0; k < d; ++k) acc += bf16_bits_to_double(w[k]) * s[k];
                u[j] = acc;
                ss += acc * acc;
            }
            const double inv = 1.0 / sqrt(ss / d + c->rms_eps);
            for (int j = 0; j < d; ++j) {
                const double yd = u[j] * inv * bf16_bits_to_double(gamma[j]);
                const double y = c->round_y ? orc_bf16_round(yd) : yd;
                if (y_out) y_out[(size_t)i * d + j] = y;
                if (u_out) u_out[(size_t)i * d + j] = u[j];
                if (c->carry_hidden) hrun[(size_t)i * d + j] += u[j];
            }
        }
        free(x); free(s); free(u);
    }
}

/* ---- transformer head body (Section 3.2: fuse projection, D transformer layers, shared LM head;
 * D = 3 in Section 4.1) ----
 * The paper fixes only that outline; the layer itself is the decoder layer of the backbone's
 * model family, written out here:
 *     n   = RMSNorm(u) g1
 *     q_h = RoPE(Wq_h n, pos), k_g = RoPE(Wk_g n, pos), v_g = Wv_g n        pos = prefix_len[b] + i
 *     o_h = softmax_t( q_h . k_t / sqrt(hd) ) v_t    over the prefix cache of kv head g = h / (nh / nkv)
 *                                                    and the L rows of the block (no mask inside the block)
 *     a   = u + Wo [o_0 .. o_{nh-1}]
 *     m   = RMSNorm(a) g2
 *     u'  = a + Wdown ( SiLU(Wgate m) * (Wup m) )
 * Wqkv rows: nh query heads, then nkv key heads, then nkv value heads (hd rows each).  Wgu rows:
 * d_ff gate rows, then d_ff up rows.  The prefix cache holds bf16 keys (already rotated) and values,
 * [B][P_max][nkv][hd], of which sequence b uses the first prefix_len[b] positions. */
typedef struct {
    int D, n_heads, n_kv_heads, head_dim, d_ff, P_max;
    double rope_theta;
} orc_tcfg;

/* rotate-half convention: entry j pairs with entry j + hd/2, angle pos * theta^(-2j/hd) */
void orc_rope(double *x, int hd, double pos, double theta) {
    const int half = hd / 2;
    for (int j = 0; j < half; ++j) {
        const double ang = pos * pow(theta, -2.0 * (double)j / (double)hd);
        const double cs = cos(ang), sn = sin(ang);
        const double a = x[j], b = x[j + half];
        x[j] = a * cs - b * sn;
        x[j + half] = b * cs + a * sn;
    }
}

static void rmsnorm_gain(const double *x, const uint16_t *g, int d, double eps, double *out) {
    double ss = 0.0;
    for (int j = 0; j < d; ++j) ss += x[j] * x[j];
    const double inv = 1.0 / sqrt(ss / d + eps);
    for (int j = 0; j < d; ++j) out[j] = x[j] * inv * bf16_bits_to_double(g[j]);
}

static void matvec_bf16(const uint16_t *W, int rows, int cols, const double *x, double *out) {
    for (int r = 0; r < rows; ++r) {
        const uint16_t *w = W + (size_t)r * cols;
        double acc = 0.0;
        for (int k = 0; k < cols; ++k) acc += bf16_bits_to_double(w[k]) * x[k];
        out[r] = acc;
    }
}

/* One transformer layer over the L rows U [L][d] of sequence b (in place). */
void orc_tlayer(const orc_tcfg *t, int d, int L, double eps, const uint16_t *Wqkv, const uint16_t *Wo,
                const uint16_t *Wgu, const uint16_t *Wdown, const uint16_t *g1, const uint16_t *g2,
                const uint16_t *kc_b, const uint16_t *vc_b, int P, double *U) {
    const int nh = t->n_heads, nkv = t->n_kv_heads, hd = t->head_dim, ff = t->d_ff;
    const int qd = nh * hd, kvd = nkv * hd, rep = nh / nkv, T = P + L;
    double *n = (double *)malloc(sizeof(double) * d);
    double *qkv = (double *)malloc(sizeof(double) * (size_t)L * (qd + 2 * kvd));
    double *o = (double *)malloc(sizeof(double) * qd);
    double *sc = (double *)malloc(sizeof(double) * T);
    double *tmp = (double *)malloc(sizeof(double) * (d > 2 * ff ? d : 2 * ff));
    double *act = (double *)malloc(sizeof(double) * ff);
    double *A = (double *)malloc(sizeof(double) * (size_t)L * d);
    for (int i = 0; i < L; ++i) {
        double *r = qkv + (size_t)i * (qd + 2 * kvd);
        rmsnorm_gain(U + (size_t)i * d, g1, d, eps, n);
        matvec_bf16(Wqkv, qd + 2 * kvd, d, n, r);
        for (int h = 0; h < nh; ++h) orc_rope(r + h * hd, hd, (double)(P + i), t->rope_theta);
        for (int g = 0; g < nkv; ++g) orc_rope(r + qd + g * hd, hd, (double)(P + i), t->rope_theta);
    }
    for (int i = 0; i < L; ++i) {
        const double *qi = qkv + (size_t)i * (qd + 2 * kvd);
        for (int h = 0; h < nh; ++h) {
            const int g = h / rep;
            const double *q = qi + h * hd;
            double mx = -INFINITY;
            for (int tt = 0; tt < T; ++tt) {
                double acc = 0.0;
                if (tt < P) {
                    const uint16_t *k = kc_b + ((size_t)tt * nkv + g) * hd;
                    for (int e = 0; e < hd; ++e) acc += q[e] * bf16_bits_to_double(k[e]);
                } else {
                    const double *k = qkv + (size_t)(tt - P) * (qd + 2 * kvd) + qd + g * hd;
                    for (int e = 0; e < hd; ++e) acc += q[e] * k[e];
                }
                sc[tt] = acc / sqrt((double)hd);
                if (sc[tt] > mx) mx = sc[tt];
            }
            double den = 0.0;
            for (int tt = 0; tt < T; ++tt) { sc[tt] = exp(sc[tt] - mx); den += sc[tt]; }
            double *oh = o + h * hd;
            for (int e = 0; e < hd; ++e) oh[e] = 0.0;
            for (int tt = 0; tt < T; ++tt) {
                const double pr = sc[tt] / den;
                if (tt < P) {
                    const uint16_t *v = vc_b + ((size_t)tt * nkv + g) * hd;
                    for (int e = 0; e < hd; ++e) oh[e] += pr * bf16_bits_to_double(v[e]);
                } else {
                    const double *v = qkv + (size_t)(tt - P) * (qd + 2 * kvd) + qd + kvd + g * hd;
                    for (int e = 0; e < hd; ++e) oh[e] += pr * v[e];
                }
            }
        }
        matvec_bf16(Wo, d, qd, o, tmp);
        for (int j = 0; j < d; ++j) A[(size_t)i * d + j] = U[(size_t)i * d + j] + tmp[j];
    }
    for (int i = 0; i < L; ++i) {
        double *a = A + (size_t)i * d;
        rmsnorm_gain(a, g2, d, eps, n);
        matvec_bf16(Wgu, 2 * ff, d, n, tmp);
        for (int j = 0; j < ff; ++j) act[j] = tmp[j] / (1.0 + exp(-tmp[j])) * tmp[ff + j];
        matvec_bf16(Wdown, d, ff, act, n);
        for (int j = 0; j < d; ++j) U[(size_t)i * d + j] = a[j] + n[j];
    }
    free(n); free(qkv); free(o); free(sc); free(tmp); free(act); free(A);
}

/* Transformer head body for every sequence: u0 = Wf [hrun ; e], D layers, then as the MLP body:
 * y = RMSNorm(u_D) gamma (rounded to bf16 when round_y is set), hrun += u_D if carry_hidden.  The per-layer arrays have D entries. */
void orc_head_transformer(const orc_cfg *c, const orc_tcfg *t, const uint16_t *Wf,
                          const uint16_t *const *Wqkv, const uint16_t *const *Wo, const uint16_t *const *Wgu,
                          const uint16_t *const *Wdown, const uint16_t *const *g1, const uint16_t *const *g2,
                          const uint16_t *const *kc, const uint16_t *const *vc, const int32_t *prefix_len,
                          const uint16_t *gamma, const uint16_t *E, const int32_t *cond_tok, double *hrun,
                          double *u_out, double *y_out) {
    const int d = c->d, L = c->L;
    const size_t cache_b = (size_t)t->P_max * t->n_kv_heads * t->head_dim;
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < c->B; ++b) {
        double *x = (double *)malloc(sizeof(double) * 2 * d);
        double *U = (double *)malloc(sizeof(double) * (size_t)L * d);
        double *yn = (double *)malloc(sizeof(double) * d);
        const uint16_t *e = E + (size_t)cond_tok[b] * d;
        for (int i = 0; i < L; ++i) {
            for (int j = 0; j < d; ++j) x[j] = hrun[((size_t)b * L + i) * d + j];
            for (int j = 0; j < d; ++j) x[d + j] = bf16_bits_to_double(e[j]);
            matvec_bf16(Wf, d, 2 * d, x, U + (size_t)i * d);
        }
        for (int l = 0; l < t->D; ++l)
            orc_tlayer(t, d, L, c->rms_eps, Wqkv[l], Wo[l], Wgu[l], Wdown[l], g1[l], g2[l], kc[l] + b * cache_b,
                       vc[l] + b * cache_b, prefix_len[b], U);
        for (int i = 0; i < L; ++i) {
            const size_t row = (size_t)b * L + i;
            rmsnorm_gain(U + (size_t)i * d, gamma, d, c->rms_eps, yn);
            for (int j = 0; j < d; ++j) {
                if (y_out) y_out[row * d + j] = c->round_y ? orc_bf16_round(yn[j]) : yn[j];
                if (u_out) u_out[row * d + j] = U[(size_t)i * d + j];
                if (c->carry_hidden) hrun[row * d + j] += U[(size_t)i * d + j];
            }
        }
        free(x); free(U); free(yn);
    }
}

/* z[i][v] += sum_c W_lm[v][c] * y[i][c]   (shared LM head, residual add) */
void orc_lm_head_add(const uint16_t *W_lm, const double *y, double *z, int M, int V, int d) {
#pragma omp parallel for collapse(2) schedule(static)
    for (int i = 0; i < M; ++i) {
        for (int v = 0; v < V; ++v) {
            const uint16_t *w = W_lm + (size_t)v * d;
            const double *yi = y + (size_t)i * d;
            double acc = 0.0;
            for (int k = 0; k < d; ++k) acc += bf16_bits_to_double(w[k]) * yi[k];
            z[(size_t)i * V + v] += acc;
        }
    }
}

/* a before b in "most confident" order: higher confidence, then lower position */
static int more_confident(const double *conf, int a, int b) {
    if (conf[a] != conf[b]) return conf[a] > conf[b];
    return a < b;
}

int orc_max_accept_cap(int n_masked, int L) {
    int m = (7 * n_masked) / 10;       /* floor(0.7 n) in integers */
    if (m < 5) m = 5;
    if (m > L) m = L;
    return m;
}

/* Reveal rule for one state, all sequences.  conf/tok are this state's. */
void orc_reveal(const orc_cfg *c, int state, const double *conf, const int32_t *tok,
                uint8_t *masked, int8_t *revealed_at, int32_t *draft_pos, int32_t *draft_tok,
                int32_t *cond_tok, int32_t *top_pos /* [B] or NULL */) {
    const int L = c->L;
    int *sel = (int *)malloc(sizeof(int) * L);
    int *cand = (int *)malloc(sizeof(int) * L);
    for (int b = 0; b < c->B; ++b) {
        const double *cf = conf + (size_t)b * L;
        uint8_t *mk = masked + (size_t)b * L;
        int nc = 0;
        for (int p = 0; p < L; ++p) if (mk[p]) cand[nc++] = p;
        draft_pos[b] = -1; draft_tok[b] = -1;
        if (top_pos) top_pos[b] = -1;
        if (nc == 0) continue;
        /* candidates in most-confident-first order (insertion sort) */
        for (int a = 1; a < nc; ++a) {
            int p = cand[a], q = a - 1;
            while (q >= 0 && more_confident(cf, p, cand[q])) { cand[q + 1] = cand[q]; --q; }
            cand[q + 1] = p;
        }
        int ns = 0;
        for (int a = 0; a < nc; ++a) if (cf[cand[a]] > c->tau) sel[ns++] = cand[a];
        if (c->max_accept) {
            int m = orc_max_accept_cap(nc, L);
            if (ns > m) ns = m;        /* sel is already most-confident-first */
        }
        if (ns < c->r_min) {
            ns = c->r_min < nc ? c->r_min : nc;
            for (int a = 0; a < ns; ++a) sel[a] = cand[a];
        }
        if (ns == 0) continue;
        for (int a = 0; a < ns; ++a) {
            mk[sel[a]] = 0;
            revealed_at[(size_t)b * L + sel[a]] = (int8_t)state;
        }
        const int top = sel[0];
        draft_pos[b] = top;
        draft_tok[b] = tok[(size_t)b * L + top];
        cond_tok[b] = tok[(size_t)b * L + top];
        if (top_pos) top_pos[b] = top;
    }
    free(sel); free(cand);
}

/* Remask rule for one state: rows revealed at a state in [0, state-1] of this
 * chain step, not the protected position, whose confidence is < tau_remask. */
void orc_remask(int B, int L, int state, const double *conf, double tau_remask,
                const int32_t *protect_pos, uint8_t *masked, int8_t *revealed_at,
                uint8_t *remasked) {
    for (int b = 0; b < B; ++b)
        for (int p = 0; p < L; ++p) {
            const size_t i = (size_t)b * L + p;
            remasked[i] = 0;
            const int ra = revealed_at[i];
            if (ra < 0 || ra > state - 1) continue;
            if (protect_pos && protect_pos[b] == p) continue;
            if (conf[i] < tau_remask) { masked[i] = 1; revealed_at[i] = -1; remasked[i] = 1; }
        }
}

/* p[i] = softmax(z[i,:])[x_tok[i]] = exp(z[i][x_tok[i]] - lse[i]); 0 where no token is recorded. */
void orc_token_prob(const double *z, int M, int V, const double *lse, const int32_t *x_tok, double *p) {
    for (int i = 0; i < M; ++i) {
        const int t = x_tok[i];
        p[i] = (t >= 0 && t < V) ? exp(z[(size_t)i * V + t] - lse[i]) : 0.0;
    }
}

/* End of a denoising step: every position revealed in this step (revealed_at >= 0) is committed:
 * its token goes into the block (x_out), it is marked -2 (committed earlier) and stays unmasked.
 * n_masked[b] = positions of sequence b still masked. */
void orc_commit(int B, int L, const int32_t *x_tok, int8_t *revealed_at, const uint8_t *masked,
                int32_t *x_out, int32_t *n_masked) {
    for (int b = 0; b < B; ++b) {
        int n = 0;
        for (int p = 0; p < L; ++p) {
            const size_t i = (size_t)b * L + p;
            if (revealed_at[i] >= 0) { x_out[i] = x_tok[i]; revealed_at[i] = -2; }
            if (masked[i]) ++n;
        }
        n_masked[b] = n;
    }
}

/* Verify K drafts per sequence against verifier logits [B][L][V]. */
void orc_verify_accept(int B, int L, int V, int K, const float *verify, const int32_t *draft_pos,
                       const int32_t *draft_tok, uint8_t *match, int32_t *accept_len,
                       int32_t *correction_tok) {
    for (int b = 0; b < B; ++b) {
        int alen = 0, open = 1;
        correction_tok[b] = -1;
        for (int j = 0; j < K; ++j) {
            const int pos = draft_pos[(size_t)b * K + j];
            int vj = -1, ok = 0;
            if (pos >= 0) {
                const float *r = verify + ((size_t)b * L + pos) * V;
                float m = r[0];
                vj = 0;
                for (int v = 1; v < V; ++v) if (r[v] > m) { m = r[v]; vj = v; }
                ok = (vj == draft_tok[(size_t)b * K + j]);
            }
            match[(size_t)b * K + j] = (uint8_t)ok;
            if (open) {
                if (ok) ++alen;
                else { open = 0; correction_tok[b] = vj; }
            }
        }
        accept_len[b] = alen;
    }
}

/* Joint verification of the K + 1 draft candidates (Figure 1 (d)): candidate k carries the first
 * k drafts, so draft j is checked against candidate j's logits, which were computed with drafts
 * 0 .. j-1 in place and position draft_pos[j] still masked.  verify is [B][K+1][L][V].  The
 * accepted length is the longest all-matching prefix; the correction token is candidate a's
 * argmax at the first rejected draft's position (a = accepted length), -1 if all K are accepted
 * or that draft is missing. */
void orc_verify_accept_joint(int B, int L, int V, int K, const float *verify, const int32_t *draft_pos,
                             const int32_t *draft_tok, uint8_t *match, int32_t *accept_len,
                             int32_t *correction_tok) {
    for (int b = 0; b < B; ++b) {
        int alen = 0, open = 1;
        correction_tok[b] = -1;
        for (int j = 0; j < K; ++j) {
            const int pos = draft_pos[(size_t)b * K + j];
            int vj = -1, ok = 0;
            if (pos >= 0) {
                const float *r = verify + (((size_t)b * (K + 1) + j) * L + pos) * V;
                float m = r[0];
                vj = 0;
                for (int v = 1; v < V; ++v) if (r[v] > m) { m = r[v]; vj = v; }
                ok = (vj == draft_tok[(size_t)b * K + j]);
            }
            match[(size_t)b * K + j] = (uint8_t)ok;
            if (open) {
                if (ok) ++alen;
                else { open = 0; correction_tok[b] = vj; }
            }
        }
        accept_len[b] = alen;
    }
}

/* Candidate blocks of the joint verification (Figure 1 (d)): from the block x_t (tokens of its L
 * positions, masked_t = 1 where a position still holds the mask token) and the K drafts of a
 * chain step, in draft order, build the K + 1 candidates C^0 .. C^K: candidate k is x_t with the
 * first k drafts written in, everything else as in x_t.  cand_tok / cand_masked are
 * [B][K+1][L]; a masked position holds mask_token.  A missing draft (pos < 0) adds nothing, so the
 * candidates from it on repeat the one before. */
void orc_build_candidates(int B, int L, int K, const int32_t *x_t, const uint8_t *masked_t,
                          const int32_t *draft_pos, const int32_t *draft_tok, int32_t mask_token,
                          int32_t *cand_tok, uint8_t *cand_masked) {
    for (int b = 0; b < B; ++b)
        for (int k = 0; k <= K; ++k) {
            int32_t *ct = cand_tok + ((size_t)b * (K + 1) + k) * L;
            uint8_t *cm = cand_masked + ((size_t)b * (K + 1) + k) * L;
            for (int p = 0; p < L; ++p) {
                cm[p] = masked_t[(size_t)b * L + p] ? 1 : 0;
                ct[p] = cm[p] ? mask_token : x_t[(size_t)b * L + p];
            }
            for (int j = 0; j < k; ++j) {
                const int pos = draft_pos[(size_t)b * K + j];
                if (pos < 0 || pos >= L) continue;
                ct[pos] = draft_tok[(size_t)b * K + j];
                cm[pos] = 0;
            }
        }
}

/* Training objective of a head (Section 3.3, Equation 3), written as its definition: for each
 * row with row_mask != 0 (NULL: every row), p = softmax(teacher row) (the logits of denoising
 * step t-1), q = softmax(student row) (l_t + delta_t),
 *     loss[i] = scale * sum_v p_v (log p_v - log q_v),
 * and, when grad is not NULL, its derivative with respect to the student logits,
 *     grad[i][v] = scale * (q_v - p_v)
 * (from d(-sum_v p_v log q_v)/ds_u = q_u - p_u with sum_v p_v = 1).  Rows outside the mask get
 * loss 0 and gradient 0.  teacher/student are fp32 [M][V], read into fp64. */
void orc_kl_loss(int M, int V, const float *teacher, const float *student, const uint8_t *row_mask,
                 double scale, double *loss, double *grad) {
    double *lp = (double *)malloc(sizeof(double) * V), *lq = (double *)malloc(sizeof(double) * V);
    for (int i = 0; i < M; ++i) {
        const float *t = teacher + (size_t)i * V, *s = student + (size_t)i * V;
        if (row_mask && !row_mask[i]) {
            loss[i] = 0.0;
            if (grad) for (int v = 0; v < V; ++v) grad[(size_t)i * V + v] = 0.0;
            continue;
        }
        double mt = t[0], ms = s[0];
        for (int v = 1; v < V; ++v) { if (t[v] > mt) mt = t[v]; if (s[v] > ms) ms = s[v]; }
        double st = 0.0, ss = 0.0;
        for (int v = 0; v < V; ++v) { st += exp((double)t[v] - mt); ss += exp((double)s[v] - ms); }
        const double lt = mt + log(st), ls = ms + log(ss);
        double kl = 0.0;
        for (int v = 0; v < V; ++v) {
            lp[v] = (double)t[v] - lt;
            lq[v] = (double)s[v] - ls;
            kl += exp(lp[v]) * (lp[v] - lq[v]);
        }
        loss[i] = scale * kl;
        if (grad) for (int v = 0; v < V; ++v) grad[(size_t)i * V + v] = scale * (exp(lq[v]) - exp(lp[v]));
    }
    free(lp); free(lq);
}

/* Residual-magnitude measurement (Appendix B, the protocol behind Figure 2).  X holds, for each
 * of n_blocks decoded blocks, the S = block + 1 states X^(0..S-1) of one tensor (logits or hidden
 * states of the block's positions), N entries each, already in fp64.  With
 *     ||Y||_RMS = sqrt( (1/N) sum_i Y_i^2 ),
 *   rms_pair[b][t][u], u > t :  || X^(u) - X^(t) ||_RMS   (the residual delta_{t,r}, r = u - t)
 *   rms_pair[b][s][s]        :  || X^(s) ||_RMS            (entries below the diagonal: 0)
 *   rms_delta[r], r >= 1     :  mean of rms_pair[b][t][t+r] over every block b and t = 0 .. S-1-r
 *   rms_delta[0]             :  the reference line: mean of rms_pair[b][s][s] over b and s = 1 .. S-1 */
void orc_residual_rms(int n_blocks, int S, long N, const double *X, double *rms_pair, double *rms_delta) {
    for (int b = 0; b < n_blocks; ++b)
        for (int t = 0; t < S; ++t)
            for (int u = 0; u < S; ++u) {
                const double *xt = X + ((size_t)b * S + t) * N, *xu = X + ((size_t)b * S + u) * N;
                double acc = 0.0;
                if (u == t) for (long i = 0; i < N; ++i) acc += xt[i] * xt[i];
                else if (u > t) for (long i = 0; i < N; ++i) { const double dlt = xu[i] - xt[i]; acc += dlt * dlt; }
                rms_pair[((size_t)b * S + t) * S + u] = (u >= t) ? sqrt(acc / (double)N) : 0.0;
            }
    for (int r = 0; r < S; ++r) {
        double sum = 0.0;
        long cnt = 0;
        for (int b = 0; b < n_blocks; ++b)
            for (int t = (r == 0 ? 1 : 0); t + r < S; ++t) { sum += rms_pair[((size_t)b * S + t) * S + t + r]; ++cnt; }
        rms_delta[r] = cnt ? sum / (double)cnt : 0.0;
    }
}

/* One denoising step's chain.
 *   z       [M][V] fp64 in/out         hrun [M][d] fp64 in/out
 *   heads   K triples of bf16 arrays   (W1[k], W2[k], gamma[k])
 *   tok/conf/lse [(K+1)][M]; slot 0 = state 0 (untouched when resuming)
 *   masked, revealed_at [M] in/out; cond_tok, protect_pos [B] in/out
 *   draft_pos/draft_tok [B][K+1] (column = local state index)
 *   remasked [(K+1)][M] (may be NULL)
 *   y_dump  [K][M][d] (may be NULL)
 *   gap     [(K+1)][M] top-2 logit gap per state (may be NULL)
 *   x_tok   [M] in/out: token recorded when a position is revealed (may be NULL unless
 *           remask_mode is 1) */
/* Per-head transformer bodies for the chain: every array has K * D entries, head k's layer l at
 * [k * D + l] (a module applied K times repeats its pointers). */
typedef struct {
    const orc_tcfg *t;
    const uint16_t *const *Wqkv, *const *Wo, *const *Wgu, *const *Wdown, *const *g1, *const *g2, *const *kc,
        *const *vc;
    const int32_t *prefix_len;
} orc_tbody;

static void chain_impl(const orc_cfg *c, const uint16_t *E, const uint16_t *W_lm,
                    const uint16_t *const *W1, const uint16_t *const *W2,
                    const uint16_t *const *gamma, double *z, double *hrun, int32_t *tok,
                    double *conf, double *lse, uint8_t *masked, int8_t *revealed_at,
                    int32_t *cond_tok, int32_t *protect_pos, int32_t *draft_pos,
                    int32_t *draft_tok, uint8_t *remasked, double *y_dump, double *gap, int32_t *x_tok,
                    const orc_tbody *tb) {
    const int M = c->B * c->L, K = c->K, B = c->B;
    double *ptok = (c->remask_mode == 1) ? (double *)malloc(sizeof(double) * M) : NULL;
    int32_t *dp = (int32_t *)malloc(sizeof(int32_t) * B);
    int32_t *dt = (int32_t *)malloc(sizeof(int32_t) * B);
    double *y = (double *)malloc(sizeof(double) * (size_t)M * c->d);
    for (int b = 0; b < B; ++b)
        for (int k = 0; k <= K; ++k) { draft_pos[b * (K + 1) + k] = -1; draft_tok[b * (K + 1) + k] = -1; }
    if (remasked) memset(remasked, 0, (size_t)(K + 1) * M);

    if (c->run_state0) {
        if (c->fresh_block)
            for (int i = 0; i < M; ++i) { masked[i] = 1; revealed_at[i] = -1; if (x_tok) x_tok[i] = -1; }
        orc_reduce_rows(z, M, c->V, tok, conf, lse, gap);
        orc_reveal(c, c->state_offset, conf, tok, masked, revealed_at, dp, dt, cond_tok, protect_pos);
        if (x_tok)
            for (int i = 0; i < M; ++i) if (revealed_at[i] == c->state_offset) x_tok[i] = tok[i];
        for (int b = 0; b < B; ++b) { draft_pos[b * (K + 1)] = dp[b]; draft_tok[b * (K + 1)] = dt[b]; }
    }
    for (int k = 1; k <= K; ++k) {
        const int state = c->state_offset + k;
        if (tb) {
            const int o = (k - 1) * tb->t->D;
            orc_head_transformer(c, tb->t, W1[k - 1], tb->Wqkv + o, tb->Wo + o, tb->Wgu + o, tb->Wdown + o,
                                 tb->g1 + o, tb->g2 + o, tb->kc + o, tb->vc + o, tb->prefix_len, gamma[k - 1], E,
                                 cond_tok, hrun, NULL, y);
        } else {
            orc_head_mlp(c, W1[k - 1], W2[k - 1], gamma[k - 1], E, cond_tok, hrun, NULL, y);
        }
        if (y_dump) memcpy(y_dump + (size_t)(k - 1) * M * c->d, y, sizeof(double) * (size_t)M * c->d);
        orc_lm_head_add(W_lm, y, z, M, c->V, c->d);
        orc_reduce_rows(z, M, c->V, tok + (size_t)k * M, conf + (size_t)k * M, lse + (size_t)k * M,
                        gap ? gap + (size_t)k * M : NULL);
        if (c->head_reveal) {
            orc_reveal(c, state, conf + (size_t)k * M, tok + (size_t)k * M, masked, revealed_at,
                       dp, dt, cond_tok, NULL);
            for (int b = 0; b < B; ++b) { draft_pos[b * (K + 1) + k] = dp[b]; draft_tok[b * (K + 1) + k] = dt[b]; }
            if (x_tok)
                for (int i = 0; i < M; ++i) if (revealed_at[i] == state) x_tok[i] = tok[(size_t)k * M + i];
        }
        if (c->tau_remask >= 0.0) {
            uint8_t *rm = remasked ? remasked + (size_t)k * M : (uint8_t *)malloc(M);
            const double *cr = conf + (size_t)k * M;
            if (c->remask_mode == 1) {
                orc_token_prob(z, M, c->V, lse + (size_t)k * M, x_tok, ptok);
                cr = ptok;
            }
            orc_remask(B, c->L, state, cr, c->tau_remask, protect_pos, masked, revealed_at, rm);
            if (!remasked) free(rm);
        }
    }
    free(dp); free(dt); free(y); free(ptok);
}

void orc_chain_step(const orc_cfg *c, const uint16_t *E, const uint16_t *W_lm,
                    const uint16_t *const *W1, const uint16_t *const *W2,
                    const uint16_t *const *gamma, double *z, double *hrun, int32_t *tok,
                    double *conf, double *lse, uint8_t *masked, int8_t *revealed_at,
                    int32_t *cond_tok, int32_t *protect_pos, int32_t *draft_pos,
                    int32_t *draft_tok, uint8_t *remasked, double *y_dump, double *gap, int32_t *x_tok) {
    chain_impl(c, E, W_lm, W1, W2, gamma, z, hrun, tok, conf, lse, masked, revealed_at, cond_tok, protect_pos,
               draft_pos, draft_tok, remasked, y_dump, gap, x_tok, NULL);
}

/* The same chain with the transformer head body: W1[k] is head k's fuse projection, W2 is unused
 * (may be NULL). */
void orc_chain_step_tf(const orc_cfg *c, const uint16_t *E, const uint16_t *W_lm,
                       const uint16_t *const *W1, const uint16_t *const *gamma, double *z, double *hrun,
                       int32_t *tok, double *conf, double *lse, uint8_t *masked, int8_t *revealed_at,
                       int32_t *cond_tok, int32_t *protect_pos, int32_t *draft_pos, int32_t *draft_tok,
                       uint8_t *remasked, double *y_dump, double *gap, int32_t *x_tok, const orc_tbody *tb) {
    chain_impl(c, E, W_lm, W1, NULL, gamma, z, hrun, tok, conf, lse, masked, revealed_at, cond_tok, protect_pos,
               draft_pos, draft_tok, remasked, y_dump, gap, x_tok, tb);
}
