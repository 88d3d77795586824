/*
 * Sanitizer driver for the CPU oracle.  TEST INFRASTRUCTURE ONLY.
 *
 * Compiled together with mrp_oracle.c under -fsanitize=address,undefined (host code only) and run
 * by the CPU test suite: it calls every oracle function once on small, deterministic inputs whose
 * buffers have exactly the documented sizes, so that an out-of-bounds index, a leak or undefined
 * arithmetic in the oracle shows up as a sanitizer report.  It checks no values (the pins do that)
 * beyond a few sanity relations that keep the calls from being optimised away.
 */
#include <stdio.h>

#include "mrp_oracle.c"

static uint32_t rng_state = 12345u;
static double urand(void) {                      /* plain LCG in [0, 1) */
    rng_state = rng_state * 1664525u + 1013904223u;
    return (double)(rng_state >> 8) / 16777216.0;
}
static double nrand(void) {                      /* sum of uniforms, roughly normal */
    double s = 0.0;
    for (int i = 0; i < 6; ++i) s += urand();
    return (s - 3.0) * 1.4142;
}
static uint16_t bf16_of(double x) {
    float f = (float)x;
    uint32_t u;
    memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}
static uint16_t *bf16_matrix(size_t n, double std) {
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = bf16_of(nrand() * std);
    return p;
}
static double *f64_matrix(size_t n, double std) {
    double *p = (double *)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = nrand() * std;
    return p;
}

int main(void) {
    enum { d = 32, V = 96, B = 3, L = 5, K = 2, M = B * L };
    int bad = 0;
    uint16_t *E = bf16_matrix((size_t)V * d, 0.5), *W = bf16_matrix((size_t)V * d, 0.1);
    uint16_t *W1[K], *W2[K], *g[K];
    for (int k = 0; k < K; ++k) {
        W1[k] = bf16_matrix((size_t)d * 2 * d, 0.2);
        W2[k] = bf16_matrix((size_t)d * d, 0.2);
        g[k] = bf16_matrix(d, 0.0);
        for (int j = 0; j < d; ++j) g[k][j] = bf16_of(1.0);
    }
    double *z0 = f64_matrix((size_t)M * V, 2.0), *h0 = f64_matrix((size_t)M * d, 1.0);
    for (int i = 0; i < M; i += 2) z0[(size_t)i * V + (i * 7) % V] += 6.0 + i;     /* confident rows */

    for (int variant = 0; variant < 4; ++variant) {
        orc_cfg c = {d, V, B, L, K, 1e-6, 0.5, 1, variant & 1, 1, 0.3, 1, 1, 0, 1, (variant >> 1) & 1, variant & 1};
        double *z = (double *)malloc(sizeof(double) * M * V), *hr = (double *)malloc(sizeof(double) * M * d);
        memcpy(z, z0, sizeof(double) * M * V); memcpy(hr, h0, sizeof(double) * M * d);
        int32_t tok[(K + 1) * M], cond[B], prot[B], dpos[B * (K + 1)], dtok[B * (K + 1)], xtok[M];
        double conf[(K + 1) * M], lse[(K + 1) * M], gap[(K + 1) * M];
        uint8_t masked[M], rem[(K + 1) * M];
        int8_t ra[M];
        for (int b = 0; b < B; ++b) { cond[b] = 0; prot[b] = -1; }
        double *ydump = (double *)malloc(sizeof(double) * K * M * d);
        orc_chain_step(&c, E, W, (const uint16_t *const *)W1, (const uint16_t *const *)W2, (const uint16_t *const *)g, z, hr,
                       tok, conf, lse, masked, ra, cond, prot, dpos, dtok, rem, ydump, gap, xtok);
        /* the same chain resumed head by head */
        double *z2 = (double *)malloc(sizeof(double) * M * V), *hr2 = (double *)malloc(sizeof(double) * M * d);
        memcpy(z2, z0, sizeof(double) * M * V); memcpy(hr2, h0, sizeof(double) * M * d);
        int32_t tok2[2 * M], cond2[B], prot2[B], dpos2[B * 2], dtok2[B * 2], xtok2[M];
        double conf2[2 * M], lse2[2 * M];
        uint8_t masked2[M];
        int8_t ra2[M];
        for (int b = 0; b < B; ++b) { cond2[b] = 0; prot2[b] = -1; }
        orc_cfg c0 = c; c0.K = 0;
        int32_t dp0[B], dt0[B];
        orc_chain_step(&c0, E, W, NULL, NULL, NULL, z2, hr2, tok2, conf2, lse2, masked2, ra2, cond2, prot2, dp0, dt0, NULL,
                       NULL, NULL, xtok2);
        for (int k = 1; k <= K; ++k) {
            orc_cfg ck = c; ck.K = 1; ck.fresh_block = 0; ck.state_offset = k - 1; ck.run_state0 = 0;
            const uint16_t *w1 = W1[k - 1], *w2 = W2[k - 1], *gg = g[k - 1];
            orc_chain_step(&ck, E, W, &w1, &w2, &gg, z2, hr2, tok2, conf2, lse2, masked2, ra2, cond2, prot2, dpos2, dtok2,
                           NULL, NULL, NULL, xtok2);
        }
        for (int i = 0; i < M * V; ++i) bad |= (z[i] != z2[i]);
        for (int i = 0; i < M; ++i) bad |= (masked[i] != masked2[i]) | (ra[i] != ra2[i]);
        int32_t x_out[M], n_masked[B];
        for (int i = 0; i < M; ++i) x_out[i] = -1;
        orc_commit(B, L, xtok, ra, masked, x_out, n_masked);
        free(z); free(hr); free(z2); free(hr2); free(ydump);
    }

    /* stand-alone pieces */
    {
        double conf[M]; int32_t tok[M]; uint8_t masked[M], rm[M]; int8_t ra[M]; int32_t dp[B], dt[B], cond[B], top[B];
        for (int i = 0; i < M; ++i) { conf[i] = urand(); tok[i] = i % V; masked[i] = (i % 3) != 0; ra[i] = masked[i] ? -1 : 0; }
        for (int b = 0; b < B; ++b) cond[b] = 1;
        orc_cfg c = {d, V, B, L, 1, 1e-6, 0.6, 2, 1, 1, 0.4, 1, 0, 0, 0, 0, 0};
        orc_reveal(&c, 1, conf, tok, masked, ra, dp, dt, cond, top);
        orc_remask(B, L, 2, conf, 0.5, top, masked, ra, rm);
        bad |= (orc_max_accept_cap(16, 16) != 11) | (orc_max_accept_cap(4, 16) != 5);
        double x[5] = {1.0, -2.5, 3e-5, 1000.0, 0.0}, y[5];
        orc_bf16_round_array(x, y, 5);
        bad |= (y[0] != 1.0);
    }
    {
        enum { VV = 40, KK = 3 };
        float *ver = (float *)malloc(sizeof(float) * B * (KK + 1) * L * VV);
        for (int i = 0; i < B * (KK + 1) * L * VV; ++i) ver[i] = (float)nrand();
        int32_t dpos[B * KK], dtok[B * KK], alen[B], corr[B];
        uint8_t match[B * KK];
        for (int i = 0; i < B * KK; ++i) { dpos[i] = (i % 4 == 3) ? -1 : i % L; dtok[i] = (i * 11) % VV; }
        orc_verify_accept(B, L, VV, KK, ver, dpos, dtok, match, alen, corr);
        orc_verify_accept_joint(B, L, VV, KK, ver, dpos, dtok, match, alen, corr);
        int32_t x_t[B * L], ct[B * (KK + 1) * L];
        uint8_t m_t[B * L], cm[B * (KK + 1) * L];
        for (int i = 0; i < B * L; ++i) { x_t[i] = i; m_t[i] = i & 1; }
        dpos[1] = L + 2;                          /* a position beyond the block is skipped */
        orc_build_candidates(B, L, KK, x_t, m_t, dpos, dtok, 999, ct, cm);
        free(ver);
    }
    {
        enum { MM = 4, VV = 50 };
        float t[MM * VV], s[MM * VV];
        for (int i = 0; i < MM * VV; ++i) { t[i] = (float)nrand(); s[i] = (float)nrand(); }
        uint8_t mask[MM] = {1, 0, 1, 1};
        double loss[MM], grad[MM * VV];
        orc_kl_loss(MM, VV, t, s, mask, 0.25, loss, grad);
        orc_kl_loss(MM, VV, t, s, NULL, 1.0, loss, NULL);
        for (int i = 0; i < MM; ++i) bad |= !(loss[i] >= 0.0);
        enum { NB = 2, S = 5, N = 33 };
        double *X = f64_matrix((size_t)NB * S * N, 1.0), pair[NB * S * S], delta[S];
        orc_residual_rms(NB, S, N, X, pair, delta);
        free(X);
        double zz[MM * VV], lse2[MM], conf2[MM], p[MM]; int32_t tk[MM], xt[MM] = {3, -1, 49, 0};
        for (int i = 0; i < MM * VV; ++i) zz[i] = t[i];
        orc_reduce_rows(zz, MM, VV, tk, conf2, lse2, NULL);
        orc_token_prob(zz, MM, VV, lse2, xt, p);
    }
    {   /* transformer head body: 2 layers, 2 query heads on 1 kv head of dimension 8, prefix lengths 0, 3, 4 */
        orc_tcfg t = {2, 2, 1, 8, 24, 4, 100.0};
        const int qd = 16, kvd = 8;
        uint16_t *Wqkv[4], *Wo[4], *Wgu[4], *Wdown[4], *g1[4], *g2[4], *kc[4], *vc[4];
        for (int n = 0; n < 4; ++n) {            /* K * D = 4 layer slots */
            Wqkv[n] = bf16_matrix((size_t)(qd + 2 * kvd) * d, 0.2); Wo[n] = bf16_matrix((size_t)d * qd, 0.2);
            Wgu[n] = bf16_matrix((size_t)2 * 24 * d, 0.2); Wdown[n] = bf16_matrix((size_t)d * 24, 0.2);
            g1[n] = bf16_matrix(d, 0.1); g2[n] = bf16_matrix(d, 0.1);
            kc[n] = bf16_matrix((size_t)B * 4 * kvd, 1.0); vc[n] = bf16_matrix((size_t)B * 4 * kvd, 1.0);
        }
        int32_t plen[B] = {0, 3, 4};
        orc_tbody tb = {&t, (const uint16_t *const *)Wqkv, (const uint16_t *const *)Wo, (const uint16_t *const *)Wgu,
                        (const uint16_t *const *)Wdown, (const uint16_t *const *)g1, (const uint16_t *const *)g2,
                        (const uint16_t *const *)kc, (const uint16_t *const *)vc, plen};
        orc_cfg c = {d, V, B, L, K, 1e-6, 0.5, 1, 0, 1, 0.3, 1, 1, 0, 1, 0, 0};
        double *z = (double *)malloc(sizeof(double) * M * V), *hr = (double *)malloc(sizeof(double) * M * d);
        memcpy(z, z0, sizeof(double) * M * V); memcpy(hr, h0, sizeof(double) * M * d);
        int32_t tok[(K + 1) * M], cond[B] = {0, 0, 0}, prot[B], dpos[B * (K + 1)], dtok[B * (K + 1)], xtok[M];
        double conf[(K + 1) * M], lse[(K + 1) * M];
        uint8_t masked[M]; int8_t ra[M];
        orc_chain_step_tf(&c, E, W, (const uint16_t *const *)W1, (const uint16_t *const *)g, z, hr, tok, conf, lse, masked, ra,
                          cond, prot, dpos, dtok, NULL, NULL, NULL, xtok, &tb);
        for (int i = 0; i < M * V; ++i) bad |= !isfinite(z[i]);
        double xr[8] = {1, 2, 3, 4, 5, 6, 7, 8};
        orc_rope(xr, 8, 3.0, 100.0);
        free(z); free(hr);
        for (int n = 0; n < 4; ++n) { free(Wqkv[n]); free(Wo[n]); free(Wgu[n]); free(Wdown[n]); free(g1[n]); free(g2[n]); free(kc[n]); free(vc[n]); }
    }
    for (int k = 0; k < K; ++k) { free(W1[k]); free(W2[k]); free(g[k]); }
    free(E); free(W); free(z0); free(h0);
    printf(bad ? "sanitize_check: INCONSISTENT\n" : "sanitize_check: ok (%d threads)\n", orc_threads());
    return bad ? 1 : 0;
}
