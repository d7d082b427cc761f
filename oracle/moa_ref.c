/*
 * moa_ref.c -- CPU oracle (fp64) for the Mixture-of-Attentions draft step.
 *
 * TEST INFRASTRUCTURE ONLY: see moa_ref.h.  Every function is the plain
 * definition from the paper written out: dense score rows, two-pass softmax
 * (row max, exp, divide), no tiling, no fusion, no algebraic reordering.
 * OpenMP is used only across units the paper states to be independent
 * (tokens in LSA; (sequence, query, head) triples in CA / verification).
 *
 * Parity with the authors' own implementation is UNPINNED (the paper prints no
 * numeric example); the pins are the closed forms / invariants / brute force in
 * tests/test_oracle_*.py.
 */
#include "moa_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------ tree */

int moa_ref_tree_build(const int32_t *parent, int B, int M, uint64_t *mask, int32_t *depth)
{
    if (!parent || !mask || !depth || B < 1 || M < 1) return MOA_REF_BAD_ARG;
    const int W = (M + 63) / 64;
    for (int b = 0; b < B; ++b) {
        const int32_t *par = parent + (int64_t)b * M;
        if (par[0] != -1) return MOA_REF_BAD_TREE;
        for (int i = 1; i < M; ++i)
            if (par[i] < 0 || par[i] >= i) return MOA_REF_BAD_TREE;
    }
    for (int b = 0; b < B; ++b) {
        const int32_t *par = parent + (int64_t)b * M;
        uint64_t *mk = mask + (int64_t)b * M * W;
        int32_t *dp = depth + (int64_t)b * M;
        for (int i = 0; i < M; ++i) {
            uint64_t *row = mk + (int64_t)i * W;
            if (i == 0) {
                for (int w = 0; w < W; ++w) row[w] = 0;
                dp[0] = 0;
            } else {
                const uint64_t *prow = mk + (int64_t)par[i] * W;
                for (int w = 0; w < W; ++w) row[w] = prow[w];
                dp[i] = dp[par[i]] + 1;
            }
            row[i >> 6] |= (uint64_t)1 << (i & 63);
        }
    }
    return MOA_REF_OK;
}

/* ---------------------------------------------------------------- linear */

int moa_ref_linear(const double *x, int64_t R, int K, const double *w, int N, double *y)
{
    if (!x || !y || R < 0 || K < 1 || N < 1) return MOA_REF_BAD_ARG;
    if (!w) {
        if (N != K) return MOA_REF_BAD_ARG;
        memcpy(y, x, sizeof(double) * (size_t)R * (size_t)K);
        return MOA_REF_OK;
    }
    /* rows are independent; threads split them (no effect inside an outer parallel loop) */
#pragma omp parallel for schedule(static) if (R > 1)
    for (int64_t r = 0; r < R; ++r)
        for (int n = 0; n < N; ++n) {
            double acc = 0.0;
            for (int k = 0; k < K; ++k) acc += x[r * K + k] * w[(int64_t)n * K + k];
            y[r * N + n] = acc;
        }
    return MOA_REF_OK;
}

/* --------------------------------------------------------------- softmax */

/* o[dh] = sum_n softmax(scores)[n] * values[n, :]   (two-pass, dense). */
int moa_ref_softmax_weighted_sum(const double *scores, const double *values,
                                 int n, int dh, double *o, double *prob_sum)
{
    if (!scores || !values || !o || dh < 1) return MOA_REF_BAD_ARG;
    if (n < 1) return MOA_REF_EMPTY;
    double mx = scores[0];
    for (int i = 1; i < n; ++i) if (scores[i] > mx) mx = scores[i];
    double *p = (double *)malloc(sizeof(double) * (size_t)n);
    if (!p) return MOA_REF_BAD_ARG;
    double den = 0.0;
    for (int i = 0; i < n; ++i) { p[i] = exp(scores[i] - mx); den += p[i]; }
    double ps = 0.0;
    for (int i = 0; i < n; ++i) { p[i] /= den; ps += p[i]; }
    for (int c = 0; c < dh; ++c) {
        double acc = 0.0;
        for (int i = 0; i < n; ++i) acc += p[i] * values[(int64_t)i * dh + c];
        o[c] = acc;
    }
    if (prob_sum) *prob_sum = ps;
    free(p);
    return MOA_REF_OK;
}

/* Same quantity, accumulated chunk by chunk with a running max m, running
 * denominator l and un-normalised accumulator acc, rescaled whenever m grows. */
int moa_ref_softmax_weighted_sum_chunked(const double *scores, const double *values,
                                         int n, int dh, int chunk, double *o)
{
    if (!scores || !values || !o || dh < 1 || chunk < 1) return MOA_REF_BAD_ARG;
    if (n < 1) return MOA_REF_EMPTY;
    double m = -INFINITY, l = 0.0;
    for (int c = 0; c < dh; ++c) o[c] = 0.0;
    for (int s = 0; s < n; s += chunk) {
        int e = s + chunk < n ? s + chunk : n;
        double cm = scores[s];
        for (int i = s + 1; i < e; ++i) if (scores[i] > cm) cm = scores[i];
        double nm = cm > m ? cm : m;
        double scale = exp(m - nm);          /* exp(-inf) = 0 on the first chunk */
        l *= scale;
        for (int c = 0; c < dh; ++c) o[c] *= scale;
        for (int i = s; i < e; ++i) {
            double pi = exp(scores[i] - nm);
            l += pi;
            for (int c = 0; c < dh; ++c) o[c] += pi * values[(int64_t)i * dh + c];
        }
        m = nm;
    }
    for (int c = 0; c < dh; ++c) o[c] /= l;
    return MOA_REF_OK;
}

/* ------------------------------------------------------------------- LSA */

int moa_ref_lsa(const double *hs, int64_t T, int L, int d_in, int Hq, int Hkv, int dh,
                const double *wq, const double *wk, const double *wv, const double *wo,
                int d_out, double *out)
{
    if (!hs || !out || T < 0 || L < 1 || d_in < 1 || Hq < 1 || Hkv < 1 || dh < 1 || d_out < 1)
        return MOA_REF_BAD_ARG;
    if (Hq % Hkv) return MOA_REF_BAD_ARG;
    const int Eq = Hq * dh, Ekv = Hkv * dh, G = Hq / Hkv;
    if ((!wq && Eq != d_in) || (!wk && Ekv != d_in) || (!wv && Ekv != d_in) || (!wo && d_out != Eq))
        return MOA_REF_BAD_ARG;
    const double inv_sqrt = 1.0 / sqrt((double)dh);
    int bad = 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        const double *X = hs + t * (int64_t)L * d_in;
        double *Q = (double *)malloc(sizeof(double) * (size_t)L * Eq);
        double *K = (double *)malloc(sizeof(double) * (size_t)L * Ekv);
        double *V = (double *)malloc(sizeof(double) * (size_t)L * Ekv);
        double *A = (double *)malloc(sizeof(double) * (size_t)L * Eq);   /* concat of heads */
        double *Y = (double *)malloc(sizeof(double) * (size_t)L * d_out);
        double *s = (double *)malloc(sizeof(double) * (size_t)L);
        double *vg = (double *)malloc(sizeof(double) * (size_t)L * dh);
        double *oh = (double *)malloc(sizeof(double) * (size_t)dh);
        if (!Q || !K || !V || !A || !Y || !s || !vg || !oh) {
#pragma omp atomic write
            bad = 1;
        } else {
            moa_ref_linear(X, L, d_in, wq, Eq, Q);
            moa_ref_linear(X, L, d_in, wk, Ekv, K);
            moa_ref_linear(X, L, d_in, wv, Ekv, V);
            for (int h = 0; h < Hq; ++h) {
                const int g = h / G;
                for (int j = 0; j < L; ++j)
                    for (int c = 0; c < dh; ++c) vg[j * dh + c] = V[j * Ekv + g * dh + c];
                for (int i = 0; i < L; ++i) {           /* query = layer i */
                    for (int j = 0; j < L; ++j) {       /* key   = layer j, full mask */
                        double acc = 0.0;
                        for (int c = 0; c < dh; ++c)
                            acc += Q[i * Eq + h * dh + c] * K[j * Ekv + g * dh + c];
                        s[j] = acc * inv_sqrt;
                    }
                    moa_ref_softmax_weighted_sum(s, vg, L, dh, oh, NULL);
                    for (int c = 0; c < dh; ++c) A[i * Eq + h * dh + c] = oh[c];
                }
            }
            moa_ref_linear(A, L, Eq, wo, d_out, Y);
            for (int n = 0; n < d_out; ++n) {           /* mean aggregation over layers */
                double acc = 0.0;
                for (int i = 0; i < L; ++i) acc += Y[i * d_out + n];
                out[t * d_out + n] = acc / (double)L;
            }
        }
        free(Q); free(K); free(V); free(A); free(Y); free(s); free(vg); free(oh);
    }
    return bad ? MOA_REF_BAD_ARG : MOA_REF_OK;
}

/* ---------------------------------------------------------- CA kv append */

int moa_ref_ca_kv_append(const double *mem_new, int d_mem, const int32_t *tok_off, int B,
                         int Hkv, int dh, const double *wk, const double *wv,
                         double *kc, double *vc, int32_t *ca_len, int P_cap)
{
    if (!mem_new || !tok_off || !kc || !vc || !ca_len || B < 1 || Hkv < 1 || dh < 1 ||
        d_mem < 1 || P_cap < 1)
        return MOA_REF_BAD_ARG;
    const int Ekv = Hkv * dh;
    if ((!wk || !wv) && Ekv != d_mem) return MOA_REF_BAD_ARG;
    if (tok_off[0] != 0) return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        int nb = tok_off[b + 1] - tok_off[b];
        if (nb < 0 || ca_len[b] < 0) return MOA_REF_BAD_ARG;
        if (ca_len[b] + nb > P_cap) return MOA_REF_EMPTY;
    }
    double *kr = (double *)malloc(sizeof(double) * (size_t)Ekv);
    double *vr = (double *)malloc(sizeof(double) * (size_t)Ekv);
    if (!kr || !vr) { free(kr); free(vr); return MOA_REF_BAD_ARG; }
    for (int b = 0; b < B; ++b) {
        for (int r = tok_off[b]; r < tok_off[b + 1]; ++r) {
            const double *m = mem_new + (int64_t)r * d_mem;
            moa_ref_linear(m, 1, d_mem, wk, Ekv, kr);
            moa_ref_linear(m, 1, d_mem, wv, Ekv, vr);
            const int p = ca_len[b] + (r - tok_off[b]);
            for (int g = 0; g < Hkv; ++g)
                for (int c = 0; c < dh; ++c) {
                    int64_t o = (((int64_t)b * Hkv + g) * P_cap + p) * dh + c;
                    kc[o] = kr[g * dh + c];
                    vc[o] = vr[g * dh + c];
                }
        }
        ca_len[b] += tok_off[b + 1] - tok_off[b];
    }
    free(kr); free(vr);
    return MOA_REF_OK;
}

/* -------------------------------------------------------- cross-attention */

int moa_ref_cross_attn(const double *xq, int B, int Mq, int d, int H, int Hkv, int dh,
                       const double *wq, const double *wo, int d_out,
                       const double *kc, const double *vc, const int32_t *ca_len, int P_cap,
                       double *out)
{
    if (!xq || !kc || !vc || !ca_len || !out || B < 1 || Mq < 1 || d < 1 || H < 1 || Hkv < 1 ||
        dh < 1 || d_out < 1 || P_cap < 1)
        return MOA_REF_BAD_ARG;
    if (H % Hkv) return MOA_REF_BAD_ARG;
    const int E = H * dh, G = H / Hkv;
    if ((!wq && E != d) || (!wo && d_out != E)) return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        if (ca_len[b] < 0 || ca_len[b] > P_cap) return MOA_REF_BAD_ARG;
        if (ca_len[b] == 0) return MOA_REF_EMPTY;
    }
    const double inv_sqrt = 1.0 / sqrt((double)dh);
    const int64_t R = (int64_t)B * Mq;
    double *Q = (double *)malloc(sizeof(double) * (size_t)R * E);
    double *A = (double *)malloc(sizeof(double) * (size_t)R * E);
    if (!Q || !A) { free(Q); free(A); return MOA_REF_BAD_ARG; }
    moa_ref_linear(xq, R, d, wq, E, Q);

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rh = 0; rh < R * H; ++rh) {
        const int64_t r = rh / H;
        const int h = (int)(rh % H), g = h / G, b = (int)(r / Mq);
        const int n = ca_len[b];
        const double *Kg = kc + ((int64_t)b * Hkv + g) * P_cap * dh;
        const double *Vg = vc + ((int64_t)b * Hkv + g) * P_cap * dh;
        const double *q = Q + r * E + h * dh;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        for (int p = 0; p < n; ++p) {                 /* every cached row, no mask */
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * Kg[(int64_t)p * dh + c];
            s[p] = acc * inv_sqrt;
        }
        moa_ref_softmax_weighted_sum(s, Vg, n, dh, A + r * E + h * dh, NULL);
        free(s);
    }
    moa_ref_linear(A, R, E, wo, d_out, out);
    free(Q); free(A);
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ draft self-attention */

int moa_ref_self_attn_draft(const double *emb, int B, int M, int node0, int Mn, int d, int H, int Hkv, int dh,
                            const double *wq, const double *wk, const double *wv,
                            const double *wo, int d_out,
                            const double *kcache, const double *vcache,
                            const int32_t *prefix_len, int P_cap, const int32_t *parent,
                            double *out, double *k_draft, double *v_draft)
{
    if (!emb || !prefix_len || !parent || !out || !k_draft || !v_draft || B < 1 || M < 1 || Mn < 1 ||
        M > 4096 || node0 < 0 || node0 + Mn > M || d < 1 || H < 1 || Hkv < 1 || dh < 1 || d_out < 1 || P_cap < 0)
        return MOA_REF_BAD_ARG;
    if (H % Hkv) return MOA_REF_BAD_ARG;
    const int E = H * dh, Ekv = Hkv * dh, G = H / Hkv;
    if ((!wq && E != d) || (!wk && Ekv != d) || (!wv && Ekv != d) || (!wo && d_out != E))
        return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        if (prefix_len[b] < 0 || prefix_len[b] > P_cap) return MOA_REF_BAD_ARG;
        if (prefix_len[b] > 0 && (!kcache || !vcache)) return MOA_REF_BAD_ARG;
        if (parent[(int64_t)b * M] != -1) return MOA_REF_BAD_TREE;
        for (int i = 1; i < M; ++i)
            if (parent[(int64_t)b * M + i] < 0 || parent[(int64_t)b * M + i] >= i) return MOA_REF_BAD_TREE;
    }
    const double inv_sqrt = 1.0 / sqrt((double)dh);
    const int64_t R = (int64_t)B * Mn;
    double *Q = (double *)malloc(sizeof(double) * (size_t)R * E);
    double *Kn = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *Vn = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *A = (double *)malloc(sizeof(double) * (size_t)R * E);
    if (!Q || !Kn || !Vn || !A) { free(Q); free(Kn); free(Vn); free(A); return MOA_REF_BAD_ARG; }
    moa_ref_linear(emb, R, d, wq, E, Q);
    moa_ref_linear(emb, R, d, wk, Ekv, Kn);
    moa_ref_linear(emb, R, d, wv, Ekv, Vn);

    /* the new nodes' keys / values join the draft cache of this cycle */
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g)
            for (int t = 0; t < Mn; ++t)
                for (int c = 0; c < dh; ++c) {
                    const int64_t o = (((int64_t)b * Hkv + g) * M + node0 + t) * dh + c;
                    k_draft[o] = Kn[((int64_t)b * Mn + t) * Ekv + g * dh + c];
                    v_draft[o] = Vn[((int64_t)b * Mn + t) * Ekv + g * dh + c];
                }

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rh = 0; rh < R * H; ++rh) {
        const int64_t r = rh / H;
        const int h = (int)(rh % H), g = h / G, b = (int)(r / Mn), i = node0 + (int)(r % Mn);
        const int P = prefix_len[b];
        const double *q = Q + r * E + h * dh;
        /* the drafted tokens before node i in its own sequence: i, parent(i), ..., root */
        int path[4096];
        int np = 0;
        for (int j = i; j >= 0 && np < 4096; j = parent[(int64_t)b * M + j]) path[np++] = j;
        const int n = P + np;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        double *vv = (double *)malloc(sizeof(double) * (size_t)n * dh);
        for (int p = 0; p < P; ++p) {
            const double *kr = kcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            const double *vr = vcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[p] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)p * dh + c] = vr[c];
        }
        for (int u = 0; u < np; ++u) {                /* root first, node i last: sequence order */
            const int j = path[np - 1 - u];
            const double *kr = k_draft + (((int64_t)b * Hkv + g) * M + j) * dh;
            const double *vr = v_draft + (((int64_t)b * Hkv + g) * M + j) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[P + u] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)(P + u) * dh + c] = vr[c];
        }
        moa_ref_softmax_weighted_sum(s, vv, n, dh, A + r * E + h * dh, NULL);
        free(s); free(vv);
    }
    moa_ref_linear(A, R, E, wo, d_out, out);
    free(Q); free(Kn); free(Vn); free(A);
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ reused decoder layer (TLI) */

void moa_ref_rope(double *v, int dh, double pos, double theta)
{
    const int half = dh / 2;
    for (int c = 0; c < half; ++c) {
        const double ang = pos * pow(theta, -2.0 * (double)c / (double)dh);
        const double cs = cos(ang), sn = sin(ang);
        const double a = v[c], b = v[c + half];
        v[c] = a * cs - b * sn;
        v[c + half] = b * cs + a * sn;
    }
}

static void ref_rmsnorm(const double *x, int64_t R, int d, const double *g, double eps, double *y)
{
    for (int64_t r = 0; r < R; ++r) {
        double ss = 0.0;
        for (int c = 0; c < d; ++c) ss += x[r * d + c] * x[r * d + c];
        const double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (int c = 0; c < d; ++c) y[r * d + c] = x[r * d + c] * inv * g[c];
    }
}

int moa_ref_rmsnorm(const double *x, int64_t R, int d, const double *g, double eps, double *out)
{
    if (!x || !g || !out || R < 0 || d < 1 || !(eps >= 0.0)) return MOA_REF_BAD_ARG;
    ref_rmsnorm(x, R, d, g, eps, out);
    return MOA_REF_OK;
}

int moa_ref_mlp_block(const double *x, const double *res, int64_t R, int d, int d_ff, const double *g,
                      const double *w_gate, const double *w_up, const double *w_down, double eps, double *out)
{
    if (!x || !g || !w_gate || !w_up || !w_down || !out || R < 0 || d < 1 || d_ff < 1 || !(eps >= 0.0))
        return MOA_REF_BAD_ARG;
    if (R == 0) return MOA_REF_OK;
    double *h = (double *)malloc(sizeof(double) * (size_t)R * d);
    double *n = (double *)malloc(sizeof(double) * (size_t)R * d);
    double *gt = (double *)malloc(sizeof(double) * (size_t)R * d_ff);
    double *up = (double *)malloc(sizeof(double) * (size_t)R * d_ff);
    if (!h || !n || !gt || !up) { free(h); free(n); free(gt); free(up); return MOA_REF_BAD_ARG; }
    for (int64_t e = 0; e < R * d; ++e) h[e] = x[e] + (res ? res[e] : 0.0);     /* the stream the block sits on */
    ref_rmsnorm(h, R, d, g, eps, n);
    moa_ref_linear(n, R, d, w_gate, d_ff, gt);
    moa_ref_linear(n, R, d, w_up, d_ff, up);
    for (int64_t e = 0; e < R * d_ff; ++e) gt[e] = gt[e] / (1.0 + exp(-gt[e])) * up[e];   /* silu(gate) * up */
    moa_ref_linear(gt, R, d_ff, w_down, d, out);
    for (int64_t e = 0; e < R * d; ++e) out[e] += h[e];
    free(h); free(n); free(gt); free(up);
    return MOA_REF_OK;
}

int moa_ref_tli_decoder_layer(const double *x, int B, int M, int node0, int Mn, int d, int H, int Hkv, int dh,
                              int d_ff, double rms_eps, double rope_theta,
                              const double *g_attn, const double *wq, const double *wk, const double *wv,
                              const double *wo, const double *g_mlp, const double *w_gate, const double *w_up,
                              const double *w_down, const double *kcache, const double *vcache,
                              const int32_t *prefix_len, int P_cap, const int32_t *parent,
                              double *out, double *k_draft, double *v_draft)
{
    if (!x || !g_attn || !wq || !wk || !wv || !wo || !g_mlp || !w_gate || !w_up || !w_down || !prefix_len ||
        !parent || !out || !k_draft || !v_draft)
        return MOA_REF_BAD_ARG;
    if (B < 1 || M < 1 || M > 4096 || Mn < 1 || node0 < 0 || node0 + Mn > M || d < 1 || H < 1 || Hkv < 1 ||
        dh < 2 || (dh & 1) || d_ff < 1 || P_cap < 0 || H % Hkv || !(rms_eps >= 0.0) || !(rope_theta > 0.0))
        return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        if (prefix_len[b] < 0 || prefix_len[b] > P_cap) return MOA_REF_BAD_ARG;
        if (prefix_len[b] > 0 && (!kcache || !vcache)) return MOA_REF_BAD_ARG;
        if (parent[(int64_t)b * M] != -1) return MOA_REF_BAD_TREE;
        for (int i = 1; i < M; ++i)
            if (parent[(int64_t)b * M + i] < 0 || parent[(int64_t)b * M + i] >= i) return MOA_REF_BAD_TREE;
    }
    const int E = H * dh, Ekv = Hkv * dh, G = H / Hkv;
    const double inv_sqrt = 1.0 / sqrt((double)dh);
    const int64_t R = (int64_t)B * Mn;
    double *n1 = (double *)malloc(sizeof(double) * (size_t)R * d);
    double *Q = (double *)malloc(sizeof(double) * (size_t)R * E);
    double *Kn = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *Vn = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *A = (double *)malloc(sizeof(double) * (size_t)R * E);
    double *h1 = (double *)malloc(sizeof(double) * (size_t)R * d);
    double *gt = (double *)malloc(sizeof(double) * (size_t)R * d_ff);
    double *up = (double *)malloc(sizeof(double) * (size_t)R * d_ff);
    if (!n1 || !Q || !Kn || !Vn || !A || !h1 || !gt || !up) {
        free(n1); free(Q); free(Kn); free(Vn); free(A); free(h1); free(gt); free(up);
        return MOA_REF_BAD_ARG;
    }
    ref_rmsnorm(x, R, d, g_attn, rms_eps, n1);
    moa_ref_linear(n1, R, d, wq, E, Q);
    moa_ref_linear(n1, R, d, wk, Ekv, Kn);
    moa_ref_linear(n1, R, d, wv, Ekv, Vn);

    /* positions: a node sits depth(node) tokens after the verified prefix */
    for (int64_t r = 0; r < R; ++r) {
        const int b = (int)(r / Mn), i = node0 + (int)(r % Mn);
        int depth = 0;
        for (int j = parent[(int64_t)b * M + i]; j >= 0; j = parent[(int64_t)b * M + j]) ++depth;
        const double pos = (double)prefix_len[b] + (double)depth;
        for (int h = 0; h < H; ++h) moa_ref_rope(Q + r * E + h * dh, dh, pos, rope_theta);
        for (int g = 0; g < Hkv; ++g) moa_ref_rope(Kn + r * Ekv + g * dh, dh, pos, rope_theta);
    }
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g)
            for (int t = 0; t < Mn; ++t)
                for (int c = 0; c < dh; ++c) {
                    const int64_t o = (((int64_t)b * Hkv + g) * M + node0 + t) * dh + c;
                    k_draft[o] = Kn[((int64_t)b * Mn + t) * Ekv + g * dh + c];
                    v_draft[o] = Vn[((int64_t)b * Mn + t) * Ekv + g * dh + c];
                }

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rh = 0; rh < R * H; ++rh) {
        const int64_t r = rh / H;
        const int h = (int)(rh % H), g = h / G, b = (int)(r / Mn), i = node0 + (int)(r % Mn);
        const int P = prefix_len[b];
        const double *q = Q + r * E + h * dh;
        int path[4096];
        int np = 0;
        for (int j = i; j >= 0 && np < 4096; j = parent[(int64_t)b * M + j]) path[np++] = j;
        const int n = P + np;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        double *vv = (double *)malloc(sizeof(double) * (size_t)n * dh);
        for (int p = 0; p < P; ++p) {
            const double *kr = kcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            const double *vr = vcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[p] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)p * dh + c] = vr[c];
        }
        for (int u = 0; u < np; ++u) {
            const int j = path[np - 1 - u];
            const double *kr = k_draft + (((int64_t)b * Hkv + g) * M + j) * dh;
            const double *vr = v_draft + (((int64_t)b * Hkv + g) * M + j) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[P + u] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)(P + u) * dh + c] = vr[c];
        }
        moa_ref_softmax_weighted_sum(s, vv, n, dh, A + r * E + h * dh, NULL);
        free(s); free(vv);
    }
    moa_ref_linear(A, R, E, wo, d, h1);
    for (int64_t e = 0; e < R * d; ++e) h1[e] += x[e];                     /* first residual */

    ref_rmsnorm(h1, R, d, g_mlp, rms_eps, n1);
    moa_ref_linear(n1, R, d, w_gate, d_ff, gt);
    moa_ref_linear(n1, R, d, w_up, d_ff, up);
    for (int64_t e = 0; e < R * d_ff; ++e) gt[e] = gt[e] / (1.0 + exp(-gt[e])) * up[e];   /* silu(gate) * up */
    moa_ref_linear(gt, R, d_ff, w_down, d, out);
    for (int64_t e = 0; e < R * d; ++e) out[e] += h1[e];                  /* second residual */
    free(n1); free(Q); free(Kn); free(Vn); free(A); free(h1); free(gt); free(up);
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ draft-tree construction */

/* a ranks before b: larger joint log-probability, then lower index */
static int cand_before(const float *lp, int a, int b)
{
    if (lp[a] != lp[b]) return lp[a] > lp[b];
    return a < b;
}

int moa_ref_tree_expand_level(int level, int Bw, const float *child_logp, const int32_t *child_tok,
                              float *cand_logp, int32_t *cand_tok, int32_t *cand_parent, int32_t *frontier)
{
    if (level < 1 || Bw < 1 || !child_logp || !child_tok || !cand_logp || !cand_tok || !cand_parent || !frontier)
        return MOA_REF_BAD_ARG;
    const int F = level == 1 ? 1 : Bw;
    const int base = level == 1 ? 0 : Bw + (level - 2) * Bw * Bw;
    const int n = F * Bw;
    for (int f = 0; f < F; ++f)
        for (int j = 0; j < Bw; ++j) {
            const int c = base + f * Bw + j;
            float lp = child_logp[f * Bw + j];
            if (!(lp == lp)) lp = -INFINITY;                     /* NaN counts as impossible */
            if (lp > 0.0f) lp = 0.0f;
            if (level == 1) {
                cand_logp[c] = lp;
                cand_parent[c] = -1;
            } else {
                cand_logp[c] = cand_logp[frontier[f]] + lp;      /* one single-precision addition */
                cand_parent[c] = frontier[f];
            }
            cand_tok[c] = child_tok[f * Bw + j];
        }
    /* the Bw best of this level's expansions, best first (all of them at level 1) */
    int32_t *next = (int32_t *)malloc(sizeof(int32_t) * (size_t)Bw);
    if (!next) return MOA_REF_BAD_ARG;
    const int keep = n < Bw ? n : Bw;
    for (int r = 0; r < keep; ++r) {
        int best = -1;
        for (int c = base; c < base + n; ++c) {
            int taken = 0;
            for (int q = 0; q < r; ++q) if (next[q] == c) taken = 1;
            if (taken) continue;
            if (best < 0 || cand_before(cand_logp, c, best)) best = c;
        }
        next[r] = best;
    }
    for (int r = 0; r < keep; ++r) frontier[r] = next[r];
    free(next);
    return MOA_REF_OK;
}

int moa_ref_tree_finalize(int n_cand, int m, int32_t root_tok, const float *cand_logp, const int32_t *cand_tok,
                          const int32_t *cand_parent, int32_t *parent, int32_t *tok, int32_t *node_cand,
                          int32_t *M_out)
{
    if (n_cand < 0 || m < 0 || !parent || !tok || !node_cand || !M_out) return MOA_REF_BAD_ARG;
    if (n_cand > 0 && (!cand_logp || !cand_tok || !cand_parent)) return MOA_REF_BAD_ARG;
    const int keep = m < n_cand ? m : n_cand;
    /* rank of every candidate = how many rank before it */
    int32_t *node_of = (int32_t *)malloc(sizeof(int32_t) * (size_t)(n_cand > 0 ? n_cand : 1));
    if (!node_of) return MOA_REF_BAD_ARG;
    int M = 1;
    parent[0] = -1;
    tok[0] = root_tok;
    node_cand[0] = -1;
    for (int c = 0; c < n_cand; ++c) {
        int rank = 0;
        for (int u = 0; u < n_cand; ++u) if (u != c && cand_before(cand_logp, u, c)) ++rank;
        node_of[c] = -1;
        if (rank < keep) {                            /* kept; candidate order is node order */
            const int p = cand_parent[c];
            if (p >= c || (p >= 0 && node_of[p] < 0)) { free(node_of); return MOA_REF_BAD_TREE; }
            node_of[c] = M;
            parent[M] = p < 0 ? 0 : node_of[p];
            tok[M] = cand_tok[c];
            node_cand[M] = c;
            ++M;
        }
    }
    *M_out = M;
    free(node_of);
    return MOA_REF_OK;
}

int moa_ref_topk_logprob(const double *logits, int F, int V, int Bw, int32_t *tok, double *logp)
{
    if (!logits || !tok || !logp || F < 1 || V < 1 || Bw < 1 || Bw > V) return MOA_REF_BAD_ARG;
    for (int f = 0; f < F; ++f) {
        const double *row = logits + (int64_t)f * V;
        double mx = row[0];
        for (int v = 1; v < V; ++v) if (row[v] > mx) mx = row[v];
        double den = 0.0;
        for (int v = 0; v < V; ++v) den += exp(row[v] - mx);
        const double lse = mx + log(den);
        for (int r = 0; r < Bw; ++r) {
            int best = -1;
            for (int v = 0; v < V; ++v) {
                int taken = 0;
                for (int q = 0; q < r; ++q) if (tok[f * Bw + q] == v) taken = 1;
                if (taken) continue;
                if (best < 0 || row[v] > row[best]) best = v;      /* strict: the lower id wins a tie */
            }
            tok[f * Bw + r] = best;
            logp[f * Bw + r] = row[best] - lse;
        }
    }
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ LM head, greedy token */

int moa_ref_lm_head_argmax(const double *x, int R, int d, const double *w, int V, int32_t *tgt, double *best)
{
    if (!x || !w || !tgt || R < 1 || d < 1 || V < 1) return MOA_REF_BAD_ARG;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < R; ++r) {
        int arg = 0;
        double top = 0.0;
        for (int v = 0; v < V; ++v) {
            double acc = 0.0;
            for (int k = 0; k < d; ++k) acc += x[(int64_t)r * d + k] * w[(int64_t)v * d + k];
            if (v == 0 || acc > top) { top = acc; arg = v; }        /* strict: the lower id wins a tie */
        }
        tgt[r] = arg;
        if (best) best[r] = top;
    }
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ client-server messages */

int moa_ref_msg_pack_tree(const int32_t *tok, const int32_t *parent, int B, int M, uint8_t *msg)
{
    if (!tok || !parent || !msg || B < 1 || M < 1 || M > 256) return MOA_REF_BAD_ARG;
    for (int64_t i = 0; i < (int64_t)B * M; ++i) {
        const int32_t t = tok[i], p = parent[i];
        if (t < 0 || t >= (1 << 24) || p < -1 || p >= 255) return MOA_REF_BAD_ARG;
        msg[4 * i + 0] = (uint8_t)(t & 0xff);
        msg[4 * i + 1] = (uint8_t)((t >> 8) & 0xff);
        msg[4 * i + 2] = (uint8_t)((t >> 16) & 0xff);
        msg[4 * i + 3] = p < 0 ? 0xff : (uint8_t)p;
    }
    return MOA_REF_OK;
}

int moa_ref_msg_unpack_tree(const uint8_t *msg, int B, int M, int32_t *tok, int32_t *parent)
{
    if (!tok || !parent || !msg || B < 1 || M < 1 || M > 256) return MOA_REF_BAD_ARG;
    for (int64_t i = 0; i < (int64_t)B * M; ++i) {
        tok[i] = (int32_t)msg[4 * i] | ((int32_t)msg[4 * i + 1] << 8) | ((int32_t)msg[4 * i + 2] << 16);
        parent[i] = msg[4 * i + 3] == 0xff ? -1 : (int32_t)msg[4 * i + 3];
    }
    return MOA_REF_OK;
}

int moa_ref_msg_pack_accept(const int32_t *tok, const float *x, int A, int n_vec, int n, uint8_t *msg)
{
    if (!tok || !x || !msg || A < 0 || n_vec < 0 || n < 1) return MOA_REF_BAD_ARG;
    const int64_t per = 3 + (int64_t)n_vec * (4 + n);
    for (int a = 0; a < A; ++a) {
        uint8_t *m = msg + a * per;
        const int32_t t = tok[a];
        if (t < 0 || t >= (1 << 24)) return MOA_REF_BAD_ARG;
        m[0] = (uint8_t)(t & 0xff); m[1] = (uint8_t)((t >> 8) & 0xff); m[2] = (uint8_t)((t >> 16) & 0xff);
        for (int v = 0; v < n_vec; ++v) {
            const float *xv = x + ((int64_t)a * n_vec + v) * n;
            uint8_t *mv = m + 3 + (int64_t)v * (4 + n);
            float amax = 0.0f;
            for (int c = 0; c < n; ++c) { const float ab = fabsf(xv[c]); if (ab > amax) amax = ab; }
            const float scale = amax / 127.0f;
            memcpy(mv, &scale, 4);
            for (int c = 0; c < n; ++c) {
                float q = scale > 0.0f ? rintf(xv[c] / scale) : 0.0f;
                if (q > 127.0f) q = 127.0f;
                if (q < -127.0f) q = -127.0f;
                mv[4 + c] = (uint8_t)(int8_t)q;
            }
        }
    }
    return MOA_REF_OK;
}

int moa_ref_msg_unpack_accept(const uint8_t *msg, int A, int n_vec, int n, int32_t *tok, float *x)
{
    if (!tok || !x || !msg || A < 0 || n_vec < 0 || n < 1) return MOA_REF_BAD_ARG;
    const int64_t per = 3 + (int64_t)n_vec * (4 + n);
    for (int a = 0; a < A; ++a) {
        const uint8_t *m = msg + a * per;
        tok[a] = (int32_t)m[0] | ((int32_t)m[1] << 8) | ((int32_t)m[2] << 16);
        for (int v = 0; v < n_vec; ++v) {
            const uint8_t *mv = m + 3 + (int64_t)v * (4 + n);
            float scale;
            memcpy(&scale, mv, 4);
            float *xv = x + ((int64_t)a * n_vec + v) * n;
            for (int c = 0; c < n; ++c) xv[c] = (float)(int8_t)mv[4 + c] * scale;
        }
    }
    return MOA_REF_OK;
}

/* ------------------------------------------------------------ tree verify */

int moa_ref_tree_verify_attn(const double *x, int B, int M, int d, int H, int Hkv, int dh,
                             const double *wq, const double *wk, const double *wv,
                             const double *wo, int d_out,
                             const double *kcache, const double *vcache,
                             const int32_t *prefix_len, int P_cap, const uint64_t *mask,
                             double *out, double *k_tree, double *v_tree)
{
    if (!x || !prefix_len || !mask || !out || !k_tree || !v_tree || B < 1 || M < 1 || d < 1 ||
        H < 1 || Hkv < 1 || dh < 1 || d_out < 1 || P_cap < 0)
        return MOA_REF_BAD_ARG;
    if (H % Hkv) return MOA_REF_BAD_ARG;
    const int E = H * dh, Ekv = Hkv * dh, G = H / Hkv, W = (M + 63) / 64;
    if ((!wq && E != d) || (!wk && Ekv != d) || (!wv && Ekv != d) || (!wo && d_out != E))
        return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        if (prefix_len[b] < 0 || prefix_len[b] > P_cap) return MOA_REF_BAD_ARG;
        if (prefix_len[b] > 0 && (!kcache || !vcache)) return MOA_REF_BAD_ARG;
    }
    const double inv_sqrt = 1.0 / sqrt((double)dh);
    const int64_t R = (int64_t)B * M;
    double *Q = (double *)malloc(sizeof(double) * (size_t)R * E);
    double *Kt = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *Vt = (double *)malloc(sizeof(double) * (size_t)R * Ekv);
    double *A = (double *)malloc(sizeof(double) * (size_t)R * E);
    if (!Q || !Kt || !Vt || !A) { free(Q); free(Kt); free(Vt); free(A); return MOA_REF_BAD_ARG; }
    moa_ref_linear(x, R, d, wq, E, Q);
    moa_ref_linear(x, R, d, wk, Ekv, Kt);
    moa_ref_linear(x, R, d, wv, Ekv, Vt);

    /* tree rows' own keys / values, laid out like one more slab of the cache */
    for (int b = 0; b < B; ++b)
        for (int g = 0; g < Hkv; ++g)
            for (int j = 0; j < M; ++j)
                for (int c = 0; c < dh; ++c) {
                    int64_t o = (((int64_t)b * Hkv + g) * M + j) * dh + c;
                    k_tree[o] = Kt[((int64_t)b * M + j) * Ekv + g * dh + c];
                    v_tree[o] = Vt[((int64_t)b * M + j) * Ekv + g * dh + c];
                }

    int empty = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t rh = 0; rh < R * H; ++rh) {
        const int64_t r = rh / H;
        const int h = (int)(rh % H), g = h / G, b = (int)(r / M), i = (int)(r % M);
        const int P = prefix_len[b];
        const uint64_t *mrow = mask + ((int64_t)b * M + i) * W;
        const double *q = Q + r * E + h * dh;
        /* gather the visible key set: prefix rows, then visible tree rows */
        double *s = (double *)malloc(sizeof(double) * (size_t)(P + M));
        double *vv = (double *)malloc(sizeof(double) * (size_t)(P + M) * dh);
        int n = 0;
        for (int p = 0; p < P; ++p) {
            const double *kr = kcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            const double *vr = vcache + (((int64_t)b * Hkv + g) * P_cap + p) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[n] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)n * dh + c] = vr[c];
            ++n;
        }
        for (int j = 0; j < M; ++j) {
            if (!((mrow[j >> 6] >> (j & 63)) & 1)) continue;
            const double *kr = k_tree + (((int64_t)b * Hkv + g) * M + j) * dh;
            const double *vr = v_tree + (((int64_t)b * Hkv + g) * M + j) * dh;
            double acc = 0.0;
            for (int c = 0; c < dh; ++c) acc += q[c] * kr[c];
            s[n] = acc * inv_sqrt;
            for (int c = 0; c < dh; ++c) vv[(int64_t)n * dh + c] = vr[c];
            ++n;
        }
        if (n == 0) {
#pragma omp atomic write
            empty = 1;
        } else {
            moa_ref_softmax_weighted_sum(s, vv, n, dh, A + r * E + h * dh, NULL);
        }
        free(s); free(vv);
    }
    int rc = MOA_REF_OK;
    if (empty) rc = MOA_REF_EMPTY;
    else moa_ref_linear(A, R, E, wo, d_out, out);
    free(Q); free(Kt); free(Vt); free(A);
    return rc;
}

/* ----------------------------------------------------------------- accept */

int moa_ref_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt,
                        int B, int M, int32_t *path, int32_t *n_path, int32_t *bonus)
{
    if (!parent || !tok || !tgt || !path || !n_path || !bonus || B < 1 || M < 1)
        return MOA_REF_BAD_ARG;
    for (int b = 0; b < B; ++b) {
        const int32_t *par = parent + (int64_t)b * M;
        if (par[0] != -1) return MOA_REF_BAD_TREE;
        for (int i = 1; i < M; ++i)
            if (par[i] < 0 || par[i] >= i) return MOA_REF_BAD_TREE;
    }
    for (int b = 0; b < B; ++b) {
        const int32_t *par = parent + (int64_t)b * M;
        const int32_t *tk = tok + (int64_t)b * M;
        const int32_t *tg = tgt + (int64_t)b * M;
        int32_t *pt = path + (int64_t)b * M;
        for (int i = 0; i < M; ++i) pt[i] = -1;
        int cur = 0, n = 0;
        pt[n++] = 0;
        for (;;) {
            int next = -1;
            for (int c = cur + 1; c < M; ++c)
                if (par[c] == cur && tk[c] == tg[cur]) { next = c; break; }
            if (next < 0) break;
            cur = next;
            pt[n++] = cur;
        }
        n_path[b] = n;
        bonus[b] = tg[cur];
    }
    return MOA_REF_OK;
}
