/*
 * sanitize_driver.c -- runs every function of the CPU oracle once on small, exactly sized heap buffers.
 *
 * TEST INFRASTRUCTURE ONLY.  Built together with moa_ref.c under -fsanitize=address,undefined (a CPU test
 * does that and runs the result): an access past a buffer, a misaligned access, a signed overflow or a bad shift
 * anywhere in the oracle aborts the run.  It checks no values beyond a few invariants that fall out for free;
 * the oracle's arithmetic is pinned by the Python tests.  Shapes are ragged on purpose (odd head_dim, M not a
 * multiple of 64, empty token ranges, one-node trees).
 */
#include "moa_ref.h"

#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

static uint64_t g_state = 0x9E3779B97F4A7C15ull;

static double rnd(void)      /* uniform in (-1, 1), a 64-bit LCG: only needs to be deterministic */
{
    g_state = g_state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)((g_state >> 11) & ((1ull << 52) - 1)) / (double)(1ull << 51) - 1.0;
}

static double *buf(size_t n)
{
    double *p = (double *)malloc(sizeof(double) * (n ? n : 1));
    if (!p) { fprintf(stderr, "out of memory\n"); exit(2); }
    for (size_t i = 0; i < n; ++i) p[i] = rnd();
    return p;
}

static int32_t *random_tree(int B, int M)
{
    int32_t *parent = (int32_t *)calloc((size_t)B * M, sizeof(int32_t));
    for (int b = 0; b < B; ++b) {
        parent[b * M] = -1;
        for (int i = 1; i < M; ++i) parent[b * M + i] = (int32_t)((rnd() * 0.5 + 0.5) * i) % i;
    }
    return parent;
}

#define CHECK(call)                                                              \
    do {                                                                         \
        int rc_ = (call);                                                        \
        if (rc_ != MOA_REF_OK) { fprintf(stderr, "%s -> %d\n", #call, rc_); return 1; } \
    } while (0)

static int attention_group(int B, int M, int d, int H, int Hkv, int dh, int P_cap)
{
    const int E = H * dh, Ekv = Hkv * dh, W = (M + 63) / 64;
    int32_t *parent = random_tree(B, M);
    uint64_t *mask = (uint64_t *)malloc(sizeof(uint64_t) * (size_t)B * M * W);
    int32_t *depth = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M);
    CHECK(moa_ref_tree_build(parent, B, M, mask, depth));
    int32_t *len = (int32_t *)malloc(sizeof(int32_t) * B);
    for (int b = 0; b < B; ++b) len[b] = 1 + (int32_t)((rnd() * 0.5 + 0.5) * (P_cap - 1));
    len[0] = P_cap;                                   /* a full cache */
    double *x = buf((size_t)B * M * d), *wq = buf((size_t)E * d), *wk = buf((size_t)Ekv * d), *wv = buf((size_t)Ekv * d);
    double *wo = buf((size_t)d * E), *kc = buf((size_t)B * Hkv * P_cap * dh), *vc = buf((size_t)B * Hkv * P_cap * dh);
    double *out = buf((size_t)B * M * d), *kt = buf((size_t)B * Hkv * M * dh), *vt = buf((size_t)B * Hkv * M * dh);
    CHECK(moa_ref_cross_attn(x, B, M, d, H, Hkv, dh, wq, wo, d, kc, vc, len, P_cap, out));
    CHECK(moa_ref_tree_verify_attn(x, B, M, d, H, Hkv, dh, wq, wk, wv, wo, d, kc, vc, len, P_cap, mask, out, kt, vt));
    len[B - 1] = 0;                                   /* an empty prefix is valid for the tree forms */
    CHECK(moa_ref_tree_verify_attn(x, B, M, d, H, Hkv, dh, wq, wk, wv, wo, d, kc, vc, len, P_cap, mask, out, kt, vt));
    /* level by level: nodes [0, M/2) then [M/2, M) */
    const int half = M / 2 > 0 ? M / 2 : M;
    CHECK(moa_ref_self_attn_draft(x, B, M, 0, half, d, H, Hkv, dh, wq, wk, wv, wo, d, kc, vc, len, P_cap, parent, out, kt, vt));
    if (M - half > 0)
        CHECK(moa_ref_self_attn_draft(x, B, M, half, M - half, d, H, Hkv, dh, wq, wk, wv, wo, d, kc, vc, len, P_cap, parent, out, kt, vt));
    if (dh % 2 == 0) {
        const int dff = 3 * d / 2 + 1;
        double *g1 = buf(d), *g2 = buf(d), *wg = buf((size_t)dff * d), *wu = buf((size_t)dff * d), *wd = buf((size_t)d * dff);
        double *wo2 = buf((size_t)d * E);
        CHECK(moa_ref_tli_decoder_layer(x, B, M, 0, M, d, H, Hkv, dh, dff, 1e-5, 5e5, g1, wq, wk, wv, wo2, g2, wg, wu, wd,
                                        kc, vc, len, P_cap, parent, out, kt, vt));
        CHECK(moa_ref_mlp_block(x, out, (int64_t)B * M, d, dff, g1, wg, wu, wd, 1e-5, out));
        CHECK(moa_ref_mlp_block(x, NULL, (int64_t)B * M, d, dff, g1, wg, wu, wd, 0.0, out));
        CHECK(moa_ref_rmsnorm(x, (int64_t)B * M, d, g1, 1e-5, out));
        moa_ref_rope(x, dh, 12345.0, 5e5);
        free(g1); free(g2); free(wg); free(wu); free(wd); free(wo2);
    }
    /* accept walk and the tree message on the same trees */
    int32_t *tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M), *tgt = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M);
    for (int i = 0; i < B * M; ++i) { tok[i] = (int32_t)((rnd() * 0.5 + 0.5) * 16777215.0); tgt[i] = tok[(i + 1) % (B * M)]; }
    int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M), *np = (int32_t *)malloc(sizeof(int32_t) * B);
    int32_t *bonus = (int32_t *)malloc(sizeof(int32_t) * B);
    CHECK(moa_ref_tree_accept(parent, tok, tgt, B, M, path, np, bonus));
    for (int b = 0; b < B; ++b)
        if (np[b] < 1 || np[b] > M || path[b * M] != 0) { fprintf(stderr, "accept path\n"); return 1; }
    if (M <= 255) {
        uint8_t *msg = (uint8_t *)malloc((size_t)B * 4 * M);
        int32_t *tok2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M), *par2 = (int32_t *)malloc(sizeof(int32_t) * (size_t)B * M);
        CHECK(moa_ref_msg_pack_tree(tok, parent, B, M, msg));
        CHECK(moa_ref_msg_unpack_tree(msg, B, M, tok2, par2));
        if (memcmp(tok, tok2, sizeof(int32_t) * (size_t)B * M) || memcmp(parent, par2, sizeof(int32_t) * (size_t)B * M)) {
            fprintf(stderr, "tree message round trip\n");
            return 1;
        }
        free(msg); free(tok2); free(par2);
    }
    free(parent); free(mask); free(depth); free(len); free(x); free(wq); free(wk); free(wv); free(wo); free(kc); free(vc);
    free(out); free(kt); free(vt); free(tok); free(tgt); free(path); free(np); free(bonus);
    return 0;
}

static int lsa_group(int64_t T, int L, int d_in, int Hq, int Hkv, int dh, int B, int P_cap)
{
    const int Eq = Hq * dh, Ekv = Hkv * dh;
    double *hs = buf((size_t)T * L * d_in), *wq = buf((size_t)Eq * d_in), *wk = buf((size_t)Ekv * d_in);
    double *wv = buf((size_t)Ekv * d_in), *wo = buf((size_t)Eq * Eq), *out = buf((size_t)T * Eq);
    CHECK(moa_ref_lsa(hs, T, L, d_in, Hq, Hkv, dh, wq, wk, wv, wo, Eq, out));
    /* append the rows to a memory, ragged (sequence 1 gets none), ending exactly at the capacity for sequence 0 */
    int32_t *off = (int32_t *)malloc(sizeof(int32_t) * (B + 1)), *len = (int32_t *)malloc(sizeof(int32_t) * B);
    off[0] = 0;
    for (int b = 0; b < B; ++b) off[b + 1] = (b == 1) ? off[b] : (int32_t)(off[b] + (T - off[b]) / (B - b));
    off[B] = (int32_t)T;
    for (int b = 0; b < B; ++b) len[b] = P_cap - (off[b + 1] - off[b]) - (b ? 1 : 0);
    double *mk = buf((size_t)Ekv * Eq), *mv = buf((size_t)Ekv * Eq);
    double *kc = buf((size_t)B * Hkv * P_cap * dh), *vc = buf((size_t)B * Hkv * P_cap * dh);
    CHECK(moa_ref_ca_kv_append(out, Eq, off, B, Hkv, dh, mk, mv, kc, vc, len, P_cap));
    if (len[0] != P_cap) { fprintf(stderr, "append length\n"); return 1; }
    free(hs); free(wq); free(wk); free(wv); free(wo); free(out); free(off); free(len); free(mk); free(mv); free(kc); free(vc);
    return 0;
}

static int draft_tree_group(int Bw, int D, int m, int V)
{
    const int n_max = Bw + (D - 1) * Bw * Bw;
    float *clp = (float *)malloc(sizeof(float) * n_max), *lp = (float *)malloc(sizeof(float) * (size_t)Bw * Bw);
    int32_t *ctok = (int32_t *)malloc(sizeof(int32_t) * n_max), *cpar = (int32_t *)malloc(sizeof(int32_t) * n_max);
    int32_t *front = (int32_t *)malloc(sizeof(int32_t) * Bw), *tk = (int32_t *)malloc(sizeof(int32_t) * (size_t)Bw * Bw);
    double *logits = buf((size_t)Bw * V), *lpd = (double *)malloc(sizeof(double) * (size_t)Bw * Bw);
    for (int level = 1; level <= D; ++level) {
        const int F = level == 1 ? 1 : Bw;
        for (size_t i = 0; i < (size_t)Bw * V; ++i) logits[i] = 4.0 * rnd();
        CHECK(moa_ref_topk_logprob(logits, F, V, Bw, tk, lpd));
        for (int i = 0; i < F * Bw; ++i) lp[i] = (float)lpd[i];
        CHECK(moa_ref_tree_expand_level(level, Bw, lp, tk, clp, ctok, cpar, front));
    }
    int32_t *parent = (int32_t *)malloc(sizeof(int32_t) * (1 + m)), *tok = (int32_t *)malloc(sizeof(int32_t) * (1 + m));
    int32_t *nc = (int32_t *)malloc(sizeof(int32_t) * (1 + m)), M = 0;
    CHECK(moa_ref_tree_finalize(n_max, m, 7, clp, ctok, cpar, parent, tok, nc, &M));
    if (M != 1 + (m < n_max ? m : n_max) || parent[0] != -1) { fprintf(stderr, "finalize\n"); return 1; }
    for (int i = 1; i < M; ++i)
        if (parent[i] < 0 || parent[i] >= i) { fprintf(stderr, "finalize: parent order\n"); return 1; }
    free(clp); free(lp); free(ctok); free(cpar); free(front); free(tk); free(logits); free(lpd); free(parent); free(tok); free(nc);
    return 0;
}

static int misc_group(void)
{
    /* LM head, accept message, the two softmax forms, a plain projection with and without weights */
    const int R = 5, d = 24, V = 301;
    double *x = buf((size_t)R * d), *w = buf((size_t)V * d), *best = buf(R), *y = buf((size_t)R * V);
    int32_t *tgt = (int32_t *)malloc(sizeof(int32_t) * R);
    CHECK(moa_ref_lm_head_argmax(x, R, d, w, V, tgt, best));
    CHECK(moa_ref_linear(x, R, d, w, V, y));
    for (int r = 0; r < R; ++r)
        if (tgt[r] < 0 || tgt[r] >= V || y[(size_t)r * V + tgt[r]] != best[r]) { fprintf(stderr, "lm head\n"); return 1; }
    CHECK(moa_ref_linear(x, R, d, NULL, d, y));
    const int A = 3, nv = 4, n = 37;
    float *xa = (float *)malloc(sizeof(float) * A * nv * n), *xb = (float *)malloc(sizeof(float) * A * nv * n);
    for (int i = 0; i < A * nv * n; ++i) xa[i] = (float)(20.0 * rnd());
    for (int i = 0; i < n; ++i) xa[i] = 0.f;                       /* an all-zero vector */
    int32_t tok[3] = {0, 128255, 16777215}, tok2[3];
    uint8_t *msg = (uint8_t *)malloc((size_t)A * (3 + nv * (4 + n)));
    CHECK(moa_ref_msg_pack_accept(tok, xa, A, nv, n, msg));
    CHECK(moa_ref_msg_unpack_accept(msg, A, nv, n, tok2, xb));
    if (memcmp(tok, tok2, sizeof(tok))) { fprintf(stderr, "accept message\n"); return 1; }
    const int ns = 77, dh = 9;
    double *s = buf(ns), *vals = buf((size_t)ns * dh), o1[9], o2[9], psum = 0.0;
    s[3] = 700.0;                                                   /* would overflow exp() without the max */
    CHECK(moa_ref_softmax_weighted_sum(s, vals, ns, dh, o1, &psum));
    CHECK(moa_ref_softmax_weighted_sum_chunked(s, vals, ns, dh, 10, o2));
    if (fabs(psum - 1.0) > 1e-12) { fprintf(stderr, "softmax sum\n"); return 1; }
    for (int c = 0; c < dh; ++c)
        if (fabs(o1[c] - o2[c]) > 1e-12) { fprintf(stderr, "chunked softmax\n"); return 1; }
    free(x); free(w); free(best); free(y); free(tgt); free(xa); free(xb); free(msg); free(s); free(vals);
    return 0;
}

int main(void)
{
    if (attention_group(3, 70, 24, 6, 3, 4, 19)) return 1;       /* two mask words, GQA, tiny heads */
    if (attention_group(2, 1, 10, 2, 2, 5, 3)) return 1;         /* one-node trees, odd head_dim */
    if (attention_group(1, 130, 16, 4, 1, 4, 2)) return 1;       /* three mask words, a single KV head */
    if (lsa_group(7, 5, 12, 4, 2, 3, 3, 9)) return 1;
    if (lsa_group(2, 1, 8, 2, 2, 4, 2, 4)) return 1;             /* a single layer */
    if (draft_tree_group(3, 4, 11, 50)) return 1;
    if (draft_tree_group(1, 3, 8, 5)) return 1;                  /* breadth 1: a chain; m above the candidate count */
    if (misc_group()) return 1;
    printf("sanitize_driver: ok\n");
    return 0;
}
