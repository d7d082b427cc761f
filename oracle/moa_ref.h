/*
 * moa_ref.h -- CPU oracle for the Mixture-of-Attentions draft step.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64, written from the paper's
 * definitions.  Nothing in the product path may include, link or call this;
 * only the test-suite, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code with the GPU library (own header, own status codes).
 *
 * All pointers are HOST pointers.  All floating-point tensors are fp64,
 * row-major, dense.  Weights are [out_features, in_features].
 * A NULL weight means "this projection is the identity" (the input is taken
 * as already projected; widths must then agree).
 *
 * Value-level parity with the paper authors' implementation is UNPINNED for
 * every floating-point function here: the paper prints no numeric example of
 * LSA, CA or tree attention.  The functions are pinned by closed forms,
 * invariants, library cross-checks and brute force (tests/test_oracle_*.py).
 */
#ifndef MOA_REF_H
#define MOA_REF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOA_REF_OK = 0,
    MOA_REF_BAD_ARG = 1,   /* null pointer, non-positive size, widths that do not agree */
    MOA_REF_BAD_TREE = 2,  /* parent[0] != -1 or parent[i] outside [0, i)               */
    MOA_REF_EMPTY = 3,     /* softmax over an empty key set, or cache overflow          */
};

/* Draft tree (Sec. 2.2 "tree drafting", Tree Attention): node 0 is the root,
 * parent[i] < i.  depth[0] = 0, depth[i] = depth[parent[i]] + 1.
 * mask[b][i] is the set {i} U ancestors(i) as a bitset of W = ceil(M/64)
 * 64-bit words: node j lives in word j>>6, bit j&63. */
int moa_ref_tree_build(const int32_t *parent /*[B,M]*/, int B, int M,
                       uint64_t *mask /*[B,M,W]*/, int32_t *depth /*[B,M]*/);

/* y[R,N] = x[R,K] * w[N,K]^T  (w == NULL: N must equal K, y = x). */
int moa_ref_linear(const double *x, int64_t R, int K, const double *w, int N, double *y);

/* Layer Self-Attention followed by mean aggregation (Sec. 3.1.1 "Layer
 * Self-Attention"; Alg. 1 "LSA_layer_with_mean").  Every token is independent;
 * attention runs over the L layer rows of that token with a full mask.
 *   Q = X wq^T [L, Hq*dh],  K = X wk^T, V = X wv^T [L, Hkv*dh]
 *   head h reads KV head h / (Hq/Hkv);  S = Q_h K_g^T / sqrt(dh);  P = softmax rows
 *   Y = concat_h(P V_g) wo^T  [L, d_out];   out[t] = mean over the L rows of Y. */
int moa_ref_lsa(const double *hs /*[T,L,d_in]*/, int64_t T, int L, int d_in,
                int Hq, int Hkv, int dh,
                const double *wq /*[Hq*dh,d_in]*/, const double *wk /*[Hkv*dh,d_in]*/,
                const double *wv /*[Hkv*dh,d_in]*/, const double *wo /*[d_out,Hq*dh]*/,
                int d_out, double *out /*[T,d_out]*/);

/* Cross-Attention memory: project newly verified LSA rows to keys and values and
 * append them to each sequence's cache (Sec. 3.1.2 "Cross-Attention": keys and
 * values come from the output of LSA; Alg. 1 "kv <- (kv, kv')").
 * Rows tok_off[b] .. tok_off[b+1]-1 of mem_new belong to sequence b and land at
 * cache rows ca_len[b] ..; ca_len[b] is advanced. */
int moa_ref_ca_kv_append(const double *mem_new /*[T,d_mem]*/, int d_mem,
                         const int32_t *tok_off /*[B+1]*/, int B, int Hkv, int dh,
                         const double *wk /*[Hkv*dh,d_mem]*/, const double *wv,
                         double *kc, double *vc /*[B,Hkv,P_cap,dh]*/,
                         int32_t *ca_len /*[B] in/out*/, int P_cap);

/* Cross-Attention of the draft model at generation time (Sec. 3.1.2; Alg. 1
 * "CA_layer(q, kv)"): every query attends ALL ca_len[b] cached rows, no mask.
 * ca_len[b] == 0 -> MOA_REF_EMPTY. */
int moa_ref_cross_attn(const double *xq /*[B,Mq,d]*/, int B, int Mq, int d,
                       int H, int Hkv, int dh,
                       const double *wq /*[H*dh,d]*/, const double *wo /*[d_out,H*dh]*/, int d_out,
                       const double *kc, const double *vc /*[B,Hkv,P_cap,dh]*/,
                       const int32_t *ca_len /*[B]*/, int P_cap,
                       double *out /*[B,Mq,d_out]*/);

/* Tree-masked verification attention of one LLM layer (Sec. 2.2 Tree Attention;
 * Alg. 1 verification forward pass; the attention inside every reused layer of
 * Target Layer Inference, Sec. 3.2).  Node i, head h attends cache rows
 * 0..prefix_len[b]-1 and tree rows j with bit j of mask[b][i] set.
 * Also returns the tree rows' own projected keys/values. */
int moa_ref_tree_verify_attn(const double *x /*[B,M,d]*/, int B, int M, int d,
                             int H, int Hkv, int dh,
                             const double *wq /*[H*dh,d]*/, const double *wk /*[Hkv*dh,d]*/,
                             const double *wv, const double *wo /*[d_out,H*dh]*/, int d_out,
                             const double *kcache, const double *vcache /*[B,Hkv,P_cap,dh]*/,
                             const int32_t *prefix_len /*[B]*/, int P_cap,
                             const uint64_t *mask /*[B,M,W]*/,
                             double *out /*[B,M,d_out]*/,
                             double *k_tree, double *v_tree /*[B,Hkv,M,dh]*/);

/* Self-Attention layer of the draft model on draft-token embeddings, tree form
 * (Sec. 3.1 "Self-Attention": a causal self-attention on the CA queries, so that a
 * drafted token knows the tokens drafted before it; Alg. 1 "q <- SA_layer(token_embed(y))";
 * widths from the appendix table: embedding 4096, keys/values 512).  Causal over the
 * token sequence that leads to a node: node i attends the verified tokens' cached
 * keys/values (rows 0..prefix_len[b]-1) and the nodes on its own path root..i, found by
 * walking parent[] (no bitset here).  Drafting goes level by level: this call handles
 * the nodes node0 .. node0+Mn-1 (emb holds only their rows), writes their projected
 * keys/values into rows node0.. of the per-cycle draft cache and reads the earlier
 * rows of that cache as they are.  Every ancestor of a new node must be < node0+Mn. */
int moa_ref_self_attn_draft(const double *emb /*[B,Mn,d]*/, int B, int M, int node0, int Mn, int d,
                            int H, int Hkv, int dh,
                            const double *wq /*[H*dh,d]*/, const double *wk /*[Hkv*dh,d]*/,
                            const double *wv, const double *wo /*[d_out,H*dh]*/, int d_out,
                            const double *kcache, const double *vcache /*[B,Hkv,P_cap,dh]*/,
                            const int32_t *prefix_len /*[B]*/, int P_cap,
                            const int32_t *parent /*[B,M]*/,
                            double *out /*[B,Mn,d_out]*/,
                            double *k_draft, double *v_draft /*[B,Hkv,M,dh] in/out*/);

/* One reused LLM decoder layer under Target Layer Inference (Sec. 3.2: f^l_decoder((h^l_<=t, h^l_draft), o^l),
 * applied to the drafted tokens with the layer's KV cache of the verified ones), tree form.
 * The layer itself is the LLM's, a Llama-family pre-norm block (the paper's base models):
 *   n1 = rmsnorm(x) * g_attn;  q, k, v = n1 Wq^T, n1 Wk^T, n1 Wv^T;
 *   q, k rotated (RoPE, half-split pairs (c, c + dh/2), angle pos * theta^(-2c/dh)) at position
 *   pos = prefix_len[b] + depth(node) -- the place the token would have in its own sequence;
 *   h1 = x + concat_h(softmax(q K^T / sqrt(dh)) V) Wo^T over the cached rows and the node's own path;
 *   n2 = rmsnorm(h1) * g_mlp;  out = h1 + (silu(n2 Wgate^T) * (n2 Wup^T)) Wdown^T.
 * rmsnorm(x) = x / sqrt(mean(x^2) + eps).  The cache holds keys already rotated at their positions.
 * Node range, draft cache and parent[] as for moa_ref_self_attn_draft (k_draft holds rotated keys). */
int moa_ref_tli_decoder_layer(const double *x /*[B,Mn,d]*/, int B, int M, int node0, int Mn, int d,
                              int H, int Hkv, int dh, int d_ff, double rms_eps, double rope_theta,
                              const double *g_attn /*[d]*/, const double *wq, const double *wk,
                              const double *wv, const double *wo /*[d,H*dh]*/,
                              const double *g_mlp /*[d]*/, const double *w_gate /*[d_ff,d]*/,
                              const double *w_up, const double *w_down /*[d,d_ff]*/,
                              const double *kcache, const double *vcache /*[B,Hkv,P_cap,dh]*/,
                              const int32_t *prefix_len, int P_cap, const int32_t *parent /*[B,M]*/,
                              double *out /*[B,Mn,d]*/, double *k_draft, double *v_draft /*[B,Hkv,M,dh]*/);

/* The drafter's own layers (Sec. 3.1: Layer Self-Attention, Self-Attention, Cross-Attention) each come with an MLP
 * (appendix architecture table: projection sizes 6144, 512 and 7168); the paper states neither its form nor the
 * normalisation and residual wiring.  Reading taken: the form of the LLM's own block (above), i.e. a pre-norm
 * residual sub-block with a gated MLP,
 *   h = x + res (res may be NULL);  n = rmsnorm(h) * g;  out = h + (silu(n Wgate^T) * (n Wup^T)) Wdown^T,
 * where res is the output of the attention sub-layer that precedes the MLP and x the stream it was added to. */
int moa_ref_mlp_block(const double *x /*[R,d]*/, const double *res /*[R,d] or NULL*/, int64_t R, int d, int d_ff,
                      const double *g /*[d]*/, const double *w_gate /*[d_ff,d]*/, const double *w_up,
                      const double *w_down /*[d,d_ff]*/, double eps, double *out /*[R,d]*/);
/* out = x / sqrt(mean(x^2) + eps) * g, row by row: the pre-norm in front of an attention sub-layer. */
int moa_ref_rmsnorm(const double *x /*[R,d]*/, int64_t R, int d, const double *g /*[d]*/, double eps,
                    double *out /*[R,d]*/);

/* Rotary position embedding of one head vector in place (the convention above). */
void moa_ref_rope(double *v /*[dh]*/, int dh, double pos, double theta);

/* ---- draft-tree construction (Sec. 2.2, tree drafting as in EAGLE-2: from the root the Bw most
 * probable tokens; then, level by level, each of the Bw current branches proposes its Bw most probable
 * children, the Bw*Bw expansions are ranked by joint probability and the best Bw become the branches of
 * the next level; at the end the m most probable of all Bw + (D-1) Bw^2 candidates are kept).
 * Joint probabilities are sums of log-probabilities in SINGLE precision (one addition per candidate), so
 * that a device implementation takes every ranking decision on identical numbers.  Ties: lower candidate
 * index first.  Candidates are numbered level by level: level 1 -> 0..Bw-1, level l >= 2 ->
 * Bw + (l-2) Bw^2 + f*Bw + j for child j of the f-th branch.  Per sequence:
 *   cand_logp/tok/parent [n_max]  (parent = candidate index, -1 for children of the root)
 *   frontier [Bw] = candidate indices of the current branches, best first. */

/* One level.  level == 1: child_logp/tok hold one row (the root's children); level >= 2: Bw rows,
 * row f = children of frontier[f].  Log-probabilities above 0 are taken as 0, NaN as -inf. */
int moa_ref_tree_expand_level(int level, int Bw, const float *child_logp /*[F,Bw]*/,
                              const int32_t *child_tok /*[F,Bw]*/, float *cand_logp, int32_t *cand_tok,
                              int32_t *cand_parent, int32_t *frontier /*[Bw] in/out*/);

/* Keep the m best of the first n_cand candidates; nodes are the root (token root_tok) followed by the
 * kept candidates in candidate order (which is depth order).  Writes parent[] (node indices, -1 for the
 * root), tok[], node_cand[] (candidate index of each node, -1 for the root) for M = 1 + min(m, n_cand)
 * nodes and returns M in *M_out.  A kept candidate's parent is always kept (its joint probability is not
 * smaller and its index is lower). */
int moa_ref_tree_finalize(int n_cand, int m, int32_t root_tok, const float *cand_logp,
                          const int32_t *cand_tok, const int32_t *cand_parent,
                          int32_t *parent /*[1+m]*/, int32_t *tok, int32_t *node_cand, int32_t *M_out);

/* The Bw most probable tokens of each row of logits with their log-probabilities
 * logit - logsumexp(row) (fp64 here).  Ties: lower token id first. */
int moa_ref_topk_logprob(const double *logits /*[F,V]*/, int F, int V, int Bw,
                         int32_t *tok /*[F,Bw]*/, double *logp /*[F,Bw]*/);

/* Greedy token of the LLM at every tree node: tgt[r] = argmax_v (x[r] . W[v]) over the vocabulary
 * (Sec. 2.1: y ~ Softmax(LM_head(o)); greedy verification takes the arg max; the result is the tgt[]
 * that the accept walk reads).  Ties: lower token id.  Also returns the winning logit. */
int moa_ref_lm_head_argmax(const double *x /*[R,d]*/, int R, int d, const double *w /*[V,d]*/, int V,
                           int32_t *tgt /*[R]*/, double *best /*[R]*/);

/* ---- client-server messages (Sec. 4.2 and the table of message lengths in the appendix).
 * Client -> server: every node of the draft tree as 3 bytes of token id (little-endian, id < 2^24)
 * and 1 byte for its position in the tree = the index of its parent (0xFF for the root): 4 M bytes.
 * Server -> client: per accepted token 3 bytes of token id and its activations, (TLI+1) vectors of
 * 2 E_kv values, quantised to 8 bits.  The paper does not say how; here: per vector, symmetric,
 * scale = absmax / 127 in single precision, code = rint(x / scale) clamped to [-127, 127] (0 when the
 * vector is all zero), the scale sent as 4 bytes in front of the vector's codes.  Token layout:
 * [3 B id][n_vec x ([4 B scale][n codes])].  All arithmetic in single precision. */
int moa_ref_msg_pack_tree(const int32_t *tok, const int32_t *parent /*[B,M]*/, int B, int M, uint8_t *msg /*[B,4M]*/);
int moa_ref_msg_unpack_tree(const uint8_t *msg, int B, int M, int32_t *tok, int32_t *parent);
int moa_ref_msg_pack_accept(const int32_t *tok /*[A]*/, const float *x /*[A,n_vec,n]*/, int A, int n_vec, int n,
                            uint8_t *msg /*[A, 3 + n_vec (4 + n)]*/);
int moa_ref_msg_unpack_accept(const uint8_t *msg, int A, int n_vec, int n, int32_t *tok, float *x);

/* Greedy acceptance (Sec. 2.2: everything after the first mismatch is dropped).
 * tok[i] is the token drafted at node i; tgt[i] is the LLM's greedy token after
 * node i.  Walk from the root to the lowest-index child whose token equals the
 * current node's tgt; stop when none does.  path = visited nodes (unused = -1),
 * n_path >= 1, bonus = tgt of the last visited node. */
int moa_ref_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt /*[B,M]*/,
                        int B, int M, int32_t *path /*[B,M]*/, int32_t *n_path /*[B]*/,
                        int32_t *bonus /*[B]*/);

/* Self-check variant of the attention reduction: same result as the two-pass
 * softmax used above, computed chunk by chunk with a running max / sum and a
 * final merge.  scores[n], values[n,dh] -> o[dh].  Used only by a test that
 * shows the chunked merge formula is exact. */
int moa_ref_softmax_weighted_sum_chunked(const double *scores, const double *values,
                                         int n, int dh, int chunk, double *o);
int moa_ref_softmax_weighted_sum(const double *scores, const double *values,
                                 int n, int dh, double *o, double *prob_sum);

#ifdef __cplusplus
}
#endif
#endif
