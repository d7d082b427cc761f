/*
 * moa.h -- C ABI of libmoa: the single-device hot path of one draft step of the
 * Mixture-of-Attentions speculative-decoding method, hand-written for gfx950.
 *
 * Conventions
 *  - Every function returns an int32 status: MOA_OK (0) or a negative MOA_ERR_*.
 *    moa_last_error() gives a thread-local detail string for the last failure.
 *  - Pointers are DEVICE pointers unless the name ends in _host.  The caller owns
 *    every buffer (inputs, outputs, caches, workspace); the library allocates no
 *    device memory and never frees.  What it keeps per device for the life of the
 *    process: the fixed scratch array of moa_tree_verify_attn_noalloc, and, once
 *    MOA_SCHED_TWO_STREAM has been used, one stream and three events.
 *  - All work is enqueued on the caller's hipStream_t (passed as void*, NULL = the
 *    default stream).  No host synchronisation happens inside.  Argument checks
 *    that need only host values run before anything is launched; a failed check
 *    launches nothing.
 *  - Values that live in device memory (parent[], prefix_len[], ca_len[]) are
 *    checked on the device: kernels clamp what they read so that no access leaves
 *    the caller's buffers, and OR a MOA_DEV_* bit into *dev_status (may be NULL;
 *    the caller zeroes it and reads it back when it wants to know).
 *  - dtype: MOA_F32 or MOA_BF16 is the storage type of every floating-point
 *    tensor of the call (activations, weights, caches, outputs).  Accumulation,
 *    scores, softmax max/sum and probabilities are fp32 in both cases.
 *  - Weights are row-major [out_features, in_features].  A NULL weight means the
 *    projection is the identity: the input is taken as already projected (the
 *    widths must then agree).
 *  - Attention scale is 1/sqrt(head_dim).  Query head h reads KV head
 *    h / (n_q_heads / n_kv_heads).  No positional encoding is applied inside.
 *  - Workspace: moa_workspace_bytes() gives a size that suffices for every call
 *    with sizes up to the ones queried; ws must be 256-byte aligned.
 */
#ifndef MOA_H
#define MOA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    MOA_OK = 0,
    MOA_ERR_NULL = -1,      /* a required pointer is NULL                                  */
    MOA_ERR_SHAPE = -2,     /* unsupported or inconsistent dimensions                      */
    MOA_ERR_TREE = -3,      /* (host-visible) tree argument invalid                        */
    MOA_ERR_RANGE = -4,     /* a length exceeds its capacity                               */
    MOA_ERR_DTYPE = -5,     /* dtype is neither MOA_F32 nor MOA_BF16                       */
    MOA_ERR_WORKSPACE = -6, /* workspace NULL, misaligned or too small                     */
    MOA_ERR_HIP = -7,       /* a HIP call (launch) failed                                  */
};

enum { MOA_F32 = 0, MOA_BF16 = 1 };

/* bits OR-ed into *dev_status by kernels */
enum {
    MOA_DEV_BAD_PARENT = 1,   /* parent[0] != -1 or parent[i] outside [0, i)                */
    MOA_DEV_BAD_LENGTH = 2,   /* prefix_len / ca_len outside [0, P_cap] (clamped)           */
    MOA_DEV_EMPTY_KEYS = 4,   /* cross-attention over an empty memory (output row = 0)      */
    MOA_DEV_CACHE_FULL = 8,   /* kv append would pass P_cap (rows beyond it are dropped)    */
    MOA_DEV_BAD_MESSAGE = 16, /* a token id or tree position does not fit its message field */
};

#define MOA_MAX_TREE 256      /* a tree position fits one byte (client message format, Sec. 4.2) */

typedef struct {
    int32_t n_layers;      /* L   : LLM layers stacked on LSA's layer axis                  */
    int32_t d_model;       /* d   : LLM hidden size E                                       */
    int32_t n_q_heads;     /* H   : query heads of CA and of the LLM's attention            */
    int32_t n_kv_heads;    /* Hkv : key/value heads                                         */
    int32_t head_dim;      /* dh                                                            */
    int32_t d_lsa_in;      /* d_in: width of one layer row given to LSA (2*E_kv in the paper) */
    int32_t lsa_q_heads;   /* H_l : LSA query heads; LSA output width d_lsa = H_l * dh      */
    int32_t lsa_kv_heads;  /* Hkv_l                                                         */
    int32_t dtype;         /* MOA_F32 | MOA_BF16                                            */
} moa_shape_t;

const char *moa_status_str(int32_t status);
const char *moa_last_error(void);

/* Workspace bytes sufficient for any call below with batch <= B, cache capacity <= P_cap,
 * tree size / query count <= M and LSA token count <= T_lsa.  Host-only, launches nothing. */
int32_t moa_workspace_bytes(const moa_shape_t *shape, int32_t B, int32_t P_cap, int32_t M,
                            int64_t T_lsa, size_t *bytes_host);

/* Draft tree structure (Sec. 2.2, tree drafting / Tree Attention).
 * parent[b][0] = -1 (root = the last token sampled by the LLM), 0 <= parent[b][i] < i.
 * mask[b][i] = bitset of {i} U ancestors(i), W = ceil(M/64) words per row, node j in word
 * j>>6 bit j&63; depth[b][0] = 0.  Integer results, exact.  An invalid parent entry sets
 * MOA_DEV_BAD_PARENT and the row keeps only the ancestors reached before it. */
int32_t moa_tree_build(const int32_t *parent /*[B,M]*/, int32_t B, int32_t M,
                       uint64_t *mask /*[B,M,W]*/, int32_t *depth /*[B,M]*/,
                       int32_t *dev_status, void *stream);

/* Greedy acceptance (Sec. 2.2: all tokens after the first mismatch are discarded; Alg. 1,
 * verification step).  tok[i] = token drafted at node i, tgt[i] = the LLM's greedy token
 * after node i.  From the root, step to the lowest-index child c with tok[c] == tgt[cur];
 * stop when there is none.  path[b] = visited nodes then -1, n_path[b] >= 1,
 * bonus[b] = tgt of the last visited node.  Integer results, exact. */
int32_t moa_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt /*[B,M]*/,
                        int32_t B, int32_t M, int32_t *path /*[B,M]*/, int32_t *n_path /*[B]*/,
                        int32_t *bonus /*[B]*/, void *stream);

/* Layer Self-Attention with mean aggregation (Sec. 3.1.1 "Layer Self-Attention"; Alg. 1,
 * LSA_layer_with_mean).  For every token independently: full (unmasked) self-attention over
 * its L layer rows, output projection, then the mean over the L rows.
 *   hs [T, L, d_in]  ->  out [T, H_l*dh]
 *   wq [H_l*dh, d_in], wk, wv [Hkv_l*dh, d_in], wo [H_l*dh, H_l*dh]
 * The kernels use mean_l(P V) Wo^T = ((1^T P / L) V) Wo^T, exact in real arithmetic. */
int32_t moa_lsa(const moa_shape_t *shape, const void *hs, int64_t T,
                const void *wq, const void *wk, const void *wv, const void *wo,
                void *out, void *ws, size_t ws_bytes, void *stream);

/* The same Layer Self-Attention (Sec. 3.1.1; Alg. 1, LSA_layer_with_mean) with Wq, Wk, Wv rearranged once, at load
 * time, into the order in which the matrix cores consume them, so that the one-kernel form (see
 * moa_debug_force_lsa_kernel) reads every weight straight into the register it is used from instead of staging it
 * in LDS.  Shapes: those that form takes -- bf16, head_dim 128, n_layers <= 96, d_lsa_in >= 128 and a multiple of
 * 64, an even number of LSA query heads per KV head; others are refused with MOA_ERR_SHAPE.  Results are the bits
 * moa_lsa gives for the same weights.
 *   moa_lsa_packed_weight_bytes: size of the packed buffer (host only, launches nothing).
 *   moa_lsa_pack_weights: wq [H_l*dh, d_in], wk, wv [Hkv_l*dh, d_in] -> packed (device, caller-owned, 16-byte
 *     aligned, at least that many bytes, else MOA_ERR_WORKSPACE); one launch; layout: per unit of two query heads
 *     with their key and value head, per wavefront (64 of the unit's 512 rows), per 64 columns, the 16-byte operand
 *     pieces in lane order.  The plain matrices are not needed afterwards by moa_lsa_packed.
 *   moa_lsa_packed: moa_lsa with w_packed in place of wq / wk / wv (all other arguments, workspace size and errors
 *     as there; hs, w_packed and out 16-byte aligned). */
int32_t moa_lsa_packed_weight_bytes(const moa_shape_t *shape, size_t *bytes_host);
int32_t moa_lsa_pack_weights(const moa_shape_t *shape, const void *wq, const void *wk, const void *wv,
                             void *packed, size_t packed_bytes, void *stream);
int32_t moa_lsa_packed(const moa_shape_t *shape, const void *hs, int64_t T, const void *w_packed,
                       const void *wo, void *out, void *ws, size_t ws_bytes, void *stream);

/* Cross-attention memory append (Sec. 3.1.2: CA keys and values come from the output of
 * LSA; Alg. 1, kv <- (kv, kv')).  Rows tok_off[b] .. tok_off[b+1]-1 of mem_new belong to
 * sequence b (tok_off is a device array, tok_off[0] = 0, non-decreasing, tok_off[B] <= T;
 * rows owned by no sequence are ignored); their projections are written to cache rows
 * ca_len[b] .. and ca_len[b] is advanced.  Rows that would pass P_cap are dropped and
 * MOA_DEV_CACHE_FULL is set.  The workspace is optional here (NULL: a slower projection kernel).
 *   mem_new [T, d_mem], wk, wv [Hkv*dh, d_mem], kc, vc [B, Hkv, P_cap, dh] */
int32_t moa_ca_kv_append(const moa_shape_t *shape, const void *mem_new, int64_t T, int32_t d_mem,
                         const int32_t *tok_off /*[B+1]*/, int32_t B,
                         const void *wk, const void *wv, void *kc, void *vc,
                         int32_t *ca_len /*[B] in/out*/, int32_t P_cap,
                         int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* The draft model's Cross-Attention at generation time (Sec. 3.1.2; Alg. 1, CA_layer(q, kv)):
 * every query row attends all ca_len[b] cached rows, no mask; queries do not see each other
 * (input-independence, Property 3).
 *   xq [B, Mq, d], wq [H*dh, d], wo [d, H*dh], kc, vc [B, Hkv, P_cap, dh] -> out [B, Mq, d] */
int32_t moa_cross_attn_draft(const moa_shape_t *shape, const void *xq, int32_t B, int32_t Mq,
                             const void *wq, const void *wo, const void *kc, const void *vc,
                             const int32_t *ca_len /*[B]*/, int32_t P_cap, void *out,
                             int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* Tree-masked verification attention of one LLM layer (Sec. 2.2 Tree Attention; Alg. 1,
 * verification forward pass; also the attention inside each reused layer under Target Layer
 * Inference, Sec. 3.2).  Node i, head h attends cache rows 0..prefix_len[b]-1 and the tree
 * rows j with bit j of mask[b][i] set; one softmax over the union.
 *   x [B, M, d]; wq [H*dh, d], wk, wv [Hkv*dh, d], wo [d, H*dh]
 *   kcache, vcache [B, Hkv, P_cap, dh]; mask [B, M, W] as written by moa_tree_build
 *   -> out [B, M, d]; k_tree, v_tree [B, Hkv, M, dh] (the tree rows' own keys / values; the
 *      caller commits the accepted ones to its cache). */
int32_t moa_tree_verify_attn(const moa_shape_t *shape, const void *x, int32_t B, int32_t M,
                             const void *wq, const void *wk, const void *wv, const void *wo,
                             const void *kcache, const void *vcache,
                             const int32_t *prefix_len /*[B]*/, int32_t P_cap,
                             const uint64_t *mask, void *out, void *k_tree, void *v_tree,
                             int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* moa_tree_verify_attn for callers that cannot allocate device memory and so cannot bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without ws / ws_bytes, same
 * kernels, same results bit for bit.  The scratch (projected queries, heads, partial sums, partial attention results)
 * is a fixed 32 MiB array in the library's own device memory, one copy per GPU, held until the process ends; the call
 * itself allocates and frees nothing.  MOA_ERR_WORKSPACE when the call would need more than that (what
 * moa_workspace_bytes(shape, B, P_cap, M, 0) reports; the Llama-3-8B shape with one sequence, a tree of 64 and 4096
 * cached tokens needs about 12 MiB) -- use moa_tree_verify_attn then.  Every call on a GPU shares that GPU's array:
 * calls that overlap in time on one GPU (different streams, different host threads) race; calls on one stream do not.
 * The array keeps the previous call's contents and nothing in it has to start at zero. */
int32_t moa_tree_verify_attn_noalloc(const moa_shape_t *shape, const void *x, int32_t B, int32_t M,
                                     const void *wq, const void *wk, const void *wv, const void *wo,
                                     const void *kcache, const void *vcache,
                                     const int32_t *prefix_len /*[B]*/, int32_t P_cap,
                                     const uint64_t *mask, void *out, void *k_tree, void *v_tree,
                                     int32_t *dev_status, void *stream);

/* Self-Attention layer of the draft model on draft-token embeddings, tree form (Sec. 3.1,
 * "Self-Attention": a causal self-attention on the queries of the Cross-Attention, so that a
 * drafted token is aware of the tokens drafted before it; Alg. 1, q <- SA_layer(token_embed(y));
 * appendix table: embedding 4096, keys/values 512, i.e. shape->n_kv_heads = 4 at head_dim 128).
 * Causal over the token sequence that leads to a node: node i attends the layer's cached keys /
 * values of the verified tokens (rows 0..prefix_len[b]-1) and the drafted nodes on its own path
 * (bit j of mask[b][i]).  Drafting proceeds level by level, so a call covers the Mn nodes
 * node_begin .. node_begin+Mn-1 of a tree of M nodes:
 *   emb [B, Mn, d] (rows of the new nodes only); mask [B, M, W] of the whole tree (rows of
 *   nodes not yet drafted are not read; every ancestor of a new node is < node_begin+Mn);
 *   k_draft, v_draft [B, Hkv, M, dh]: the per-cycle draft cache; rows node_begin.. are written
 *   (the new nodes' projected keys / values), rows below are read as earlier calls left them;
 *   the caller drops the cache after verification (Alg. 1, "discard")
 *   -> out [B, Mn, d]: the Cross-Attention queries of the new nodes.
 * node_begin = 0, Mn = M handles a whole tree at once.  MOA_ERR_RANGE if the node range leaves
 * the tree.  Weights, caches, workspace and dev_status as for moa_tree_verify_attn (workspace:
 * moa_workspace_bytes with this shape, Mn as the tree size is enough; M always is). */
int32_t moa_self_attn_draft(const moa_shape_t *shape, const void *emb, int32_t B, int32_t M,
                            int32_t node_begin, int32_t Mn,
                            const void *wq, const void *wk, const void *wv, const void *wo,
                            const void *kcache, const void *vcache,
                            const int32_t *prefix_len /*[B]*/, int32_t P_cap,
                            const uint64_t *mask, void *out, void *k_draft, void *v_draft,
                            int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* One reused LLM decoder layer under Target Layer Inference (Sec. 3.2: the last TLI layers of the
 * LLM, f^l_decoder, run on the drafted tokens with their KV cache of the verified ones; Alg. 1, the
 * loop over l = L-N .. L).  The layer is the LLM's own; for the paper's base models that is a
 * Llama-family pre-norm block, which is what is built:
 *   n1 = rmsnorm(x) * g_attn; q, k, v = n1 Wq^T, n1 Wk^T, n1 Wv^T; q and k rotated (rotary
 *   embedding, pairs (c, c + dh/2), angle pos * theta^(-2c/dh)) at pos = prefix_len[b] + depth of the
 *   node; h1 = x + TreeAttention(q; cache, draft rows on the node's path) Wo^T;
 *   n2 = rmsnorm(h1) * g_mlp; out = h1 + (silu(n2 Wgate^T) * (n2 Wup^T)) Wdown^T,
 *   rmsnorm(x) = x / sqrt(mean(x^2) + rms_eps).
 * Node range, mask and per-cycle draft cache as for moa_self_attn_draft (k_draft holds rotated keys,
 * the cache too, as the LLM stored them); depth [B, M] as written by moa_tree_build.
 *   x [B, Mn, d]; g_attn, g_mlp [d]; wq [H*dh, d], wk, wv [Hkv*dh, d], wo [d, H*dh];
 *   w_gate, w_up [d_ff, d], w_down [d, d_ff] -> out [B, Mn, d].
 * All weights are required.  Workspace: moa_tli_workspace_bytes (host only, launches nothing). */
typedef struct { int32_t d_ff; float rms_eps; float rope_theta; } moa_decoder_cfg_t;
int32_t moa_tli_workspace_bytes(const moa_shape_t *shape, const moa_decoder_cfg_t *cfg, int32_t B,
                                int32_t P_cap, int32_t M, size_t *bytes_host);
int32_t moa_tli_decoder_layer(const moa_shape_t *shape, const moa_decoder_cfg_t *cfg, const void *x,
                              int32_t B, int32_t M, int32_t node_begin, int32_t Mn,
                              const void *g_attn, const void *wq, const void *wk, const void *wv,
                              const void *wo, const void *g_mlp, const void *w_gate, const void *w_up,
                              const void *w_down, const void *kcache, const void *vcache,
                              const int32_t *prefix_len /*[B]*/, int32_t P_cap, const uint64_t *mask,
                              const int32_t *depth, void *out, void *k_draft, void *v_draft,
                              int32_t *dev_status, void *ws, size_t ws_bytes, void *stream);

/* The wrappers of the drafter's own layers (Sec. 3.1: Layer Self-Attention, Self-Attention,
 * Cross-Attention; appendix architecture table: an MLP projection of 6144 after LSA, 512 after SA, 7168
 * after CA).  The paper states neither the MLP's form nor the normalisation and residual wiring; the
 * form of the LLM's own block (moa_tli_decoder_layer) is taken: a pre-norm residual sub-block with a
 * gated MLP,
 *   h = x + res (res may be NULL);  n = rmsnorm(h) * g;  out = h + (silu(n Wgate^T) * (n Wup^T)) Wdown^T,
 * where res is the output of the attention sub-layer in front of the MLP and x the stream that output
 * is added to; moa_rmsnorm is the pre-norm in front of such an attention sub-layer:
 *   out = x / sqrt(mean(x^2) + rms_eps) * g.
 * A drafter layer is then  a = Attn(moa_rmsnorm(x));  y = moa_mlp_block(x, a)  with Attn one of
 * moa_self_attn_draft / moa_cross_attn_draft, and  mem = moa_mlp_block(moa_lsa(...), NULL)  for LSA, whose
 * mean over the layers leaves no stream to add to.
 *   x, res, out [R, d] (device, `dtype`; out may alias x or res); g [d]; w_gate, w_up [d_ff, d];
 *   w_down [d, d_ff]; the stream h is kept in single precision between the two halves.
 * R = 0 is a no-op.  Workspace: moa_mlp_block_workspace_bytes (host only, launches nothing); the caller
 * owns it.  Errors: MOA_ERR_NULL / _DTYPE / _SHAPE / _WORKSPACE before anything is launched. */
int32_t moa_mlp_block_workspace_bytes(int32_t dtype, int64_t R, int32_t d, int32_t d_ff, size_t *bytes_host);
int32_t moa_mlp_block(int32_t dtype, const void *x, const void *res, int64_t R, int32_t d, int32_t d_ff,
                      const void *g, const void *w_gate, const void *w_up, const void *w_down,
                      float rms_eps, void *out, void *ws, size_t ws_bytes, void *stream);
int32_t moa_rmsnorm(int32_t dtype, const void *x, int64_t R, int32_t d, const void *g, float rms_eps,
                    void *out, void *stream);

/* Draft-tree construction on the device (Sec. 2.2, tree drafting as in EAGLE-2: from the root the Bw
 * most probable tokens; then, level by level, each of the Bw current branches proposes its Bw most
 * probable children, the Bw*Bw expansions are ranked by joint probability and the best Bw become the
 * branches of the next level; at the end the m most probable of all Bw + (D-1) Bw^2 candidates are
 * kept for verification).  Joint probabilities are sums of log-probabilities in single precision, one
 * addition per candidate; ties go to the lower candidate index; a log-probability above 0 counts as 0
 * and NaN as -inf, so a child is never ranked before its parent and the kept set is always a tree.
 * Candidates are numbered level by level: level 1 -> 0..Bw-1; level l >= 2 -> Bw + (l-2) Bw^2 + f Bw + j
 * for child j of the f-th branch.  State per sequence b (device, caller-owned, row length n_max >=
 * Bw + (D-1) Bw^2): cand_logp (fp32), cand_tok, cand_parent (candidate index, -1 = child of the root),
 * and frontier [B, Bw] = candidate indices of the current branches, best first.
 * moa_tree_expand_level: child_logp / child_tok [B, F, Bw] with F = 1 at level 1 (the root's children)
 *   and F = Bw above (row f = children of frontier[f]); writes the level's candidates and the new
 *   frontier.  1 <= Bw <= 16.  MOA_ERR_RANGE if the level does not fit n_max.
 * moa_tree_finalize: of the first n_cand candidates (<= 4096) keeps the min(m, n_cand) best; node 0 is
 *   the root (token root_tok[b]), the kept candidates follow in candidate order, which is depth order.
 *   Writes parent / tok / node_cand [B, 1+m] (node_cand = candidate index of the node, -1 for the
 *   root); rows have M = 1 + min(m, n_cand) valid entries, 1 + m <= MOA_MAX_TREE.  parent[] is exactly
 *   what moa_tree_build takes.  If the candidate arrays were not written by moa_tree_expand_level and a
 *   kept candidate's parent is not kept, the node hangs off the root and MOA_DEV_BAD_PARENT is set.
 * moa_topk_logprob: the Bw most probable tokens of each row of logits [F, V] (dtype MOA_F32 or
 *   MOA_BF16) with log-probabilities logit - logsumexp(row) in fp32; ties go to the lower token id.
 *   tok, logp [F, Bw]: the child_tok / child_logp of the next moa_tree_expand_level.  Logits are
 *   expected finite.  Workspace: moa_topk_workspace_bytes(F, V, Bw), 256-byte aligned. */
int32_t moa_tree_expand_level(int32_t level, int32_t B, int32_t Bw, int32_t n_max,
                              const float *child_logp, const int32_t *child_tok,
                              float *cand_logp, int32_t *cand_tok, int32_t *cand_parent,
                              int32_t *frontier, void *stream);
int32_t moa_tree_finalize(int32_t B, int32_t n_cand, int32_t n_max, int32_t m, const int32_t *root_tok,
                          const float *cand_logp, const int32_t *cand_tok, const int32_t *cand_parent,
                          int32_t *parent, int32_t *tok, int32_t *node_cand, int32_t *dev_status,
                          void *stream);
int32_t moa_topk_workspace_bytes(int32_t F, int32_t V, int32_t Bw, size_t *bytes_host);
int32_t moa_topk_logprob(int32_t dtype, const void *logits, int32_t F, int32_t V, int32_t Bw,
                         int32_t *tok, float *logp, void *ws, size_t ws_bytes, void *stream);

/* Greedy token of the LLM at every tree node (Sec. 2.1, y ~ Softmax(LM_head(o)); greedy verification
 * takes the arg max): tgt[r] = argmax_v x[r] . w[v] over the vocabulary, the tgt[] the accept walk
 * reads.  The logits are never stored: one pass over w per 64 rows.  Ties: lower token id.
 *   x [R, d], w [V, d] (bf16, 16-byte aligned, d a multiple of 128) -> tgt [R] (int32) and, if best
 *   is not NULL, best [R] (fp32: the winning logit).  Workspace: moa_lm_head_workspace_bytes(V),
 *   256-byte aligned.  MOA_ERR_DTYPE for fp32 inputs (project and reduce them on the caller's side). */
int32_t moa_lm_head_workspace_bytes(int32_t V, size_t *bytes_host);
int32_t moa_lm_head_argmax(int32_t dtype, const void *x, int32_t R, int32_t d, const void *w, int32_t V,
                           int32_t *tgt, float *best, void *ws, size_t ws_bytes, void *stream);

/* Client-server messages (Sec. 4.2; appendix table of message lengths).
 * Client -> server: each node of the draft tree as 3 bytes of token id (little-endian) and 1 byte for
 * its position in the tree = the index of its parent, 0xFF for the root: msg [B, 4 M] bytes (4-byte
 * aligned).  A token id outside [0, 2^24) or a parent outside [-1, 254] sets MOA_DEV_BAD_MESSAGE (the
 * low bits are sent).  moa_msg_unpack_tree is the inverse.
 * Server -> client: per accepted token 3 bytes of token id and its activations, n_vec vectors of n
 * values (for this method n_vec = TLI + 1 and n = 2 E_kv), 8 bits per value.  The paper does not give
 * the quantiser; this one is per vector and symmetric: scale = absmax / 127 in single precision,
 * code = rint(x / scale) clamped to [-127, 127] (0 for an all-zero vector), the scale sent as 4
 * bytes in front of the vector's codes.  Layout of a token: [3 B id][n_vec x ([4 B scale][n codes])];
 * msg holds moa_msg_accept_bytes(A, n_vec, n) bytes.  x [A, n_vec, n] in `dtype`;
 * moa_msg_unpack_accept returns fp32 values code * scale.  The gzip pass over the first message of a
 * conversation is moa_msg_gzip below. */
int32_t moa_msg_pack_tree(const int32_t *tok, const int32_t *parent, int32_t B, int32_t M, void *msg,
                          int32_t *dev_status, void *stream);
int32_t moa_msg_unpack_tree(const void *msg, int32_t B, int32_t M, int32_t *tok, int32_t *parent,
                            void *stream);
int32_t moa_msg_accept_bytes(int32_t A, int32_t n_vec, int32_t n, size_t *bytes_host);
int32_t moa_msg_pack_accept(int32_t dtype, const int32_t *tok, const void *x, int32_t A, int32_t n_vec,
                            int32_t n, void *msg, int32_t *dev_status, void *stream);
int32_t moa_msg_unpack_accept(const void *msg, int32_t A, int32_t n_vec, int32_t n, int32_t *tok,
                              float *x, void *stream);

/* The server's first message of a conversation carries the activations of the whole prompt and is gzip-compressed
 * after quantisation (Sec. 4.2).  Host-side byte work: msg_host is the message moa_msg_pack_accept wrote, copied to
 * the host on its way to the network.  The gzip container (RFC 1952) around a DEFLATE stream (RFC 1951), header
 * fields empty, so the output depends on the message bytes alone.  All pointers are HOST pointers.
 *   moa_msg_gzip_bound : an output size that always suffices for an n-byte message.
 *   moa_msg_gzip       : out_host[0 .. *out_bytes_host) = the compressed message.  MOA_ERR_RANGE if cap is too small.
 *   moa_msg_gunzip     : the inverse; checks the stream's CRC-32 and length.  MOA_ERR_SHAPE for a truncated or
 *                        corrupt stream, MOA_ERR_RANGE if the message does not fit cap.
 * Messages are limited to 2 GiB. */
int32_t moa_msg_gzip_bound(size_t n, size_t *bytes_host);
int32_t moa_msg_gzip(const void *msg_host, size_t n, void *out_host, size_t cap, size_t *out_bytes_host);
int32_t moa_msg_gunzip(const void *gz_host, size_t n, void *out_host, size_t cap, size_t *out_bytes_host);

/* y = x w^T, the projection every layer of the path is made of, for the ones the path leaves to the
 * caller (the drafter's LM head when the logits themselves are wanted, Sec. 2.1 LM_head(o); an MLP).
 *   x [R, K], w [N, K] row-major -> y [R, N], all in `dtype`.  Workspace optional
 *   (moa_linear_workspace_bytes; without it short-and-wide shapes take a slower kernel). */
int32_t moa_linear_workspace_bytes(int32_t dtype, int64_t R, int32_t K, int32_t N, size_t *bytes_host);
int32_t moa_linear(int32_t dtype, const void *x, int64_t R, int32_t K, const void *w, int32_t N, void *y,
                   void *ws, size_t ws_bytes, void *stream);

/* out [N, K] = w_outer [N, J] w_inner [J, K]: the product of two projection matrices that are applied
 * one after the other, computed once (fp32 accumulation, result in `dtype`).  Not on the hot path. */
int32_t moa_fold_projection(int32_t dtype, const void *w_outer, const void *w_inner, int32_t N, int32_t J,
                            int32_t K, void *out, void *stream);

/* One pass of the whole path on one stream (Alg. 1, one iteration of the outer loop with the
 * tree form of drafting): tree mask -> LSA of T_lsa new tokens -> CA memory append ->
 * CA of Mq query rows per sequence -> n_verify_layers tree-verify attentions -> accept walk;
 * optionally (sa_emb != NULL) the drafter's Self-Attention layer produces the CA's queries first.
 * The *_host members are HOST arrays of n_verify_layers device pointers.
 * Scheduling (`schedule`), all with the same ordering as seen from `stream`:
 *  MOA_SCHED_GROUPED (0, default): calls of the step that do not depend on each other and have the
 *    same shape share a launch: the CA query projection with the first verification layer's Q/K/V
 *    projection (the integer work -- tree masks, accept walk, memory lengths -- rides in the first
 *    workgroups of that grid); the two attention cores; the two output projections.
 *    Needs Mq == M, n_verify_layers >= 1, non-NULL CA and first-layer weights and the workspace
 *    moa_workspace_bytes asks for; otherwise the step runs as MOA_SCHED_SEQUENTIAL.  tok[], tgt[]
 *    and ca_len[] are read by the first launch of the step, so nothing in the step may produce them.
 *  MOA_SCHED_TWO_STREAM (1): the grouped launches, with the first of them (the CA query and first-layer
 *    Q/K/V projections, which depend on nothing else in the step) and the pass that adds up its slices on a
 *    second, library-owned stream that is forked from and joined back into `stream` with one event each,
 *    beside the LSA kernel on `stream`.  With lsa_w_packed the LSA kernel runs in a lean form that shares
 *    its compute units with the projection kernel; without, with its largest token tile, so that compute
 *    units are left over.  Same requirements as MOA_SCHED_GROUPED.  One side stream exists per device:
 *    steps of several host threads on one device are enqueued one after the other (a mutex), and the
 *    branch is joined back even when a launch fails half way.
 *    With the Self-Attention layer (sa_emb != NULL) and the LSA as one kernel, the branches are cut differently:
 *    `stream` carries the step's one long chain (tree masks, the Self-Attention layer, the CA query projection,
 *    the CA core and its output projection), the library's stream the LSA with the memory append and then the
 *    verification layers; a third event tells the CA core that the memory is complete.  The two attention
 *    cores are then launches of their own.
 *  MOA_SCHED_SEQUENTIAL (2): every stage enqueued on `stream` in the order above, one launch
 *    per stage, exactly as the single entry points would.
 * Integer results are identical under all three; floating-point results of 0 and 1 are
 * bit-identical (without the Self-Attention layer), those of 2, and of 1 with that layer, differ from
 * them only where the two attention cores end up with a different number of key slices (partials
 * merged in another order). */
enum { MOA_SCHED_GROUPED = 0, MOA_SCHED_TWO_STREAM = 1, MOA_SCHED_SEQUENTIAL = 2 };

typedef struct {
    const moa_shape_t *shape;
    int32_t B, M, Mq;
    /* tree */
    const int32_t *parent;  uint64_t *mask;  int32_t *depth;
    /* LSA */
    const void *lsa_hs;  int64_t T_lsa;
    const void *lsa_wq, *lsa_wk, *lsa_wv, *lsa_wo;
    void *lsa_out;                                /* [T_lsa, H_l*dh]; also the CA memory rows */
    /* CA memory append */
    const int32_t *tok_off;                       /* device [B+1], tok_off[B] <= T_lsa        */
    const void *ca_wk, *ca_wv;  void *ca_k, *ca_v;  int32_t *ca_len;  int32_t ca_P_cap;
    /* CA */
    const void *ca_xq, *ca_wq, *ca_wo;  void *ca_out;
    /* verification */
    int32_t n_verify_layers;
    const void *const *v_x_host, *const *v_wq_host, *const *v_wk_host, *const *v_wv_host, *const *v_wo_host;
    const void *const *v_kcache_host, *const *v_vcache_host;
    void *const *v_out_host, *const *v_ktree_host, *const *v_vtree_host;
    const int32_t *prefix_len;  int32_t P_cap;
    /* accept */
    const int32_t *tok, *tgt;  int32_t *path, *n_path, *bonus;
    int32_t *dev_status;  void *ws;  size_t ws_bytes;  void *stream;
    int32_t schedule;             /* MOA_SCHED_*                                                     */
    /* optional Self-Attention layer in front of the CA (Alg. 1: q <- SA_layer(token_embed(y)), then
     * CA_layer(q, kv)): with sa_emb != NULL the step first runs moa_self_attn_draft on the whole
     * tree (after the tree mask) and the CA takes sa_out as its queries; ca_xq is then ignored and
     * Mq must equal M.  sa_shape is `shape` with the layer's own n_kv_heads.                        */
    const moa_shape_t *sa_shape;
    const void *sa_emb;                           /* [B, M, d] token embeddings of the tree nodes    */
    const void *sa_wq, *sa_wk, *sa_wv, *sa_wo;
    const void *sa_kcache, *sa_vcache;            /* [B, Hkv_sa, sa_P_cap, dh], prefix_len[b] rows   */
    int32_t sa_P_cap;
    void *sa_k_draft, *sa_v_draft;                /* [B, Hkv_sa, M, dh] per-cycle draft cache (out)  */
    void *sa_out;                                 /* [B, M, d]: the CA's queries                     */
    /* optional: the products ca_wk lsa_wo and ca_wv lsa_wo ([Hkv*dh, H_l*dh], computed once with
     * moa_fold_projection).  With both, the grouped and two-stream schedules project the memory's new
     * keys / values straight from LSA's mean-folded heads in the launch that also applies lsa_wo
     * ((a Wo^T) Wk^T = a (Wk Wo)^T, exact in real arithmetic); lsa_out is still written.            */
    const void *ca_wk_lsa_wo, *ca_wv_lsa_wo;
    /* optional: lsa_wq / lsa_wk / lsa_wv packed by moa_lsa_pack_weights.  The step then runs the LSA's one-kernel
     * form from the packed copy wherever it runs that form at all; lsa_wq / lsa_wk / lsa_wv are still required
     * (the other form reads them).  Ignored for shapes that cannot be packed.                        */
    const void *lsa_w_packed;
} moa_step_args_t;

int32_t moa_draft_step(const moa_step_args_t *args);

/* Measurement aid (not part of the method; paper Appendix "Complexity Analysis" is the only place
 * that discusses where time goes).  When enabled, every kernel launch -- or, with only_kernel >= 0,
 * every launch of that kernel -- carries a start and a stop hipEvent attached to the dispatch
 * itself, so their difference is the kernel's own begin-to-end time on the device and a benchmark
 * can attribute time to single kernels.  Off by default; events are created on first use and
 * recycled.  moa_profile_collect waits for the recorded events (host synchronisation), sums them
 * per (launch site, kernel) into rows_host and forgets them.
 * moa_profile_sample_every(n) times only every n-th eligible launch (n >= 1, default 1).
 * Kernel and site ids are the indices accepted by the *_name functions ("?" past the end). */
typedef struct { int32_t site, kernel; int64_t launches; double total_ms; } moa_profile_row_t;
int32_t moa_profile_enable(int32_t on, int32_t only_kernel);
int32_t moa_profile_sample_every(int32_t n);
int32_t moa_profile_collect(moa_profile_row_t *rows_host, int32_t max_rows, int32_t *n_rows_host);
const char *moa_profile_kernel_name(int32_t kernel);
const char *moa_profile_site_name(int32_t site);

/* Testing aid (not part of the method).  The attention core of moa_cross_attn_draft, moa_tree_verify_attn,
 * moa_self_attn_draft, moa_tli_decoder_layer and moa_draft_step has two matrix-core forms for bf16 with head_dim 64
 * or 128 and picks one from the call's shape: one workgroup per 32 query rows walking the whole key range (short key
 * ranges, few workgroups) or the key range split over workgroups with a merging pass (everything else).  Both compute
 * the attention of Sec. 2.2 / 3.1.2; they differ in the order partial sums are merged.  This call forces one of them
 * for every later call of the process (MOA_ATTN_KERNEL_AUTO restores the choice by shape) so that a parity test can
 * run each case through both.  A forced form that a call cannot take (fp32, other head_dim, workspace too small for
 * the split form) falls back as the automatic choice would.  Host only, launches nothing; MOA_ERR_SHAPE for another
 * value.  Not thread-safe against calls in flight on other host threads (they see either value). */
enum { MOA_ATTN_KERNEL_AUTO = 0, MOA_ATTN_KERNEL_WHOLE = 1, MOA_ATTN_KERNEL_SPLIT = 2 };
int32_t moa_debug_force_attn_kernel(int32_t form);

/* The same for the Layer Self-Attention (moa_lsa, moa_draft_step): for bf16 with head_dim 128, at most 96 layers, an
 * input width in 64s and an even number of query heads per KV head, projection, attention over the layers and mean
 * run as ONE kernel that keeps the projected rows on the compute unit; other shapes take three kernels with the
 * projected rows in the workspace.  Both give the same bits where the three-kernel form also projects on the matrix
 * cores (d_lsa_in a multiple of 128), and agree within rounding otherwise.  MOA_LSA_KERNEL_SEPARATE forces the three-kernel form,
 * MOA_LSA_KERNEL_FUSED the one-kernel form wherever it applies; left to itself (_AUTO) the library takes the
 * one-kernel form except for at most 192 rows (T * n_layers) and for more than 1024 workgroups' worth of tokens whose
 * layer count leaves over a tenth of its last 32-row block empty, where the three kernels measured faster. */
enum { MOA_LSA_KERNEL_AUTO = 0, MOA_LSA_KERNEL_FUSED = 1, MOA_LSA_KERNEL_SEPARATE = 2 };
int32_t moa_debug_force_lsa_kernel(int32_t form);

/* Two probes of what the device delivers in practice, timed like any other kernel through the aid
 * above (kernels "k_probe_read", "k_probe_mfma"); a benchmark prints them beside the published
 * peaks.  moa_probe_read streams `bytes` (multiple of 16, 16-byte aligned device buffer) once with
 * plain coalesced loads.  moa_probe_mfma runs iters x 4 independent register-resident bf16
 * 32x32x16 MFMAs in each of 4096 wavefronts and returns the flop count in *flops_host.
 * scratch4: 4 writable device bytes (never written in practice).  Not part of the method. */
int32_t moa_probe_read(const void *buf, size_t bytes, void *scratch4, void *stream);
int32_t moa_probe_mfma(int32_t iters, void *scratch4, int64_t *flops_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif
