// C ABI of libmoa: argument checks on the host, workspace carving, kernel launches on the
// caller's stream.  No device allocation, no host synchronisation.
#include "../../include/moa.h"
#include "moa_common.h"

#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>

using namespace moa;

namespace {

thread_local char g_err[320] = "";

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

}  // namespace

// the same error record for entry points that live in other files
namespace moa {
int32_t api_fail(int32_t code, const char *msg) { return fail(code, "%s", msg); }
}  // namespace moa

namespace {

int32_t hip_fail(hipError_t e, const char *where)
{
    return fail(MOA_ERR_HIP, "%s: %s", where, hipGetErrorString(e));
}

// While a whole step is being validated no launch may happen: moa_draft_step runs every stage
// once with g_dry set (checks only), then for real.
thread_local bool g_dry = false;

#define MOA_TRY_HIP(expr, where)                              \
    do {                                                      \
        if (!g_dry) {                                         \
            hipError_t e_ = (expr);                           \
            if (e_ != hipSuccess) return hip_fail(e_, where); \
        }                                                     \
    } while (0)

size_t esize(int dtype) { return dtype == MOA_BF16 ? 2 : 4; }
size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

int32_t check_shape(const moa_shape_t *s, bool need_lsa)
{
    if (!s) return fail(MOA_ERR_NULL, "shape is NULL");
    if (s->dtype != MOA_F32 && s->dtype != MOA_BF16) return fail(MOA_ERR_DTYPE, "dtype %d", s->dtype);
    if (s->head_dim < 1 || s->head_dim > 256) return fail(MOA_ERR_SHAPE, "head_dim %d outside [1,256]", s->head_dim);
    if (need_lsa) {
        if (s->n_layers < 1 || s->d_lsa_in < 1 || s->lsa_q_heads < 1 || s->lsa_kv_heads < 1 ||
            s->lsa_q_heads % s->lsa_kv_heads)
            return fail(MOA_ERR_SHAPE, "LSA dims L=%d d_in=%d H_l=%d Hkv_l=%d", s->n_layers, s->d_lsa_in,
                        s->lsa_q_heads, s->lsa_kv_heads);
    } else {
        if (s->d_model < 1 || s->n_q_heads < 1 || s->n_kv_heads < 1 || s->n_q_heads % s->n_kv_heads)
            return fail(MOA_ERR_SHAPE, "dims d=%d H=%d Hkv=%d", s->d_model, s->n_q_heads, s->n_kv_heads);
    }
    return MOA_OK;
}

StoreSpec row_store(void *dst, int64_t ld)
{
    StoreSpec st = {};
    st.mode = StoreSpec::ROW;
    st.dst = dst;
    st.ld = ld;
    st.dh = 1;
    return st;
}

StoreSpec heads_store(void *dst, int heads, int dh, int cap, int rows_per_seq)
{
    StoreSpec st = {};
    st.mode = StoreSpec::HEADS;
    st.dst = dst;
    st.heads = heads;
    st.dh = dh;
    st.cap = cap;
    st.rows_per_seq = rows_per_seq;
    return st;
}

constexpr int64_t LSA_CHUNK = 256;    // tokens projected per pass (bounds the Q/K/V scratch)
constexpr int64_t LSA_OBLOCK = 4096;  // tokens per output-projection pass (one GEMM over many chunks' mean-folded heads)

size_t max2(size_t a, size_t b) { return a > b ? a : b; }

size_t lsa_ws_bytes(const moa_shape_t *s, int64_t T)
{
    const int64_t tc = T < LSA_CHUNK ? T : LSA_CHUNK, ob = T < LSA_OBLOCK ? T : LSA_OBLOCK;
    const size_t eq = (size_t)s->lsa_q_heads * s->head_dim, ekv = (size_t)s->lsa_kv_heads * s->head_dim;
    // the projections of a short chunk (the first and the last one can be) stream the weights and keep partial sums
    const int64_t tail = T % LSA_CHUNK;
    // the output projection may carry the memory's folded K/V projections as two more segments (draft step)
    size_t lin = linear_workspace_bytes(s->dtype, ob, (int)eq, (int)(eq + 2 * (size_t)s->n_kv_heads * s->head_dim));
    lin = max2(lin, linear_workspace_bytes(s->dtype, ob, (int)eq, (int)eq));
    lin = max2(lin, linear_workspace_bytes(s->dtype, tc * s->n_layers, s->d_lsa_in, (int)(eq + 2 * ekv)));
    if (tail) lin = max2(lin, linear_workspace_bytes(s->dtype, tail * s->n_layers, s->d_lsa_in, (int)(eq + 2 * ekv)));
    return align256((size_t)tc * s->n_layers * (eq + 2 * ekv) * esize(s->dtype)) + align256((size_t)ob * eq * esize(s->dtype)) +
           align256(lin);
}

// scratch shared by the projections' split-K partials and the attention core's split-KV partials
size_t attn_scratch_bytes(const moa_shape_t *s, int B, int Mq, int P_cap, bool tree)
{
    const int e = s->n_q_heads * s->head_dim, ekv = s->n_kv_heads * s->head_dim;
    const int64_t R = (int64_t)B * Mq;
    size_t n = attn_workspace_bytes(s->dtype, B, Mq, s->n_q_heads, s->n_kv_heads, s->head_dim, P_cap);
    n = max2(n, linear_workspace_bytes(s->dtype, R, s->d_model, e + (tree ? 2 * ekv : 0)));
    n = max2(n, linear_workspace_bytes(s->dtype, R, s->d_model, e));
    n = max2(n, linear_workspace_bytes(s->dtype, R, s->d_model, 2 * ekv));
    n = max2(n, linear_workspace_bytes(s->dtype, R, s->d_model, ekv));
    n = max2(n, linear_workspace_bytes(s->dtype, R, e, s->d_model));
    return align256(n);
}

size_t attn_ws_bytes(const moa_shape_t *s, int B, int Mq, int P_cap)
{
    const size_t e = (size_t)s->n_q_heads * s->head_dim;
    return 2 * align256((size_t)B * Mq * e * esize(s->dtype)) + attn_scratch_bytes(s, B, Mq, P_cap, true);
}

size_t append_ws_bytes(const moa_shape_t *s, int64_t T, int d_mem)
{
    const int ekv = s->n_kv_heads * s->head_dim;
    return align256(max2(linear_workspace_bytes(s->dtype, T, d_mem, 2 * ekv), linear_workspace_bytes(s->dtype, T, d_mem, ekv)));
}

// workspace split of the grouped step:
// [old lengths | CA queries | CA heads | verify queries | verify heads | scratch shared by every stage in turn]
struct GroupLayout {
    size_t len_bytes, qa, attn_each, scratch;
    size_t total() const { return len_bytes + 4 * qa + scratch; }
};

GroupLayout group_layout(const moa_shape_t *s, int B, int M, int P_cap, int ca_P_cap, int64_t T)
{
    GroupLayout L;
    const int e = s->n_q_heads * s->head_dim, ekv = s->n_kv_heads * s->head_dim;
    const int64_t R = (int64_t)B * M;
    L.len_bytes = align256((size_t)B * sizeof(int32_t));
    L.qa = align256((size_t)R * e * esize(s->dtype));
    const int cap = P_cap > ca_P_cap ? P_cap : ca_P_cap;
    L.attn_each = align256(attn_workspace_bytes(s->dtype, B, M, s->n_q_heads, s->n_kv_heads, s->head_dim, cap));
    size_t n = 2 * L.attn_each;
    n = max2(n, linear_workspace_bytes(s->dtype, R, s->d_model, 2 * e + 2 * ekv));
    n = max2(n, linear_workspace_bytes(s->dtype, R, e, 2 * s->d_model));
    n = max2(n, attn_ws_bytes(s, B, M, P_cap));                       // verification layers after the first
    n = max2(n, attn_ws_bytes(s, B, M, ca_P_cap));
    if (T > 0) {
        n = max2(n, lsa_ws_bytes(s, T));
        n = max2(n, append_ws_bytes(s, T, s->lsa_q_heads * s->head_dim));
    }
    L.scratch = align256(n);
    return L;
}

int32_t check_ws(const void *ws, size_t have, size_t need)
{
    if (need == 0) return MOA_OK;
    if (!ws) return fail(MOA_ERR_WORKSPACE, "workspace is NULL (%zu bytes needed)", need);
    if (((uintptr_t)ws) & 255) return fail(MOA_ERR_WORKSPACE, "workspace not 256-byte aligned");
    if (have < need) return fail(MOA_ERR_WORKSPACE, "workspace %zu bytes, %zu needed", have, need);
    return MOA_OK;
}

}  // namespace

extern "C" {

const char *moa_status_str(int32_t status)
{
    switch (status) {
    case MOA_OK: return "MOA_OK";
    case MOA_ERR_NULL: return "MOA_ERR_NULL";
    case MOA_ERR_SHAPE: return "MOA_ERR_SHAPE";
    case MOA_ERR_TREE: return "MOA_ERR_TREE";
    case MOA_ERR_RANGE: return "MOA_ERR_RANGE";
    case MOA_ERR_DTYPE: return "MOA_ERR_DTYPE";
    case MOA_ERR_WORKSPACE: return "MOA_ERR_WORKSPACE";
    case MOA_ERR_HIP: return "MOA_ERR_HIP";
    default: return "MOA_ERR_UNKNOWN";
    }
}

const char *moa_last_error(void) { return g_err; }

int32_t moa_workspace_bytes(const moa_shape_t *shape, int32_t B, int32_t P_cap, int32_t M, int64_t T_lsa,
                            size_t *bytes_host)
{
    if (!bytes_host) return fail(MOA_ERR_NULL, "bytes_host is NULL");
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (B < 1 || M < 1 || P_cap < 0 || T_lsa < 0) return fail(MOA_ERR_SHAPE, "B=%d M=%d P_cap=%d T_lsa=%lld", B, M, P_cap, (long long)T_lsa);
    size_t need = attn_ws_bytes(shape, B, M, P_cap);
    if (T_lsa > 0) {
        rc = check_shape(shape, true);
        if (rc) return rc;
        need = max2(need, lsa_ws_bytes(shape, T_lsa));
        need = max2(need, append_ws_bytes(shape, T_lsa, shape->lsa_q_heads * shape->head_dim));
        need = max2(need, append_ws_bytes(shape, T_lsa, shape->d_model));
        // moa_draft_step: grouped buffers, plus a second scratch region when it runs two branches side by side
        const GroupLayout L = group_layout(shape, B, M, P_cap, P_cap, T_lsa);
        need = max2(need, L.total() + L.scratch);
    }
    *bytes_host = need;
    return MOA_OK;
}

int32_t moa_tree_build(const int32_t *parent, int32_t B, int32_t M, uint64_t *mask, int32_t *depth,
                       int32_t *dev_status, void *stream)
{
    if (!parent || !mask || !depth) return fail(MOA_ERR_NULL, "tree_build: NULL pointer");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE) return fail(MOA_ERR_SHAPE, "tree_build: B=%d M=%d (M <= %d)", B, M, MOA_MAX_TREE);
    prof_set_site(S_TREE_BUILD);
    MOA_TRY_HIP(launch_tree_build(parent, B, M, mask, depth, dev_status, (hipStream_t)stream), "tree_build");
    return MOA_OK;
}

int32_t moa_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt, int32_t B, int32_t M,
                        int32_t *path, int32_t *n_path, int32_t *bonus, void *stream)
{
    if (!parent || !tok || !tgt || !path || !n_path || !bonus) return fail(MOA_ERR_NULL, "tree_accept: NULL pointer");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE) return fail(MOA_ERR_SHAPE, "tree_accept: B=%d M=%d (M <= %d)", B, M, MOA_MAX_TREE);
    prof_set_site(S_TREE_ACCEPT);
    MOA_TRY_HIP(launch_tree_accept(parent, tok, tgt, B, M, path, n_path, bonus, (hipStream_t)stream), "tree_accept");
    return MOA_OK;
}

}  // extern "C"

// Segments a caller inside the library adds to the LSA output projection's launch (same activations: the
// mean-folded heads); only honoured when all tokens fall into one output-projection block.  *taken reports it.
static thread_local const LinSeg *t_lsa_extra = nullptr;
static thread_local int t_lsa_nextra = 0;
static thread_local bool t_lsa_extra_taken = false;

// which form the Layer Self-Attention takes: 0 = the one-kernel form wherever its shapes allow, 1 = the same (a call
// it cannot take still falls back), 2 = always projection, attention and mean as separate kernels
static std::atomic<int> g_lsa_form{0};

// Whether a Layer Self-Attention pass over T tokens runs as the one kernel.  Left to itself the library keeps the
// separate kernels in two corners where they measured faster: a handful of rows (T L <= 192: the weight-streaming
// projection spreads the weights over every compute unit, the one-kernel form over T x 8 workgroups only -- 28 against
// 48 us for 5 tokens at the Llama-3-8B shape), and many tokens whose layer count fills its last 32-row block badly
// (L = 80 in 96 rows: 535 against 492 us for 256 tokens at the Llama-2-70B shape).
static bool lsa_takes_fused(const moa_shape_t *shape, int64_t T, const void *hs, const void *wq, const void *wk,
                            const void *wv, const void *abar)
{
    const int form = g_lsa_form.load(std::memory_order_relaxed);
    if (form == MOA_LSA_KERNEL_SEPARATE) return false;
    if (!(wq && wk && wv &&
          lsa_fused_ok(shape->dtype, shape->n_layers, shape->d_lsa_in, shape->lsa_q_heads, shape->lsa_kv_heads,
                       shape->head_dim, hs, wq, wk, wv, abar)))
        return false;
    if (form == MOA_LSA_KERNEL_FUSED) return true;
    const int64_t L = shape->n_layers, padded = (L + 31) / 32 * 32;
    if (T * L <= 192) return false;
    if (10 * padded > 11 * L && T * (shape->lsa_q_heads / 2) > 1024) return false;
    return true;
}

static LsaFusedCall lsa_fused_call(const moa_shape_t *shape, const void *hs, int64_t t0, int64_t tc, const void *wq,
                                   const void *wk, const void *wv, void *abar, const void *w_packed = nullptr)
{
    LsaFusedCall c = {};
    c.w_packed = w_packed;
    c.dtype = shape->dtype;
    c.hs = (const char *)hs + (size_t)t0 * shape->n_layers * shape->d_lsa_in * esize(shape->dtype);
    c.wq = wq;
    c.wk = wk;
    c.wv = wv;
    c.abar = abar;
    c.T = tc;
    c.L = shape->n_layers;
    c.d_in = shape->d_lsa_in;
    c.Hq = shape->lsa_q_heads;
    c.Hkv = shape->lsa_kv_heads;
    c.dh = shape->head_dim;
    return c;
}

// ---- the LSA stage in pieces: moa_lsa runs them in order; the grouped draft step puts other launches between them
static int32_t lsa_check(const moa_shape_t *shape, const void *hs, int64_t T, const void *wq, const void *wk,
                         const void *wv, const void *out, const void *ws, size_t ws_bytes)
{
    int32_t rc = check_shape(shape, true);
    if (rc) return rc;
    if (!hs || !out) return fail(MOA_ERR_NULL, "lsa: hs / out is NULL");
    if (T < 0) return fail(MOA_ERR_SHAPE, "lsa: T=%lld", (long long)T);
    const int L = shape->n_layers, dh = shape->head_dim, d_in = shape->d_lsa_in;
    const int eq = shape->lsa_q_heads * dh, ekv = shape->lsa_kv_heads * dh;
    if ((!wq && eq != d_in) || (!wk && ekv != d_in) || (!wv && ekv != d_in))
        return fail(MOA_ERR_SHAPE, "lsa: NULL weight needs matching widths (d_in=%d, H_l*dh=%d, Hkv_l*dh=%d)", d_in, eq, ekv);
    if (lsa_attn_lds_bytes(shape->dtype, L, dh) > 150 * 1024)
        return fail(MOA_ERR_SHAPE, "lsa: L=%d x head_dim=%d does not fit the LDS-resident score tile", L, dh);
    if (T == 0) return MOA_OK;
    return check_ws(ws, ws_bytes, lsa_ws_bytes(shape, T));
}

struct LsaBufs {
    char *qkv;        // [chunk tokens * L, eq + 2 ekv] projected rows of one chunk
    char *abar0;      // [output block tokens, eq] mean-folded heads
    char *lin_ws;     // partial sums of the projections
    size_t lin_ws_bytes;
};

static LsaBufs lsa_carve(const moa_shape_t *shape, int64_t T, void *ws, size_t ws_bytes)
{
    const size_t es = esize(shape->dtype);
    const int eq = shape->lsa_q_heads * shape->head_dim, ekv = shape->lsa_kv_heads * shape->head_dim;
    const int64_t tc_max = T < LSA_CHUNK ? T : LSA_CHUNK, ob_max = T < LSA_OBLOCK ? T : LSA_OBLOCK;
    LsaBufs b;
    b.qkv = (char *)ws;
    b.abar0 = b.qkv + align256((size_t)tc_max * shape->n_layers * (eq + 2 * ekv) * es);
    b.lin_ws = b.abar0 + align256((size_t)ob_max * eq * es);
    b.lin_ws_bytes = ws_bytes - (size_t)(b.lin_ws - (char *)ws);
    return b;
}

// tokens t0 .. t0 + tc: the Q/K/V projection (la->nseg == 0: nothing to project) and the attention over the layers
// that follows it.  The attention writes the mean-folded heads into `abar`.
static void lsa_chunk_args(const moa_shape_t *shape, const void *hs, int64_t t0, int64_t tc, const void *wq,
                           const void *wk, const void *wv, void *abar, const LsaBufs &b, LinArgs *la, LsaAttnArgs *aa)
{
    const int L = shape->n_layers, dh = shape->head_dim, d_in = shape->d_lsa_in;
    const int eq = shape->lsa_q_heads * dh, ekv = shape->lsa_kv_heads * dh, wide = eq + 2 * ekv;
    const size_t es = esize(shape->dtype);
    const char *x = (const char *)hs + (size_t)t0 * L * d_in * es;
    *la = LinArgs{};
    la->X = x;
    la->R = tc * L;
    la->K = d_in;
    la->ldx = d_in;
    la->ws = b.lin_ws;
    la->ws_bytes = b.lin_ws_bytes;
    *aa = LsaAttnArgs{};
    aa->dtype = shape->dtype;
    auto add = [&](const void *w, int n, int col, const void **ptr, int64_t *ldp) {
        if (w) {
            la->seg[la->nseg].W = w;
            la->seg[la->nseg].N = n;
            la->seg[la->nseg].st = row_store(b.qkv + (size_t)col * es, wide);
            ++la->nseg;
            *ptr = b.qkv + (size_t)col * es;
            *ldp = wide;
        } else {
            *ptr = x;
            *ldp = d_in;
        }
    };
    add(wq, eq, 0, &aa->q, &aa->ldq);
    add(wk, ekv, eq, &aa->k, &aa->ldk);
    add(wv, ekv, eq + ekv, &aa->v, &aa->ldv);
    aa->T = tc;
    aa->L = L;
    aa->Hq = shape->lsa_q_heads;
    aa->Hkv = shape->lsa_kv_heads;
    aa->dh = dh;
    aa->abar = abar;
}

// W_o on `rows` mean-folded tokens starting at token b0, plus up to three more segments on the same activations
static LinArgs lsa_oproj_args(const moa_shape_t *shape, int64_t b0, int64_t rows, const void *wo, void *out,
                              const LsaBufs &b, const LinSeg *extra, int nextra)
{
    const int eq = shape->lsa_q_heads * shape->head_dim;
    LinArgs lo = {};
    lo.X = b.abar0;
    lo.R = rows;
    lo.K = eq;
    lo.ldx = eq;
    lo.nseg = 1;
    lo.seg[0].W = wo;
    lo.seg[0].N = eq;
    lo.seg[0].st = row_store((char *)out + (size_t)b0 * eq * esize(shape->dtype), eq);
    for (int i = 0; i < nextra && lo.nseg < 4; ++i) lo.seg[lo.nseg++] = extra[i];
    lo.ws = b.lin_ws;
    lo.ws_bytes = b.lin_ws_bytes;
    return lo;
}

extern "C" {

// the LSA pass behind moa_lsa and moa_lsa_packed (arguments checked by the caller); with w_packed the one-kernel
// form runs whatever the token count, since the other form reads the plain matrices
static int32_t lsa_run(const moa_shape_t *shape, const void *hs, int64_t T, const void *wq, const void *wk, const void *wv,
                       const void *w_packed, const void *wo, void *out, void *ws, size_t ws_bytes, void *stream)
{
    const int dt = shape->dtype, eq = shape->lsa_q_heads * shape->head_dim;
    hipStream_t st = (hipStream_t)stream;
    const size_t es = esize(dt);
    const LsaBufs b = lsa_carve(shape, T, ws, ws_bytes);

    // One kernel for projection, attention over the layers and mean where the shapes allow: no projected row ever
    // reaches memory, so a pass covers a whole output-projection block of tokens; else chunks of LSA_CHUNK tokens
    // whose Q/K/V rows go through the workspace.
    const bool fused = w_packed || lsa_takes_fused(shape, T, hs, wq, wk, wv, wo ? (const void *)b.abar0 : out);
    const int64_t step = fused ? LSA_OBLOCK : LSA_CHUNK;
    for (int64_t t0 = 0; t0 < T; t0 += step) {
        const int64_t tc = (T - t0) < step ? (T - t0) : step;
        const int64_t b0 = (t0 / LSA_OBLOCK) * LSA_OBLOCK;            // first token of this output-projection block
        char *abar = wo ? b.abar0 + (size_t)(t0 - b0) * eq * es : (char *)out + (size_t)t0 * eq * es;
        if (fused) {
            prof_set_site(S_LSA_FUSED);
            MOA_TRY_HIP(launch_lsa_fused(lsa_fused_call(shape, hs, t0, tc, wq, wk, wv, abar, w_packed), st), "lsa: fused kernel");
        } else {
            LinArgs la;
            LsaAttnArgs aa;
            lsa_chunk_args(shape, hs, t0, tc, wq, wk, wv, abar, b, &la, &aa);
            prof_set_site(S_LSA_QKV);
            if (la.nseg) MOA_TRY_HIP(launch_linear(dt, la, st), "lsa: projection");
            prof_set_site(S_LSA_ATTN);
            MOA_TRY_HIP(launch_lsa_attn(aa, st), "lsa: attention over layers");
        }
        const bool block_done = t0 + tc >= T || (t0 + tc) % LSA_OBLOCK == 0;
        if (wo && block_done) {                                      // W_o once per block, on one row per token
            const bool extras = t_lsa_nextra > 0 && T <= LSA_OBLOCK;
            const LinArgs lo = lsa_oproj_args(shape, b0, t0 + tc - b0, wo, out, b, t_lsa_extra, extras ? t_lsa_nextra : 0);
            if (extras) t_lsa_extra_taken = true;
            prof_set_site(S_LSA_OPROJ);
            MOA_TRY_HIP(launch_linear(dt, lo, st), "lsa: output projection");
        }
    }
    return MOA_OK;
}

int32_t moa_lsa(const moa_shape_t *shape, const void *hs, int64_t T, const void *wq, const void *wk,
                const void *wv, const void *wo, void *out, void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = lsa_check(shape, hs, T, wq, wk, wv, out, ws, ws_bytes);
    if (rc || T == 0) return rc;
    return lsa_run(shape, hs, T, wq, wk, wv, nullptr, wo, out, ws, ws_bytes, stream);
}

// shapes whose LSA weights can be packed: exactly those the one-kernel form takes
static int32_t lsa_pack_check(const moa_shape_t *shape, const char *who)
{
    int32_t rc = check_shape(shape, true);
    if (rc) return rc;
    if (!lsa_fused_shape_ok(shape->dtype, shape->n_layers, shape->d_lsa_in, shape->lsa_q_heads, shape->lsa_kv_heads, shape->head_dim))
        return fail(MOA_ERR_SHAPE, "%s: packed LSA weights need bf16, head_dim 128, n_layers <= 96, d_lsa_in >= 128 in 64s and "
                                   "an even number of query heads per KV head", who);
    return MOA_OK;
}

int32_t moa_lsa_packed_weight_bytes(const moa_shape_t *shape, size_t *bytes_host)
{
    if (!bytes_host) return fail(MOA_ERR_NULL, "lsa_packed_weight_bytes: bytes_host is NULL");
    int32_t rc = lsa_pack_check(shape, "lsa_packed_weight_bytes");
    if (rc) return rc;
    *bytes_host = lsa_packed_weight_bytes(shape->d_lsa_in, shape->lsa_q_heads, shape->lsa_kv_heads, shape->head_dim);
    return MOA_OK;
}

int32_t moa_lsa_pack_weights(const moa_shape_t *shape, const void *wq, const void *wk, const void *wv, void *packed,
                             size_t packed_bytes, void *stream)
{
    int32_t rc = lsa_pack_check(shape, "lsa_pack_weights");
    if (rc) return rc;
    if (!wq || !wk || !wv || !packed) return fail(MOA_ERR_NULL, "lsa_pack_weights: NULL pointer");
    if ((((uintptr_t)wq) | ((uintptr_t)wk) | ((uintptr_t)wv) | ((uintptr_t)packed)) & 15)
        return fail(MOA_ERR_SHAPE, "lsa_pack_weights: pointers must be 16-byte aligned");
    const size_t need = lsa_packed_weight_bytes(shape->d_lsa_in, shape->lsa_q_heads, shape->lsa_kv_heads, shape->head_dim);
    if (packed_bytes < need) return fail(MOA_ERR_WORKSPACE, "lsa_pack_weights: packed buffer has %zu bytes, %zu needed", packed_bytes, need);
    prof_set_site(S_LSA_FUSED);
    MOA_TRY_HIP(launch_lsa_pack_weights(wq, wk, wv, packed, shape->d_lsa_in, shape->lsa_q_heads, shape->lsa_kv_heads, (hipStream_t)stream),
                "lsa_pack_weights");
    return MOA_OK;
}

int32_t moa_lsa_packed(const moa_shape_t *shape, const void *hs, int64_t T, const void *w_packed, const void *wo,
                       void *out, void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = lsa_pack_check(shape, "lsa_packed");
    if (rc) return rc;
    if (!hs || !out || !w_packed) return fail(MOA_ERR_NULL, "lsa_packed: hs / w_packed / out is NULL");
    if (T < 0) return fail(MOA_ERR_SHAPE, "lsa_packed: T=%lld", (long long)T);
    if ((((uintptr_t)hs) | ((uintptr_t)w_packed) | ((uintptr_t)out)) & 15)
        return fail(MOA_ERR_SHAPE, "lsa_packed: pointers must be 16-byte aligned");
    if (T == 0) return MOA_OK;
    rc = check_ws(ws, ws_bytes, lsa_ws_bytes(shape, T));
    if (rc) return rc;
    return lsa_run(shape, hs, T, nullptr, nullptr, nullptr, w_packed, wo, out, ws, ws_bytes, stream);
}

int32_t moa_debug_force_lsa_kernel(int32_t form)
{
    if (form < MOA_LSA_KERNEL_AUTO || form > MOA_LSA_KERNEL_SEPARATE)
        return fail(MOA_ERR_SHAPE, "debug_force_lsa_kernel: form must be MOA_LSA_KERNEL_AUTO / _FUSED / _SEPARATE");
    g_lsa_form.store(form, std::memory_order_relaxed);
    return MOA_OK;
}

int32_t moa_ca_kv_append(const moa_shape_t *shape, const void *mem_new, int64_t T, int32_t d_mem,
                         const int32_t *tok_off, int32_t B, const void *wk, const void *wv, void *kc, void *vc,
                         int32_t *ca_len, int32_t P_cap, int32_t *dev_status, void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!mem_new || !tok_off || !kc || !vc || !ca_len) return fail(MOA_ERR_NULL, "ca_kv_append: NULL pointer");
    if (ws && (((uintptr_t)ws) & 255)) return fail(MOA_ERR_WORKSPACE, "workspace not 256-byte aligned");
    if (B < 1 || T < 0 || d_mem < 1 || P_cap < 1) return fail(MOA_ERR_SHAPE, "ca_kv_append: B=%d T=%lld d_mem=%d P_cap=%d", B, (long long)T, d_mem, P_cap);
    const int dh = shape->head_dim, ekv = shape->n_kv_heads * dh, dt = shape->dtype;
    if ((!wk || !wv) && ekv != d_mem) return fail(MOA_ERR_SHAPE, "ca_kv_append: NULL weight needs d_mem == Hkv*dh");
    hipStream_t st = (hipStream_t)stream;
    StoreSpec sp = {};
    sp.mode = StoreSpec::APPEND;
    sp.heads = shape->n_kv_heads;
    sp.dh = dh;
    sp.cap = P_cap;
    sp.B = B;
    sp.row_base = ca_len;
    sp.tok_off = tok_off;
    sp.dev_status = dev_status;
    prof_set_site(S_APPEND_KV);
    if (T > 0) {
        LinArgs la = {};
        la.X = mem_new;
        la.R = T;
        la.K = d_mem;
        la.ldx = d_mem;
        la.ws = ws;              // optional here: without it the projection takes the slower kernel
        la.ws_bytes = ws_bytes;
        const void *w[2] = {wk, wv};
        void *dst[2] = {kc, vc};
        for (int i = 0; i < 2; ++i) {
            sp.dst = dst[i];
            if (w[i]) {
                la.seg[la.nseg].W = w[i];
                la.seg[la.nseg].N = ekv;
                la.seg[la.nseg].st = sp;
                ++la.nseg;
            } else {
                MOA_TRY_HIP(launch_scatter_copy(dt, mem_new, T, ekv, d_mem, sp, st), "ca_kv_append: copy");
            }
        }
        if (la.nseg) MOA_TRY_HIP(launch_linear(dt, la, st), "ca_kv_append: projection");
    }
    prof_set_site(S_APPEND_LEN);
    MOA_TRY_HIP(launch_append_lengths(tok_off, B, ca_len, P_cap, dev_status, st), "ca_kv_append: lengths");
    return MOA_OK;
}

// ---- one attention layer = projections, then core + output projection.  Shared by cross-attention
// (mask == NULL: no K/V projection, no tree rows) and tree verification.  The two halves can be put on
// different streams by moa_draft_step; each gets its own scratch.
struct AttnBufs {
    char *qbuf;        // [B*M, H*dh] projected queries
    char *abuf;        // [B*M, H*dh] concatenated heads before W_o
    char *scratch_p;   // split-K partials of the projections
    size_t scratch_p_bytes;
    char *scratch_c;   // split-KV partials of the core, then split-K partials of W_o
    size_t scratch_c_bytes;
};

// launch sites of the layer being run, {projections, core, output projection}; nullptr = by kind of layer
static thread_local const int *t_sites = nullptr;

static int32_t attn_check(const char *who, const moa_shape_t *shape, const void *wq, const void *wk, const void *wv,
                          bool tree)
{
    const int dh = shape->head_dim, e = shape->n_q_heads * dh, ekv = shape->n_kv_heads * dh, d = shape->d_model;
    if (!wq && e != d) return fail(MOA_ERR_SHAPE, "%s: NULL wq needs d == H*dh", who);
    if (tree && ((!wk || !wv) && ekv != d)) return fail(MOA_ERR_SHAPE, "%s: NULL wk/wv needs d == Hkv*dh", who);
    return MOA_OK;
}

// Q (and, for verification, the tree rows' K/V) projections; *q_out = where the queries are
// A call may cover only the nodes node0 .. node0+M-1 of a tree of M_total nodes (0 = the whole tree): the new
// rows' K/V then go to rows node0.. of slabs that hold M_total rows.
static int32_t attn_stage_project(const char *who, const moa_shape_t *shape, const void *x, int32_t B, int32_t M,
                                  const void *wq, const void *wk, const void *wv, bool tree, void *k_tree,
                                  void *v_tree, const AttnBufs &bf, hipStream_t st, const void **q_out,
                                  int32_t M_total = 0, int32_t node0 = 0, const RopeArgs *rope = nullptr)
{
    const int dh = shape->head_dim, H = shape->n_q_heads, Hkv = shape->n_kv_heads, d = shape->d_model;
    const int e = H * dh, ekv = Hkv * dh, dt = shape->dtype;
    const int64_t R = (int64_t)B * M;
    prof_set_site(t_sites ? t_sites[0] : (tree ? S_VERIFY_QKV : S_CA_QPROJ));
    LinArgs la = {};
    la.X = x;
    la.R = R;
    la.K = d;
    la.ldx = d;
    la.ws = bf.scratch_p;
    la.ws_bytes = bf.scratch_p_bytes;
    *q_out = x;
    if (wq) {
        la.seg[la.nseg].W = wq;
        la.seg[la.nseg].N = e;
        la.seg[la.nseg].st = row_store(bf.qbuf, e);
        ++la.nseg;
        *q_out = bf.qbuf;
    }
    if (tree) {
        const void *w[2] = {wk, wv};
        const size_t skip = (size_t)node0 * dh * esize(dt);          // first new row inside every slab
        void *dst[2] = {(char *)k_tree + skip, (char *)v_tree + skip};
        for (int i = 0; i < 2; ++i) {
            const StoreSpec sp = heads_store(dst[i], Hkv, dh, M_total ? M_total : M, M);
            if (w[i]) {
                la.seg[la.nseg].W = w[i];
                la.seg[la.nseg].N = ekv;
                la.seg[la.nseg].st = sp;
                ++la.nseg;
            } else {
                MOA_TRY_HIP(launch_scatter_copy(dt, x, R, ekv, d, sp, st), who);
            }
        }
    }
    // rotary positions (a reused decoder layer): on the way out of the projection where all three are projected here
    if (rope && la.nseg == 3) {
        la.epi = LinArgs::EPI_ROPE;
        la.rope = *rope;
    }
    if (la.nseg) MOA_TRY_HIP(launch_linear(dt, la, st), who);
    if (rope && la.nseg != 3 && !g_dry) {
        prof_set_site(S_TLI_ROPE);
        MOA_TRY_HIP(launch_rope(dt, rope->q, rope->k_draft, rope->prefix_len, rope->depth, rope->B, rope->Mn, rope->M, rope->node0,
                                rope->H, rope->Hkv, rope->dh, rope->theta, rope->P_cap, st), who);
    }
    return MOA_OK;
}

static AttnArgs attn_core_args(const moa_shape_t *shape, const void *q, int32_t B, int32_t M, const void *kcache,
                               const void *vcache, const int32_t *len, int32_t P_cap, const uint64_t *mask, void *dst,
                               void *k_tree, void *v_tree, int32_t *dev_status, void *scratch, size_t scratch_bytes,
                               int32_t M_total = 0, int32_t node0 = 0)
{
    AttnArgs aa = {};
    aa.dtype = shape->dtype;
    aa.q = q;
    aa.kcache = kcache;
    aa.vcache = vcache;
    aa.ktree = mask ? k_tree : nullptr;
    aa.vtree = mask ? v_tree : nullptr;
    aa.len = len;
    aa.mask = mask;
    aa.out = dst;
    aa.B = B;
    aa.Mq = M;
    aa.Mt = mask ? node0 + M : 0;        // keys: every node up to the last new one
    if (mask && M_total) {
        aa.tree_cap = M_total;
        aa.mask_rows = M_total;
        aa.mask_row0 = node0;
    }
    aa.H = shape->n_q_heads;
    aa.Hkv = shape->n_kv_heads;
    aa.dh = shape->head_dim;
    aa.P_cap = P_cap;
    aa.empty_is_error = mask ? 0 : 1;
    aa.dev_status = dev_status;
    aa.ws = scratch;
    aa.ws_bytes = scratch_bytes;
    return aa;
}

static LinSeg oproj_seg(const moa_shape_t *shape, const void *heads, const void *wo, void *out)
{
    LinSeg sg = {};
    sg.W = wo;
    sg.N = shape->d_model;
    sg.st = row_store(out, shape->d_model);
    sg.X = heads;
    sg.ldx = (int64_t)shape->n_q_heads * shape->head_dim;
    return sg;
}

static int32_t attn_stage_core(const char *who, const moa_shape_t *shape, const void *q, int32_t B, int32_t M,
                               const void *wo, const void *kcache, const void *vcache, const int32_t *len,
                               int32_t P_cap, const uint64_t *mask, void *out, void *k_tree, void *v_tree,
                               int32_t *dev_status, const AttnBufs &bf, hipStream_t st, int32_t M_total = 0,
                               int32_t node0 = 0, const NormArgs *norm = nullptr)
{
    const int e = shape->n_q_heads * shape->head_dim, dt = shape->dtype;
    const AttnArgs aa = attn_core_args(shape, q, B, M, kcache, vcache, len, P_cap, mask, wo ? (void *)bf.abuf : out,
                                       k_tree, v_tree, dev_status, bf.scratch_c, bf.scratch_c_bytes, M_total, node0);
    prof_set_site(t_sites ? t_sites[1] : (mask ? S_VERIFY_CORE : S_CA_CORE));
    MOA_TRY_HIP(launch_attn(aa, st), who);
    if (wo) {
        LinArgs lo = {};
        lo.X = bf.abuf;
        lo.R = (int64_t)B * M;
        lo.K = e;
        lo.ldx = e;
        lo.nseg = 1;
        lo.seg[0] = oproj_seg(shape, nullptr, wo, out);
        lo.seg[0].ldx = 0;
        lo.ws = bf.scratch_c;
        lo.ws_bytes = bf.scratch_c_bytes;
        if (norm) {                          // the block's residual and next norm on the way out (a reused decoder layer)
            lo.epi = LinArgs::EPI_ADD_NORM;
            lo.norm = *norm;
        }
        prof_set_site(t_sites ? t_sites[2] : (mask ? S_VERIFY_OPROJ : S_CA_OPROJ));
        MOA_TRY_HIP(launch_linear(dt, lo, st), who);
    }
    return MOA_OK;
}

// carve [qbuf | abuf | scratch] out of one region; projections and core share the scratch (same stream)
static AttnBufs attn_carve(const moa_shape_t *shape, int32_t B, int32_t M, void *ws, size_t ws_bytes)
{
    const size_t qa = align256((size_t)B * M * shape->n_q_heads * shape->head_dim * esize(shape->dtype));
    AttnBufs bf;
    bf.qbuf = (char *)ws;
    bf.abuf = bf.qbuf + qa;
    bf.scratch_p = bf.scratch_c = bf.abuf + qa;
    bf.scratch_p_bytes = bf.scratch_c_bytes = ws_bytes - 2 * qa;
    return bf;
}

static int32_t attention_layer(const char *who, const moa_shape_t *shape, const void *x, int32_t B, int32_t M,
                               const void *wq, const void *wk, const void *wv, const void *wo,
                               const void *kcache, const void *vcache, const int32_t *len, int32_t P_cap,
                               const uint64_t *mask, void *out, void *k_tree, void *v_tree, int32_t *dev_status,
                               void *ws, size_t ws_bytes, hipStream_t st, int32_t M_total = 0, int32_t node0 = 0)
{
    int32_t rc = attn_check(who, shape, wq, wk, wv, mask != nullptr);
    if (rc) return rc;
    rc = check_ws(ws, ws_bytes, attn_ws_bytes(shape, B, M, P_cap));
    if (rc) return rc;
    const AttnBufs bf = attn_carve(shape, B, M, ws, ws_bytes);
    const void *q = nullptr;
    rc = attn_stage_project(who, shape, x, B, M, wq, wk, wv, mask != nullptr, k_tree, v_tree, bf, st, &q, M_total, node0);
    if (rc) return rc;
    return attn_stage_core(who, shape, q, B, M, wo, kcache, vcache, len, P_cap, mask, out, k_tree, v_tree, dev_status,
                           bf, st, M_total, node0);
}

int32_t moa_cross_attn_draft(const moa_shape_t *shape, const void *xq, int32_t B, int32_t Mq, const void *wq,
                             const void *wo, const void *kc, const void *vc, const int32_t *ca_len, int32_t P_cap,
                             void *out, int32_t *dev_status, void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!xq || !kc || !vc || !ca_len || !out) return fail(MOA_ERR_NULL, "cross_attn_draft: NULL pointer");
    if (B < 1 || Mq < 1 || P_cap < 1) return fail(MOA_ERR_SHAPE, "cross_attn_draft: B=%d Mq=%d P_cap=%d", B, Mq, P_cap);
    if (!wo && shape->n_q_heads * shape->head_dim != shape->d_model)
        return fail(MOA_ERR_SHAPE, "cross_attn_draft: NULL wo needs d == H*dh");
    return attention_layer("cross_attn_draft", shape, xq, B, Mq, wq, nullptr, nullptr, wo, kc, vc, ca_len, P_cap,
                           nullptr, out, nullptr, nullptr, dev_status, ws, ws_bytes, (hipStream_t)stream);
}

int32_t moa_tree_verify_attn(const moa_shape_t *shape, const void *x, int32_t B, int32_t M, const void *wq,
                             const void *wk, const void *wv, const void *wo, const void *kcache,
                             const void *vcache, const int32_t *prefix_len, int32_t P_cap, const uint64_t *mask,
                             void *out, void *k_tree, void *v_tree, int32_t *dev_status, void *ws, size_t ws_bytes,
                             void *stream)
{
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!x || !prefix_len || !mask || !out || !k_tree || !v_tree) return fail(MOA_ERR_NULL, "tree_verify_attn: NULL pointer");
    if (P_cap > 0 && (!kcache || !vcache)) return fail(MOA_ERR_NULL, "tree_verify_attn: cache is NULL with P_cap > 0");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE || P_cap < 0) return fail(MOA_ERR_SHAPE, "tree_verify_attn: B=%d M=%d P_cap=%d (M <= %d)", B, M, P_cap, MOA_MAX_TREE);
    if (!wo && shape->n_q_heads * shape->head_dim != shape->d_model)
        return fail(MOA_ERR_SHAPE, "tree_verify_attn: NULL wo needs d == H*dh");
    return attention_layer("tree_verify_attn", shape, x, B, M, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap, mask,
                           out, k_tree, v_tree, dev_status, ws, ws_bytes, (hipStream_t)stream);
}

// ---- the same layer for callers that cannot bring a workspace: its scratch is a fixed array in device memory that
// belongs to the library's code object (every GPU that loads the library holds its own copy until the process ends).
// In host code the array's name is only a handle for hipGetSymbolAddress; the address a kernel can use is looked up
// once per device, with that device current, and kept.
#define MOA_NOALLOC_SCRATCH_BYTES ((size_t)32 << 20)
static __device__ __align__(256) unsigned char scratch[MOA_NOALLOC_SCRATCH_BYTES];

static int32_t noalloc_scratch_for_current_device(void **out)
{
    static std::mutex mu;
    static void *addr[16] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_fail(e, "tree_verify_attn_noalloc: hipGetDevice");
    if (dev < 0 || dev >= 16) return fail(MOA_ERR_HIP, "tree_verify_attn_noalloc: device %d outside the 16 supported", dev);
    std::lock_guard<std::mutex> lk(mu);
    if (!addr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) return hip_fail(e, "tree_verify_attn_noalloc: hipGetSymbolAddress(scratch)");
        addr[dev] = p;
    }
    *out = addr[dev];
    return MOA_OK;
}

int32_t moa_tree_verify_attn_noalloc(const moa_shape_t *shape, const void *x, int32_t B, int32_t M, const void *wq,
                                     const void *wk, const void *wv, const void *wo, const void *kcache,
                                     const void *vcache, const int32_t *prefix_len, int32_t P_cap,
                                     const uint64_t *mask, void *out, void *k_tree, void *v_tree,
                                     int32_t *dev_status, void *stream)
{
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!x || !prefix_len || !mask || !out || !k_tree || !v_tree) return fail(MOA_ERR_NULL, "tree_verify_attn_noalloc: NULL pointer");
    if (P_cap > 0 && (!kcache || !vcache)) return fail(MOA_ERR_NULL, "tree_verify_attn_noalloc: cache is NULL with P_cap > 0");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE || P_cap < 0)
        return fail(MOA_ERR_SHAPE, "tree_verify_attn_noalloc: B=%d M=%d P_cap=%d (M <= %d)", B, M, P_cap, MOA_MAX_TREE);
    if (!wo && shape->n_q_heads * shape->head_dim != shape->d_model)
        return fail(MOA_ERR_SHAPE, "tree_verify_attn_noalloc: NULL wo needs d == H*dh");
    const size_t need = attn_ws_bytes(shape, B, M, P_cap);
    if (need > MOA_NOALLOC_SCRATCH_BYTES)
        return fail(MOA_ERR_WORKSPACE, "tree_verify_attn_noalloc: this call needs %zu bytes of scratch, the built-in array holds %zu; "
                                       "use moa_tree_verify_attn with a workspace", need, MOA_NOALLOC_SCRATCH_BYTES);
    void *ws = nullptr;
    rc = noalloc_scratch_for_current_device(&ws);
    if (rc) return rc;
    // Nothing in the scratch has to start at zero: the projected queries, the heads and every partial sum or partial
    // attention result a later kernel reads are written by an earlier kernel of this same call.
    return attention_layer("tree_verify_attn_noalloc", shape, x, B, M, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap,
                           mask, out, k_tree, v_tree, dev_status, ws, MOA_NOALLOC_SCRATCH_BYTES, (hipStream_t)stream);
}

int32_t moa_self_attn_draft(const moa_shape_t *shape, const void *emb, int32_t B, int32_t M, int32_t node_begin,
                            int32_t Mn, const void *wq, const void *wk, const void *wv, const void *wo,
                            const void *kcache, const void *vcache, const int32_t *prefix_len, int32_t P_cap,
                            const uint64_t *mask, void *out, void *k_draft, void *v_draft, int32_t *dev_status,
                            void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!emb || !prefix_len || !mask || !out || !k_draft || !v_draft) return fail(MOA_ERR_NULL, "self_attn_draft: NULL pointer");
    if (P_cap > 0 && (!kcache || !vcache)) return fail(MOA_ERR_NULL, "self_attn_draft: cache is NULL with P_cap > 0");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE || P_cap < 0)
        return fail(MOA_ERR_SHAPE, "self_attn_draft: B=%d M=%d P_cap=%d (M <= %d)", B, M, P_cap, MOA_MAX_TREE);
    if (node_begin < 0 || Mn < 1 || node_begin + Mn > M)
        return fail(MOA_ERR_RANGE, "self_attn_draft: nodes %d..%d of a tree of %d", node_begin, node_begin + Mn - 1, M);
    if (!wo && shape->n_q_heads * shape->head_dim != shape->d_model)
        return fail(MOA_ERR_SHAPE, "self_attn_draft: NULL wo needs d == H*dh");
    static const int sites[3] = {S_SA_QKV, S_SA_CORE, S_SA_OPROJ};
    t_sites = sites;
    rc = attention_layer("self_attn_draft", shape, emb, B, Mn, wq, wk, wv, wo, kcache, vcache, prefix_len, P_cap, mask,
                         out, k_draft, v_draft, dev_status, ws, ws_bytes, (hipStream_t)stream, M, node_begin);
    t_sites = nullptr;
    return rc;
}

// the optional Self-Attention layer in front of the cross-attention: tree mask, then the layer on the whole tree
static int32_t step_self_attn_check(const moa_step_args_t *a)
{
    if (!a->sa_shape || !a->sa_out) return fail(MOA_ERR_NULL, "draft_step: sa_shape / sa_out is NULL");
    if (a->Mq != a->M) return fail(MOA_ERR_SHAPE, "draft_step: the Self-Attention layer needs Mq == M");
    if (a->sa_shape->d_model != a->shape->d_model || a->sa_shape->dtype != a->shape->dtype)
        return fail(MOA_ERR_SHAPE, "draft_step: sa_shape must have the step's d_model and dtype");
    return MOA_OK;
}

static int32_t step_self_attn_layer(const moa_step_args_t *a, void *ws, size_t ws_bytes, void *stream)
{
    return moa_self_attn_draft(a->sa_shape, a->sa_emb, a->B, a->M, 0, a->M, a->sa_wq, a->sa_wk, a->sa_wv, a->sa_wo,
                               a->sa_kcache, a->sa_vcache, a->prefix_len, a->sa_P_cap, a->mask, a->sa_out,
                               a->sa_k_draft, a->sa_v_draft, a->dev_status, ws, ws_bytes, stream);
}

static int32_t step_self_attn(const moa_step_args_t *a)
{
    int32_t rc = step_self_attn_check(a);
    if (rc) return rc;
    rc = moa_tree_build(a->parent, a->B, a->M, a->mask, a->depth, a->dev_status, a->stream);
    if (rc) return rc;
    return step_self_attn_layer(a, a->ws, a->ws_bytes, a->stream);
}

// ---- a reused LLM decoder layer (Target Layer Inference)
// workspace: [attention stage (queries | heads | scratch) | split-K scratch of the MLP projections |
//             normed rows | projection result | residual stream (fp32) | gate, up | activation]
// scratch of the MLP half of a pre-norm block
struct MlpBufs {
    char *lin;        // partial sums of the projections
    size_t lin_bytes;
    char *n;          // [R, d] normalised stream
    char *tmp;        // [R, d] down projection where no kernel adds the residual on the way out
    float *h;         // [R, d] the stream in single precision
    char *gu;         // [R, 2 d_ff] gate | up where no kernel applies the activation on the way out
    char *act;        // [R, d_ff]
};

// h = x + res (res may be NULL); out = h + Wdown(silu(Wgate n) * Wup n), n = rmsnorm(h) * g.
// sites = launch sites of {norm, gate/up projection, down projection}
static int32_t mlp_block_run(const char *who, int dt, const void *x, const void *res, int64_t R, int d, int d_ff,
                             const void *g, const void *w_gate, const void *w_up, const void *w_down, float eps, void *out,
                             const MlpBufs &b, const int *sites, hipStream_t st, bool normed = false)
{
    const size_t es = esize(dt);
    if (!normed) {                           // else b.h and b.n are there already (the projection in front made them)
        prof_set_site(sites[0]);
        MOA_TRY_HIP(launch_rmsnorm(dt, x, res, R, d, g, eps, b.h, b.n, st), who);
    }
    LinArgs lg = {};
    lg.X = b.n;
    lg.R = R;
    lg.K = d;
    lg.ldx = d;
    lg.nseg = 2;
    lg.seg[0].W = w_gate;
    lg.seg[0].N = d_ff;
    lg.seg[0].st = row_store(b.gu, 2 * (int64_t)d_ff);
    lg.seg[1].W = w_up;
    lg.seg[1].N = d_ff;
    lg.seg[1].st = row_store(b.gu + (size_t)d_ff * es, 2 * (int64_t)d_ff);
    lg.ws = b.lin;
    lg.ws_bytes = b.lin_bytes;
    lg.epi = LinArgs::EPI_SWIGLU;            // act = silu(gate) * up, by the kernel that sums the K slices when there is one
    lg.epi_out = b.act;
    prof_set_site(sites[1]);
    MOA_TRY_HIP(launch_linear(dt, lg, st), who);
    LinArgs ld = {};
    ld.X = b.act;
    ld.R = R;
    ld.K = d_ff;
    ld.ldx = d_ff;
    ld.nseg = 1;
    ld.seg[0].W = w_down;
    ld.seg[0].N = d;
    ld.seg[0].st = row_store(b.tmp, d);
    ld.ws = b.lin;
    ld.ws_bytes = b.lin_bytes;
    ld.epi = LinArgs::EPI_ADD_F32;           // out = h + down projection (the block's residual)
    ld.epi_res = b.h;
    ld.epi_out = out;
    prof_set_site(sites[2]);
    MOA_TRY_HIP(launch_linear(dt, ld, st), who);
    return MOA_OK;
}

struct TliBufs {
    char *attn, *lin, *n, *tmp, *gu, *act;
    float *h1;
    size_t attn_bytes, lin_bytes, total;
};

static TliBufs tli_carve(const moa_shape_t *s, int32_t d_ff, int32_t B, int32_t Mn, int32_t P_cap, void *ws)
{
    const int64_t R = (int64_t)B * Mn;
    const size_t es = esize(s->dtype), d = (size_t)s->d_model;
    TliBufs t;
    size_t off = 0;
    // (sizes are measured with ws == NULL: no pointer arithmetic on a null base)
    auto take = [&](size_t bytes) { char *p = ws ? (char *)ws + off : nullptr; off += align256(bytes); return p; };
    t.attn_bytes = align256(attn_ws_bytes(s, B, Mn, P_cap));
    t.attn = take(t.attn_bytes);
    t.lin_bytes = align256(max2(linear_workspace_bytes(s->dtype, R, s->d_model, 2 * d_ff),
                                linear_workspace_bytes(s->dtype, R, d_ff, s->d_model)));
    t.lin = take(t.lin_bytes);
    t.n = take((size_t)R * d * es);
    t.tmp = take((size_t)R * d * es);
    t.h1 = (float *)take((size_t)R * d * sizeof(float));
    t.gu = take((size_t)R * 2 * d_ff * es);
    t.act = take((size_t)R * d_ff * es);
    t.total = off;
    return t;
}

int32_t moa_tli_workspace_bytes(const moa_shape_t *shape, const moa_decoder_cfg_t *cfg, int32_t B, int32_t P_cap,
                                int32_t M, size_t *bytes_host)
{
    if (!bytes_host || !cfg) return fail(MOA_ERR_NULL, "tli_workspace_bytes: NULL pointer");
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (B < 1 || M < 1 || P_cap < 0 || cfg->d_ff < 1) return fail(MOA_ERR_SHAPE, "B=%d M=%d P_cap=%d d_ff=%d", B, M, P_cap, cfg->d_ff);
    *bytes_host = tli_carve(shape, cfg->d_ff, B, M, P_cap, nullptr).total;
    return MOA_OK;
}

int32_t moa_tli_decoder_layer(const moa_shape_t *shape, const moa_decoder_cfg_t *cfg, const void *x, int32_t B,
                              int32_t M, int32_t node_begin, int32_t Mn, const void *g_attn, const void *wq,
                              const void *wk, const void *wv, const void *wo, const void *g_mlp, const void *w_gate,
                              const void *w_up, const void *w_down, const void *kcache, const void *vcache,
                              const int32_t *prefix_len, int32_t P_cap, const uint64_t *mask, const int32_t *depth,
                              void *out, void *k_draft, void *v_draft, int32_t *dev_status, void *ws, size_t ws_bytes,
                              void *stream)
{
    const char *who = "tli_decoder_layer";
    int32_t rc = check_shape(shape, false);
    if (rc) return rc;
    if (!cfg || !x || !g_attn || !wq || !wk || !wv || !wo || !g_mlp || !w_gate || !w_up || !w_down || !prefix_len ||
        !mask || !depth || !out || !k_draft || !v_draft)
        return fail(MOA_ERR_NULL, "%s: NULL pointer", who);
    if (P_cap > 0 && (!kcache || !vcache)) return fail(MOA_ERR_NULL, "%s: cache is NULL with P_cap > 0", who);
    if (B < 1 || M < 1 || M > MOA_MAX_TREE || P_cap < 0)
        return fail(MOA_ERR_SHAPE, "%s: B=%d M=%d P_cap=%d (M <= %d)", who, B, M, P_cap, MOA_MAX_TREE);
    if (node_begin < 0 || Mn < 1 || node_begin + Mn > M)
        return fail(MOA_ERR_RANGE, "%s: nodes %d..%d of a tree of %d", who, node_begin, node_begin + Mn - 1, M);
    if (cfg->d_ff < 1 || !(cfg->rms_eps >= 0.f) || !(cfg->rope_theta > 0.f) || (shape->head_dim & 1))
        return fail(MOA_ERR_SHAPE, "%s: d_ff=%d rms_eps=%g rope_theta=%g head_dim=%d (even)", who, cfg->d_ff,
                    (double)cfg->rms_eps, (double)cfg->rope_theta, shape->head_dim);
    const TliBufs t = tli_carve(shape, cfg->d_ff, B, Mn, P_cap, ws);
    rc = check_ws(ws, ws_bytes, t.total);
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const int dt = shape->dtype, d = shape->d_model, d_ff = cfg->d_ff;
    const int64_t R = (int64_t)B * Mn;

    // attention block: norm, Q/K/V, rotary positions, tree attention over cache + own path, output projection
    prof_set_site(S_TLI_NORM);
    MOA_TRY_HIP(launch_rmsnorm(dt, x, nullptr, R, d, g_attn, cfg->rms_eps, nullptr, t.n, st), who);
    static const int sites[3] = {S_TLI_QKV, S_TLI_CORE, S_TLI_OPROJ};
    t_sites = sites;
    const AttnBufs bf = attn_carve(shape, B, Mn, t.attn, t.attn_bytes);
    const void *q = nullptr;
    RopeArgs rope = {};
    rope.q = bf.qbuf;
    rope.k_draft = k_draft;
    rope.prefix_len = prefix_len;
    rope.depth = depth;
    rope.B = B;
    rope.Mn = Mn;
    rope.M = M;
    rope.node0 = node_begin;
    rope.H = shape->n_q_heads;
    rope.Hkv = shape->n_kv_heads;
    rope.dh = shape->head_dim;
    rope.P_cap = P_cap;
    rope.theta = (double)cfg->rope_theta;
    rc = attn_stage_project(who, shape, t.n, B, Mn, wq, wk, wv, true, k_draft, v_draft, bf, st, &q, M, node_begin, &rope);
    // W_o, then the residual and the MLP's norm: h1 = x + attention output, n = rmsnorm(h1) g_mlp
    NormArgs nm = {};
    nm.x = x;
    nm.g = g_mlp;
    nm.eps = cfg->rms_eps;
    nm.h = t.h1;
    nm.n = t.n;
    if (rc == MOA_OK)
        rc = attn_stage_core(who, shape, q, B, Mn, wo, kcache, vcache, prefix_len, P_cap, mask, t.tmp, k_draft, v_draft,
                             dev_status, bf, st, M, node_begin, &nm);
    t_sites = nullptr;
    if (rc) return rc;

    // MLP block: residual + norm, gate and up projections side by side, gated activation, down projection, residual
    MlpBufs mb;
    mb.lin = t.lin;
    mb.lin_bytes = t.lin_bytes;
    mb.n = t.n;
    mb.tmp = t.tmp;
    mb.h = t.h1;
    mb.gu = t.gu;
    mb.act = t.act;
    static const int mlp_sites[3] = {S_TLI_NORM, S_TLI_GATE_UP, S_TLI_DOWN};
    return mlp_block_run(who, dt, x, t.tmp, R, d, d_ff, g_mlp, w_gate, w_up, w_down, cfg->rms_eps, out, mb, mlp_sites, st, true);
}

// ---- the drafter's own layers: pre-norm in front of an attention sub-layer, MLP sub-block behind it
static MlpBufs mlp_carve(int dtype, int64_t R, int d, int d_ff, void *ws, size_t *total)
{
    const size_t es = esize(dtype);
    MlpBufs b;
    size_t off = 0;
    auto take = [&](size_t bytes) { char *p = ws ? (char *)ws + off : nullptr; off += align256(bytes); return p; };
    b.lin_bytes = align256(max2(linear_workspace_bytes(dtype, R, d, 2 * d_ff), linear_workspace_bytes(dtype, R, d_ff, d)));
    b.lin = take(b.lin_bytes);
    b.n = take((size_t)R * d * es);
    b.tmp = take((size_t)R * d * es);
    b.h = (float *)take((size_t)R * d * sizeof(float));
    b.gu = take((size_t)R * 2 * d_ff * es);
    b.act = take((size_t)R * d_ff * es);
    *total = off;
    return b;
}

static int32_t mlp_check(const char *who, int32_t dtype, int64_t R, int32_t d, int32_t d_ff, float eps)
{
    if (dtype != MOA_F32 && dtype != MOA_BF16) return fail(MOA_ERR_DTYPE, "%s: dtype %d", who, dtype);
    const int64_t widest = 2 * (int64_t)d_ff > d ? 2 * (int64_t)d_ff : d;      // longest row any kernel of the block walks
    if (R < 0 || d < 1 || d_ff < 1 || R > ((int64_t)1 << 40) / widest)
        return fail(MOA_ERR_SHAPE, "%s: R=%lld d=%d d_ff=%d", who, (long long)R, d, d_ff);
    if (!(eps >= 0.f)) return fail(MOA_ERR_SHAPE, "%s: rms_eps=%g", who, (double)eps);
    return MOA_OK;
}

int32_t moa_mlp_block_workspace_bytes(int32_t dtype, int64_t R, int32_t d, int32_t d_ff, size_t *bytes_host)
{
    if (!bytes_host) return fail(MOA_ERR_NULL, "mlp_block_workspace_bytes: NULL pointer");
    int32_t rc = mlp_check("mlp_block_workspace_bytes", dtype, R, d, d_ff, 0.f);
    if (rc) return rc;
    mlp_carve(dtype, R, d, d_ff, nullptr, bytes_host);
    return MOA_OK;
}

int32_t moa_mlp_block(int32_t dtype, const void *x, const void *res, int64_t R, int32_t d, int32_t d_ff, const void *g,
                      const void *w_gate, const void *w_up, const void *w_down, float rms_eps, void *out, void *ws,
                      size_t ws_bytes, void *stream)
{
    const char *who = "mlp_block";
    int32_t rc = mlp_check(who, dtype, R, d, d_ff, rms_eps);
    if (rc) return rc;
    if (R == 0) return MOA_OK;             // nothing is touched, so nothing has to be there
    if (!x || !g || !w_gate || !w_up || !w_down || !out) return fail(MOA_ERR_NULL, "%s: NULL pointer", who);
    size_t need = 0;
    const MlpBufs mb = mlp_carve(dtype, R, d, d_ff, ws, &need);
    rc = check_ws(ws, ws_bytes, need);
    if (rc) return rc;
    static const int sites[3] = {S_MLP_NORM, S_MLP_GATE_UP, S_MLP_DOWN};
    return mlp_block_run(who, dtype, x, res, R, d, d_ff, g, w_gate, w_up, w_down, rms_eps, out, mb, sites, (hipStream_t)stream);
}

int32_t moa_rmsnorm(int32_t dtype, const void *x, int64_t R, int32_t d, const void *g, float rms_eps, void *out, void *stream)
{
    int32_t rc = mlp_check("rmsnorm", dtype, R, d, 1, rms_eps);
    if (rc) return rc;
    if (R == 0) return MOA_OK;
    if (!x || !g || !out) return fail(MOA_ERR_NULL, "rmsnorm: NULL pointer");
    prof_set_site(S_MLP_NORM);
    MOA_TRY_HIP(launch_rmsnorm(dtype, x, nullptr, R, d, g, rms_eps, nullptr, out, (hipStream_t)stream), "rmsnorm");
    return MOA_OK;
}

int32_t moa_fold_projection(int32_t dtype, const void *w_outer, const void *w_inner, int32_t N, int32_t J, int32_t K,
                            void *out, void *stream)
{
    if (!w_outer || !w_inner || !out) return fail(MOA_ERR_NULL, "fold_projection: NULL pointer");
    if (dtype != MOA_F32 && dtype != MOA_BF16) return fail(MOA_ERR_DTYPE, "dtype %d", dtype);
    if (N < 1 || J < 1 || K < 1) return fail(MOA_ERR_SHAPE, "fold_projection: N=%d J=%d K=%d", N, J, K);
    MOA_TRY_HIP(launch_fold_weights(dtype, w_outer, w_inner, N, J, K, out, (hipStream_t)stream), "fold_projection");
    return MOA_OK;
}

int32_t moa_linear_workspace_bytes(int32_t dtype, int64_t R, int32_t K, int32_t N, size_t *bytes_host)
{
    if (!bytes_host) return fail(MOA_ERR_NULL, "linear_workspace_bytes: bytes_host is NULL");
    if (dtype != MOA_F32 && dtype != MOA_BF16) return fail(MOA_ERR_DTYPE, "dtype %d", dtype);
    if (R < 0 || K < 1 || N < 1) return fail(MOA_ERR_SHAPE, "linear_workspace_bytes: R=%lld K=%d N=%d", (long long)R, K, N);
    *bytes_host = align256(linear_workspace_bytes(dtype, R, K, N));
    return MOA_OK;
}

int32_t moa_linear(int32_t dtype, const void *x, int64_t R, int32_t K, const void *w, int32_t N, void *y, void *ws,
                   size_t ws_bytes, void *stream)
{
    if (!x || !w || !y) return fail(MOA_ERR_NULL, "linear: NULL pointer");
    if (dtype != MOA_F32 && dtype != MOA_BF16) return fail(MOA_ERR_DTYPE, "dtype %d", dtype);
    if (R < 0 || K < 1 || N < 1) return fail(MOA_ERR_SHAPE, "linear: R=%lld K=%d N=%d", (long long)R, K, N);
    if (ws && (((uintptr_t)ws) & 255)) return fail(MOA_ERR_WORKSPACE, "workspace not 256-byte aligned");
    if (R == 0) return MOA_OK;
    LinArgs la = {};
    la.X = x;
    la.R = R;
    la.K = K;
    la.ldx = K;
    la.nseg = 1;
    la.seg[0].W = w;
    la.seg[0].N = N;
    la.seg[0].st = row_store(y, N);
    la.ws = ws;                      // optional: without it a slower kernel takes the short-and-wide shapes
    la.ws_bytes = ws_bytes;
    prof_set_site(S_LINEAR);
    MOA_TRY_HIP(launch_linear(dtype, la, (hipStream_t)stream), "linear");
    return MOA_OK;
}

// The packed copy of the LSA weights a step may use: only where the one-kernel form runs anyway (the other form
// reads the plain matrices), and only if it is aligned like every other operand of that kernel.
static const void *step_lsa_packed(const moa_step_args_t *a)
{
    if (!a->lsa_w_packed || (((uintptr_t)a->lsa_w_packed) & 15)) return nullptr;
    return lsa_takes_fused(a->shape, a->T_lsa, a->lsa_hs, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->ws) ? a->lsa_w_packed : nullptr;
}

// moa_lsa for a step: the same checks, and the packed weights where they apply
static int32_t step_lsa(const moa_step_args_t *a, void *ws, size_t ws_bytes, void *stream)
{
    int32_t rc = lsa_check(a->shape, a->lsa_hs, a->T_lsa, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->lsa_out, ws, ws_bytes);
    if (rc || a->T_lsa == 0) return rc;
    return lsa_run(a->shape, a->lsa_hs, a->T_lsa, a->lsa_wq, a->lsa_wk, a->lsa_wv, step_lsa_packed(a), a->lsa_wo, a->lsa_out,
                   ws, ws_bytes, stream);
}

static int32_t draft_step_stages(const moa_step_args_t *a)
{
    int32_t rc = moa_tree_build(a->parent, a->B, a->M, a->mask, a->depth, a->dev_status, a->stream);
    if (rc) return rc;
    rc = step_lsa(a, a->ws, a->ws_bytes, a->stream);
    if (rc) return rc;
    const int d_mem = a->shape->lsa_q_heads * a->shape->head_dim;
    rc = moa_ca_kv_append(a->shape, a->lsa_out, a->T_lsa, d_mem, a->tok_off, a->B, a->ca_wk, a->ca_wv, a->ca_k,
                          a->ca_v, a->ca_len, a->ca_P_cap, a->dev_status, a->ws, a->ws_bytes, a->stream);
    if (rc) return rc;
    rc = moa_cross_attn_draft(a->shape, a->ca_xq, a->B, a->Mq, a->ca_wq, a->ca_wo, a->ca_k, a->ca_v, a->ca_len,
                              a->ca_P_cap, a->ca_out, a->dev_status, a->ws, a->ws_bytes, a->stream);
    if (rc) return rc;
    for (int l = 0; l < a->n_verify_layers; ++l) {
        rc = moa_tree_verify_attn(a->shape, a->v_x_host[l], a->B, a->M, a->v_wq_host[l], a->v_wk_host[l],
                                  a->v_wv_host[l], a->v_wo_host[l], a->v_kcache_host[l], a->v_vcache_host[l],
                                  a->prefix_len, a->P_cap, a->mask, a->v_out_host[l], a->v_ktree_host[l],
                                  a->v_vtree_host[l], a->dev_status, a->ws, a->ws_bytes, a->stream);
        if (rc) return rc;
    }
    return moa_tree_accept(a->parent, a->tok, a->tgt, a->B, a->M, a->path, a->n_path, a->bonus, a->stream);
}

// ---- the step with its independent pieces launched together.
// Two calls that do not depend on each other and have the same shape share one launch: the three integer
// kernels; the cross-attention query projection with the first verification layer's Q/K/V projection; the two
// attention cores; the two output projections.  At decode sizes each of these kernels is short enough that
// launch latency and the ramp-up/drain of a grid are a visible part of it, and the two halves of a pair fill
// the chip better than either alone.  Per-output arithmetic is that of the separate launches (same kernels,
// same split counts along K).  The pieces below are shared by the one-stream (grouped) and the two-stream
// schedule.
struct StepBufs {
    int32_t *old_len;              // memory lengths before this step's append
    char *q_ca, *h_ca, *q_v, *h_v; // projected queries / concatenated heads of the CA and of verification layer 0
};

static bool pieces_ok(const moa_step_args_t *a)
{
    if (a->n_verify_layers < 1 || a->Mq != a->M) return false;
    return a->ca_wq && a->ca_wo && a->v_wq_host[0] && a->v_wk_host[0] && a->v_wv_host[0] && a->v_wo_host[0];
}

// tree masks, accepted paths, memory lengths (the old lengths are kept for the append)
static StepSmallArgs small_args(const moa_step_args_t *a, const StepBufs &bf)
{
    StepSmallArgs sm = {};
    sm.parent = a->parent;
    sm.tok = a->tok;
    sm.tgt = a->tgt;
    sm.tok_off = a->tok_off;
    sm.mask = a->mask;
    sm.depth = a->depth;
    sm.path = a->path;
    sm.n_path = a->n_path;
    sm.bonus = a->bonus;
    sm.ca_len = a->ca_len;
    sm.old_len = bf.old_len;
    sm.dev_status = a->dev_status;
    sm.B = a->B;
    sm.M = a->M;
    sm.cap = a->ca_P_cap;
    return sm;
}

static int32_t piece_small(const moa_step_args_t *a, const StepBufs &bf, hipStream_t st)
{
    prof_set_site(S_STEP_SMALL);
    MOA_TRY_HIP(launch_step_small(small_args(a, bf), st), "draft_step: tree/lengths");
    return MOA_OK;
}

// cross-attention queries + first verification layer's Q/K/V in one launch (which = 3), or the queries (1) or the
// verification layer's three (2) alone
// with_small: the integer work rides in spare workgroups of this launch's grid instead of being a launch of its
// own (nothing before the LSA chain's append and the attention cores needs its results).  sum_out: the pass that
// adds up this projection's K slices is left to the caller (scr is then a region nobody else writes until that pass
// has run).
static int32_t piece_projections(const moa_step_args_t *a, const StepBufs &bf, void *scr, size_t scr_bytes, hipStream_t st,
                                 bool with_small, SumArgs *sum_out = nullptr, int which = 3)
{
    const moa_shape_t *sh = a->shape;
    const int dh = sh->head_dim, Hkv = sh->n_kv_heads, d = sh->d_model, M = a->M;
    const int e = sh->n_q_heads * dh, ekv = Hkv * dh;
    LinArgs la = {};
    la.R = (int64_t)a->B * M;
    la.K = d;
    la.ldx = d;
    la.ws = scr;
    la.ws_bytes = scr_bytes;
    if (which & 1) {
        LinSeg &q = la.seg[la.nseg++];
        q.W = a->ca_wq;
        q.N = e;
        q.st = row_store(bf.q_ca, e);
        q.X = a->ca_xq;
        q.ldx = d;
    }
    if (which & 2) {
        const void *w[3] = {a->v_wq_host[0], a->v_wk_host[0], a->v_wv_host[0]};
        const StoreSpec st3[3] = {row_store(bf.q_v, e), heads_store(a->v_ktree_host[0], Hkv, dh, M, M),
                                  heads_store(a->v_vtree_host[0], Hkv, dh, M, M)};
        for (int i = 0; i < 3; ++i) {
            LinSeg &g = la.seg[la.nseg++];
            g.W = w[i];
            g.N = i == 0 ? e : ekv;
            g.st = st3[i];
            g.X = a->v_x_host[0];
            g.ldx = d;
        }
    }
    la.X = la.seg[0].X;
    la.seg[0].X = nullptr;               // the first segment reads the launch's own rows
    if (with_small) {
        la.rider = small_args(a, bf);
        la.rider_units = 2 * a->B + 1;
    }
    la.sum_out = sum_out;
    prof_set_site(which == 3 ? S_PAIR_QKV : which == 1 ? S_CA_QPROJ : S_VERIFY_QKV);
    MOA_TRY_HIP(launch_linear(sh->dtype, la, st), "draft_step: projections");
    return MOA_OK;
}

// where the memory's new rows go: appended at the lengths from before this step
static StoreSpec append_spec(const moa_step_args_t *a, const StepBufs &bf)
{
    StoreSpec sp = {};
    sp.mode = StoreSpec::APPEND;
    sp.heads = a->shape->n_kv_heads;
    sp.dh = a->shape->head_dim;
    sp.cap = a->ca_P_cap;
    sp.B = a->B;
    sp.row_base = bf.old_len;
    sp.tok_off = a->tok_off;
    sp.dev_status = a->dev_status;
    return sp;
}

// With the products ca_wk lsa_wo and ca_wv lsa_wo at hand, the memory's keys / values are projected straight from
// the mean-folded heads, in the launch that also projects the LSA output: (a Wo^T) Wk^T = a (Wk Wo)^T.
// Fills folded[2] and returns true when that applies.
static bool folded_segments(const moa_step_args_t *a, const StepBufs &bf, LinSeg *folded)
{
    if (!(a->ca_wk_lsa_wo && a->ca_wv_lsa_wo && a->lsa_wo && a->ca_wk && a->ca_wv)) return false;
    const void *wf[2] = {a->ca_wk_lsa_wo, a->ca_wv_lsa_wo};
    void *dstf[2] = {a->ca_k, a->ca_v};
    for (int i = 0; i < 2; ++i) {
        folded[i] = LinSeg{};
        folded[i].W = wf[i];
        folded[i].N = a->shape->n_kv_heads * a->shape->head_dim;
        folded[i].st = append_spec(a, bf);
        folded[i].st.dst = dstf[i];
    }
    return true;
}

// the LSA output's rows projected (or copied) into the memory
static int32_t piece_append(const moa_step_args_t *a, const StepBufs &bf, void *scr, size_t scr_bytes, hipStream_t st)
{
    const moa_shape_t *sh = a->shape;
    const int dh = sh->head_dim, ekv = sh->n_kv_heads * dh, dt = sh->dtype, d_mem = sh->lsa_q_heads * dh;
    StoreSpec sp = append_spec(a, bf);
    LinArgs la = {};
    la.X = a->lsa_out;
    la.R = a->T_lsa;
    la.K = d_mem;
    la.ldx = d_mem;
    la.ws = scr;
    la.ws_bytes = scr_bytes;
    const void *w[2] = {a->ca_wk, a->ca_wv};
    void *dst[2] = {a->ca_k, a->ca_v};
    prof_set_site(S_APPEND_KV);
    for (int i = 0; i < 2; ++i) {
        sp.dst = dst[i];
        if (w[i]) {
            la.seg[la.nseg].W = w[i];
            la.seg[la.nseg].N = ekv;
            la.seg[la.nseg].st = sp;
            ++la.nseg;
        } else {
            MOA_TRY_HIP(launch_scatter_copy(dt, a->lsa_out, a->T_lsa, ekv, d_mem, sp, st), "draft_step: append copy");
        }
    }
    if (la.nseg) MOA_TRY_HIP(launch_linear(dt, la, st), "draft_step: append projection");
    return MOA_OK;
}

// layer self-attention, then its rows appended to the memory at the old lengths
static int32_t piece_lsa_append(const moa_step_args_t *a, const StepBufs &bf, void *scr, size_t scr_bytes, hipStream_t st)
{
    LinSeg folded[2];
    if (folded_segments(a, bf, folded)) {
        t_lsa_extra = folded;
        t_lsa_nextra = 2;
    }
    t_lsa_extra_taken = false;
    int32_t rc = step_lsa(a, scr, scr_bytes, st);
    t_lsa_extra = nullptr;
    t_lsa_nextra = 0;
    if (rc || a->T_lsa <= 0 || (t_lsa_extra_taken && !g_dry)) return rc;
    return piece_append(a, bf, scr, scr_bytes, st);
}

// The step's first projections and an LSA chain that is one pass (at most LSA_CHUNK tokens, or an output-projection
// block of them in the one-kernel form), with the small kernels riding in launches that do not depend on them:
//   1. CA query + verification Q/K/V projections  + the step's integer work
//   2. LSA in one kernel (or its Q/K/V projection) + the pass that adds up launch 1's K slices (the one-kernel form and
//                                                    the tiled kernel carry it; else that pass is a launch of its own)
//   3. (attention over the layers, when apart)     4. LSA W_o (+ the memory's folded K/V)
// scr2 is the second scratch region: launch 1's partial sums live there while the LSA chain uses the first.
static int32_t piece_lsa_interleaved(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes, char *scr2,
                                     hipStream_t st)
{
    const moa_shape_t *sh = a->shape;
    const int dt = sh->dtype;
    const int64_t T = a->T_lsa;
    int32_t rc = lsa_check(sh, a->lsa_hs, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->lsa_out, scr, scr_bytes);
    if (rc) return rc;
    SumArgs sum_pair = {};
    rc = piece_projections(a, bf, scr2, scr_bytes, st, true, &sum_pair);
    if (rc) return rc;
    const LsaBufs b = lsa_carve(sh, T, scr, scr_bytes);
    void *abar = a->lsa_wo ? (void *)b.abar0 : a->lsa_out;
    if (lsa_takes_fused(sh, T, a->lsa_hs, a->lsa_wq, a->lsa_wk, a->lsa_wv, abar)) {
        LsaFusedCall fc = lsa_fused_call(sh, a->lsa_hs, 0, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, abar, step_lsa_packed(a));
        fc.carry_sum = &sum_pair;
        prof_set_site(S_LSA_FUSED);
        MOA_TRY_HIP(launch_lsa_fused(fc, st), "lsa: fused kernel");
    } else {
        LinArgs la;
        LsaAttnArgs aa;
        lsa_chunk_args(sh, a->lsa_hs, 0, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, abar, b, &la, &aa);
        if (la.nseg) {
            la.carry_sum = &sum_pair;
            prof_set_site(S_LSA_QKV);
            MOA_TRY_HIP(launch_linear(dt, la, st), "lsa: projection");
        } else {
            prof_set_site(S_PAIR_QKV);
            MOA_TRY_HIP(launch_splitk_sum(sum_pair, st), "draft_step: projections");
        }
        prof_set_site(S_LSA_ATTN);
        MOA_TRY_HIP(launch_lsa_attn(aa, st), "lsa: attention over layers");
    }
    LinSeg folded[2];
    const bool fold = a->lsa_wo && folded_segments(a, bf, folded);
    if (a->lsa_wo) {
        const LinArgs lo = lsa_oproj_args(sh, 0, T, a->lsa_wo, a->lsa_out, b, folded, fold ? 2 : 0);
        prof_set_site(S_LSA_OPROJ);
        MOA_TRY_HIP(launch_linear(dt, lo, st), "lsa: output projection");
    }
    if (fold) return MOA_OK;
    return piece_append(a, bf, scr, scr_bytes, st);
}

static AttnArgs piece_ca_core_args(const moa_step_args_t *a, const StepBufs &bf, void *scr, size_t scr_bytes)
{
    return attn_core_args(a->shape, bf.q_ca, a->B, a->M, a->ca_k, a->ca_v, a->ca_len, a->ca_P_cap, nullptr, bf.h_ca,
                          nullptr, nullptr, a->dev_status, scr, scr_bytes);
}

static AttnArgs piece_verify_core_args(const moa_step_args_t *a, const StepBufs &bf, void *scr, size_t scr_bytes)
{
    return attn_core_args(a->shape, bf.q_v, a->B, a->M, a->v_kcache_host[0], a->v_vcache_host[0], a->prefix_len,
                          a->P_cap, a->mask, bf.h_v, a->v_ktree_host[0], a->v_vtree_host[0], a->dev_status, scr,
                          scr_bytes);
}

// output projections: which = 1 (cross-attention), 2 (verification layer 0) or 3 (both in one launch)
static int32_t piece_oproj(const moa_step_args_t *a, const StepBufs &bf, int which, void *scr, size_t scr_bytes, hipStream_t st)
{
    const moa_shape_t *sh = a->shape;
    const int e = sh->n_q_heads * sh->head_dim;
    LinArgs lo = {};
    lo.R = (int64_t)a->B * a->M;
    lo.K = e;
    lo.ldx = e;
    lo.ws = scr;
    lo.ws_bytes = scr_bytes;
    if (which & 1) lo.seg[lo.nseg++] = oproj_seg(sh, bf.h_ca, a->ca_wo, a->ca_out);
    if (which & 2) lo.seg[lo.nseg++] = oproj_seg(sh, bf.h_v, a->v_wo_host[0], a->v_out_host[0]);
    lo.X = lo.seg[0].X;
    prof_set_site(which == 3 ? S_PAIR_OPROJ : which == 1 ? S_CA_OPROJ : S_VERIFY_OPROJ);
    MOA_TRY_HIP(launch_linear(sh->dtype, lo, st), "draft_step: output projections");
    return MOA_OK;
}

static int32_t piece_more_verify_layers(const moa_step_args_t *a, void *scr, size_t scr_bytes, hipStream_t st)
{
    for (int l = 1; l < a->n_verify_layers; ++l) {
        int32_t rc = attention_layer("tree_verify_attn", a->shape, a->v_x_host[l], a->B, a->M, a->v_wq_host[l],
                                     a->v_wk_host[l], a->v_wv_host[l], a->v_wo_host[l], a->v_kcache_host[l],
                                     a->v_vcache_host[l], a->prefix_len, a->P_cap, a->mask, a->v_out_host[l],
                                     a->v_ktree_host[l], a->v_vtree_host[l], a->dev_status, scr, scr_bytes, st);
        if (rc) return rc;
    }
    return MOA_OK;
}

static StepBufs carve_step_bufs(const moa_step_args_t *a, const GroupLayout &L, char **scr)
{
    char *p = (char *)a->ws;
    StepBufs bf;
    bf.old_len = (int32_t *)p;
    bf.q_ca = p + L.len_bytes;
    bf.h_ca = bf.q_ca + L.qa;
    bf.q_v = bf.h_ca + L.qa;
    bf.h_v = bf.q_v + L.qa;
    *scr = bf.h_v + L.qa;
    return bf;
}

static bool can_group(const moa_step_args_t *a)
{
    return pieces_ok(a) && a->ws_bytes >= group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa).total();
}

static int32_t draft_step_grouped(const moa_step_args_t *a)
{
    hipStream_t st = (hipStream_t)a->stream;
    const GroupLayout L = group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa);
    char *scr = nullptr;
    const StepBufs bf = carve_step_bufs(a, L, &scr);
    // With room for a second scratch region (the first projections keep their partial sums there while the LSA chain
    // uses the first) and all LSA tokens in one chunk, the two are interleaved; else one after the other.
    int32_t rc;
    const bool one_pass = a->T_lsa <= LSA_CHUNK ||
                          (a->T_lsa <= LSA_OBLOCK && lsa_takes_fused(a->shape, a->T_lsa, a->lsa_hs, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->ws));
    if (a->T_lsa > 0 && one_pass && a->ws_bytes >= L.total() + L.scratch) {
        rc = piece_lsa_interleaved(a, bf, scr, L.scratch, scr + L.scratch, st);
        if (rc) return rc;
    } else {
        rc = piece_projections(a, bf, scr, L.scratch, st, true);
        if (rc) return rc;
        rc = piece_lsa_append(a, bf, scr, L.scratch, st);
        if (rc) return rc;
    }
    const AttnArgs ca = piece_ca_core_args(a, bf, scr, L.attn_each);
    const AttnArgs ve = piece_verify_core_args(a, bf, scr + L.attn_each, L.attn_each);
    prof_set_site(S_PAIR_CORE);
    MOA_TRY_HIP(launch_attn_pair(ca, ve, st), "draft_step: attention cores");
    rc = piece_oproj(a, bf, 3, scr, L.scratch, st);
    if (rc) return rc;
    return piece_more_verify_layers(a, scr, L.scratch, st);
}

// ---- the same pieces on two streams.
// Dependencies inside one step: the LSA kernel depends on nothing else in the step, and neither do the projections of
// the cross-attention queries and the first verification layer.  The LSA kernel is bound by the matrix cores and the
// L2, those projections by HBM, so the two want different parts of the chip.  From packed weights the LSA kernel has a
// lean form (a third of a SIMD's registers per wavefront, 67 KB of LDS) beside which a compute unit still holds a
// workgroup of the weight-streaming kernel, so the two launches run on the same compute units at the same time; from
// plain weights the LSA kernel fills the LDS and runs with its largest token tile instead, which at decode sizes leaves
// half of the compute units to the other launch.  The projections run on a library-owned stream that is forked from
// and joined back into the caller's stream with one event each (an edge between two hardware queues costs several
// microseconds, so there are only these two), and the caller still sees one stream's worth of ordering (a stream
// capture records both branches).
//   side: E_fork -> [CA query + verification Q/K/V projections] -> [sum of its K slices] -> E_join
//   main: E_fork -> [LSA + the step's integer work] -> LSA W_o + memory append -> wait E_join -> both attention cores
//         -> both output projections -> further verification layers
// (When the LSA cannot run as the one kernel, the integer work rides with the projections and the main branch waits
// for E_join before the memory append.)
// One side stream and its events (fork, join, and one more for the schedule with the Self-Attention layer) exist per device; a mutex is held while a step is being enqueued, so steps of
// several host threads on one device are enqueued one after the other.
struct SideStream {
    hipStream_t stream = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, mid = nullptr;
    bool ok = false;
    std::mutex enqueue;
};

// The two events order work of one device against work of the same device: no system-scope fence (which writes the
// caches back for the host and other devices to see) is needed for that, and none is asked for.
static constexpr unsigned kEdgeFlags = hipEventDisableTiming | hipEventDisableSystemFence;

static SideStream *side_stream_for_current_device()
{
    static std::mutex mu;
    static SideStream pool[16];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return nullptr;
    std::lock_guard<std::mutex> lk(mu);
    SideStream &s = pool[dev];
    if (!s.stream) {
        s.ok = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) == hipSuccess &&
               hipEventCreateWithFlags(&s.fork, kEdgeFlags) == hipSuccess &&
               hipEventCreateWithFlags(&s.join, kEdgeFlags) == hipSuccess &&
               hipEventCreateWithFlags(&s.mid, kEdgeFlags) == hipSuccess;
    }
    return s.ok ? &s : nullptr;
}

// the grouped layout with a second scratch region for the side branch
static size_t two_stream_bytes(const moa_step_args_t *a)
{
    const GroupLayout L = group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa);
    return L.total() + L.scratch;
}

// side branch
static int32_t two_stream_side(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes, SideStream *ss,
                               bool with_small)
{
    hipStream_t side = ss->stream;
    SumArgs sum_pair = {};
    int32_t rc = piece_projections(a, bf, scr, scr_bytes, side, with_small, &sum_pair);
    if (rc) return rc;
    prof_set_site(S_PAIR_QKV);
    MOA_TRY_HIP(launch_splitk_sum(sum_pair, side), "draft_step: projections");
    return MOA_OK;
}

// whether the main branch of a two-stream step runs the LSA as the one kernel (which then also carries the step's
// integer work, so that nothing in the LSA chain has to wait for the other branch)
static bool two_stream_lsa_fused(const moa_step_args_t *a)
{
    return a->T_lsa > 0 && a->T_lsa <= LSA_OBLOCK &&
           lsa_takes_fused(a->shape, a->T_lsa, a->lsa_hs, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->ws);
}

static int32_t two_stream_main(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes, size_t attn_each,
                               SideStream *ss, bool fused)
{
    hipStream_t main = (hipStream_t)a->stream;
    const moa_shape_t *sh = a->shape;
    const int64_t T = a->T_lsa;
    int32_t rc = lsa_check(sh, a->lsa_hs, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->lsa_out, scr, scr_bytes);
    if (rc) return rc;
    if (fused) {
        const LsaBufs b = lsa_carve(sh, T, scr, scr_bytes);
        void *abar = a->lsa_wo ? (void *)b.abar0 : a->lsa_out;
        LsaFusedCall fc = lsa_fused_call(sh, a->lsa_hs, 0, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, abar, step_lsa_packed(a));
        fc.leave_room = 1;                   // the form that shares the chip with the other branch
        fc.rider = small_args(a, bf);        // tree masks, accept walk, old memory lengths
        fc.rider_units = 2 * a->B + 1;
        prof_set_site(S_LSA_FUSED);
        MOA_TRY_HIP(launch_lsa_fused(fc, main), "lsa: fused kernel");
        LinSeg folded[2];
        const bool fold = a->lsa_wo && folded_segments(a, bf, folded);
        if (a->lsa_wo) {
            const LinArgs lo = lsa_oproj_args(sh, 0, T, a->lsa_wo, a->lsa_out, b, folded, fold ? 2 : 0);
            prof_set_site(S_LSA_OPROJ);
            MOA_TRY_HIP(launch_linear(sh->dtype, lo, main), "lsa: output projection");
        }
        if (!fold) {
            rc = piece_append(a, bf, scr, scr_bytes, main);
            if (rc) return rc;
        }
        // the cores need the other branch's queries; by now it has usually finished, so the wait costs nothing
        MOA_TRY_HIP(hipStreamWaitEvent(main, ss->join, 0), "draft_step: join");
    } else {
        MOA_TRY_HIP(hipStreamWaitEvent(main, ss->join, 0), "draft_step: join");      // the append needs the old lengths
        rc = piece_lsa_append(a, bf, scr, scr_bytes, main);
        if (rc) return rc;
    }
    const AttnArgs ca = piece_ca_core_args(a, bf, scr, attn_each);
    const AttnArgs ve = piece_verify_core_args(a, bf, scr + attn_each, attn_each);
    prof_set_site(S_PAIR_CORE);
    MOA_TRY_HIP(launch_attn_pair(ca, ve, main), "draft_step: attention cores");
    rc = piece_oproj(a, bf, 3, scr, scr_bytes, main);
    if (rc) return rc;
    return piece_more_verify_layers(a, scr, scr_bytes, main);
}

static int32_t draft_step_concurrent(const moa_step_args_t *a, SideStream *ss)
{
    const LinearLeaveRoom share_the_compute_units;
    hipStream_t main = (hipStream_t)a->stream, side = ss->stream;
    const GroupLayout L = group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa);
    char *scr_main = nullptr;
    const StepBufs bf = carve_step_bufs(a, L, &scr_main);
    char *scr_side = scr_main + L.scratch;
    std::lock_guard<std::mutex> lk(ss->enqueue);

    MOA_TRY_HIP(hipEventRecord(ss->fork, main), "draft_step: fork");
    MOA_TRY_HIP(hipStreamWaitEvent(side, ss->fork, 0), "draft_step: fork");
    // Whatever happens from here on, the side stream is joined back into the caller's (a stream capture must not be
    // left with an unjoined branch): the main branch waits for the join event on its way; when either branch fails,
    // the wait is enqueued here (a second wait for the same event is harmless).
    const bool fused = two_stream_lsa_fused(a);
    int32_t rc = two_stream_side(a, bf, scr_side, L.scratch, ss, !fused);
    const hipError_t ej = hipEventRecord(ss->join, side);
    if (rc == MOA_OK && ej != hipSuccess) rc = hip_fail(ej, "draft_step: join");
    if (rc == MOA_OK) {
        rc = two_stream_main(a, bf, scr_main, L.scratch, L.attn_each, ss, fused);
        if (rc == MOA_OK) return rc;
    }
    if (ej == hipSuccess) (void)hipStreamWaitEvent(main, ss->join, 0);
    return rc;
}

// ---- two streams with the Self-Attention layer.
// With that layer the step has one long chain -- tree masks -> SA projections -> SA core -> SA output projection ->
// cross-attention query projection -> cross-attention core -> its output projection -- of launches that each leave
// most of the chip idle, and two shorter chains nothing in front of the cross-attention core depends on: the LSA with
// the memory append (needed by that core only) and the first verification layer.  The long chain stays on the
// caller's stream; the other two run one after the other on the library's:
//   main: tree masks -> E_fork -> SA layer -> CA query projection -> wait E_mid -> CA core -> CA output projection
//         -> wait E_join
//   side: wait E_fork -> [LSA + the step's other integer work] -> LSA W_o + memory append -> E_mid
//         -> verification Q/K/V -> verification core -> its output projection -> further layers -> E_join
// The masks are built once, in front of the fork, for both branches to read.
static bool two_stream_takes_sa(const moa_step_args_t *args, const moa_step_args_t *a)
{
    if (!two_stream_lsa_fused(a) || a->n_verify_layers < 1) return false;
    const GroupLayout L = group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa);
    return attn_ws_bytes(args->sa_shape, args->B, args->M, args->sa_P_cap) <= L.scratch;
}

// The side branch in the three parts the enqueue order below needs.
struct SaSideState {
    LsaBufs b;
    bool fold;
    LinSeg folded[2];
};

static int32_t two_stream_sa_side_lsa(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes,
                                      hipStream_t side, SaSideState *st)
{
    const moa_shape_t *sh = a->shape;
    const int64_t T = a->T_lsa;
    int32_t rc = lsa_check(sh, a->lsa_hs, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, a->lsa_out, scr, scr_bytes);
    if (rc) return rc;
    st->b = lsa_carve(sh, T, scr, scr_bytes);
    void *abar = a->lsa_wo ? (void *)st->b.abar0 : a->lsa_out;
    LsaFusedCall fc = lsa_fused_call(sh, a->lsa_hs, 0, T, a->lsa_wq, a->lsa_wk, a->lsa_wv, abar, step_lsa_packed(a));
    fc.leave_room = 1;
    fc.rider = small_args(a, bf);        // accept walk, old memory lengths
    fc.rider.skip_masks = 1;             // built in front of the fork
    fc.rider_units = 2 * a->B + 1;
    prof_set_site(S_LSA_FUSED);
    MOA_TRY_HIP(launch_lsa_fused(fc, side), "lsa: fused kernel");
    return MOA_OK;
}

static int32_t two_stream_sa_side_memory(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes,
                                         hipStream_t side, SaSideState *st)
{
    const moa_shape_t *sh = a->shape;
    st->fold = a->lsa_wo && folded_segments(a, bf, st->folded);
    if (a->lsa_wo) {
        const LinArgs lo = lsa_oproj_args(sh, 0, a->T_lsa, a->lsa_wo, a->lsa_out, st->b, st->folded, st->fold ? 2 : 0);
        prof_set_site(S_LSA_OPROJ);
        MOA_TRY_HIP(launch_linear(sh->dtype, lo, side), "lsa: output projection");
    }
    return st->fold ? MOA_OK : piece_append(a, bf, scr, scr_bytes, side);
}

static int32_t two_stream_sa_side_verify(const moa_step_args_t *a, const StepBufs &bf, char *scr, size_t scr_bytes,
                                         size_t attn_each, hipStream_t side)
{
    int32_t rc = piece_projections(a, bf, scr, scr_bytes, side, false, nullptr, 2);
    if (rc) return rc;
    const AttnArgs ve = piece_verify_core_args(a, bf, scr, attn_each);
    prof_set_site(S_VERIFY_CORE);
    MOA_TRY_HIP(launch_attn(ve, side), "draft_step: verification core");
    rc = piece_oproj(a, bf, 2, scr, scr_bytes, side);
    if (rc) return rc;
    return piece_more_verify_layers(a, scr, scr_bytes, side);
}

// Enqueue order matters beyond the order inside each stream: the runtime settles where in the producing stream a
// cross-stream wait takes hold when the waiting stream's next launch is submitted, and takes that stream's tail at that
// moment.  So each wait is followed at once by the launch that needs it, before the producing stream is given
// anything further (measured: with the whole main chain enqueued ahead of the side branch's first launch, that
// launch started only after the chain, 59 us late).
static int32_t draft_step_concurrent_sa(const moa_step_args_t *args, const moa_step_args_t *a, SideStream *ss)
{
    const LinearLeaveRoom share_the_compute_units;
    hipStream_t main = (hipStream_t)a->stream, side = ss->stream;
    const GroupLayout L = group_layout(a->shape, a->B, a->M, a->P_cap, a->ca_P_cap, a->T_lsa);
    char *scr_main = nullptr;
    const StepBufs bf = carve_step_bufs(a, L, &scr_main);
    char *scr_side = scr_main + L.scratch;
    std::lock_guard<std::mutex> lk(ss->enqueue);

    int32_t rc = moa_tree_build(a->parent, a->B, a->M, a->mask, a->depth, a->dev_status, main);
    if (rc) return rc;
    MOA_TRY_HIP(hipEventRecord(ss->fork, main), "draft_step: fork");
    MOA_TRY_HIP(hipStreamWaitEvent(side, ss->fork, 0), "draft_step: fork");
    // From here on the side stream is joined back into the caller's whatever happens (see draft_step_concurrent).
    SaSideState st;
    rc = two_stream_sa_side_lsa(a, bf, scr_side, L.scratch, side, &st);
    if (rc == MOA_OK) rc = step_self_attn_layer(args, scr_main, L.scratch, main);
    if (rc == MOA_OK) rc = piece_projections(a, bf, scr_main, L.scratch, main, false, nullptr, 1);
    if (rc == MOA_OK) rc = two_stream_sa_side_memory(a, bf, scr_side, L.scratch, side, &st);
    if (rc == MOA_OK) {
        hipError_t e = hipEventRecord(ss->mid, side);
        if (e == hipSuccess) e = hipStreamWaitEvent(main, ss->mid, 0);
        if (e != hipSuccess) rc = hip_fail(e, "draft_step: memory ready");
    }
    if (rc == MOA_OK) {
        const AttnArgs ca = piece_ca_core_args(a, bf, scr_main, L.attn_each);
        prof_set_site(S_CA_CORE);
        const hipError_t e = launch_attn(ca, main);
        if (e != hipSuccess) rc = hip_fail(e, "draft_step: cross-attention core");
    }
    if (rc == MOA_OK) rc = two_stream_sa_side_verify(a, bf, scr_side, L.scratch, L.attn_each, side);
    const hipError_t ej = hipEventRecord(ss->join, side);
    if (rc == MOA_OK && ej != hipSuccess) rc = hip_fail(ej, "draft_step: join");
    if (rc == MOA_OK) rc = piece_oproj(a, bf, 1, scr_main, L.scratch, main);
    if (ej == hipSuccess) {
        const hipError_t e = hipStreamWaitEvent(main, ss->join, 0);
        if (rc == MOA_OK && e != hipSuccess) rc = hip_fail(e, "draft_step: join");
    }
    return rc;
}

int32_t moa_draft_step(const moa_step_args_t *args)
{
    if (!args) return fail(MOA_ERR_NULL, "draft_step: args is NULL");
    if (!args->shape) return fail(MOA_ERR_NULL, "draft_step: shape is NULL");
    if (args->n_verify_layers < 0) return fail(MOA_ERR_SHAPE, "draft_step: n_verify_layers=%d", args->n_verify_layers);
    if (args->schedule < MOA_SCHED_GROUPED || args->schedule > MOA_SCHED_SEQUENTIAL) return fail(MOA_ERR_SHAPE, "draft_step: schedule=%d", args->schedule);
    if (args->n_verify_layers > 0 &&
        (!args->v_x_host || !args->v_wq_host || !args->v_wk_host || !args->v_wv_host || !args->v_wo_host || !args->v_kcache_host ||
         !args->v_vcache_host || !args->v_out_host || !args->v_ktree_host || !args->v_vtree_host))
        return fail(MOA_ERR_NULL, "draft_step: a per-layer pointer array is NULL");
    // With the Self-Attention layer in front, the cross-attention's queries are that layer's output.
    const bool sa = args->sa_emb != nullptr;
    moa_step_args_t with_sa;
    const moa_step_args_t *a = args;
    if (sa) {
        with_sa = *args;
        with_sa.ca_xq = args->sa_out;
        a = &with_sa;
    }
    g_dry = true;                       // every stage's host checks first: a bad argument launches nothing
    int32_t rc = sa ? step_self_attn(args) : MOA_OK;
    if (rc == MOA_OK) rc = draft_step_stages(a);
    g_dry = false;
    if (rc) return rc;
    // grouped launches by default; two streams on request when the workspace has room for both branches'
    // scratch; otherwise one stage after another
    const bool two = a->schedule == MOA_SCHED_TWO_STREAM && pieces_ok(a) && a->ws_bytes >= two_stream_bytes(a);
    SideStream *ss = two ? side_stream_for_current_device() : nullptr;
    // On two streams the layer is one branch's first piece; otherwise it runs in front of whichever schedule follows
    // (whose first launch writes the same masks again).
    if (sa && ss && two_stream_takes_sa(args, a)) return draft_step_concurrent_sa(args, a, ss);
    if (sa) {
        rc = step_self_attn(args);
        if (rc) return rc;
    }
    if (ss) return draft_step_concurrent(a, ss);
    if (a->schedule != MOA_SCHED_SEQUENTIAL && can_group(a)) return draft_step_grouped(a);
    return draft_step_stages(a);
}

}  // extern "C"
