// Draft-tree construction on the device (Sec. 2.2, tree drafting as in EAGLE-2): per level, the joint
// log-probabilities of the Bw*Bw expansions and the best Bw of them; at the end the m best of all candidates,
// relabelled so that parents come first; and the Bw most probable tokens of a row of logits.
// Every ranking decision is taken on single-precision numbers formed by one addition, ties to the lower index,
// so results are a pure function of the inputs.  These are latency-sized kernels: one workgroup per sequence
// (or per row of logits), everything in LDS / registers.
#include "moa_common.h"
#include "../../include/moa.h"

namespace moa {

constexpr int TREE_MAX_BREADTH = 16;      // Bw*Bw expansions fit one 256-thread workgroup
constexpr int TREE_MAX_CAND = 4096;       // candidates ranked in LDS by moa_tree_finalize

__device__ __forceinline__ bool ranks_before(float a, int ia, float b, int ib) { return a > b || (a == b && ia < ib); }

// a float as an unsigned integer of the same order (-inf lowest)
__device__ __forceinline__ uint32_t orderable(float v)
{
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float from_orderable(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

// (value, index) as one 64-bit key whose unsigned order is "ranks before": larger value first, then smaller index.
// -0 and +0 are one value.  NaN never gets here (callers map it to -inf first).
__device__ __forceinline__ uint64_t rank_key(float v, int idx)
{
    return ((uint64_t)orderable(v + 0.0f) << 32) | (uint64_t)(0xffffffffu - (uint32_t)idx);
}
__device__ __forceinline__ float key_value(uint64_t k) { return from_orderable((uint32_t)(k >> 32)); }
__device__ __forceinline__ int key_index(uint64_t k) { return (int)(0xffffffffu - (uint32_t)k); }

// how many of keys[0..n) rank before `mine`; keys is a 16-byte aligned LDS array, read two keys at a time (every
// lane reads the same address: a broadcast)
typedef __attribute__((ext_vector_type(2))) uint64_t u64x2;
__device__ __forceinline__ int rank_among(const uint64_t *keys, int n, uint64_t mine)
{
    int rank = 0;
    const int n2 = n & ~1;
#pragma unroll 4
    for (int u = 0; u < n2; u += 2) {
        const u64x2 a = *(const u64x2 *)&keys[u];
        rank += (a[0] > mine ? 1 : 0) + (a[1] > mine ? 1 : 0);
    }
    if (n2 < n) rank += keys[n2] > mine ? 1 : 0;
    return rank;
}

__global__ __launch_bounds__(256) void k_tree_expand(int level, int Bw, int n_max, const float *__restrict__ child_logp,
                                                     const int32_t *__restrict__ child_tok, float *__restrict__ cand_logp,
                                                     int32_t *__restrict__ cand_tok, int32_t *__restrict__ cand_parent,
                                                     int32_t *__restrict__ frontier)
{
    __shared__ __attribute__((aligned(16))) uint64_t lp[256];
    const int b = blockIdx.x, t = threadIdx.x;
    const int F = level == 1 ? 1 : Bw, n = F * Bw;
    const int base = level == 1 ? 0 : Bw + (level - 2) * Bw * Bw;
    float *clp = cand_logp + (int64_t)b * n_max;
    int32_t *ctk = cand_tok + (int64_t)b * n_max, *cpr = cand_parent + (int64_t)b * n_max, *fr = frontier + (int64_t)b * Bw;
    uint64_t mine = 0;
    if (t < n) {
        const int f = t / Bw;
        float v = child_logp[(int64_t)b * n + t];
        v = v == v ? fminf(v, 0.0f) : -INFINITY;          // a child is never more likely than its parent
        int par = -1;
        if (level > 1) {
            par = fr[f];
            par = par < 0 ? 0 : (par >= base ? base - 1 : par);      // a corrupt frontier cannot leave the array
            v = clp[par] + v;                                        // one single-precision addition
        }
        clp[base + t] = v;
        ctk[base + t] = child_tok[(int64_t)b * n + t];
        cpr[base + t] = par;
        mine = rank_key(v, t);
        lp[t] = mine;
    }
    __syncthreads();                                       // every read of the old frontier is done
    if (t < n) {
        const int rank = rank_among(lp, n, mine);
        if (rank < Bw) fr[rank] = base + t;
    }
}

__global__ __launch_bounds__(256) void k_tree_finalize(int n, int n_max, int keep, int ld_out, const int32_t *__restrict__ root_tok,
                                                       const float *__restrict__ cand_logp, const int32_t *__restrict__ cand_tok,
                                                       const int32_t *__restrict__ cand_parent, int32_t *__restrict__ parent,
                                                       int32_t *__restrict__ tok, int32_t *__restrict__ node_cand,
                                                       int32_t *dev_status)
{
    __shared__ __attribute__((aligned(16))) uint64_t lp[TREE_MAX_CAND];
    __shared__ int32_t node_of[TREE_MAX_CAND];
    __shared__ int32_t cnt[256];
    const int b = blockIdx.x, t = threadIdx.x;
    const float *clp = cand_logp + (int64_t)b * n_max;
    const int32_t *ctk = cand_tok + (int64_t)b * n_max, *cpr = cand_parent + (int64_t)b * n_max;
    int32_t *po = parent + (int64_t)b * ld_out, *to = tok + (int64_t)b * ld_out, *no = node_cand + (int64_t)b * ld_out;
    for (int c = t; c < n; c += 256) {
        const float v = clp[c];
        lp[c] = rank_key(v == v ? v : -INFINITY, c);
    }
    __syncthreads();
    // each thread owns a run of consecutive candidates, so that node numbers follow candidate order
    const int per = (n + 255) / 256, c0 = t * per, c1 = min(c0 + per, n);
    int kept = 0;
    for (int c = c0; c < c1; ++c) {
        const bool k = rank_among(lp, n, lp[c]) < keep;
        node_of[c] = k ? 1 : 0;
        kept += k ? 1 : 0;
    }
    // exclusive prefix sum of the 256 counts, starting at 1 (node 0 is the root): within a wave by shuffles, the
    // four wave totals through LDS
    int incl = kept;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int up = __shfl_up(incl, o);
        if ((t & 63) >= o) incl += up;
    }
    if ((t & 63) == 63) cnt[t >> 6] = incl;
    if (t == 0) {
        po[0] = -1;
        to[0] = root_tok[b];
        no[0] = -1;
    }
    __syncthreads();
    int next = 1 + incl - kept;
    for (int w = 0; w < (t >> 6); ++w) next += cnt[w];
    for (int c = c0; c < c1; ++c) node_of[c] = node_of[c] ? next++ : -1;
    __syncthreads();
    for (int c = c0; c < c1; ++c) {
        const int i = node_of[c];
        if (i < 0) continue;
        const int p = cpr[c];
        int pn = 0;
        if (p >= 0) {
            pn = (p < c) ? node_of[p] : -1;
            if (pn < 0) {                                  // cannot happen with arrays written by k_tree_expand
                pn = 0;
                if (dev_status) atomicOr(dev_status, MOA_DEV_BAD_PARENT);
            }
        }
        po[i] = pn;
        to[i] = ctk[c];
        no[i] = c;
    }
}

// ---- the Bw most probable tokens of a row of logits, with log-probabilities
// A row of the vocabulary is cut into S slices, one workgroup each, so that a handful of rows still fills the chip.
// A thread holds its (at most 32) values in registers and sorts them once, best first (value descending, id
// ascending: a total order, so ties need no care); the slice's Bw best are then found by Bw rounds that compare only
// the heads of the 256 lists (one workgroup-wide reduction per round).  A second kernel ranks the S*Bw survivors of
// a row and merges the slices' (max, sum of exponentials).

// Wavefront-wide maximum / minimum of an unsigned value by data-parallel-primitive moves inside the vector ALU (four
// shifts within the rows of 16 lanes, then two row broadcasts), read from lane 63: a dozen ALU instructions where
// the shuffle form makes six trips through the LDS crossbar.  Lanes a move does not reach keep their own value,
// which is harmless for max and min.
template <bool MAX>
__device__ __forceinline__ uint32_t wave_reduce_u32(uint32_t x)
{
#define MOA_DPP_STEP(ctrl)                                                                                   \
    {                                                                                                        \
        const uint32_t o = (uint32_t)__builtin_amdgcn_update_dpp((int)x, (int)x, ctrl, 0xf, 0xf, false);     \
        x = MAX ? (o > x ? o : x) : (o < x ? o : x);                                                         \
    }
    MOA_DPP_STEP(0x111)   // row_shr:1
    MOA_DPP_STEP(0x112)   // row_shr:2
    MOA_DPP_STEP(0x114)   // row_shr:4
    MOA_DPP_STEP(0x118)   // row_shr:8   -> lane 15 of a row holds the row's result
    MOA_DPP_STEP(0x142)   // row_bcast:15 -> lane 31: rows 0-1, lane 63: rows 2-3
    MOA_DPP_STEP(0x143)   // row_bcast:31 -> lane 63: all four rows
#undef MOA_DPP_STEP
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

constexpr int TOPK_EPT = 32;              // values a thread keeps
constexpr int TOPK_MIN_SLICES = 32;

static int topk_slices(int V)
{
    const int need = (V + 256 * TOPK_EPT - 1) / (256 * TOPK_EPT);
    return need > TOPK_MIN_SLICES ? need : TOPK_MIN_SLICES;
}

// scratch per (row, slice): Bw values, Bw ids, max, sum
template <int EPT>
__global__ __launch_bounds__(256) void k_topk_slices(int is_bf16, const void *__restrict__ logits, int V, int Bw, int S,
                                                     float *__restrict__ sval, int32_t *__restrict__ sid,
                                                     float *__restrict__ smax, float *__restrict__ ssum)
{
    __shared__ float wv[4], wm[4], wsum[4];
    __shared__ int wi[4];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int s = blockIdx.x % S;
    const int64_t r = blockIdx.x / S;
    const int Vs = (V + S - 1) / S, v0 = s * Vs, v1 = min(v0 + Vs, V);
    const float *rf = (const float *)logits + r * V;
    const bf16_t *rb = (const bf16_t *)logits + r * V;
    float x[EPT];
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int v = v0 + t + 256 * i;
        x[i] = v < v1 ? (is_bf16 ? bf2f(rb[v]) : rf[v]) : -INFINITY;
    }
    // the slice's log-sum-exp pieces
    float m = -INFINITY;
#pragma unroll
    for (int i = 0; i < EPT; ++i) m = fmaxf(m, x[i]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) wm[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(wm[0], wm[1]), fmaxf(wm[2], wm[3]));
    float sum = 0.f;
    if (m > -INFINITY) {
#pragma unroll
        for (int i = 0; i < EPT; ++i) sum += __expf(x[i] - m);      // exp(-inf) = 0 for the padding
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) wsum[wave] = sum;
    __syncthreads();
    const int64_t slot = r * S + s;
    if (t == 0) { smax[slot] = m; ssum[slot] = (wsum[0] + wsum[1]) + (wsum[2] + wsum[3]); }
    // Each thread sorts its own values once (a bitonic network on registers: no lane does anything another does not),
    // best first; a round then only compares the heads of the 256 lists, and the one thread that wins moves its list up.
    int id[EPT];
#pragma unroll
    for (int i = 0; i < EPT; ++i) {
        const int v = v0 + t + 256 * i;
        id[i] = v < v1 ? v : 0x7fffffff;
    }
#pragma unroll
    for (int k = 2; k <= EPT; k <<= 1)
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1)
#pragma unroll
            for (int i = 0; i < EPT; ++i) {
                const int l = i ^ j;
                if (l > i) {
                    const bool up = (i & k) == 0;              // this pair ends with the better element first
                    const bool swap = up ? ranks_before(x[l], id[l], x[i], id[i]) : ranks_before(x[i], id[i], x[l], id[l]);
                    const float xi = x[i], xl = x[l];
                    const int ii = id[i], il = id[l];
                    x[i] = swap ? xl : xi;
                    x[l] = swap ? xi : xl;
                    id[i] = swap ? il : ii;
                    id[l] = swap ? ii : il;
                }
            }
    for (int round = 0; round < Bw; ++round) {
        float bv = x[0];
        int bi = id[0];
        // the wavefront's best: the largest value, then the smallest id among the lanes that hold it
        const uint32_t key = orderable(bv + 0.0f);         // -0 and +0 are the same value, as in every comparison here
        const uint32_t kmax = wave_reduce_u32<true>(key);
        bi = (int)wave_reduce_u32<false>(key == kmax ? (uint32_t)bi : 0x7fffffffu);
        bv = from_orderable(kmax);
        __syncthreads();
        if (lane == 0) { wv[wave] = bv; wi[wave] = bi; }
        __syncthreads();
        bv = wv[0];
        bi = wi[0];
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (ranks_before(wv[w], wi[w], bv, bi)) { bv = wv[w]; bi = wi[w]; }
        if (t == 0) { sval[slot * Bw + round] = bv; sid[slot * Bw + round] = bi; }   // (-inf, INT_MAX) when the slice ran out
        if (id[0] == bi && bi != 0x7fffffff) {             // the winner's list moves up
#pragma unroll
            for (int i = 0; i + 1 < EPT; ++i) { x[i] = x[i + 1]; id[i] = id[i + 1]; }
            x[EPT - 1] = -INFINITY;
            id[EPT - 1] = 0x7fffffff;
        }
    }
}

// one workgroup per row: rank the S*Bw survivors, merge the log-sum-exp
__global__ __launch_bounds__(256) void k_topk_merge(int Bw, int S, const float *__restrict__ sval, const int32_t *__restrict__ sid,
                                                    const float *__restrict__ smax, const float *__restrict__ ssum,
                                                    int32_t *__restrict__ tok, float *__restrict__ logp)
{
    extern __shared__ __attribute__((aligned(16))) uint64_t ck[];   // [n] order keys, then [S] slice maxima, [S] slice sums
    __shared__ float red[4];
    __shared__ float lse_s;
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const int64_t r = blockIdx.x;
    const int n = S * Bw;
    float *sm = (float *)(ck + n), *ss = sm + S;
    // everything the row needs is requested at once: one trip to memory instead of three
    for (int c = t; c < n; c += 256) ck[c] = rank_key(sval[r * n + c], sid[r * n + c]);
    for (int k = t; k < S; k += 256) { sm[k] = smax[r * S + k]; ss[k] = ssum[r * S + k]; }
    __syncthreads();
    float m = -INFINITY;
    for (int k = t; k < S; k += 256) m = fmaxf(m, sm[k]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) m = fmaxf(m, __shfl_xor(m, o));
    if (lane == 0) red[wave] = m;
    __syncthreads();
    m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float sum = 0.f;
    for (int k = t; k < S; k += 256) {
        const float mk = sm[k];
        if (mk > -INFINITY) sum += ss[k] * __expf(mk - m);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red[wave] = sum;
    __syncthreads();
    if (t == 0) lse_s = m + __logf((red[0] + red[1]) + (red[2] + red[3]));
    __syncthreads();
    const float lse = lse_s;
    for (int c = t; c < n; c += 256) {
        const uint64_t mine = ck[c];
        const int id = key_index(mine);
        if (id == 0x7fffffff) continue;                    // an exhausted slice's filler
        const int rank = rank_among(ck, n, mine);
        if (rank < Bw) { tok[r * Bw + rank] = id; logp[r * Bw + rank] = key_value(mine) - lse; }
    }
}

}  // namespace moa

using namespace moa;

extern "C" {

static int32_t tree_fail(int32_t code, const char *msg) { return moa::api_fail(code, msg); }

int32_t moa_tree_expand_level(int32_t level, int32_t B, int32_t Bw, int32_t n_max, const float *child_logp,
                              const int32_t *child_tok, float *cand_logp, int32_t *cand_tok, int32_t *cand_parent,
                              int32_t *frontier, void *stream)
{
    if (!child_logp || !child_tok || !cand_logp || !cand_tok || !cand_parent || !frontier) return tree_fail(MOA_ERR_NULL, "tree_expand_level: NULL pointer");
    if (level < 1 || B < 1 || Bw < 1 || Bw > TREE_MAX_BREADTH) return tree_fail(MOA_ERR_SHAPE, "tree_expand_level: level >= 1, B >= 1, 1 <= breadth <= 16");
    const int64_t end = level == 1 ? Bw : (int64_t)Bw + (int64_t)(level - 1) * Bw * Bw;
    if (end > n_max) return tree_fail(MOA_ERR_RANGE, "tree_expand_level: the level's candidates do not fit n_max");
    prof_set_site(S_TREE_EXPAND);
    prof_begin(K_TREE_EXPAND, (hipStream_t)stream);
    MOA_KLAUNCH(k_tree_expand, dim3(B), dim3(256), 0, (hipStream_t)stream, level, Bw, n_max, child_logp, child_tok, cand_logp,
                cand_tok, cand_parent, frontier);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : tree_fail(MOA_ERR_HIP, "tree_expand_level: launch failed");
}

int32_t moa_tree_finalize(int32_t B, int32_t n_cand, int32_t n_max, int32_t m, const int32_t *root_tok,
                          const float *cand_logp, const int32_t *cand_tok, const int32_t *cand_parent, int32_t *parent,
                          int32_t *tok, int32_t *node_cand, int32_t *dev_status, void *stream)
{
    if (!root_tok || !cand_logp || !cand_tok || !cand_parent || !parent || !tok || !node_cand) return tree_fail(MOA_ERR_NULL, "tree_finalize: NULL pointer");
    if (B < 1 || n_cand < 0 || n_cand > n_max || n_cand > TREE_MAX_CAND || m < 0 || 1 + m > MOA_MAX_TREE)
        return tree_fail(MOA_ERR_SHAPE, "tree_finalize: 0 <= n_cand <= min(n_max, 4096), 1 + m <= 256");
    const int keep = m < n_cand ? m : n_cand;
    prof_set_site(S_TREE_FINALIZE);
    prof_begin(K_TREE_FINALIZE, (hipStream_t)stream);
    MOA_KLAUNCH(k_tree_finalize, dim3(B), dim3(256), 0, (hipStream_t)stream, n_cand, n_max, keep, 1 + m, root_tok, cand_logp,
                cand_tok, cand_parent, parent, tok, node_cand, dev_status);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : tree_fail(MOA_ERR_HIP, "tree_finalize: launch failed");
}

int32_t moa_topk_workspace_bytes(int32_t F, int32_t V, int32_t Bw, size_t *bytes_host)
{
    if (!bytes_host) return tree_fail(MOA_ERR_NULL, "topk_workspace_bytes: bytes_host is NULL");
    if (F < 1 || V < 1 || Bw < 1 || Bw > TREE_MAX_BREADTH) return tree_fail(MOA_ERR_SHAPE, "topk_workspace_bytes: F >= 1, V >= 1, 1 <= breadth <= 16");
    const size_t S = (size_t)topk_slices(V);
    *bytes_host = (size_t)F * S * ((size_t)Bw * 8 + 8);
    return MOA_OK;
}

int32_t moa_topk_logprob(int32_t dtype, const void *logits, int32_t F, int32_t V, int32_t Bw, int32_t *tok, float *logp,
                         void *ws, size_t ws_bytes, void *stream)
{
    if (!logits || !tok || !logp) return tree_fail(MOA_ERR_NULL, "topk_logprob: NULL pointer");
    if (dtype != MOA_F32 && dtype != MOA_BF16) return tree_fail(MOA_ERR_DTYPE, "topk_logprob: dtype");
    if (F < 1 || V < 1 || Bw < 1 || Bw > TREE_MAX_BREADTH || Bw > V) return tree_fail(MOA_ERR_SHAPE, "topk_logprob: F >= 1, 1 <= breadth <= min(16, V)");
    const int S = topk_slices(V);
    const size_t n = (size_t)F * S;
    if ((int64_t)F * S > 0x7fffffff) return tree_fail(MOA_ERR_SHAPE, "topk_logprob: too many rows");
    const size_t need = n * ((size_t)Bw * 8 + 8);
    if (!ws || (((uintptr_t)ws) & 255) || ws_bytes < need) return tree_fail(MOA_ERR_WORKSPACE, "topk_logprob: workspace NULL, misaligned or smaller than moa_topk_workspace_bytes");
    float *sval = (float *)ws;
    int32_t *sid = (int32_t *)(sval + n * Bw);
    float *smax = (float *)(sid + n * Bw);
    float *ssum = smax + n;
    hipStream_t st = (hipStream_t)stream;
    prof_set_site(S_TOPK_LOGPROB);
    prof_begin(K_TOPK_LOGPROB, st);
    if ((V + S - 1) / S <= 256 * 16)         // half-filled slices (few rows, many slices): half the registers to walk per round
        MOA_KLAUNCH(k_topk_slices<16>, dim3((unsigned)n), dim3(256), 0, st, dtype == MOA_BF16 ? 1 : 0, logits, V, Bw, S, sval, sid, smax, ssum);
    else
        MOA_KLAUNCH(k_topk_slices<TOPK_EPT>, dim3((unsigned)n), dim3(256), 0, st, dtype == MOA_BF16 ? 1 : 0, logits, V, Bw, S, sval, sid, smax, ssum);
    prof_end(st);
    if (hipGetLastError() != hipSuccess) return tree_fail(MOA_ERR_HIP, "topk_logprob: launch failed");
    const size_t lds = (size_t)S * Bw * 8 + (size_t)S * 8;
    if (lds > 60 * 1024) return tree_fail(MOA_ERR_SHAPE, "topk_logprob: vocabulary too large for the merge");
    prof_begin(K_TOPK_MERGE, st);
    MOA_KLAUNCH(k_topk_merge, dim3(F), dim3(256), lds, st, Bw, S, sval, sid, smax, ssum, tok, logp);
    prof_end(st);
    return hipGetLastError() == hipSuccess ? MOA_OK : tree_fail(MOA_ERR_HIP, "topk_logprob: launch failed");
}

}  // extern "C"
