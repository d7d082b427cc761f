// Internal declarations shared by the libmoa translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>

namespace moa {

typedef uint16_t bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
// 16-byte register chunk.  HIP's own uint4 is a class; arrays of it are not promoted to registers
// (they end up in scratch memory), so staging buffers use this plain vector type instead.
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

enum { DT_F32 = 0, DT_BF16 = 1 };

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round to nearest even; NaN stays NaN.  The hardware's own conversion (v_cvt_pk_bf16_f32 on this target): one
// instruction per pair of values, where the integer formulation costs a dozen and a branch for the NaN case.
typedef __attribute__((ext_vector_type(2))) float f32x2_cvt;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_cvt;
__device__ __forceinline__ bf16_t f2bf(float f)
{
    const __bf16 h = (__bf16)f;
    return __builtin_bit_cast(bf16_t, h);
}
// two values rounded and packed: `lo` in bits 0..15, `hi` in bits 16..31
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    const f32x2_cvt v = {lo, hi};
    const bf16x2_cvt h = __builtin_convertvector(v, bf16x2_cvt);
    return __builtin_bit_cast(uint32_t, h);
}

// x summed over the 32 lanes that share lane / 32 (every one of them gets the sum).  Four of the five levels are
// DPP moves inside the vector ALU -- neighbours in a quad, the other pair of the quad, then the mirror images within 8
// and within 16 lanes, which after the levels before them hold exactly what the lanes 4 and 8 away hold -- and only the
// last one (16 lanes away) goes through the LDS crossbar.  A butterfly of five shuffles costs five crossbar round trips.
template <int CTRL>
__device__ __forceinline__ float dpp_move_f32(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float sum_over_lanes32(float x)
{
    x += dpp_move_f32<0xB1>(x);     // quad_perm [1, 0, 3, 2]
    x += dpp_move_f32<0x4E>(x);     // quad_perm [2, 3, 0, 1]
    x += dpp_move_f32<0x141>(x);    // row_half_mirror
    x += dpp_move_f32<0x140>(x);    // row_mirror
    x += __shfl_xor(x, 16);
    return x;
}

template <typename T> __device__ __forceinline__ float ld(const T *p);
template <> __device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld<bf16_t>(const bf16_t *p) { return bf2f(*p); }
template <typename T> __device__ __forceinline__ void st(T *p, float v);
template <> __device__ __forceinline__ void st<float>(float *p, float v) { *p = v; }
template <> __device__ __forceinline__ void st<bf16_t>(bf16_t *p, float v) { *p = f2bf(v); }

// Where a projection's output element (row r, feature n) goes.
//  ROW    : dst[r*ld + n]
//  HEADS  : r = b*rows_per_seq + m, n = g*dh + c -> dst[((b*heads + g)*cap + m)*dh + c]
//           (the tree rows' K/V slabs)
//  APPEND : r belongs to the sequence b with tok_off[b] <= r < tok_off[b+1]; position
//           pos = row_base[b] + r - tok_off[b]; dropped when pos >= cap (cache append)
struct StoreSpec {
    enum { ROW = 0, HEADS = 1, APPEND = 2 };
    int mode;
    void *dst;
    int64_t ld;
    int heads, dh, cap, rows_per_seq, B;
    const int32_t *row_base;  // APPEND: ca_len
    const int32_t *tok_off;   // APPEND
    int32_t *dev_status;
};

// The element offset of (r, n) is store_row_part(r) + store_feat_part(n); a negative row part means the row is
// dropped.  Kernels that store many features of one row compute the row part once (for an append it contains
// the search for the row's sequence).
__device__ __forceinline__ int64_t store_row_part(const StoreSpec &s, int64_t r)
{
    if (s.mode == StoreSpec::ROW) return r * s.ld;
    if (s.mode == StoreSpec::HEADS) {
        const int64_t b = r / s.rows_per_seq;
        const int m = (int)(r - b * s.rows_per_seq);
        return (b * s.heads * (int64_t)s.cap + m) * s.dh;
    }
    int b = -1;
    for (int i = 0; i < s.B; ++i) {
        if (r >= s.tok_off[i] && r < s.tok_off[i + 1]) { b = i; break; }
    }
    if (b < 0) return -1;
    int base = s.row_base[b];
    if (base < 0) base = 0;
    const int64_t pos = (int64_t)base + (r - s.tok_off[b]);
    if (pos >= s.cap) return -1;
    return ((int64_t)b * s.heads * (int64_t)s.cap + pos) * s.dh;
}

__device__ __forceinline__ int64_t store_feat_part(const StoreSpec &s, int n)
{
    if (s.mode == StoreSpec::ROW) return n;
    const int g = n / s.dh, c = n - g * s.dh;
    return (int64_t)g * s.cap * s.dh + c;
}

// element offset of (r, n) or -1 when the element is dropped
__device__ __forceinline__ int64_t store_offset(const StoreSpec &s, int64_t r, int n)
{
    const int64_t rp = store_row_part(s, r);
    return rp < 0 ? -1 : rp + store_feat_part(s, n);
}

// ---- optional per-launch timing (hipEvents around single kernels), used by the benchmark only
enum KernelId {
    K_TREE_BUILD = 0, K_TREE_ACCEPT, K_APPEND_LEN, K_LIN_GENERIC, K_LIN_SKINNY, K_LIN_SPLITK, K_LIN_REDUCE, K_LIN_TILED, K_SCATTER,
    K_ATTN_GENERIC, K_ATTN_MFMA, K_ATTN_MERGE, K_LSA_ATTN, K_LSA_ATTN_MFMA, K_STEP_SMALL, K_ATTN_FUSED, K_PROBE_READ, K_PROBE_MFMA,
    K_RMSNORM, K_ROPE, K_SWIGLU, K_ADD_OUT, K_TREE_EXPAND, K_TREE_FINALIZE, K_TOPK_LOGPROB,
    K_LM_HEAD, K_LM_HEAD_REDUCE, K_TOPK_MERGE, K_MSG_TREE, K_MSG_ACCEPT, K_LIN_SPLITK_CHUNKED, K_LSA_FUSED, K_LSA_FUSED_PK, K_LSA_PACK, K_LSA_FUSED_PK_LEAN, K_LIN_SPLITK_XRES, K_COUNT
};
enum SiteId {
    S_NONE = 0, S_TREE_BUILD, S_LSA_QKV, S_LSA_ATTN, S_LSA_OPROJ, S_APPEND_KV, S_APPEND_LEN, S_CA_QPROJ, S_CA_CORE,
    S_CA_OPROJ, S_VERIFY_QKV, S_VERIFY_CORE, S_VERIFY_OPROJ, S_TREE_ACCEPT, S_STEP_SMALL, S_PAIR_QKV, S_PAIR_CORE,
    S_PAIR_OPROJ, S_PROBE, S_SA_QKV, S_SA_CORE, S_SA_OPROJ, S_TLI_QKV, S_TLI_CORE, S_TLI_OPROJ, S_TLI_NORM, S_TLI_ROPE,
    S_TLI_GATE_UP, S_TLI_ACT, S_TLI_DOWN, S_TLI_ADD, S_TREE_EXPAND, S_TREE_FINALIZE, S_TOPK_LOGPROB, S_LM_HEAD, S_MSG, S_LINEAR, S_MLP_NORM, S_MLP_GATE_UP, S_MLP_DOWN, S_LSA_FUSED, S_COUNT
};
// records the message moa_last_error returns and hands the code back (entry points outside moa_api.hip)
int32_t api_fail(int32_t code, const char *msg);
void prof_set_site(int site);
void prof_begin(int kernel, hipStream_t stream);   // no-ops unless profiling is enabled
void prof_end(hipStream_t stream);
// Events of the launch opened by prof_begin (nullptr when it is not being timed).  They are attached to the
// dispatch itself, so they carry the kernel's own begin and end timestamps and cost the stream nothing.
hipEvent_t prof_start_event();
hipEvent_t prof_stop_event();
#define MOA_KLAUNCH(kernel, grid, block, lds, stream, ...)                                                      \
    do {                                                                                                        \
        hipEvent_t e0_ = ::moa::prof_start_event(), e1_ = ::moa::prof_stop_event();                             \
        if (e0_ && e1_) hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, e0_, e1_, 0, __VA_ARGS__);      \
        else hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                                 \
    } while (0)

// Raises a kernel's dynamic-LDS limit the first time it is launched on a device (done[] belongs to that kernel).
// Two threads racing here set the same value twice.
inline hipError_t raise_lds_limit_once(bool (&done)[16], const void *kernel, size_t bytes)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 16 && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e == hipSuccess && dev >= 0 && dev < 16) done[dev] = true;
    return e;
}

// the integer work of a step (tree masks, accept walk, memory lengths): 2 B + 1 units of one wavefront each
struct StepSmallArgs {
    const int32_t *parent, *tok, *tgt, *tok_off;
    uint64_t *mask;
    int32_t *depth, *path, *n_path, *bonus, *ca_len, *old_len, *dev_status;
    int B, M, cap;
    int skip_masks;          // the tree masks are built elsewhere in the step: units [0, B) do nothing
};
hipError_t launch_step_small(const StepSmallArgs &a, hipStream_t stream);

// ---- LSA attention over the layer axis with the mean folded in:
// abar[t, h*dh + c] = sum_j (1/L sum_i softmax_i(S)[i][j]) V[t, j, g, c]
struct LsaAttnArgs {
    int dtype;
    const void *q, *k, *v;   // row (t*L + l): q + row*ldq + h*dh ; k, v + row*ldk + g*dh
    int64_t ldq, ldk, ldv;
    int64_t T;
    int L, Hq, Hkv, dh;
    void *abar;              // [T, Hq*dh]
};

// The pass that adds up the K slices of a weight-streaming projection, as data: what launch_linear leaves behind
// when asked not to launch it (LinArgs::sum_out), what another launch can carry (LinArgs::carry_sum) and what
// launch_splitk_sum runs.
// Rotary position embedding of a decoder layer's queries and draft keys (position = clamped prefix length + depth of
// the node; the pair (c, c + dh/2) of every head is rotated by position * theta^(-2c/dh), the angle in double
// precision): everything launch_rope needs, so that a projection can apply it on the way out.
struct RopeArgs {
    void *q;                     // [B*Mn, H*dh]
    void *k_draft;               // [B, Hkv, M, dh] slabs; rows node0 .. node0 + Mn - 1 are this call's
    const int32_t *prefix_len, *depth;
    int B, Mn, M, node0, H, Hkv, dh, P_cap;
    double theta;
};

// Residual + RMS norm behind a projection (a pre-norm block's second half begins with it): h = x + y in single
// precision, n = h / sqrt(mean(h^2) + eps) * g in the storage type -- what launch_rmsnorm makes of x and the stored y.
struct NormArgs {
    const void *x;       // [R, N] the block's input (storage type)
    const void *g;       // [N]
    float eps;
    float *h;            // [R, N] out
    void *n;             // [R, N] out
};

struct SumArgs {
    int blocks;          // workgroups of 256 threads; 0 = nothing to do
    int64_t R;
    int nseg;
    StoreSpec st[4];     // where each segment's sums go
    int tile_begin[5];   // first 64-feature tile of each segment; [nseg] = total tiles
    int splits, ntot;    // K slices; total features = row length of the partial buffer
    const float *part;   // [row tiles][splits][64][ntot]
    int epi;             // LinArgs::EPI_*
    const float *epi_res;
    void *epi_out;
    RopeArgs rope;       // EPI_ROPE
    double rope_log_theta;
    NormArgs norm;       // EPI_ADD_NORM: one workgroup per row (blocks = R)
};
hipError_t launch_splitk_sum(const SumArgs &s, hipStream_t stream);

struct LinSeg {
    const void *W;  // [N, K] row-major
    int N;
    StoreSpec st;
    const void *X;  // this segment's own activations [R, K] (nullptr: LinArgs::X); same R and K for all segments
    int64_t ldx;
};

struct LinArgs {
    const void *X;  // [R, K] with row stride ldx
    int64_t R;
    int K;
    int64_t ldx;
    int nseg;
    LinSeg seg[4];
    void *ws;          // optional scratch for the split-K kernel (linear_workspace_bytes)
    size_t ws_bytes;
    StepSmallArgs rider;   // optional: integer work carried in rider_units spare workgroups of the projection's grid
    int rider_units;       // 0 = none; the work is done when the projection kernel has finished
    // Optional row-wise step on the projection's result.  Where partial sums are added up by a second kernel that
    // kernel does it and the projected values themselves are never stored; on the other paths the projection is
    // stored as its segments say and a small kernel follows.
    //  EPI_ADD_F32: one segment; epi_out[r, n] = epi_res[r, n] + y[r, n]   (row length N)
    //  EPI_SWIGLU : two segments of equal N stored side by side in one row of 2N; epi_out[r, j] = silu(y0[r, j]) * y1[r, j]
    //  EPI_ROPE   : three segments -- queries (row store), draft keys (head slabs), draft values; the first two get
    //               their rotary position embedding (`rope`), exactly as launch_rope would apply it to the stored result
    //  EPI_ADD_NORM: one segment of N <= 8192 features; `norm`: h = x + y, n = rmsnorm(h) g; y itself is stored (where the
    //               segment says) only on the paths that finish with a kernel of their own
    enum { EPI_NONE = 0, EPI_ADD_F32 = 1, EPI_SWIGLU = 2, EPI_ROPE = 3, EPI_ADD_NORM = 4 };
    int epi;
    const float *epi_res;
    void *epi_out;
    RopeArgs rope;
    NormArgs norm;
    // The summing pass of an earlier weight-streaming projection, carried in spare workgroups at the front of this
    // launch's grid: it is done when this launch has finished, and must neither feed this projection nor depend on
    // it.  Only the tiled kernel carries; on the other paths the pass is launched apart, first.  A host pointer, read
    // during the call; NULL or blocks == 0 = nothing.
    const SumArgs *carry_sum;
    // Weight-streaming path only: do not launch the pass that adds up the K slices but describe it here (blocks = 0
    // when another kernel ran and nothing is left to do).  The caller has it carried by a later launch or runs
    // launch_splitk_sum; the partial sums (ws) must stay untouched until then.
    SumArgs *sum_out;
};

// Y_s = X_s W_s^T for up to four weight matrices (one launch on the fast paths; segments usually share X).
hipError_t launch_linear(int dtype, const LinArgs &a, hipStream_t stream);
// While an object of this type lives, this thread's projections keep to kernels that leave LDS and registers for a
// second kernel on the same compute units (the two-stream schedule runs its branches side by side).
struct LinearLeaveRoom {
    LinearLeaveRoom();
    ~LinearLeaveRoom();
    bool before;
};
// scratch the fast weight-streaming path wants for R rows and ntot output features in total (0 = not used)
size_t linear_workspace_bytes(int dtype, int64_t R, int K, int ntot);

// dst(store spec) = X, element by element (NULL-weight projections that still change layout)
hipError_t launch_scatter_copy(int dtype, const void *X, int64_t R, int N, int64_t ldx, const StoreSpec &st,
                               hipStream_t stream);

// ---- tree
hipError_t launch_tree_build(const int32_t *parent, int B, int M, uint64_t *mask, int32_t *depth,
                             int32_t *dev_status, hipStream_t stream);
hipError_t launch_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt, int B, int M,
                              int32_t *path, int32_t *n_path, int32_t *bonus, hipStream_t stream);
hipError_t launch_append_lengths(const int32_t *tok_off, int B, int32_t *ca_len, int cap, int32_t *dev_status,
                                 hipStream_t stream);
// tree mask + accept walk + cache length update of one step in a single launch; old_len[B] receives the
// (clamped) lengths from before the update, which is where the append writes its rows


// ---- attention core (cross-attention when mask == nullptr / Mt == 0)
struct AttnArgs {
    int dtype;
    const void *q;        // [B*Mq, H*dh] row-major
    const void *kcache;   // [B, Hkv, P_cap, dh]
    const void *vcache;
    const void *ktree;    // [B, Hkv, Mt, dh] or nullptr
    const void *vtree;
    const int32_t *len;   // [B] visible cache rows
    const uint64_t *mask; // [B, Mq, W] or nullptr
    void *out;            // [B*Mq, H*dh]
    int B, Mq, Mt, H, Hkv, dh, P_cap;
    // A call on part of a tree (level-by-level drafting): the Mq queries are the nodes mask_row0 .. of a tree of
    // mask_rows nodes (mask is [B, mask_rows, ceil(mask_rows/64)]), the tree slabs have tree_cap rows of which the
    // first Mt are keys.  Zero = the whole tree: mask_rows = Mq, tree_cap = Mt (filled in by launch_attn).
    int tree_cap, mask_rows, mask_row0;
    int empty_is_error;   // cross-attention: len == 0 -> flag + zeros
    int32_t *dev_status;
    void *ws;
    size_t ws_bytes;
};
size_t attn_workspace_bytes(int dtype, int B, int Mq, int H, int Hkv, int dh, int P_cap);
hipError_t launch_attn(const AttnArgs &a, hipStream_t stream);
// Two independent cores of the same shape (cross-attention and one verification layer) in one launch; P_cap may
// differ, each call's ws must hold attn_workspace_bytes for the larger one.  Falls back to two launches.
hipError_t launch_attn_pair(const AttnArgs &a0, const AttnArgs &a1, hipStream_t stream);

// ---- row-wise pieces of a reused decoder layer
hipError_t launch_rmsnorm(int dtype, const void *x, const void *res, int64_t R, int d, const void *g, float eps,
                          float *h_out, void *n_out, hipStream_t stream);
hipError_t launch_rope(int dtype, void *q, void *k_draft, const int32_t *prefix_len, const int32_t *depth, int B, int Mn,
                       int M, int node0, int H, int Hkv, int dh, double theta, int P_cap, hipStream_t stream);
hipError_t launch_fold_weights(int dtype, const void *a, const void *b, int N, int J, int K, void *out, hipStream_t stream);
hipError_t launch_swiglu(int dtype, const void *gu, int64_t R, int d_ff, void *act, hipStream_t stream);
hipError_t launch_add_out(int dtype, const float *h, const void *t, int64_t n, void *out, hipStream_t stream);

// ---- LSA in one kernel: projection of a token's layer rows, attention over the layers, mean; writes the mean-folded
// heads abar [T, Hq*dh] (the output projection is a launch of its own, on one row per token).  rider / carry_sum as in
// LinArgs: work of other calls carried in spare workgroups at the front of the grid.
struct LsaFusedCall {
    int dtype;
    const void *hs, *wq, *wk, *wv;
    const void *w_packed;    // wq / wk / wv in the order launch_lsa_pack_weights writes, or NULL; when given, wq / wk / wv are not read
    void *abar;
    int64_t T;
    int L, d_in, Hq, Hkv, dh;
    StepSmallArgs rider;
    int rider_units;
    const SumArgs *carry_sum;
    int leave_room;      // take the largest token tile: fewest workgroups, so that another stream's kernels find free compute units
};
// shapes and alignments the kernel takes (bf16, head_dim 128, L <= 96, d_in in 64s, an even number of query heads per KV head)
bool lsa_fused_ok(int dtype, int L, int d_in, int Hq, int Hkv, int dh, const void *hs, const void *wq, const void *wk,
                  const void *wv, const void *abar);
bool lsa_fused_shape_ok(int dtype, int L, int d_in, int Hq, int Hkv, int dh);
hipError_t launch_lsa_fused(const LsaFusedCall &c, hipStream_t stream);
// the weights of those shapes rearranged once into MFMA-operand order, for the form of the kernel that keeps them in registers
size_t lsa_packed_weight_bytes(int d_in, int Hq, int Hkv, int dh);
hipError_t launch_lsa_pack_weights(const void *wq, const void *wk, const void *wv, void *out, int d_in, int Hq, int Hkv,
                                   hipStream_t stream);

// ---- LSA attention over the layer axis (LsaAttnArgs is declared above, beside the projections that can carry it)
size_t lsa_attn_lds_bytes(int dtype, int L, int dh);
hipError_t launch_lsa_attn(const LsaAttnArgs &a, hipStream_t stream);

}  // namespace moa
