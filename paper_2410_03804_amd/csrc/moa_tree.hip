// Draft-tree integer kernels: ancestor bitsets + depths, greedy accept walk, cache length update.
// One 64-lane wavefront per sequence; a mask row is at most 4 x 64-bit words (M <= 256).
#include "moa_common.h"
#include "../../include/moa.h"

namespace moa {

// Tree structure (paper Sec. 2.2, tree drafting): mask[i] = {i} U ancestors(i).
// Lane t walks the parent chain of nodes t, t+64, ...; a walk is at most M steps because a
// valid parent index is smaller than its child, and it stops at the first invalid entry.
__device__ __forceinline__ void tree_build_block(int b, const int32_t *__restrict__ parent, int M,
                                                 uint64_t *__restrict__ mask, int32_t *__restrict__ depth,
                                                 int32_t *dev_status, int32_t *par /* LDS [MOA_MAX_TREE] */)
{
    const int W = (M + 63) >> 6;
    const int32_t *p = parent + (int64_t)b * M;
    bool bad = false;
    for (int i = threadIdx.x; i < M; i += 64) {
        const int32_t v = p[i];
        par[i] = v;
        if (i == 0 ? (v != -1) : (v < 0 || v >= i)) bad = true;
    }
    __syncthreads();
    for (int i = threadIdx.x; i < M; i += 64) {
        uint64_t row[MOA_MAX_TREE / 64] = {0, 0, 0, 0};
        int cur = i, steps = 0;
        while (steps <= M) {
            row[cur >> 6] |= 1ull << (cur & 63);
            ++steps;
            if (cur == 0) break;
            const int nxt = par[cur];
            if (nxt < 0 || nxt >= cur) break;   // invalid entry: flagged above, walk ends here
            cur = nxt;
        }
        for (int w = 0; w < W; ++w) mask[((int64_t)b * M + i) * W + w] = row[w];
        depth[(int64_t)b * M + i] = steps - 1;
    }
    if (bad && dev_status) atomicOr(dev_status, MOA_DEV_BAD_PARENT);
}

__global__ __launch_bounds__(64) void k_tree_build(const int32_t *__restrict__ parent, int M,
                                                   uint64_t *__restrict__ mask, int32_t *__restrict__ depth,
                                                   int32_t *dev_status)
{
    __shared__ int32_t par[MOA_MAX_TREE];
    tree_build_block(blockIdx.x, parent, M, mask, depth, dev_status, par);
}

// Greedy acceptance (paper Sec. 2.2: everything after the first mismatch is discarded).
// The 64 lanes test 64 candidate children at a time; the lowest matching index wins.
__device__ __forceinline__ void tree_accept_block(int b, const int32_t *__restrict__ parent,
                                                  const int32_t *__restrict__ tok, const int32_t *__restrict__ tgt,
                                                  int M, int32_t *__restrict__ path, int32_t *__restrict__ n_path,
                                                  int32_t *__restrict__ bonus, int32_t *par, int32_t *tk /* LDS */)
{
    const int lane = threadIdx.x;
    for (int i = lane; i < M; i += 64) {
        par[i] = parent[(int64_t)b * M + i];
        tk[i] = tok[(int64_t)b * M + i];
        path[(int64_t)b * M + i] = -1;
    }
    __syncthreads();
    int cur = 0, n = 1;
    if (lane == 0) path[(int64_t)b * M] = 0;
    for (int step = 1; step < M; ++step) {          // a path has at most M nodes
        const int want = tgt[(int64_t)b * M + cur];
        int next = -1;
        for (int base = cur + 1 - ((cur + 1) & 63); base < M; base += 64) {
            const int c = base + lane;
            const bool hit = c > cur && c < M && par[c] == cur && tk[c] == want;
            const uint64_t votes = __ballot(hit);
            if (votes) { next = base + __ffsll((long long)votes) - 1; break; }
        }
        if (next < 0) break;
        cur = next;
        if (lane == 0) path[(int64_t)b * M + n] = cur;
        ++n;
    }
    if (lane == 0) {
        n_path[b] = n;
        bonus[b] = tgt[(int64_t)b * M + cur];
    }
}

__global__ __launch_bounds__(64) void k_tree_accept(const int32_t *__restrict__ parent,
                                                    const int32_t *__restrict__ tok,
                                                    const int32_t *__restrict__ tgt, int M,
                                                    int32_t *__restrict__ path, int32_t *__restrict__ n_path,
                                                    int32_t *__restrict__ bonus)
{
    __shared__ int32_t par[MOA_MAX_TREE], tk[MOA_MAX_TREE];
    tree_accept_block(blockIdx.x, parent, tok, tgt, M, path, n_path, bonus, par, tk);
}

// ca_len[b] += rows appended for sequence b (clamped to the capacity), after the projection
// kernel that read the old lengths.
__device__ __forceinline__ void append_length_one(int b, const int32_t *__restrict__ tok_off, int32_t *ca_len,
                                                  int cap, int32_t *old_len, int32_t *dev_status)
{
    int base = ca_len[b];
    int flag = 0;
    if (base < 0 || base > cap) { flag |= MOA_DEV_BAD_LENGTH; base = base < 0 ? 0 : cap; }
    int add = tok_off[b + 1] - tok_off[b];
    if (add < 0) add = 0;
    if ((int64_t)base + add > cap) { flag |= MOA_DEV_CACHE_FULL; add = cap - base; }
    if (old_len) old_len[b] = base;
    ca_len[b] = base + add;
    if (flag && dev_status) atomicOr(dev_status, flag);
}

__global__ void k_append_lengths(const int32_t *__restrict__ tok_off, int B, int32_t *ca_len, int cap,
                                 int32_t *dev_status)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) append_length_one(b, tok_off, ca_len, cap, nullptr, dev_status);
}

// The three integer pieces of a step in one launch: blocks [0, B) build the tree masks, blocks [B, 2B) walk the
// accepted paths, the last block advances the cross-attention memory lengths (keeping the old ones for the
// projection that appends the rows).
__global__ __launch_bounds__(64) void k_step_small(StepSmallArgs a)
{
    __shared__ int32_t par[MOA_MAX_TREE], tk[MOA_MAX_TREE];
    const int blk = blockIdx.x;
    if (blk < a.B) {
        tree_build_block(blk, a.parent, a.M, a.mask, a.depth, a.dev_status, par);
    } else if (blk < 2 * a.B) {
        tree_accept_block(blk - a.B, a.parent, a.tok, a.tgt, a.M, a.path, a.n_path, a.bonus, par, tk);
    } else {
        for (int b = threadIdx.x; b < a.B; b += 64) append_length_one(b, a.tok_off, a.ca_len, a.cap, a.old_len, a.dev_status);
    }
}

hipError_t launch_tree_build(const int32_t *parent, int B, int M, uint64_t *mask, int32_t *depth,
                             int32_t *dev_status, hipStream_t stream)
{
    { prof_begin(K_TREE_BUILD, stream); MOA_KLAUNCH(k_tree_build, dim3(B), dim3(64), 0, stream, parent, M, mask, depth, dev_status); prof_end(stream); }
    return hipGetLastError();
}

hipError_t launch_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt, int B, int M,
                              int32_t *path, int32_t *n_path, int32_t *bonus, hipStream_t stream)
{
    { prof_begin(K_TREE_ACCEPT, stream); MOA_KLAUNCH(k_tree_accept, dim3(B), dim3(64), 0, stream, parent, tok, tgt, M, path, n_path, bonus); prof_end(stream); }
    return hipGetLastError();
}

hipError_t launch_step_small(const StepSmallArgs &a, hipStream_t stream)
{
    prof_begin(K_STEP_SMALL, stream);
    MOA_KLAUNCH(k_step_small, dim3(2 * a.B + 1), dim3(64), 0, stream, a);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_append_lengths(const int32_t *tok_off, int B, int32_t *ca_len, int cap, int32_t *dev_status,
                                 hipStream_t stream)
{
    { prof_begin(K_APPEND_LEN, stream); MOA_KLAUNCH(k_append_lengths, dim3((B + 63) / 64), dim3(64), 0, stream, tok_off, B, ca_len, cap,
                       dev_status); prof_end(stream); }
    return hipGetLastError();
}

}  // namespace moa
