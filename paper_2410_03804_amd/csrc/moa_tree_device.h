// Device-side bodies of the draft-tree integer work, shared by the stand-alone kernels and by the projection
// kernels that carry this work in spare workgroups of their grid.  Each body is written for ONE 64-lane
// wavefront (threadIdx.x < 64) and synchronises at wavefront level only.
#ifndef MOA_TREE_DEVICE_H
#define MOA_TREE_DEVICE_H
#include "moa_common.h"
#include "../../include/moa.h"

namespace moa {

// LDS traffic of one wavefront is processed in order; this keeps the compiler from moving a read of another
// lane's data above the write that produced it
__device__ __forceinline__ void tree_wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

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
    tree_wave_sync();
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
    tree_wave_sync();
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

// One unit of the three integer pieces of a step: units [0, B) build the tree masks, [B, 2B) walk the accepted
// paths, unit 2B advances the cross-attention memory lengths (keeping the old ones for the projection that
// appends the rows).  par / tk: LDS, MOA_MAX_TREE ints each.
__device__ __forceinline__ void step_small_unit(const StepSmallArgs &a, int unit, int32_t *par, int32_t *tk)
{
    if (unit < a.B) {
        if (!a.skip_masks) tree_build_block(unit, a.parent, a.M, a.mask, a.depth, a.dev_status, par);
    } else if (unit < 2 * a.B) {
        tree_accept_block(unit - a.B, a.parent, a.tok, a.tgt, a.M, a.path, a.n_path, a.bonus, par, tk);
    } else {
        for (int b = threadIdx.x; b < a.B; b += 64) append_length_one(b, a.tok_off, a.ca_len, a.cap, a.old_len, a.dev_status);
    }
}

}  // namespace moa
#endif
