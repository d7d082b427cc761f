// Greedy token of the LLM at every tree node: tgt[r] = argmax_v x[r] . W[v] over the vocabulary (Sec. 2.1,
// y ~ Softmax(LM_head(o)); greedy verification takes the arg max).  The logits are never stored: the head is one
// pass over its weights ([V, d], 1 GiB at the Llama-3 shape, the largest single read of a decoding cycle), each
// workgroup reduces its 128 tokens to one (logit, id) pair per row and a second small kernel reduces the pairs.
// Weight streaming as in the split-K projections (64 contiguous bytes per lane straight into MFMA operands, the
// next K chunk requested before this one is used), but a workgroup walks the whole K range, so there are no
// partial sums to write: with V/128 = 1002 workgroups the grid is deep enough without splitting K.
#include "moa_common.h"
#include "../../include/moa.h"

namespace moa {

struct LmHeadArgs {
    const bf16_t *X;      // [R, K]
    const bf16_t *W;      // [V, K]
    int R, K, V;
    float *pval;          // [tiles, 64]
    int32_t *pid;         // [tiles, 64]
};

__device__ __forceinline__ bool better(float a, int ia, float b, int ib) { return a > b || (a == b && ia < ib); }

// TG groups of 16 tokens per wavefront: a workgroup's tile is 64 TG tokens, and the activation chunk it stages per K
// chunk serves that many -- with TG = 1 the workgroups pull as many activation bytes out of the L2 as weight bytes out
// of HBM (one 480 KB pass over X per 64 tokens).
template <int NQ, int TG, int NW>
__global__ __launch_bounds__(64 * NW, 2) void k_lm_head_argmax(LmHeadArgs a)
{
    constexpr int KS = 128 * NQ, LDK = KS + 8, CPR = KS / 8, NT = 64 * NW, XL = (64 * CPR) / NT;
    extern __shared__ __attribute__((aligned(16))) bf16_t Xs[];   // [64][LDK]; reused for the per-wave bests at the end
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, kg = lane >> 4;
    const int tile = blockIdx.x;
    const int n0 = (tile * NW + wave) * 16 * TG;
    const bf16_t *wp[TG];
#pragma unroll
    for (int t = 0; t < TG; ++t) {
        int wrow = n0 + 16 * t + li;
        if (wrow > a.V - 1) wrow = a.V - 1;                 // tokens past the end repeat the last one; masked below
        wp[t] = a.W + (int64_t)wrow * a.K + 8 * kg;         // k slot (q, j, kg) is k = 128 q + 32 j + 8 kg
    }
    const int nchunk = a.K / KS;

    // Piece c = tid + NT i of the slice is row c / CPR, 16-byte column c % CPR: the column and the row's remainder
    // are the same for every i, so one 32-bit lane offset serves all loads and the per-i part of the address is
    // uniform (a scalar base): sixteen 64-bit lane addresses kept alive across the chunk loop would not fit the
    // register budget of two workgroups per CU, and reloading spilled ones waits for every load in flight.
    static_assert(NT % CPR == 0, "rows advance by a whole number per NT pieces");
    constexpr int RSTEP = NT / CPR;                         // rows between piece i and piece i + 1
    const uint32_t xoff = (uint32_t)(((tid / CPR) * a.K + 8 * (tid % CPR)) * (int)sizeof(bf16_t));
    u32x4 xr[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) xr[i] = u32x4{0u, 0u, 0u, 0u};   // rows past the end stay zero; never used
    auto load_x = [&](int kc) {
        const char *xb = (const char *)(a.X + (int64_t)kc * KS);
#pragma unroll
        for (int i = 0; i < XL; ++i)
            if (tid / CPR + RSTEP * i < a.R)
                xr[i] = *(const u32x4 *)(xb + (int64_t)i * RSTEP * a.K * (int64_t)sizeof(bf16_t) + xoff);
    };
    bf16x8 wf[2][TG][NQ][4];
    auto load_w = [&](int set, int kc) {
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) wf[set][t][q][j] = *(const bf16x8 *)(wp[t] + (int64_t)kc * KS + 128 * q + 32 * j);
    };
    load_x(0);
    load_w(0, 0);
    f32x4 acc[TG][4];
#pragma unroll
    for (int t = 0; t < TG; ++t)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[t][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    auto chunk = [&](int set, int kc) {
        if (kc + 1 < nchunk) load_w(set ^ 1, kc + 1);       // the next chunk's weights are on their way
        // Bare barriers (LDS traffic drained, then s_barrier): __syncthreads() also waits for every outstanding
        // global load, which would hold each chunk until the weights just requested for the next one have arrived.
        if (kc > 0) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // every wave is done reading the previous slice
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int c = tid + NT * i;
            *(u32x4 *)&Xs[(c / CPR) * LDK + 8 * (c % CPR)] = xr[i];
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (kc + 1 < nchunk) load_x(kc + 1);
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x8 xf[4];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) xf[rb] = *(const bf16x8 *)&Xs[(16 * rb + li) * LDK + 128 * q + 32 * j + 8 * kg];
#pragma unroll
                for (int t = 0; t < TG; ++t)
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        acc[t][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[set][t][q][j], xf[rb], acc[t][rb], 0, 0, 0);
            }
    };
    for (int kc = 0; kc < nchunk; kc += 2) {                // two chunks per trip: the register sets alternate statically
        chunk(0, kc);
        if (kc + 1 < nchunk) chunk(1, kc + 1);
    }

    // lane holds tokens n0 + 16 t + 4 kg .. + 3 for row 16 rb + li: best of the workgroup's tokens per row
    __syncthreads();
    float *wv = (float *)Xs;                                 // [NW waves][64 rows]
    int32_t *wi = (int32_t *)(wv + 64 * NW);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
        float bv = -INFINITY;
        int bi = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < TG; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int id = n0 + 16 * t + 4 * kg + e;
                const float v = acc[t][rb][e];
                if (id < a.V && better(v, id, bv, bi)) { bv = v; bi = id; }
            }
#pragma unroll
        for (int o = 16; o <= 32; o <<= 1) {
            const float ov = __shfl_xor(bv, o);
            const int oi = __shfl_xor(bi, o);
            if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
        }
        if (kg == 0) { wv[wave * 64 + 16 * rb + li] = bv; wi[wave * 64 + 16 * rb + li] = bi; }
    }
    __syncthreads();
    if (tid < 64) {
        float bv = wv[tid];
        int bi = wi[tid];
#pragma unroll
        for (int w = 1; w < NW; ++w)
            if (better(wv[w * 64 + tid], wi[w * 64 + tid], bv, bi)) { bv = wv[w * 64 + tid]; bi = wi[w * 64 + tid]; }
        a.pval[(int64_t)tile * 64 + tid] = bv;
        a.pid[(int64_t)tile * 64 + tid] = bi;
    }
}

// one workgroup per row: the best of the tiles' pairs
__global__ __launch_bounds__(256) void k_lm_head_reduce(const float *__restrict__ pval, const int32_t *__restrict__ pid, int tiles,
                                                        int32_t *__restrict__ tgt, float *__restrict__ best)
{
    __shared__ float sv[4];
    __shared__ int si[4];
    const int r = blockIdx.x, t = threadIdx.x;
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int k = t; k < tiles; k += 256) {
        const float v = pval[(int64_t)k * 64 + r];
        const int i = pid[(int64_t)k * 64 + r];
        if (better(v, i, bv, bi)) { bv = v; bi = i; }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        const float ov = __shfl_xor(bv, o);
        const int oi = __shfl_xor(bi, o);
        if (better(ov, oi, bv, bi)) { bv = ov; bi = oi; }
    }
    if ((t & 63) == 0) { sv[t >> 6] = bv; si[t >> 6] = bi; }
    __syncthreads();
    if (t == 0) {
#pragma unroll
        for (int w = 1; w < 4; ++w)
            if (better(sv[w], si[w], bv, bi)) { bv = sv[w]; bi = si[w]; }
        tgt[r] = bi;
        if (best) best[r] = bv;
    }
}

}  // namespace moa

using namespace moa;

extern "C" {

int32_t moa_lm_head_workspace_bytes(int32_t V, size_t *bytes_host)
{
    if (!bytes_host) return api_fail(MOA_ERR_NULL, "lm_head_workspace_bytes: bytes_host is NULL");
    if (V < 1) return api_fail(MOA_ERR_SHAPE, "lm_head_workspace_bytes: V < 1");
    *bytes_host = (size_t)((V + 63) / 64) * 64 * (sizeof(float) + sizeof(int32_t));
    return MOA_OK;
}

int32_t moa_lm_head_argmax(int32_t dtype, const void *x, int32_t R, int32_t d, const void *w, int32_t V, int32_t *tgt,
                           float *best, void *ws, size_t ws_bytes, void *stream)
{
    if (!x || !w || !tgt) return api_fail(MOA_ERR_NULL, "lm_head_argmax: NULL pointer");
    if (dtype != MOA_BF16) return api_fail(MOA_ERR_DTYPE, "lm_head_argmax: bf16 only");
    if (R < 1 || V < 1 || d < 128 || d % 128) return api_fail(MOA_ERR_SHAPE, "lm_head_argmax: R >= 1, V >= 1, d a multiple of 128");
    if ((((uintptr_t)x) | ((uintptr_t)w)) & 15) return api_fail(MOA_ERR_SHAPE, "lm_head_argmax: x and w must be 16-byte aligned");
    constexpr int TG = 2, NW = 4;               // 128 tokens per workgroup (eight wavefronts, 256 tokens: 223 against 214 us)
    const int tiles = (V + 16 * TG * NW - 1) / (16 * TG * NW);
    const size_t need = (size_t)tiles * 64 * (sizeof(float) + sizeof(int32_t));
    if (!ws || (((uintptr_t)ws) & 255) || ws_bytes < need) return api_fail(MOA_ERR_WORKSPACE, "lm_head_argmax: workspace NULL, misaligned or smaller than moa_lm_head_workspace_bytes");
    hipStream_t st = (hipStream_t)stream;
    // 256-wide K chunks: with 512-wide ones the two weight sets and the staged activations no longer fit the registers
    // of two workgroups per CU, and every reload of a spilled value waits for all loads in flight (measured 319 us
    // against 241 us at 60 x 4096 x 128256)
    const int nq = d % 256 == 0 ? 2 : 1;
    const size_t lds = (size_t)64 * (128 * nq + 8) * sizeof(bf16_t);
    // 64 rows per pass (the weights are streamed once per pass; a tree has at most 256 nodes)
    for (int r0 = 0; r0 < R; r0 += 64) {
        LmHeadArgs a;
        a.X = (const bf16_t *)x + (int64_t)r0 * d;
        a.W = (const bf16_t *)w;
        a.R = R - r0 < 64 ? R - r0 : 64;
        a.K = d;
        a.V = V;
        a.pval = (float *)ws;
        a.pid = (int32_t *)((float *)ws + (size_t)tiles * 64);
        prof_set_site(S_LM_HEAD);
        prof_begin(K_LM_HEAD, st);
        if (nq == 2) MOA_KLAUNCH((k_lm_head_argmax<2, TG, NW>), dim3(tiles), dim3(64 * NW), lds, st, a);
        else MOA_KLAUNCH((k_lm_head_argmax<1, TG, NW>), dim3(tiles), dim3(64 * NW), lds, st, a);
        prof_end(st);
        if (hipGetLastError() != hipSuccess) return api_fail(MOA_ERR_HIP, "lm_head_argmax: launch failed");
        prof_begin(K_LM_HEAD_REDUCE, st);
        MOA_KLAUNCH(k_lm_head_reduce, dim3(a.R), dim3(256), 0, st, a.pval, a.pid, tiles, tgt + r0, best ? best + r0 : nullptr);
        prof_end(st);
        if (hipGetLastError() != hipSuccess) return api_fail(MOA_ERR_HIP, "lm_head_argmax: launch failed");
    }
    return MOA_OK;
}

}  // extern "C"
