// Attention core shared by the draft model's cross-attention (no mask, cache rows only) and the
// tree-masked verification attention (cache rows, then the tree rows filtered by the ancestor
// bitset).  Input Q is already projected; the output is the concatenated heads before W_o.
//
//   k_attn_generic   any dtype / head_dim <= 256: one wavefront per (sequence, query, head),
//                    64 keys per step, exact online softmax with wavefront shuffles.
//   k_attn_mfma      bf16, head_dim 64 / 128: split-KV.  A workgroup owns one (sequence, KV head),
//                    one slice of the key range and up to 128*NBLK query rows (the GQA group's heads
//                    times the tree tokens are folded into the row dimension, so K/V are read once for
//                    all of them).  K/V tiles of 32 keys are staged in LDS by 16-byte loads; scores are
//                    computed transposed (S^T = K Q^T) so that a lane owns one query column and the
//                    softmax max/sum need a single cross-lane exchange; P^T feeds the second MFMA
//                    straight from registers and V is transposed on its way into LDS.
//   k_attn_merge     combines the per-slice (max, sum, accumulator) triples.
#include "moa_common.h"
#include "../../include/moa.h"

#include <math.h>
#include <stdlib.h>

namespace moa {

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ int clamp_len(int len, int cap, int32_t *dev_status)
{
    if (len < 0 || len > cap) {
        if (dev_status) atomicOr(dev_status, MOA_DEV_BAD_LENGTH);
        len = len < 0 ? 0 : cap;
    }
    return len;
}

// ------------------------------------------------------------------ generic
template <typename T>
__global__ __launch_bounds__(64) void k_attn_generic(AttnArgs a)
{
    __shared__ float qs[256];
    const int lane = threadIdx.x;
    const int h = blockIdx.x % a.H;
    const int m = (blockIdx.x / a.H) % a.Mq;
    const int b = blockIdx.x / (a.H * a.Mq);
    const int g = h / (a.H / a.Hkv);
    const int dh = a.dh, W = (a.Mq + 63) >> 6;
    const float scale = 1.0f / sqrtf((float)dh);

    const T *q = (const T *)a.q + (((int64_t)b * a.Mq + m) * a.H + h) * dh;
    for (int c = lane; c < dh; c += 64) qs[c] = ld<T>(q + c);
    __syncthreads();

    const int len = clamp_len(a.len[b], a.P_cap, lane == 0 ? a.dev_status : nullptr);
    const int Mt = a.mask ? a.Mt : 0;
    const int total = len + Mt;
    const T *kc = (const T *)a.kcache + ((int64_t)b * a.Hkv + g) * (int64_t)a.P_cap * dh;
    const T *vc = (const T *)a.vcache + ((int64_t)b * a.Hkv + g) * (int64_t)a.P_cap * dh;
    const T *kt = (const T *)a.ktree + ((int64_t)b * a.Hkv + g) * (int64_t)a.Mt * dh;
    const T *vt = (const T *)a.vtree + ((int64_t)b * a.Hkv + g) * (int64_t)a.Mt * dh;
    const uint64_t *mrow = a.mask ? a.mask + ((int64_t)b * a.Mq + m) * W : nullptr;

    float mrun = -INFINITY, lrun = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int base = 0; base < total; base += 64) {
        const int kidx = base + lane;
        float s = -INFINITY;
        if (kidx < total) {
            const T *krow = nullptr;
            if (kidx < len) {
                krow = kc + (int64_t)kidx * dh;
            } else {
                const int j = kidx - len;
                if ((mrow[j >> 6] >> (j & 63)) & 1) krow = kt + (int64_t)j * dh;
            }
            if (krow) {
                float d = 0.f;
                for (int c = 0; c < dh; ++c) d = fmaf(qs[c], ld<T>(krow + c), d);
                s = d * scale;
            }
        }
        const float mnew = fmaxf(mrun, wave_max(s));
        if (mnew == -INFINITY) continue;   // nothing visible yet (same decision in every lane)
        const float p = (s == -INFINITY) ? 0.f : expf(s - mnew);
        const float corr = expf(mrun - mnew);
        lrun = lrun * corr + wave_sum(p);
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[c] *= corr;
        const int nk = min(64, total - base);
        for (int kk = 0; kk < nk; ++kk) {
            const float pk = __shfl(p, kk);
            if (pk == 0.f) continue;
            const int ki = base + kk;
            const T *vrow = ki < len ? vc + (int64_t)ki * dh : vt + (int64_t)(ki - len) * dh;
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (lane + 64 * c < dh) acc[c] = fmaf(pk, ld<T>(vrow + lane + 64 * c), acc[c]);
        }
        mrun = mnew;
    }
    T *o = (T *)a.out + (((int64_t)b * a.Mq + m) * a.H + h) * dh;
    const float inv = lrun > 0.f ? 1.0f / lrun : 0.f;
    for (int c = 0; c < 4; ++c)
        if (lane + 64 * c < dh) st<T>(o + lane + 64 * c, acc[c] * inv);
    if (lrun == 0.f && a.empty_is_error && lane == 0 && a.dev_status) atomicOr(a.dev_status, MOA_DEV_EMPTY_KEYS);
}

// ------------------------------------------------------------------ MFMA split-KV
struct SplitGeom {
    int nsplit;     // key-range slices
    int rowtiles;   // workgroups along the G*Mq rows of one (sequence, KV head)
    int rows_pad;   // rowtiles * rows per workgroup
};

typedef _Float16 f16_t;
typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;

// up to two independent calls of the same shape in one launch (blockIdx.z / nbg picks the call)
struct AttnGroup {
    AttnArgs a[2];
    int nbg;   // B * Hkv of one call
};

constexpr int KT = 32;        // keys per tile
constexpr int VLD = KT + 8;   // padded row of the transposed V tile

// position of key k (0..31) inside a transposed V row: bits 2 and 3 swapped, so that the eight
// keys one lane contributes to a 16-deep MFMA step are contiguous
__device__ __forceinline__ int vpos(int k) { return (k & ~12) | ((k & 4) << 1) | ((k & 8) >> 1); }

template <int DH, int NBLK>
__global__ __launch_bounds__(256) void k_attn_mfma(AttnGroup grp, SplitGeom geo)
{
    const int call = blockIdx.z / grp.nbg;
    const AttnArgs &a = grp.a[call];
    f16_t *__restrict__ part_o = (f16_t *)a.ws;
    float *__restrict__ part_ml = (float *)(part_o + (size_t)grp.nbg * geo.nsplit * geo.rows_pad * DH);
    constexpr int KLD = DH + 8;           // padded K row (bf16)
    constexpr int NKS = DH / 16;          // MFMA steps along head_dim
    constexpr int NDB = DH / 32;          // 32-wide blocks of head_dim in the output
    constexpr int CPK = DH / 8;           // 16-byte chunks per key row
    constexpr int NLD = (KT * CPK) / 256; // chunks per thread per tile (1 for DH 64, 2 for DH 128)
    __shared__ __attribute__((aligned(16))) bf16_t Ks[KT][KLD];
    __shared__ __attribute__((aligned(16))) bf16_t Vt[DH][VLD];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int split = blockIdx.x, rowtile = blockIdx.y;
    const int bg = blockIdx.z - call * grp.nbg, b = bg / a.Hkv, g = bg % a.Hkv;
    const int G = a.H / a.Hkv, RG = G * a.Mq, W = (a.Mq + 63) >> 6;
    const float sc = 1.4426950408889634f / sqrtf((float)DH);   // scores are kept in the log2 domain

    const int len = clamp_len(a.len[b], a.P_cap, tid == 0 ? a.dev_status : nullptr);
    const int nt = (len + KT - 1) / KT;
    const int per = (nt + geo.nsplit - 1) / geo.nsplit;
    const int t0 = min(split * per, nt), t1 = min(t0 + per, nt);
    const int Mt = a.mask ? a.Mt : 0;
    const int ntree = (split == geo.nsplit - 1) ? (Mt + KT - 1) / KT : 0;
    const int ntiles = (t1 - t0) + ntree;

    const bf16_t *kc = (const bf16_t *)a.kcache + (int64_t)bg * a.P_cap * DH;
    const bf16_t *vc = (const bf16_t *)a.vcache + (int64_t)bg * a.P_cap * DH;
    const bf16_t *ktp = (const bf16_t *)a.ktree + (int64_t)bg * a.Mt * DH;
    const bf16_t *vtp = (const bf16_t *)a.vtree + (int64_t)bg * a.Mt * DH;

    // query fragments (B operand of S^T = K Q^T): lane = query column l32, 8 head_dim values
    const int rowbase = rowtile * (128 * NBLK) + wave * (32 * NBLK);
    bf16x8 qf[NBLK][NKS];
    int mrow_of[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        int rho = rowbase + 32 * blk + l32;
        if (rho > RG - 1) rho = RG - 1;
        const int m = rho / G, hh = rho - m * G;
        mrow_of[blk] = m;
        const bf16_t *qrow = (const bf16_t *)a.q + (((int64_t)b * a.Mq + m) * a.H + g * G + hh) * DH;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[blk][ks] = *(const bf16x8 *)(qrow + 16 * ks + 8 * half);
    }

    f32x16 acc[NBLK][NDB];
    float mrun[NBLK], lrun[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        mrun[blk] = -INFINITY;
        lrun[blk] = 0.f;
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[blk][d][e] = 0.f;
    }

    // tile i of this workgroup: cache tile t0+i, or tree tile i-(t1-t0)
    u32x4 kreg[NLD], vreg[NLD];
    auto fetch = [&](int i) {
        const bool tree = i >= (t1 - t0);
        const int base = tree ? (i - (t1 - t0)) * KT : (t0 + i) * KT;
        const int limit = tree ? Mt : len;
        const bf16_t *ksrc = tree ? ktp : kc;
        const bf16_t *vsrc = tree ? vtp : vc;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int c = tid + 256 * j;
            int kr = base + c / CPK;                       // K: consecutive lanes walk along one key row
            if (kr > limit - 1) kr = limit - 1;            // rows past the end repeat the last valid row
            kreg[j] = *(const u32x4 *)(ksrc + (int64_t)kr * DH + (c % CPK) * 8);
            int vr = base + (c & 31);                      // V: consecutive lanes take consecutive keys
            if (vr > limit - 1) vr = limit - 1;
            vreg[j] = *(const u32x4 *)(vsrc + (int64_t)vr * DH + (c >> 5) * 8);
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int c = tid + 256 * j;
            *(u32x4 *)&Ks[c / CPK][(c % CPK) * 8] = kreg[j];
            const int key = vpos(c & 31), d0 = (c >> 5) * 8;
#pragma unroll
            for (int e = 0; e < 8; ++e) Vt[d0 + e][key] = (bf16_t)(vreg[j][e >> 1] >> (16 * (e & 1)));
        }
    };

    if (ntiles > 0) fetch(0);
    for (int i = 0; i < ntiles; ++i) {
        __syncthreads();          // every wave is done reading the previous tile
        stage();
        __syncthreads();
        if (i + 1 < ntiles) fetch(i + 1);

        const bool tree = i >= (t1 - t0);
        const int base = tree ? (i - (t1 - t0)) * KT : (t0 + i) * KT;
        const int limit = tree ? Mt : len;

        // S^T tile: keys x queries
        f32x16 s[NBLK];
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[blk][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 kf = *(const bf16x8 *)&Ks[l32][16 * ks + 8 * half];
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk)
                s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[blk][ks], s[blk], 0, 0, 0);
        }

        bf16x8 pf[NBLK][2];
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            // visibility of the 32 keys of this tile for this lane's query
            uint32_t vis = 0xffffffffu;
            if (tree) vis = (uint32_t)(a.mask[((int64_t)b * a.Mq + mrow_of[blk]) * W + (base >> 6)] >> (base & 63));
            const int nvalid = limit - base;               // >= 1
            if (nvalid < 32) vis &= (1u << nvalid) - 1u;
            float tmax = -INFINITY;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int key = 8 * (v >> 2) + 4 * half + (v & 3);
                const float x = ((vis >> key) & 1u) ? s[blk][v] * sc : -INFINITY;
                s[blk][v] = x;
                tmax = fmaxf(tmax, x);
            }
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float mnew = fmaxf(mrun[blk], tmax);
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
            const float corr = exp2f(mrun[blk] - msafe);
            float psum = 0.f;
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) { p[v] = exp2f(s[blk][v] - msafe); psum += p[v]; }
            psum += __shfl_xor(psum, 32);
            lrun[blk] = lrun[blk] * corr + psum;
            mrun[blk] = mnew;
#pragma unroll
            for (int d = 0; d < NDB; ++d)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[blk][d][e] *= corr;
#pragma unroll
            for (int st2 = 0; st2 < 2; ++st2)
#pragma unroll
                for (int t = 0; t < 8; ++t) pf[blk][st2][t] = (__bf16)p[8 * st2 + t];
        }

        // O^T += V^T P^T
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
            for (int st2 = 0; st2 < 2; ++st2) {
                const bf16x8 vf = *(const bf16x8 *)&Vt[32 * d + l32][16 * st2 + 8 * half];
#pragma unroll
                for (int blk = 0; blk < NBLK; ++blk)
                    acc[blk][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[blk][st2], acc[blk][d], 0, 0, 0);
            }
    }

    // partial results of this slice: the slice's own normalised output (a convex combination of V rows, so it
    // fits fp16 with 2^-12 relative rounding, eight times finer than the bf16 result), running max (log2 domain)
    // and running sum in fp32
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        const int rho = rowbase + 32 * blk + l32;
        if (rho >= RG) continue;
        const int64_t prow = ((int64_t)bg * geo.nsplit + split) * geo.rows_pad + rho;
        if (half == 0) {
            part_ml[prow * 2 + 0] = mrun[blk];
            part_ml[prow * 2 + 1] = lrun[blk];
        }
        const float inv = lrun[blk] > 0.f ? 1.0f / lrun[blk] : 0.f;
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                f16x4 v = {(f16_t)(acc[blk][d][4 * q4] * inv), (f16_t)(acc[blk][d][4 * q4 + 1] * inv),
                           (f16_t)(acc[blk][d][4 * q4 + 2] * inv), (f16_t)(acc[blk][d][4 * q4 + 3] * inv)};
                *(f16x4 *)(part_o + prow * DH + 32 * d + 8 * q4 + 4 * half) = v;
            }
    }
}

// one wavefront per (sequence, query, head)
template <int DH>
__global__ __launch_bounds__(64) void k_attn_merge(AttnGroup grp, SplitGeom geo)
{
    constexpr int CPL = DH / 64;   // components per lane
    const int lane = threadIdx.x;
    const int per_call = grp.a[0].B * grp.a[0].Mq * grp.a[0].H;
    const int call = blockIdx.x / per_call, blk = blockIdx.x - call * per_call;
    const AttnArgs &a = grp.a[call];
    const f16_t *__restrict__ part_o = (const f16_t *)a.ws;
    const float *__restrict__ part_ml = (const float *)(part_o + (size_t)grp.nbg * geo.nsplit * geo.rows_pad * DH);
    const int h = blk % a.H;
    const int m = (blk / a.H) % a.Mq;
    const int b = blk / (a.H * a.Mq);
    const int G = a.H / a.Hkv, g = h / G, rho = m * G + (h - g * G);
    const int64_t bg = (int64_t)b * a.Hkv + g;

    // slices in groups of eight: all (max, sum) pairs and accumulator rows of a group are requested before any
    // is used; groups are folded with the usual running-max rescale
    const int64_t stride = geo.rows_pad;
    const int64_t prow0 = bg * geo.nsplit * stride + rho;
    float mstar = -INFINITY, lsum = 0.f, o[CPL];
#pragma unroll
    for (int c = 0; c < CPL; ++c) o[c] = 0.f;
    for (int s0 = 0; s0 < geo.nsplit; s0 += 8) {
        float ms[8], ls[8], ov[8][CPL];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int sidx = min(s0 + u, geo.nsplit - 1);
            const int64_t prow = prow0 + sidx * stride;
            ms[u] = (s0 + u < geo.nsplit) ? part_ml[prow * 2] : -INFINITY;
            ls[u] = part_ml[prow * 2 + 1];
#pragma unroll
            for (int c = 0; c < CPL; ++c) ov[u][c] = (float)part_o[prow * DH + lane * CPL + c];
        }
        float gmax = mstar;
#pragma unroll
        for (int u = 0; u < 8; ++u) gmax = fmaxf(gmax, ms[u]);
        if (gmax == -INFINITY) continue;
        const float keep = exp2f(mstar - gmax);      // 0 on the first non-empty group
        lsum *= keep;
#pragma unroll
        for (int c = 0; c < CPL; ++c) o[c] *= keep;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float w = (ms[u] == -INFINITY) ? 0.f : exp2f(ms[u] - gmax) * ls[u];   // slice weight
            lsum += w;
#pragma unroll
            for (int c = 0; c < CPL; ++c) o[c] += w * ov[u][c];
        }
        mstar = gmax;
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16_t *dst = (bf16_t *)a.out + (((int64_t)b * a.Mq + m) * a.H + h) * DH + lane * CPL;
#pragma unroll
    for (int c = 0; c < CPL; ++c) dst[c] = f2bf(o[c] * inv);
    if (lsum == 0.f && a.empty_is_error && lane == 0 && a.dev_status) atomicOr(a.dev_status, MOA_DEV_EMPTY_KEYS);
}

// ------------------------------------------------------------------ host side
static bool mfma_ok(int dtype, int dh, const AttnArgs *a)
{
    if (dtype != DT_BF16 || (dh != 64 && dh != 128)) return false;
    if (!a) return true;
    auto al = [](const void *p) { return (((uintptr_t)p) & 15) == 0; };
    return al(a->q) && al(a->kcache) && al(a->vcache) && al(a->ktree) && al(a->vtree) && al(a->out);
}

static SplitGeom split_geometry(int B, int Mq, int H, int Hkv, int dh, int P_cap, bool tree)
{
    const int RG = (H / Hkv) * Mq;
    const int tiles_cap = (P_cap + KT - 1) / KT;
    SplitGeom g;
    const int nblk = RG > 256 ? 2 : 1;
    g.rowtiles = (RG + 128 * nblk - 1) / (128 * nblk);
    g.rows_pad = g.rowtiles * 128 * nblk;
    int want = 512 / (B * Hkv * g.rowtiles);        // about two workgroups per compute unit
    int most = tiles_cap / 2;                        // at least two tiles per slice
    if (want > most) want = most;
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    g.nsplit = want;
    return g;
}

size_t attn_workspace_bytes(int dtype, int B, int Mq, int H, int Hkv, int dh, int P_cap)
{
    if (!mfma_ok(dtype, dh, nullptr)) return 0;
    const SplitGeom g = split_geometry(B, Mq, H, Hkv, dh, P_cap, true);
    const size_t rows = (size_t)B * Hkv * g.nsplit * g.rows_pad;
    return rows * ((size_t)dh * sizeof(f16_t) + 2 * sizeof(float)) + 256;
}

static hipError_t launch_attn_generic(const AttnArgs &a, hipStream_t stream)
{
    const int nblocks = a.B * a.Mq * a.H;
    if (a.dh > 256) return hipErrorInvalidValue;
    if (a.dtype == DT_BF16) { prof_begin(K_ATTN_GENERIC, stream); hipLaunchKernelGGL(k_attn_generic<bf16_t>, dim3(nblocks), dim3(64), 0, stream, a); prof_end(stream); }
    else { prof_begin(K_ATTN_GENERIC, stream); hipLaunchKernelGGL(k_attn_generic<float>, dim3(nblocks), dim3(64), 0, stream, a); prof_end(stream); }
    return hipGetLastError();
}

static bool attn_fast_ok(const AttnArgs &a, int P_cap_geo)
{
    return mfma_ok(a.dtype, a.dh, &a) && a.ws && (((uintptr_t)a.ws) & 15) == 0 &&
           a.ws_bytes >= attn_workspace_bytes(a.dtype, a.B, a.Mq, a.H, a.Hkv, a.dh, P_cap_geo);
}

// n = 1 or 2 calls of identical shape (B, Mq, H, Hkv, dh); the slice geometry comes from the larger capacity
static hipError_t launch_attn_group(const AttnArgs *calls, int n, hipStream_t stream)
{
    const AttnArgs &a = calls[0];
    const int cap = n == 2 && calls[1].P_cap > a.P_cap ? calls[1].P_cap : a.P_cap;
    const SplitGeom g = split_geometry(a.B, a.Mq, a.H, a.Hkv, a.dh, cap, true);
    AttnGroup grp;
    grp.a[0] = calls[0];
    grp.a[1] = calls[n - 1];
    grp.nbg = a.B * a.Hkv;
    const dim3 grid(g.nsplit, g.rowtiles, n * grp.nbg);
    const int nblocks = n * a.B * a.Mq * a.H;
    const bool two = (a.H / a.Hkv) * a.Mq > 256;
    const int var = a.dh * 8 + (two ? 2 : 1);
    prof_begin(K_ATTN_MFMA + 64 * var, stream);
    if (a.dh == 128) {
        if (two) hipLaunchKernelGGL((k_attn_mfma<128, 2>), grid, dim3(256), 0, stream, grp, g);
        else hipLaunchKernelGGL((k_attn_mfma<128, 1>), grid, dim3(256), 0, stream, grp, g);
    } else {
        if (two) hipLaunchKernelGGL((k_attn_mfma<64, 2>), grid, dim3(256), 0, stream, grp, g);
        else hipLaunchKernelGGL((k_attn_mfma<64, 1>), grid, dim3(256), 0, stream, grp, g);
    }
    prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    prof_begin(K_ATTN_MERGE + 64 * (a.dh * 8), stream);
    if (a.dh == 128) hipLaunchKernelGGL(k_attn_merge<128>, dim3(nblocks), dim3(64), 0, stream, grp, g);
    else hipLaunchKernelGGL(k_attn_merge<64>, dim3(nblocks), dim3(64), 0, stream, grp, g);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_attn(const AttnArgs &a, hipStream_t stream)
{
    if (attn_fast_ok(a, a.P_cap)) return launch_attn_group(&a, 1, stream);
    return launch_attn_generic(a, stream);
}

hipError_t launch_attn_pair(const AttnArgs &a0, const AttnArgs &a1, hipStream_t stream)
{
    const int cap = a0.P_cap > a1.P_cap ? a0.P_cap : a1.P_cap;
    const bool same = a0.dtype == a1.dtype && a0.B == a1.B && a0.Mq == a1.Mq && a0.H == a1.H && a0.Hkv == a1.Hkv && a0.dh == a1.dh;
    if (same && attn_fast_ok(a0, cap) && attn_fast_ok(a1, cap)) {
        const AttnArgs both[2] = {a0, a1};
        return launch_attn_group(both, 2, stream);
    }
    hipError_t e = launch_attn(a0, stream);
    if (e != hipSuccess) return e;
    return launch_attn(a1, stream);
}

}  // namespace moa
