// Attention core shared by the draft model's cross-attention (no mask, cache rows only) and the
// tree-masked verification attention (cache rows, then the tree rows filtered by the ancestor
// bitset).  Input Q is already projected; the output is the concatenated heads before W_o.
//
//   k_attn_generic   any dtype / head_dim <= 256: one wavefront per (sequence, query, head),
//                    64 keys per step, exact online softmax with wavefront shuffles.
//   k_attn_fused     bf16, head_dim 64 / 128, short key ranges: a workgroup owns 32 query rows and the
//                    whole key range (its waves split the keys and are combined through LDS), so there
//                    are no partial results and no second launch.  Described at the kernel.
//   k_attn_mfma      bf16, head_dim 64 / 128, long key ranges: split-KV.  A workgroup owns one
//                    (sequence, KV head), one slice of the key range and up to 128*NBLK query rows (the
//                    GQA group's heads times the tree tokens are folded into the row dimension, so K/V
//                    are read once for all of them).  K/V tiles of 32 keys are staged row-major in LDS by
//                    row-contiguous 16-byte loads; scores are computed transposed (S^T = K Q^T) so that a
//                    lane owns one query column and the softmax max/sum need a single cross-lane
//                    exchange; P^T feeds the second MFMA straight from registers and V^T comes out of
//                    the LDS transpose read.
//   k_attn_merge     combines the per-slice (max, sum, accumulator) triples.
#include "moa_common.h"
#include "../../include/moa.h"

#include <math.h>

#include <atomic>

namespace moa {

// which MFMA form the attention core takes: 0 = chosen from the call's shape, 1 = whole key range per workgroup,
// 2 = split-KV + merge (moa_debug_force_attn_kernel; process-wide, read once per launch)
static std::atomic<int> g_attn_form{0};

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
    const int dh = a.dh, W = (a.mask_rows + 63) >> 6;
    const float scale = 1.0f / sqrtf((float)dh);

    const T *q = (const T *)a.q + (((int64_t)b * a.Mq + m) * a.H + h) * dh;
    for (int c = lane; c < dh; c += 64) qs[c] = ld<T>(q + c);
    __syncthreads();

    const int len = clamp_len(a.len[b], a.P_cap, lane == 0 ? a.dev_status : nullptr);
    const int Mt = a.mask ? a.Mt : 0;
    const int total = len + Mt;
    const T *kc = (const T *)a.kcache + ((int64_t)b * a.Hkv + g) * (int64_t)a.P_cap * dh;
    const T *vc = (const T *)a.vcache + ((int64_t)b * a.Hkv + g) * (int64_t)a.P_cap * dh;
    const T *kt = (const T *)a.ktree + ((int64_t)b * a.Hkv + g) * (int64_t)a.tree_cap * dh;
    const T *vt = (const T *)a.vtree + ((int64_t)b * a.Hkv + g) * (int64_t)a.tree_cap * dh;
    const uint64_t *mrow = a.mask ? a.mask + ((int64_t)b * a.mask_rows + a.mask_row0 + m) * W : nullptr;

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
    int nbg;      // B * Hkv of one call
    int ncalls;   // 1 or 2
};

typedef short i16x4 __attribute__((ext_vector_type(4)));

// 2^x by the hardware instruction alone: arguments here are <= 0 and results below the normal range may
// become 0, which a softmax weight may
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

constexpr int KT = 32;        // keys per tile

template <int DH, int NBLK>
__global__ __launch_bounds__(256, NBLK == 1 ? 2 : 1) void k_attn_mfma(AttnGroup grp, SplitGeom geo)
{
    const int call = blockIdx.z / grp.nbg;
    const AttnArgs &a = grp.a[call];
    f16_t *__restrict__ part_o = (f16_t *)a.ws;
    float *__restrict__ part_ml = (float *)(part_o + (size_t)grp.nbg * geo.nsplit * geo.rows_pad * DH);
    constexpr int KLD = DH + 8;           // padded K row (bf16): 16-byte operand reads of 16 rows hit 64 different banks
    constexpr int VSLD = DH + 32;         // padded V row: the 4 rows x 2 column groups of a transpose read hit different banks
    constexpr int NKS = DH / 16;          // MFMA steps along head_dim
    constexpr int NDB = DH / 32;          // 32-wide blocks of head_dim in the output
    constexpr int CPK = DH / 8;           // 16-byte chunks per key row
    constexpr int NLD = (KT * CPK) / 256; // chunks per thread per tile (1 for DH 64, 2 for DH 128)
    __shared__ __attribute__((aligned(16))) bf16_t Ks2[2][KT * KLD];    // two stages: one barrier per tile
    __shared__ __attribute__((aligned(16))) bf16_t Vs2[2][KT * VSLD];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int split = blockIdx.x, rowtile = blockIdx.y;
    const int bg = blockIdx.z - call * grp.nbg, b = bg / a.Hkv, g = bg % a.Hkv;
    const int G = a.H / a.Hkv, RG = G * a.Mq, W = (a.mask_rows + 63) >> 6;
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
    const bf16_t *ktp = (const bf16_t *)a.ktree + (int64_t)bg * a.tree_cap * DH;
    const bf16_t *vtp = (const bf16_t *)a.vtree + (int64_t)bg * a.tree_cap * DH;

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

    // tile i of this workgroup: cache tile t0+i, or tree tile i-(t1-t0).  K and V rows are fetched row-contiguously
    // (16 lanes cover a 256-byte row), staged row-major in LDS; V comes back transposed by the LDS transpose read.
    // A ring of RD register stages: the loads of tile i+RD are issued when tile i has been computed, so a tile has
    // RD-1 whole iterations to arrive (memory latency under load is longer than one iteration).
    constexpr int RD = 3;
    u32x4 kreg[RD][NLD], vreg[RD][NLD];
    auto full_tile = [&](int i) { return i < (t1 - t0) && (t0 + i + 1) * KT <= len; };
    auto fetch = [&](int i, u32x4 (&kr)[NLD], u32x4 (&vr)[NLD]) {
        if (full_tile(i)) {
            const int64_t off0 = (int64_t)(t0 + i) * KT * DH;
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                const int c = tid + 256 * j;
                kr[j] = *(const u32x4 *)(kc + off0 + (c / CPK) * DH + (c % CPK) * 8);
                vr[j] = *(const u32x4 *)(vc + off0 + (c / CPK) * DH + (c % CPK) * 8);
            }
            return;
        }
        const bool tree = i >= (t1 - t0);
        const int base = tree ? (i - (t1 - t0)) * KT : (t0 + i) * KT;
        const int limit = tree ? Mt : len;
        const bf16_t *ksrc = tree ? ktp : kc;
        const bf16_t *vsrc = tree ? vtp : vc;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int c = tid + 256 * j;
            int row = base + c / CPK;
            if (row > limit - 1) row = limit - 1;          // rows past the end repeat the last valid row
            kr[j] = *(const u32x4 *)(ksrc + (int64_t)row * DH + (c % CPK) * 8);
            vr[j] = *(const u32x4 *)(vsrc + (int64_t)row * DH + (c % CPK) * 8);
        }
    };
    auto stage = [&](int buf, const u32x4 (&kr)[NLD], const u32x4 (&vr)[NLD]) {
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            const int c = tid + 256 * j;
            *(u32x4 *)&Ks2[buf][(c / CPK) * KLD + (c % CPK) * 8] = kr[j];
            *(u32x4 *)&Vs2[buf][(c / CPK) * VSLD + (c % CPK) * 8] = vr[j];
        }
    };
    // transpose read: lane j of a 16-lane group addresses key (j >> 2), head_dim 4 (j & 3) of the group's 16
    const int tr_off = ((lane & 15) >> 2) * VSLD + 16 * ((lane >> 4) & 1) + 4 * (lane & 3) + 4 * half * VSLD;

    // Tile i+1 is staged into the other LDS buffer after tile i has been computed; the barrier at the end of an
    // iteration publishes it and retires the reads of tile i.  Three iterations per trip so that the register
    // stages are addressed statically.
#pragma unroll
    for (int d = 0; d < RD; ++d)
        if (d < ntiles) fetch(d, kreg[d], vreg[d]);
    if (ntiles > 0) stage(0, kreg[0], vreg[0]);
    __syncthreads();
    for (int i0 = 0; i0 < ntiles; i0 += RD) {
#pragma unroll
    for (int d = 0; d < RD; ++d) {
        const int i = i0 + d;
        if (i >= ntiles) continue;                             // same decision in the whole workgroup
        const bf16_t *Ks = Ks2[i & 1], *Vs = Vs2[i & 1];

        // S^T tile: keys x queries
        f32x16 s[NBLK];
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
            for (int e = 0; e < 16; ++e) s[blk][e] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const bf16x8 kf = *(const bf16x8 *)&Ks[l32 * KLD + 16 * ks + 8 * half];
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk)
                s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[blk][ks], s[blk], 0, 0, 0);
        }

        // keys that do not count (tree rows outside the ancestor set, rows past the end) get -inf; a cache tile
        // wholly below the length has none (the decision is the same for the whole workgroup)
        if (!full_tile(i)) {
            const bool tree = i >= (t1 - t0);
            const int base = tree ? (i - (t1 - t0)) * KT : (t0 + i) * KT;
            const int nvalid = (tree ? Mt : len) - base;       // >= 1
#pragma unroll
            for (int blk = 0; blk < NBLK; ++blk) {
                uint32_t vis = 0xffffffffu;
                if (tree) vis = (uint32_t)(a.mask[((int64_t)b * a.mask_rows + a.mask_row0 + mrow_of[blk]) * W + (base >> 6)] >> (base & 63));
                if (nvalid < 32) vis &= (1u << nvalid) - 1u;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 8 * (v >> 2) + 4 * half + (v & 3);
                    if (!((vis >> key) & 1u)) s[blk][v] = -INFINITY;
                }
            }
        }

        bf16x8 pf[NBLK][2];
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            float tmax = s[blk][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[blk][v]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float mnew = fmaxf(mrun[blk], tmax * sc);    // sc > 0: scaling keeps the order (and -inf)
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
            const float corr = fast_exp2(mrun[blk] - msafe);
            float psum = 0.f;
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) { p[v] = fast_exp2(fmaf(s[blk][v], sc, -msafe)); psum += p[v]; }
            psum += __shfl_xor(psum, 32);
            lrun[blk] = lrun[blk] * corr + psum;
            mrun[blk] = mnew;
            if (__any(corr != 1.0f)) {                          // the running max moved in some column
                asm volatile("" ::: "memory");                  // keep this a real branch: the multiplies are skipped
#pragma unroll
                for (int d = 0; d < NDB; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[blk][d][e] *= corr;
            }
#pragma unroll
            for (int st2 = 0; st2 < 2; ++st2)
#pragma unroll
                for (int t = 0; t < 8; ++t) pf[blk][st2][t] = (__bf16)p[8 * st2 + t];
        }

        // O^T += V^T P^T; P^T slot t of step st2 is key 16 st2 + 8 (t >> 2) + 4 half + (t & 3)
#pragma unroll
        for (int d = 0; d < NDB; ++d)
#pragma unroll
            for (int st2 = 0; st2 < 2; ++st2) {
                const bf16_t *vp = Vs + tr_off + 16 * st2 * VSLD + 32 * d;
                union { i16x4 h[2]; bf16x8 v; } vf;
                vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)vp);
                vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(vp + 8 * VSLD));
#pragma unroll
                for (int blk = 0; blk < NBLK; ++blk)
                    acc[blk][d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf[blk][st2], acc[blk][d], 0, 0, 0);
            }
        if (i + 1 < ntiles) stage((i + 1) & 1, kreg[(d + 1) % RD], vreg[(d + 1) % RD]);
        if (i + RD < ntiles) fetch(i + RD, kreg[d], vreg[d]);
        __syncthreads();
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


// ------------------------------------------------------------------ MFMA, whole key range in one workgroup
// One workgroup owns 32 query rows of one (sequence, KV head) and ALL of its keys: wave w takes the key tiles
// w, w + NW, ... with its own running (max, sum, accumulator), and the NW triples are combined through LDS at
// the end, in wave order, so no partial results go through HBM and no merge kernel follows.  The key loop has
// no workgroup barrier: each wave stages its tiles in a private LDS buffer.
//  - Global loads are row-contiguous (16 lanes cover 256 B): the memory pipeline handles one cache line per
//    lane group per clock, so loads in which every lane touches its own line run at a quarter of the rate.
//  - K goes to LDS row-major and comes back as MFMA operands (lane = key, 8 head_dim values).
//  - V goes to LDS row-major too and comes back TRANSPOSED by the LDS transpose read (within 16 lanes, lane i
//    receives element i%4 of the 8-byte datum addressed by lane i/4 + 4t, t = 0..3): the 16 lanes address 4
//    keys x 16 head_dim values, and lane i ends up with head_dim i for the 4 keys, which is the operand layout
//    of O^T += V^T P^T.  Two such reads (keys +0..3 and +8..11 of the lane's half) give the 8 keys that match
//    the key order of P^T in the score registers.
// Every row block re-reads the (sequence, KV head)'s K/V, which is why this form is used for short key ranges
// only; the blocks that share K/V are placed on the same XCD so that the re-reads hit its L2.
__device__ __forceinline__ void wave_lds_sync()
{
    // LDS traffic of one wavefront is processed in order; this only keeps the compiler from moving a read of
    // another lane's data above the write that produced it
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <int DH, int NW>
struct FusedLds {
    static constexpr int KLD = DH + 8;    // K / Q row (bf16): 16-byte operand reads of 16 rows hit 64 different banks
    static constexpr int VSLD = DH + 32;  // V row: the 4 rows x 2 column groups of a transpose read hit different banks
    static constexpr int NV = (DH / 32) * 16;
    static constexpr size_t q_bytes = (size_t)32 * KLD * sizeof(bf16_t);
    static constexpr size_t stage_bytes = (size_t)32 * VSLD * sizeof(bf16_t);
    static constexpr size_t loop_bytes = q_bytes + NW * stage_bytes;
    static constexpr size_t merge_bytes = ((size_t)NW * NV * 64 + 2 * NW * 32) * sizeof(float);
    static constexpr size_t bytes = loop_bytes > merge_bytes ? loop_bytes : merge_bytes;
};

template <int DH, int NW>
__global__ __launch_bounds__(64 * NW) void k_attn_fused(AttnGroup grp, int nrb)
{
    using L = FusedLds<DH, NW>;
    constexpr int KLD = L::KLD, VSLD = L::VSLD;
    constexpr int NKS = DH / 16;          // MFMA steps along head_dim
    constexpr int NDB = DH / 32;          // 32-wide blocks of head_dim in the output
    constexpr int CPK = DH / 8;           // 16-byte pieces per row
    constexpr int RPI = 64 / CPK;         // rows covered by one load instruction of the wave
    constexpr int NLD = KT / RPI;         // load instructions per tile
    constexpr int NV = L::NV;             // accumulator values per lane
    constexpr int VPW = NV / NW;          // accumulator values each wave finalises
    static_assert(VPW % 4 == 0, "finalisation stores four head_dim values at a time");
    extern __shared__ __attribute__((aligned(16))) char smem[];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    // workgroup -> (unit, row block): the hardware deals consecutive workgroups round-robin to the 8 XCDs
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int u = xcd + 8 * (slot / nrb), rb = slot - (slot / nrb) * nrb;
    if (u >= grp.ncalls * grp.nbg) return;          // the whole workgroup leaves before any barrier
    const int call = u / grp.nbg, bg = u - call * grp.nbg;
    const AttnArgs &a = grp.a[call];
    const int b = bg / a.Hkv, g = bg - b * a.Hkv;
    const int G = a.H / a.Hkv, RG = G * a.Mq, W = (a.mask_rows + 63) >> 6;
    const float sc = 1.4426950408889634f / sqrtf((float)DH);   // scores are kept in the log2 domain

    // the block's 32 query rows: requested first (they do not depend on the sequence length), row-contiguous
    constexpr int QPT = (32 * CPK + 64 * NW - 1) / (64 * NW);
    u32x4 qreg[QPT];
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int c = min(tid + 64 * NW * i, 32 * CPK - 1);
        int rq = rb * 32 + c / CPK;
        if (rq > RG - 1) rq = RG - 1;
        const int m = rq / G, hq = rq - m * G;
        const bf16_t *qrow = (const bf16_t *)a.q + (((int64_t)b * a.Mq + m) * a.H + g * G + hq) * DH;
        qreg[i] = *(const u32x4 *)(qrow + 8 * (c % CPK));
    }

    const int len = clamp_len(a.len[b], a.P_cap, tid == 0 ? a.dev_status : nullptr);
    const int Mt = a.mask ? a.Mt : 0;
    const int ntc = (len + KT - 1) / KT, nt = ntc + (Mt + KT - 1) / KT;

    const bf16_t *kc = (const bf16_t *)a.kcache + (int64_t)bg * a.P_cap * DH;
    const bf16_t *vc = (const bf16_t *)a.vcache + (int64_t)bg * a.P_cap * DH;
    const bf16_t *ktp = (const bf16_t *)a.ktree + (int64_t)bg * a.tree_cap * DH;
    const bf16_t *vtp = (const bf16_t *)a.vtree + (int64_t)bg * a.tree_cap * DH;

    // the K/V tile as the wave loads it: instruction j covers rows RPI j .. RPI j + RPI - 1, 16 bytes per lane.
    // A cache tile that lies wholly below the length needs no row clamp: one base address, constant offsets.
    const int ld_row = lane / CPK, ld_piece = lane % CPK;
    const int ld_off = ld_row * DH + 8 * ld_piece;
    u32x4 kreg[NLD], vreg[NLD];
    auto fetch = [&](int i) {
        if (i < ntc && (i + 1) * KT <= len) {
            const bf16_t *kp = kc + (int64_t)i * KT * DH + ld_off, *vp = vc + (int64_t)i * KT * DH + ld_off;
#pragma unroll
            for (int j = 0; j < NLD; ++j) {
                kreg[j] = *(const u32x4 *)(kp + j * RPI * DH);
                vreg[j] = *(const u32x4 *)(vp + j * RPI * DH);
            }
            return;
        }
        const bool tree = i >= ntc;
        const int base = tree ? (i - ntc) * KT : i * KT;
        const int limit = tree ? Mt : len;
        const bf16_t *ksrc = tree ? ktp : kc;
        const bf16_t *vsrc = tree ? vtp : vc;
#pragma unroll
        for (int j = 0; j < NLD; ++j) {
            int row = base + RPI * j + ld_row;
            if (row > limit - 1) row = limit - 1;              // rows past the end repeat the last valid row
            const int64_t off = (int64_t)row * DH + 8 * ld_piece;
            kreg[j] = *(const u32x4 *)(ksrc + off);
            vreg[j] = *(const u32x4 *)(vsrc + off);
        }
    };
    if (wave < nt) fetch(wave);

    bf16_t *Qs = (bf16_t *)smem;
#pragma unroll
    for (int i = 0; i < QPT; ++i) {
        const int c = tid + 64 * NW * i;
        if (c < 32 * CPK) *(u32x4 *)&Qs[(c / CPK) * KLD + 8 * (c % CPK)] = qreg[i];
    }
    __syncthreads();
    bf16x8 qf[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8 *)&Qs[l32 * KLD + 16 * ks + 8 * half];

    int rho = rb * 32 + l32;                        // this lane's query column
    const bool row_ok = rho < RG;
    if (!row_ok) rho = RG - 1;
    const int mrow = rho / G, hh = rho - mrow * G;

    f32x16 acc[NDB];
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[d][e] = 0.f;
    float mrun = -INFINITY, lrun = 0.f;              // running max (scaled, log2 domain) and sum

    bf16_t *stg = (bf16_t *)(smem + L::q_bytes + wave * L::stage_bytes);   // this wave's tile buffer
    // transpose read: lane j of a 16-lane group addresses key (j >> 2), head_dim 4 (j & 3) of the group's 16
    const int tr_off = ((lane & 15) >> 2) * VSLD + 16 * ((lane >> 4) & 1) + 4 * (lane & 3) + 4 * half * VSLD;

    if (wave < nt) {
        const int last = wave + ((nt - 1 - wave) / NW) * NW;
        for (int i = wave; i <= last; i += NW) {
            // K tile -> LDS -> S^T = K Q^T (keys x queries)
#pragma unroll
            for (int j = 0; j < NLD; ++j) *(u32x4 *)&stg[(RPI * j + ld_row) * KLD + 8 * ld_piece] = kreg[j];
            wave_lds_sync();
            f32x16 s;
#pragma unroll
            for (int e = 0; e < 16; ++e) s[e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const bf16x8 kf = *(const bf16x8 *)&stg[l32 * KLD + 16 * ks + 8 * half];
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
            }
            wave_lds_sync();
            // V tile into the same buffer, then the next tile's loads (clamped to the wave's last tile: a
            // repeated load of valid memory whose result is not used) fly during the softmax and the second MFMA
#pragma unroll
            for (int j = 0; j < NLD; ++j) *(u32x4 *)&stg[(RPI * j + ld_row) * VSLD + 8 * ld_piece] = vreg[j];
            wave_lds_sync();
            fetch(min(i + NW, last));

            // keys that do not count (tree rows outside the ancestor set, rows past the end) get -inf; a cache
            // tile wholly below the length has none (the decision is the same for the whole wavefront)
            if (!(i < ntc && (i + 1) * KT <= len)) {
                const bool tree = i >= ntc;
                const int base = tree ? (i - ntc) * KT : i * KT;
                const int nvalid = (tree ? Mt : len) - base;   // >= 1
                uint32_t vis = 0xffffffffu;
                if (tree) vis = (uint32_t)(a.mask[((int64_t)b * a.mask_rows + a.mask_row0 + mrow) * W + (base >> 6)] >> (base & 63));
                if (nvalid < 32) vis &= (1u << nvalid) - 1u;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 8 * (v >> 2) + 4 * half + (v & 3);
                    if (!((vis >> key) & 1u)) s[v] = -INFINITY;
                }
            }
            float tmax = s[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) tmax = fmaxf(tmax, s[v]);
            tmax = fmaxf(tmax, __shfl_xor(tmax, 32));
            const float mnew = fmaxf(mrun, tmax * sc);         // sc > 0: scaling keeps the order (and -inf)
            const float msafe = (mnew == -INFINITY) ? 0.f : mnew;
            const float corr = fast_exp2(mrun - msafe);
            float psum = 0.f;
            float p[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) { p[v] = fast_exp2(fmaf(s[v], sc, -msafe)); psum += p[v]; }
            psum += __shfl_xor(psum, 32);
            lrun = lrun * corr + psum;
            mrun = mnew;
            if (__any(corr != 1.0f)) {                          // the running max moved in some column
                asm volatile("" ::: "memory");                  // keep this a real branch: 64 multiplies skipped
#pragma unroll
                for (int d = 0; d < NDB; ++d)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[d][e] *= corr;
            }
            // O^T += V^T P^T; P^T slot t of step st2 is key 16 st2 + 8 (t >> 2) + 4 half + (t & 3)
#pragma unroll
            for (int st2 = 0; st2 < 2; ++st2) {
                bf16x8 pf;
#pragma unroll
                for (int t = 0; t < 8; ++t) pf[t] = (__bf16)p[8 * st2 + t];
#pragma unroll
                for (int d = 0; d < NDB; ++d) {
                    const bf16_t *vp = stg + tr_off + 16 * st2 * VSLD + 32 * d;
                    union { i16x4 h[2]; bf16x8 v; } vf;
                    vf.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)vp);
                    vf.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) i16x4 *)(vp + 8 * VSLD));
                    acc[d] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf.v, pf, acc[d], 0, 0, 0);
                }
            }
            wave_lds_sync();
        }
    }

    // combine the waves' triples: out = sum_w 2^(m_w - m*) acc_w / sum_w 2^(m_w - m*) l_w, waves in order
    __syncthreads();                                            // the tile buffers are dead; their memory is reused
    float *red = (float *)smem;                                 // [NW][NV][64]
    float *msh = red + NW * NV * 64;                            // [NW][32]
    float *lsh = msh + NW * 32;
    if (half == 0) {
        msh[wave * 32 + l32] = mrun;
        lsh[wave * 32 + l32] = lrun;
    }
#pragma unroll
    for (int d = 0; d < NDB; ++d)
#pragma unroll
        for (int e = 0; e < 16; ++e) red[((wave * NDB + d) * 16 + e) * 64 + lane] = acc[d][e];
    __syncthreads();

    float wgt[NW], mstar = -INFINITY, lsum = 0.f;
#pragma unroll
    for (int w = 0; w < NW; ++w) { wgt[w] = msh[w * 32 + l32]; mstar = fmaxf(mstar, wgt[w]); }
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        wgt[w] = (wgt[w] == -INFINITY) ? 0.f : exp2f(wgt[w] - mstar);
        lsum += wgt[w] * lsh[w * 32 + l32];
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    bf16_t *orow = (bf16_t *)a.out + (((int64_t)b * a.Mq + mrow) * a.H + g * G + hh) * DH;
#pragma unroll
    for (int t4 = 0; t4 < VPW / 4; ++t4) {
        const int v0 = wave * VPW + 4 * t4;                     // accumulator values v0 .. v0+3: four consecutive head_dim
        float o[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) sum += wgt[w] * red[(w * NV + v0 + t) * 64 + lane];
            o[t] = sum * inv;
        }
        const int dcol = 32 * (v0 >> 4) + 8 * ((v0 & 15) >> 2) + 4 * half;
        if (row_ok) {
            u32x2 pk;
            pk[0] = pack_bf16x2(o[0], o[1]);
            pk[1] = pack_bf16x2(o[2], o[3]);
            *(u32x2 *)(orow + dcol) = pk;
        }
    }
    if (wave == 0 && half == 0 && row_ok && lsum == 0.f && a.empty_is_error && a.dev_status)
        atomicOr(a.dev_status, MOA_DEV_EMPTY_KEYS);
}

// DH/8 lanes per (sequence, query, head) row, 8 head_dim values (one 16-byte load per slice) per lane; a
// workgroup of 256 threads folds 2048/DH rows
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;

template <int DH>
__global__ __launch_bounds__(256) void k_attn_merge(AttnGroup grp, SplitGeom geo)
{
    constexpr int LPR = DH / 8;            // lanes per row
    constexpr int RPB = 256 / LPR;         // rows per workgroup
    const int per_call = grp.a[0].B * grp.a[0].Mq * grp.a[0].H;
    const int64_t row = (int64_t)blockIdx.x * RPB + threadIdx.x / LPR;
    if (row >= (int64_t)grp.ncalls * per_call) return;
    const int call = (int)(row / per_call), blk = (int)(row - (int64_t)call * per_call);
    const int piece = threadIdx.x % LPR;
    const AttnArgs &a = grp.a[call];
    const f16_t *__restrict__ part_o = (const f16_t *)a.ws;
    const float *__restrict__ part_ml = (const float *)(part_o + (size_t)grp.nbg * geo.nsplit * geo.rows_pad * DH);
    const int h = blk % a.H;
    const int m = (blk / a.H) % a.Mq;
    const int b = blk / (a.H * a.Mq);
    const int G = a.H / a.Hkv, g = h / G, rho = m * G + (h - g * G);
    const int64_t bg = (int64_t)b * a.Hkv + g;

    // slices in groups of four: all (max, sum) pairs and accumulator pieces of a group are requested before any
    // is used; groups are folded with the usual running-max rescale
    const int64_t stride = geo.rows_pad;
    const int64_t prow0 = bg * geo.nsplit * stride + rho;
    float mstar = -INFINITY, lsum = 0.f, o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;
    for (int s0 = 0; s0 < geo.nsplit; s0 += 4) {
        float ms[4], ls[4];
        f16x8 ov[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int sidx = min(s0 + u, geo.nsplit - 1);
            const int64_t prow = prow0 + sidx * stride;
            ms[u] = (s0 + u < geo.nsplit) ? part_ml[prow * 2] : -INFINITY;
            ls[u] = part_ml[prow * 2 + 1];
            ov[u] = *(const f16x8 *)(part_o + prow * DH + 8 * piece);
        }
        float gmax = mstar;
#pragma unroll
        for (int u = 0; u < 4; ++u) gmax = fmaxf(gmax, ms[u]);
        if (gmax == -INFINITY) continue;
        const float keep = exp2f(mstar - gmax);      // 0 on the first non-empty group
        lsum *= keep;
#pragma unroll
        for (int c = 0; c < 8; ++c) o[c] *= keep;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float w = (ms[u] == -INFINITY) ? 0.f : exp2f(ms[u] - gmax) * ls[u];   // slice weight
            lsum += w;
#pragma unroll
            for (int c = 0; c < 8; ++c) o[c] += w * (float)ov[u][c];
        }
        mstar = gmax;
    }
    const float inv = lsum > 0.f ? 1.0f / lsum : 0.f;
    u32x4 pk;
#pragma unroll
    for (int w = 0; w < 4; ++w) pk[w] = pack_bf16x2(o[2 * w] * inv, o[2 * w + 1] * inv);
    *(u32x4 *)((bf16_t *)a.out + (((int64_t)b * a.Mq + m) * a.H + h) * DH + 8 * piece) = pk;
    if (lsum == 0.f && a.empty_is_error && piece == 0 && a.dev_status) atomicOr(a.dev_status, MOA_DEV_EMPTY_KEYS);
}

// ------------------------------------------------------------------ host side
static bool mfma_ok(int dtype, int dh, const AttnArgs *a)
{
    if (dtype != DT_BF16 || (dh != 64 && dh != 128)) return false;
    if (!a) return true;
    auto al = [](const void *p) { return (((uintptr_t)p) & 15) == 0; };
    return al(a->q) && al(a->kcache) && al(a->vcache) && al(a->ktree) && al(a->vtree) && al(a->out);
}

// 32-row blocks per wave of the split-KV kernel: one block per wave keeps two workgroups per CU, which measured
// 25 % faster than two blocks per wave at RG = 512 even though K/V are then read by twice as many row tiles
constexpr int ATTN_NBLK = 1;

static SplitGeom split_geometry(int B, int Mq, int H, int Hkv, int dh, int P_cap, bool tree)
{
    const int RG = (H / Hkv) * Mq;
    const int tiles_cap = (P_cap + KT - 1) / KT;
    SplitGeom g;
    g.rowtiles = (RG + 128 * ATTN_NBLK - 1) / (128 * ATTN_NBLK);
    g.rows_pad = g.rowtiles * 128 * ATTN_NBLK;
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
    if (a.dtype == DT_BF16) { prof_begin(K_ATTN_GENERIC, stream); MOA_KLAUNCH(k_attn_generic<bf16_t>, dim3(nblocks), dim3(64), 0, stream, a); prof_end(stream); }
    else { prof_begin(K_ATTN_GENERIC, stream); MOA_KLAUNCH(k_attn_generic<float>, dim3(nblocks), dim3(64), 0, stream, a); prof_end(stream); }
    return hipGetLastError();
}

static bool attn_split_ok(const AttnArgs &a, int P_cap_geo)
{
    return mfma_ok(a.dtype, a.dh, &a) && a.ws && (((uintptr_t)a.ws) & 15) == 0 &&
           a.ws_bytes >= attn_workspace_bytes(a.dtype, a.B, a.Mq, a.H, a.Hkv, a.dh, P_cap_geo);
}

// Which MFMA kernel.  The whole-key-range form needs one launch, writes no partial results and has the shorter
// fixed part, but re-reads K/V once per 32 query rows and runs one workgroup per CU: it wins while the call is
// latency-bound, i.e. while its workgroups fit the chip in one round and the key range is short (C1: 14.5 us
// against 17.8 + 6.8 us).  With more work the split form (128 rows per workgroup, two workgroups per CU, then the
// merge) is ahead (B = 16, prefixes up to 2048: 122 against 166 us).  moa_debug_force_attn_kernel overrides the
// choice (the parity tests run every case through both forms).
constexpr int FUSED_MAX_KEYS = 8192;
constexpr int FUSED_MAX_WORKGROUPS = 256;
static bool want_fused(const AttnArgs &a)
{
    const int form = g_attn_form.load(std::memory_order_relaxed);
    if (form == MOA_ATTN_KERNEL_SPLIT) return false;
    if (form == MOA_ATTN_KERNEL_WHOLE) return true;
    const int64_t wgs = (int64_t)a.B * a.Hkv * (((a.H / a.Hkv) * a.Mq + 31) / 32);
    return a.P_cap + a.Mt <= FUSED_MAX_KEYS && wgs <= FUSED_MAX_WORKGROUPS;
}

// n = 1 or 2 calls of identical shape (B, Mq, H, Hkv, dh)
template <int DH, int NW>
static hipError_t launch_fused_as(const AttnGroup &grp, int nrb, unsigned grid, hipStream_t stream)
{
    constexpr size_t lds = FusedLds<DH, NW>::bytes;
    static bool raised[16] = {};
    hipError_t e = raise_lds_limit_once(raised, (const void *)k_attn_fused<DH, NW>, lds);
    if (e != hipSuccess) return e;
    prof_begin(K_ATTN_FUSED + 64 * (DH * 8 + NW / 4), stream);
    MOA_KLAUNCH((k_attn_fused<DH, NW>), dim3(grid), dim3(64 * NW), lds, stream, grp, nrb);
    prof_end(stream);
    return hipGetLastError();
}

static hipError_t launch_attn_fused(const AttnArgs *calls, int n, hipStream_t stream)
{
    const AttnArgs &a = calls[0];
    AttnGroup grp;
    grp.a[0] = calls[0];
    grp.a[1] = calls[n - 1];
    grp.nbg = a.B * a.Hkv;
    grp.ncalls = n;
    const int nrb = ((a.H / a.Hkv) * a.Mq + 31) / 32;
    const int64_t units8 = ((int64_t)n * grp.nbg + 7) / 8;
    const int64_t grid = 8 * units8 * nrb;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    if (a.dh == 128) return launch_fused_as<128, 8>(grp, nrb, (unsigned)grid, stream);
    return launch_fused_as<64, 8>(grp, nrb, (unsigned)grid, stream);
}

static hipError_t launch_attn_split(const AttnArgs *calls, int n, hipStream_t stream)
{
    const AttnArgs &a = calls[0];
    const int cap = n == 2 && calls[1].P_cap > a.P_cap ? calls[1].P_cap : a.P_cap;
    const SplitGeom g = split_geometry(a.B, a.Mq, a.H, a.Hkv, a.dh, cap, true);
    AttnGroup grp;
    grp.a[0] = calls[0];
    grp.a[1] = calls[n - 1];
    grp.nbg = a.B * a.Hkv;
    grp.ncalls = n;
    const dim3 grid(g.nsplit, g.rowtiles, n * grp.nbg);
    const int nblocks = n * a.B * a.Mq * a.H;
    prof_begin(K_ATTN_MFMA + 64 * (a.dh * 8 + ATTN_NBLK), stream);
    if (a.dh == 128) MOA_KLAUNCH((k_attn_mfma<128, ATTN_NBLK>), grid, dim3(256), 0, stream, grp, g);
    else MOA_KLAUNCH((k_attn_mfma<64, ATTN_NBLK>), grid, dim3(256), 0, stream, grp, g);
    prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    prof_begin(K_ATTN_MERGE + 64 * (a.dh * 8), stream);
    const int rpb = 2048 / a.dh;                      // rows per merge workgroup
    const unsigned mblocks = (unsigned)(((int64_t)nblocks + rpb - 1) / rpb);
    if (a.dh == 128) MOA_KLAUNCH(k_attn_merge<128>, dim3(mblocks), dim3(256), 0, stream, grp, g);
    else MOA_KLAUNCH(k_attn_merge<64>, dim3(mblocks), dim3(256), 0, stream, grp, g);
    prof_end(stream);
    return hipGetLastError();
}

// whole-tree defaults of the tree window; false when the window does not fit its tree
static bool tree_window(AttnArgs &a)
{
    if (!a.tree_cap) a.tree_cap = a.Mt;
    if (!a.mask_rows) a.mask_rows = a.Mq;
    return a.mask_row0 >= 0 && a.mask_row0 + a.Mq <= a.mask_rows && a.Mt <= a.tree_cap;
}

hipError_t launch_attn(const AttnArgs &a_in, hipStream_t stream)
{
    AttnArgs a = a_in;
    if (!tree_window(a)) return hipErrorInvalidValue;
    if (mfma_ok(a.dtype, a.dh, &a) && want_fused(a)) return launch_attn_fused(&a, 1, stream);
    if (attn_split_ok(a, a.P_cap)) return launch_attn_split(&a, 1, stream);
    return launch_attn_generic(a, stream);
}

hipError_t launch_attn_pair(const AttnArgs &a0_in, const AttnArgs &a1_in, hipStream_t stream)
{
    AttnArgs a0 = a0_in, a1 = a1_in;
    if (!tree_window(a0) || !tree_window(a1)) return hipErrorInvalidValue;
    const int cap = a0.P_cap > a1.P_cap ? a0.P_cap : a1.P_cap;
    const bool same = a0.dtype == a1.dtype && a0.B == a1.B && a0.Mq == a1.Mq && a0.H == a1.H && a0.Hkv == a1.Hkv && a0.dh == a1.dh;
    const AttnArgs both[2] = {a0, a1};
    if (same && mfma_ok(a0.dtype, a0.dh, &a0) && mfma_ok(a1.dtype, a1.dh, &a1)) {
        if (want_fused(a0) && want_fused(a1)) return launch_attn_fused(both, 2, stream);
        if (!want_fused(a0) && !want_fused(a1) && attn_split_ok(a0, cap) && attn_split_ok(a1, cap))
            return launch_attn_split(both, 2, stream);
    }
    hipError_t e = launch_attn(a0, stream);
    if (e != hipSuccess) return e;
    return launch_attn(a1, stream);
}

}  // namespace moa

extern "C" int32_t moa_debug_force_attn_kernel(int32_t form)
{
    if (form < MOA_ATTN_KERNEL_AUTO || form > MOA_ATTN_KERNEL_SPLIT)
        return moa::api_fail(MOA_ERR_SHAPE, "debug_force_attn_kernel: form must be MOA_ATTN_KERNEL_AUTO / _WHOLE / _SPLIT");
    moa::g_attn_form.store(form, std::memory_order_relaxed);
    return MOA_OK;
}
