// Device-side body of the pass that adds up the K slices of a weight-streaming projection (fp32 partial sums, fixed
// slice order), shared by the kernel of its own and by the kernels that carry the pass in spare workgroups.
#ifndef MOA_SUM_DEVICE_H
#define MOA_SUM_DEVICE_H
#include "moa_common.h"

namespace moa {

// one thread per (row, 8 consecutive features): sum the K slices in order, round once, store
__device__ __forceinline__ void splitk_sum8(const SumArgs &sa, const float *p, f32x4 &lo, f32x4 &hi)
{
    lo = f32x4{0.f, 0.f, 0.f, 0.f};
    hi = f32x4{0.f, 0.f, 0.f, 0.f};
    const int64_t stride = (int64_t)64 * sa.ntot;
    int k = 0;
    for (; k + 8 <= sa.splits; k += 8) {        // eight slices in flight, summed in slice order
        f32x4 l8[8], h8[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) { l8[u] = *(const f32x4 *)(p + (k + u) * stride); h8[u] = *(const f32x4 *)(p + (k + u) * stride + 4); }
#pragma unroll
        for (int u = 0; u < 8; ++u) { lo += l8[u]; hi += h8[u]; }
    }
    for (; k < sa.splits; ++k) {
        lo += *(const f32x4 *)(p + k * stride);
        hi += *(const f32x4 *)(p + k * stride + 4);
    }
}

__device__ __forceinline__ u32x4 pack8(const f32x4 &lo, const f32x4 &hi)
{
    u32x4 pk;
    pk[0] = pack_bf16x2(lo[0], lo[1]);
    pk[1] = pack_bf16x2(lo[2], lo[3]);
    pk[2] = pack_bf16x2(hi[0], hi[1]);
    pk[3] = pack_bf16x2(hi[2], hi[3]);
    return pk;
}

// block: which 256-thread unit of the pass; tid: 0..255 inside it
__device__ __forceinline__ void splitk_reduce_block(const SumArgs &sa, int block, int tid)
{
    const int width = sa.epi == LinArgs::EPI_SWIGLU ? sa.ntot / 2 : sa.ntot;   // features a row of threads walks
    const int per = width / 8;
    const int64_t idx = (int64_t)block * 256 + tid;
    if (idx >= sa.R * per) return;
    const int64_t r = idx / per;
    const int nt = (int)(idx - r * per) * 8;          // feature in the concatenated space
    const int64_t rt = r >> 6, rr = r & 63;
    const float *p = sa.part + (rt * sa.splits * 64 + rr) * sa.ntot + nt;
    f32x4 lo, hi;
    splitk_sum8(sa, p, lo, hi);
    if (sa.epi == LinArgs::EPI_SWIGLU) {              // gate in the first half of the row, up in the second
        f32x4 ulo, uhi;
        splitk_sum8(sa, p + width, ulo, uhi);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            // the gate goes through the storage type, as it does when the projection is stored first
            const float gl = bf2f(f2bf(lo[e])), gh = bf2f(f2bf(hi[e]));
            lo[e] = gl / (1.0f + __expf(-gl)) * bf2f(f2bf(ulo[e]));
            hi[e] = gh / (1.0f + __expf(-gh)) * bf2f(f2bf(uhi[e]));
        }
        *(u32x4 *)((bf16_t *)sa.epi_out + r * width + nt) = pack8(lo, hi);
        return;
    }
    if (sa.epi == LinArgs::EPI_ADD_F32) {
        const float *h = sa.epi_res + r * width + nt;
        const f32x4 h0 = *(const f32x4 *)h, h1 = *(const f32x4 *)(h + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            lo[e] = h0[e] + bf2f(f2bf(lo[e]));
            hi[e] = h1[e] + bf2f(f2bf(hi[e]));
        }
        *(u32x4 *)((bf16_t *)sa.epi_out + r * width + nt) = pack8(lo, hi);
        return;
    }
    const int tile = nt >> 6;
    int s = 0;
    while (s + 1 < sa.nseg && tile >= sa.tile_begin[s + 1]) ++s;
    const int n = nt - sa.tile_begin[s] * 64;
    if (sa.epi == LinArgs::EPI_ROPE && s < 2) {       // queries and keys: this thread's 8 features and their partners
        const RopeArgs &ro = sa.rope;
        const int half = ro.dh >> 1, c = n % ro.dh;
        if (c >= half) return;                        // written by the thread that owns the lower half of the pair
        f32x4 plo, phi;
        splitk_sum8(sa, p + half, plo, phi);
        const int b = (int)(r / ro.Mn), i = ro.node0 + (int)(r - (int64_t)b * ro.Mn);
        int plen = ro.prefix_len[b];
        plen = plen < 0 ? 0 : (plen > ro.P_cap ? ro.P_cap : plen);
        const double pos = (double)plen + (double)ro.depth[(int64_t)b * ro.M + i];
        f32x4 olo, ohi, qlo, qhi;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            // through the storage type first, as when the projection is stored and rotated in place afterwards
            const float a = bf2f(f2bf(e < 4 ? lo[e] : hi[e - 4])), bb = bf2f(f2bf(e < 4 ? plo[e] : phi[e - 4]));
            const double ang = pos * exp(-2.0 * (double)(c + e) / (double)ro.dh * sa.rope_log_theta);
            double sn, cs;
            sincos(ang, &sn, &cs);
            const float x0 = (float)((double)a * cs - (double)bb * sn), x1 = (float)((double)bb * cs + (double)a * sn);
            if (e < 4) { olo[e] = x0; qlo[e] = x1; } else { ohi[e - 4] = x0; qhi[e - 4] = x1; }
        }
        const int64_t off = store_offset(sa.st[s], r, n);
        if (off < 0) return;
        *(u32x4 *)((bf16_t *)sa.st[s].dst + off) = pack8(olo, ohi);
        *(u32x4 *)((bf16_t *)sa.st[s].dst + off + half) = pack8(qlo, qhi);
        return;
    }
    const int64_t off = store_offset(sa.st[s], r, n);
    if (off < 0) return;
    *(u32x4 *)((bf16_t *)sa.st[s].dst + off) = pack8(lo, hi);
}

}  // namespace moa
#endif
