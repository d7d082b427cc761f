// Projections Y = X W^T (W row-major [N, K]) for the Q/K/V/O projections of LSA, CA and
// tree verification.  Three kernels:
//   k_linear_generic     any dtype / shape, fp32 FMA, LDS-tiled 64x64 (fp32 path and odd shapes)
//   k_linear_skinny_bf16 <=64 rows per tile: weight streaming, HBM-bound.  Operands go straight
//                        from global memory into MFMA 16x16x32 fragments (both are K-contiguous,
//                        which is exactly the fragment layout), the four waves of a workgroup
//                        split K and reduce through LDS.
//   k_linear_tiled_bf16  128x128x64 LDS-tiled MFMA 32x32x16 GEMM for many rows (LSA's T*L rows,
//                        batched configs).
// In both MFMA kernels the weight tile is the A operand and the activation tile the B operand,
// so a lane ends up holding consecutive output features of one row (vector stores).
#include "moa_common.h"
#include "moa_tree_device.h"
#include "moa_sum_device.h"

namespace moa {

// ------------------------------------------------------------------ generic
template <typename T>
__global__ __launch_bounds__(256) void k_linear_generic(const T *__restrict__ X, int64_t R, int K, int64_t ldx,
                                                        const T *__restrict__ W, int N, StoreSpec stp)
{
    __shared__ float Xs[16][65];
    __shared__ float Ws[16][65];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int64_t r0 = (int64_t)blockIdx.y * 64;
    const int n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = 0; i < 4; ++i) {
            const int idx = tid + 256 * i, rr = idx >> 4, kk = idx & 15;
            const int64_t r = r0 + rr;
            const int n = n0 + rr, k = k0 + kk;
            Xs[kk][rr] = (r < R && k < K) ? ld<T>(X + r * ldx + k) : 0.f;
            Ws[kk][rr] = (n < N && k < K) ? ld<T>(W + (int64_t)n * K + k) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = Xs[kk][ty * 4 + i]; b[i] = Ws[kk][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
    T *dst = (T *)stp.dst;
    for (int i = 0; i < 4; ++i) {
        const int64_t r = r0 + ty * 4 + i;
        if (r >= R) continue;
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            const int64_t off = store_offset(stp, r, n);
            if (off >= 0) st<T>(dst + off, acc[i][j]);
        }
    }
}

// ------------------------------------------------------------------ skinny bf16 (weight streaming)
struct SkinnyArgs {
    LinArgs a;
    int tile_begin[5];  // first feature tile of each segment, tile_begin[nseg] = total
};

template <int NB>  // 16*NB output features per workgroup
__global__ __launch_bounds__(256) void k_linear_skinny_bf16(SkinnyArgs sa)
{
    constexpr int FT = 16 * NB;
    constexpr int RS = FT + 4;  // padded row of the reduction buffer (floats)
    __shared__ float red[4][64][RS];

    const LinArgs &a = sa.a;
    int s = 0;
    while (s + 1 < a.nseg && (int)blockIdx.x >= sa.tile_begin[s + 1]) ++s;
    const int n0 = ((int)blockIdx.x - sa.tile_begin[s]) * FT;
    const int64_t r0 = (int64_t)blockIdx.y * 64;
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, li = lane & 15, kg = lane >> 4;
    const int K = a.K, kper = K >> 2;
    const bf16_t *W = (const bf16_t *)a.seg[s].W;
    const bf16_t *X = (const bf16_t *)a.X;

    const bf16_t *wp[NB];
    const bf16_t *xp[4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wp[nb] = W + (int64_t)(n0 + 16 * nb + li) * K + wave * kper + 8 * kg;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) {
        int64_t r = r0 + 16 * rb + li;
        if (r > a.R - 1) r = a.R - 1;   // rows past the end repeat the last row; never stored
        xp[rb] = X + r * a.ldx + wave * kper + 8 * kg;
    }

    f32x4 acc[NB][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[nb][rb] = f32x4{0.f, 0.f, 0.f, 0.f};

    bf16x8 wf[2][NB], xf[2][4];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) wf[0][nb] = *(const bf16x8 *)(wp[nb]);
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) xf[0][rb] = *(const bf16x8 *)(xp[rb]);

    const int nsteps = kper >> 5;   // 32 k per MFMA
    for (int step = 0; step < nsteps; step += 2) {
        // stage 1 loads (step+1) while stage 0 computes, then the other way round
        if (step + 1 < nsteps) {
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) wf[1][nb] = *(const bf16x8 *)(wp[nb] + (step + 1) * 32);
#pragma unroll
            for (int rb = 0; rb < 4; ++rb) xf[1][rb] = *(const bf16x8 *)(xp[rb] + (step + 1) * 32);
        }
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int rb = 0; rb < 4; ++rb)
                acc[nb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[0][nb], xf[0][rb], acc[nb][rb], 0, 0, 0);
        if (step + 1 < nsteps) {
            if (step + 2 < nsteps) {
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) wf[0][nb] = *(const bf16x8 *)(wp[nb] + (step + 2) * 32);
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) xf[0][rb] = *(const bf16x8 *)(xp[rb] + (step + 2) * 32);
            }
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    acc[nb][rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[1][nb], xf[1][rb], acc[nb][rb], 0, 0, 0);
        }
    }

    // lane holds features 4*kg..4*kg+3 of feature block nb for row 16*rb + li
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
            *(f32x4 *)&red[wave][16 * rb + li][16 * nb + 4 * kg] = acc[nb][rb];
    __syncthreads();

    bf16_t *dst = (bf16_t *)a.seg[s].st.dst;
    constexpr int CPR = FT / 8;  // 8-feature chunks per row
    for (int c = threadIdx.x; c < 64 * CPR; c += 256) {
        const int row = c / CPR, fc = c % CPR;
        const int64_t r = r0 + row;
        if (r >= a.R) continue;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e)
            v[e] = (red[0][row][8 * fc + e] + red[1][row][8 * fc + e]) + (red[2][row][8 * fc + e] + red[3][row][8 * fc + e]);
        const int64_t off = store_offset(a.seg[s].st, r, n0 + 8 * fc);
        if (off < 0) continue;
        u32x4 pk;
        pk[0] = pack_bf16x2(v[0], v[1]);
        pk[1] = pack_bf16x2(v[2], v[3]);
        pk[2] = pack_bf16x2(v[4], v[5]);
        pk[3] = pack_bf16x2(v[6], v[7]);
        *(u32x4 *)(dst + off) = pk;
    }
}

// ------------------------------------------------------------------ split-K bf16 (weight streaming)
// The HBM-bound projections (<= 128 rows): W is read exactly once, every load of
// a workgroup's slice issued before anything is waited for.  A workgroup owns 64 output features (16 per
// wave) and one K slice of 128*NQ; the activation slice [64 rows x 128*NQ] is requested first, parked in
// LDS and shared by the four waves, so X costs the fill path as much as W and not four times more.
// Slices are summed by k_linear_splitk_reduce (fp32 partials, fixed order: results do not depend on
// scheduling).  MFMA k-slots are permuted so that one load instruction takes a 64-byte run per feature (the
// four lanes of a feature side by side): slot (q, j, kg) reads k = 128 q + 32 j + 8 kg, and the X fragment is
// read from the same place.  With the run in one lane's four loads instead (32 kg + 8 j) every instruction
// touches twice the cache lines: 27.3 against 25.5 us for 60 x 10240 x 4096.
struct SplitKArgs {
    LinArgs a;
    int tile_begin[5];   // first 64-feature tile of each segment; [nseg] = total tiles
    int splits;          // K slices
    int ntot;            // total features (all segments), row length of the partial buffer
    float *part;         // [row tiles][splits][64][ntot]
    int lead_blocks;     // workgroups in front of the projection's own (LinArgs::rider, padded to the XCD count)
};

template <int NQ>
__global__ __launch_bounds__(256) void k_linear_splitk_bf16(SplitKArgs sa)
{
    constexpr int KS = 128 * NQ, LDK = KS + 8, CPR = KS / 8, XL = (64 * CPR) / 256;
    extern __shared__ __attribute__((aligned(16))) bf16_t Xs[];   // [64][LDK]
    const LinArgs &a = sa.a;
    if ((int)blockIdx.x < sa.lead_blocks) {        // the first workgroups of the grid carry the integer work
        if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
            step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)Xs, (int32_t *)Xs + MOA_MAX_TREE);
        return;
    }
    const int bx = (int)blockIdx.x - sa.lead_blocks;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, kg = lane >> 4;
    const int tile = bx / sa.splits, split = bx - tile * sa.splits;
    int s = 0;
    while (s + 1 < a.nseg && tile >= sa.tile_begin[s + 1]) ++s;
    const int n0 = (tile - sa.tile_begin[s]) * 64 + wave * 16;   // feature inside the segment
    const int k0 = split * KS;
    const bf16_t *X = (const bf16_t *)(a.seg[s].X ? a.seg[s].X : a.X);
    const int64_t ldx = a.seg[s].X ? a.seg[s].ldx : a.ldx;
    const bf16_t *W = (const bf16_t *)a.seg[s].W;
    const int rowtiles = (int)((a.R + 63) >> 6);

    // X slice of row tile rt into registers (rows past the end repeat the last row; never stored)
    u32x4 xr[XL];
    auto load_x = [&](int rt) {
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int c = tid + 256 * i;
            int64_t r = (int64_t)rt * 64 + c / CPR;
            if (r > a.R - 1) r = a.R - 1;
            xr[i] = *(const u32x4 *)(X + r * ldx + k0 + 8 * (c % CPR));
        }
    };
    load_x(0);
    bf16x8 wf[NQ][4];
    const bf16_t *wp = W + (int64_t)(n0 + li) * a.K + k0 + 8 * kg;
#pragma unroll
    for (int q = 0; q < NQ; ++q)
#pragma unroll
        for (int j = 0; j < 4; ++j) wf[q][j] = *(const bf16x8 *)(wp + 128 * q + 32 * j);

    // The weights stay in registers while the workgroup walks the row tiles (one at decode sizes): W is
    // streamed once however many rows there are; the next tile's X slice is requested before this one is used.
    // Bare barriers behind an LDS-only wait: __syncthreads() also waits for every outstanding global load, which
    // would hold a row tile's MFMAs until the next tile's activations, requested just before, have arrived.
    for (int rt = 0; rt < rowtiles; ++rt) {
        if (rt > 0) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // every wave is done reading the previous slice
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int c = tid + 256 * i;
            *(u32x4 *)&Xs[(c / CPR) * LDK + 8 * (c % CPR)] = xr[i];
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (rt + 1 < rowtiles) load_x(rt + 1);

        f32x4 acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x8 xf[4];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) xf[rb] = *(const bf16x8 *)&Xs[(16 * rb + li) * LDK + 128 * q + 32 * j + 8 * kg];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[q][j], xf[rb], acc[rb], 0, 0, 0);
            }

        // lane holds features 4 kg .. 4 kg + 3 of its wave's 16, for row 16 rb + li of this row tile
        float *p = sa.part + ((int64_t)rt * sa.splits + split) * 64 * sa.ntot + tile * 64 + wave * 16 + 4 * kg;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
            if ((int64_t)rt * 64 + 16 * rb + li < a.R) *(f32x4 *)(p + (int64_t)(16 * rb + li) * sa.ntot) = acc[rb];
    }
}

// The same for at most 64 rows with a workgroup walking CH consecutive 256-wide K chunks: the weights of the next
// chunk are requested before this one's MFMAs (two register sets), the activation slice of a chunk goes through a
// 33 KB LDS buffer (three workgroups per CU instead of two), and the partial sums are CH/2 times fewer.  The barriers
// are bare s_barriers behind an LDS-only wait: __syncthreads() would wait for every outstanding global load, the
// next chunk's weights included.
template <int CH>
__global__ __launch_bounds__(256, 3) void k_linear_splitk_chunked_bf16(SplitKArgs sa)
{
    constexpr int NQ = 2, KS = 128 * NQ, LDK = KS + 8, CPR = KS / 8, XL = (64 * CPR) / 256, RSTEP = 256 / CPR;
    extern __shared__ __attribute__((aligned(16))) bf16_t Xs[];   // [64][LDK]
    const LinArgs &a = sa.a;
    if ((int)blockIdx.x < sa.lead_blocks) {        // the first workgroups of the grid carry the integer work
        if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
            step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)Xs, (int32_t *)Xs + MOA_MAX_TREE);
        return;
    }
    const int bx = (int)blockIdx.x - sa.lead_blocks;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, kg = lane >> 4;
    const int tile = bx / sa.splits, split = bx - tile * sa.splits;
    int s = 0;
    while (s + 1 < a.nseg && tile >= sa.tile_begin[s + 1]) ++s;
    const int n0 = (tile - sa.tile_begin[s]) * 64 + wave * 16;   // feature inside the segment
    const int k0 = split * KS * CH;
    const bf16_t *X = (const bf16_t *)(a.seg[s].X ? a.seg[s].X : a.X);
    const int64_t ldx = a.seg[s].X ? a.seg[s].ldx : a.ldx;
    const bf16_t *wp = (const bf16_t *)a.seg[s].W + (int64_t)(n0 + li) * a.K + k0 + 8 * kg;

    // piece c = tid + 256 i of a slice is row c / CPR, 16-byte column c % CPR: one 32-bit lane offset serves all i
    const uint32_t xoff = (uint32_t)(((tid / CPR) * ldx + 8 * (tid % CPR)) * (int64_t)sizeof(bf16_t));
    u32x4 xr[XL];
#pragma unroll
    for (int i = 0; i < XL; ++i) xr[i] = u32x4{0u, 0u, 0u, 0u};   // rows past the end stay zero; never stored
    auto load_x = [&](int c) {
        const char *xb = (const char *)(X + k0 + c * KS);
#pragma unroll
        for (int i = 0; i < XL; ++i)
            if (tid / CPR + RSTEP * i < a.R)
                xr[i] = *(const u32x4 *)(xb + (int64_t)i * RSTEP * ldx * (int64_t)sizeof(bf16_t) + xoff);
    };
    bf16x8 wf[2][NQ][4];
    auto load_w = [&](int set, int c) {
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) wf[set][q][j] = *(const bf16x8 *)(wp + c * KS + 128 * q + 32 * j);
    };
    load_x(0);
    load_w(0, 0);
    f32x4 acc[4];
#pragma unroll
    for (int rb = 0; rb < 4; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int set = c & 1;
        if (c + 1 < CH) load_w(set ^ 1, c + 1);
        if (c > 0) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // every wave is done reading the previous slice
#pragma unroll
        for (int i = 0; i < XL; ++i) {
            const int cc = tid + 256 * i;
            *(u32x4 *)&Xs[(cc / CPR) * LDK + 8 * (cc % CPR)] = xr[i];
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (c + 1 < CH) load_x(c + 1);
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bf16x8 xf[4];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb) xf[rb] = *(const bf16x8 *)&Xs[(16 * rb + li) * LDK + 128 * q + 32 * j + 8 * kg];
#pragma unroll
                for (int rb = 0; rb < 4; ++rb)
                    acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[set][q][j], xf[rb], acc[rb], 0, 0, 0);
            }
    }
    // lane holds features 4 kg .. 4 kg + 3 of its wave's 16, for row 16 rb + li
    float *p = sa.part + (int64_t)split * 64 * sa.ntot + tile * 64 + wave * 16 + 4 * kg;
#pragma unroll
    for (int rb = 0; rb < 4; ++rb)
        if (16 * rb + li < a.R) *(f32x4 *)(p + (int64_t)(16 * rb + li) * sa.ntot) = acc[rb];
}

// The same sums with the activation slice resident: a workgroup owns one 1024-wide K slice of one activation matrix for
// its whole life -- the slice [64 rows x 1024] is parked in LDS once (132 KB, so one workgroup per compute unit) -- and
// its wavefronts each stream the weight rows of 16-feature groups through registers, 256 columns at a time with the
// next 256 in flight.  After the one barrier behind the staging nothing in the loop waits for another wavefront: no
// barrier per chunk, no activation re-reads (the chunked form above pulls as many activation bytes from the L2 as
// weight bytes from HBM), every wavefront keeps two chunks of loads in flight from its first instruction to its last.
// The grid is planned on the host so that every compute unit gets one workgroup and every wavefront the same number of
// groups: segments that read different activations are classes of their own, each with its share of the workgroups.
// Partial sums go where the chunked form puts them (same K slices, same order of MFMAs along K: same bits), and the
// same pass adds them up.
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

struct XresArgs {
    SplitKArgs k;
    int ncls;
    int wg0[5];          // first workgroup of each class behind the lead blocks; [ncls] = all
    int g0[5];           // first 16-feature group of each class; [ncls] = all groups
    int gpw[4];          // groups per workgroup
    const void *X[4];    // the class's activations
    int64_t ldx[4];
};

__global__ __launch_bounds__(1024) void k_linear_splitk_xres_bf16(XresArgs xa)
{
    constexpr int KS = 1024, LDK = KS + 8, CW = 256, NCH = KS / CW;
    extern __shared__ __attribute__((aligned(16))) bf16_t Xs[];   // [64][LDK]
    const SplitKArgs &sa = xa.k;
    const LinArgs &a = sa.a;
    if ((int)blockIdx.x < sa.lead_blocks) {        // the first workgroups of the grid carry the integer work
        if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
            step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)Xs, (int32_t *)Xs + MOA_MAX_TREE);
        return;
    }
    const int bx = (int)blockIdx.x - sa.lead_blocks;
    int cls = 0;
    while (cls + 1 < xa.ncls && bx >= xa.wg0[cls + 1]) ++cls;
    const int rel = bx - xa.wg0[cls];
    const int split = rel % sa.splits, fr = rel / sa.splits;
    const int nthreads = (int)blockDim.x, nw = nthreads >> 6;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, li = lane & 15, kg = lane >> 4;
    const int k0 = split * KS;
    const int gbeg = xa.g0[cls] + fr * xa.gpw[cls];
    int gend = gbeg + xa.gpw[cls];
    if (gend > xa.g0[cls + 1]) gend = xa.g0[cls + 1];
    if (gbeg >= gend) return;                       // (the host plans no such workgroup) leaves before the barrier, whole

    // weight rows of group g for this lane: k slot (q, j, kg) of chunk c is k = 256 c + 128 q + 32 j + 8 kg
    auto wrow = [&](int g) {
        if (g > gend - 1) g = gend - 1;             // a request past the wavefront's last group repeats a valid one
        const int tile = g >> 2;
        int s = 0;
        while (s + 1 < a.nseg && tile >= sa.tile_begin[s + 1]) ++s;
        const int n = (tile - sa.tile_begin[s]) * 64 + (g & 3) * 16 + li;
        return (const bf16_t *)a.seg[s].W + (int64_t)n * a.K + k0 + 8 * kg;
    };
    bf16x8 wf[2][8];
    auto load_w = [&](int set, const bf16_t *wp, int c) {
#pragma unroll
        for (int q = 0; q < 2; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) wf[set][q * 4 + j] = *(const bf16x8 *)(wp + CW * c + 128 * q + 32 * j);
    };
    int g = gbeg + wave;
    const bf16_t *wp = wrow(g);
    load_w(0, wp, 0);                               // on their way while the activations are staged

    // the activation slice, once, from global memory straight into LDS: instruction t fills the 1 KB half t % 2 of row
    // t / 2; rows past the end repeat the last row (their sums are never stored).  Nothing waits inside the loop.
    {
        const bf16_t *X = (const bf16_t *)xa.X[cls] + k0 + 8 * lane;
        const int64_t ldx = xa.ldx[cls];
        for (int t = wave; t < 128; t += nw) {
            const int row = t >> 1, h = t & 1;
            const int rsrc = row < a.R ? row : (int)a.R - 1;
            __builtin_amdgcn_global_load_lds((global_void_t *)(X + (int64_t)rsrc * ldx + 512 * h),
                                             (lds_void_t *)(Xs + row * LDK + 512 * h), 16, 0, 0);
        }
    }
    asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");

    // A wavefront's groups one after the other; the chunk after the one being multiplied is always in flight, across
    // the end of a group too.
    for (; g < gend; g += nw) {
        // (the slice in LDS does not change any more, and the compiler knows: without this it reads all of a group's
        // operand fragments ahead of the loop, into five hundred registers it does not have)
        asm volatile("" ::: "memory");
        const bf16_t *wnext = wrow(g + nw);
        f32x4 acc[4];
#pragma unroll
        for (int rb = 0; rb < 4; ++rb) acc[rb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int c = 0; c < NCH; ++c) {
            const int set = c & 1;
            if (c + 1 < NCH) load_w(set ^ 1, wp, c + 1);
            else load_w(set ^ 1, wnext, 0);
            __builtin_amdgcn_sched_barrier(0);      // the requests stay up here, a whole chunk ahead of their use
#pragma unroll
            for (int q = 0; q < 2; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bf16x8 xf[4];
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb) xf[rb] = *(const bf16x8 *)&Xs[(16 * rb + li) * LDK + CW * c + 128 * q + 32 * j + 8 * kg];
#pragma unroll
                    for (int rb = 0; rb < 4; ++rb)
                        acc[rb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[set][q * 4 + j], xf[rb], acc[rb], 0, 0, 0);
                }
        }
        // lane holds features 4 kg .. 4 kg + 3 of the group for row 16 rb + li
        float *pp = sa.part + (int64_t)split * 64 * sa.ntot + g * 16 + 4 * kg;
#pragma unroll
        for (int rb = 0; rb < 4; ++rb)
            if (16 * rb + li < a.R) *(f32x4 *)(pp + (int64_t)(16 * rb + li) * sa.ntot) = acc[rb];
        wp = wnext;
    }
}

__global__ __launch_bounds__(256) void k_linear_splitk_reduce(SumArgs sa) { splitk_reduce_block(sa, (int)blockIdx.x, (int)threadIdx.x); }

// The pass with the residual and the RMS norm behind it (LinArgs::EPI_ADD_NORM): one workgroup per row, every lane
// its 16-byte pieces of the row in registers for both halves (the sum of squares, then the scaled row).  The arithmetic
// is launch_rmsnorm's on x and the projection rounded to the storage type: the same bits as the two launches.
template <int NCH>
__global__ __launch_bounds__(256) void k_linear_splitk_reduce_norm(SumArgs sa)
{
    __shared__ float part[4];
    const int64_t r = blockIdx.x;
    const int d = sa.ntot, nch = d >> 3;
    const float *prow = sa.part + (((r >> 6) * sa.splits) * 64 + (r & 63)) * (int64_t)sa.ntot;
    const bf16_t *x = (const bf16_t *)sa.norm.x + r * d, *g = (const bf16_t *)sa.norm.g;
    float v[NCH][8];
    u32x4 gv[NCH];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + 256 * i;
        const bool live = c < nch;
        const int cc = live ? c : 0;
        f32x4 lo, hi;
        splitk_sum8(sa, prow + 8 * cc, lo, hi);
        const u32x4 yv = pack8(lo, hi);                      // the projection as it would be stored
        const u32x4 xv = *(const u32x4 *)(x + 8 * cc);
        gv[i] = *(const u32x4 *)(g + 8 * cc);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float l = __uint_as_float(xv[e] << 16) + __uint_as_float(yv[e] << 16);
            const float h = __uint_as_float(xv[e] & 0xffff0000u) + __uint_as_float(yv[e] & 0xffff0000u);
            v[i][2 * e] = l;
            v[i][2 * e + 1] = h;
            if (live) ss += l * l + h * h;
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + sa.norm.eps);
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + 256 * i;
        if (c >= nch) continue;
        u32x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float glo = __uint_as_float(gv[i][e] << 16), ghi = __uint_as_float(gv[i][e] & 0xffff0000u);
            o[e] = pack_bf16x2(v[i][2 * e] * inv * glo, v[i][2 * e + 1] * inv * ghi);
        }
        *(u32x4 *)((bf16_t *)sa.norm.n + r * d + 8 * c) = o;
        *(f32x4 *)(sa.norm.h + r * d + 8 * c) = f32x4{v[i][0], v[i][1], v[i][2], v[i][3]};
        *(f32x4 *)(sa.norm.h + r * d + 8 * c + 4) = f32x4{v[i][4], v[i][5], v[i][6], v[i][7]};
    }
}

hipError_t launch_splitk_sum(const SumArgs &sa, hipStream_t stream)
{
    if (sa.blocks <= 0) return hipSuccess;
    prof_begin(K_LIN_REDUCE, stream);
    if (sa.epi == LinArgs::EPI_ADD_NORM) {
        if (sa.ntot <= 256 * 8 * 2) MOA_KLAUNCH(k_linear_splitk_reduce_norm<2>, dim3((unsigned)sa.R), dim3(256), 0, stream, sa);
        else MOA_KLAUNCH(k_linear_splitk_reduce_norm<4>, dim3((unsigned)sa.R), dim3(256), 0, stream, sa);
        prof_end(stream);
        return hipGetLastError();
    }
    MOA_KLAUNCH(k_linear_splitk_reduce, dim3((unsigned)sa.blocks), dim3(256), 0, stream, sa);
    prof_end(stream);
    return hipGetLastError();
}

// The weight-streaming kernel walks 64-row tiles with the weights in registers.  Its fp32 partial sums are
// (row tiles * 128 / K slice) of the weight bytes.  Up to two row tiles it is always used (K slices chosen for the
// number of workgroups); at three row tiles with 512-wide K slices (partial sums three quarters of the weights):
// the tiled kernel has too few workgroups there to hide its per-tile latency (LSA on five tokens: 35 -> 17 us).
// Four row tiles would need 1024-wide slices, one workgroup per CU: measured twice as slow as the tiled kernel.
constexpr int64_t SPLITK_MAX_ROWS = 128;
constexpr int64_t SPLITK_MAX_ROWS_WIDE = 192;

static int splitk_nq(int K)
{
    for (int nq = 1; nq <= 4; nq *= 2)
        if (K % (128 * nq) == 0 && K / (128 * nq) <= 8) return nq;
    // long rows: 512-wide slices keep two workgroups per CU (1024-wide ones need 132 KB of LDS); the partial sums
    // are a quarter of the weights per row tile, whatever the number of slices
    if (K % 512 == 0) return 4;
    return (K % 1024 == 0) ? 8 : 0;
}

// K slice width (in units of 128) for R rows, 0 = do not use the weight-streaming kernel
static int splitk_plan(int64_t R, int K)
{
    if (R <= 0 || K % 128) return 0;
    const int nq0 = splitk_nq(K);
    if (!nq0 || R <= SPLITK_MAX_ROWS) return nq0;
    if (R > SPLITK_MAX_ROWS_WIDE) return 0;
    const int64_t rowtiles = (R + 63) / 64;
    for (int nq = nq0; nq <= 4; nq *= 2)
        if (K % (128 * nq) == 0 && rowtiles * 4 <= 3 * nq) return nq;      // rowtiles * 128 / (128 nq) <= 3/4
    return 0;
}

size_t linear_workspace_bytes(int dtype, int64_t R, int K, int ntot)
{
    if (dtype != DT_BF16 || ntot % 64) return 0;
    const int nq = splitk_plan(R, K);
    if (!nq) return 0;
    const size_t splits = K / (128 * nq), rowtiles = (size_t)((R + 63) / 64);
    return rowtiles * splits * 64 * (size_t)ntot * sizeof(float);
}

// ------------------------------------------------------------------ tiled bf16 (many rows)
struct TiledArgs {
    LinArgs a;
    int tile_begin[5];
    int tiles_per_xcd;   // feature tiles owned by one XCD
    int lead_blocks;     // workgroups in front of the projection's own: LinArgs::rider, then LinArgs::carry_sum
    int small_lead;      // the first of them carry LinArgs::rider (padded to the XCD count)
    int red_blocks;      // workgroups of the carried summing pass `red` (0 = none)
    SumArgs red;
};

// WF x WR = 32x32 MFMA blocks per wave along features x rows; the four waves sit 2 x 2, so the workgroup
// tile is (64 WF) features x (64 WR) rows, walked along K in tiles of 64.
// The k tiles go from global memory straight into LDS (no register staging, no LDS write instructions): one
// wave instruction moves 64 x 16 B = 8 rows of 128 B into 1 KB of contiguous LDS, so rows are unpadded, and
// the bank conflicts that would cause in the operand reads are removed by a swizzle: 16-byte chunk c of tile
// row r lives at position c ^ ((r >> 1) & 7), applied to the global address each lane fetches (the eight
// lanes of a row still cover the same 128 bytes).  The loads of tile kt+1 are issued before the MFMAs of tile
// kt and complete behind them; one barrier per k tile publishes the new tile and retires the old one.

template <int WF, int WR>
__global__ __launch_bounds__(256) void k_linear_tiled_bf16(TiledArgs ta)
{
    constexpr int BN = 64 * WF, BM = 64 * WR, BK = 64;
    constexpr int STAGE = (BN + BM) * BK;                     // bf16 elements per LDS stage: W rows, then X rows
    constexpr int NWI = BN / 32, NXI = BM / 32;               // 8-row load instructions per wave per stage
    extern __shared__ __attribute__((aligned(16))) bf16_t tsm[];   // [2][STAGE]

    const LinArgs &a = ta.a;
    if ((int)blockIdx.x < ta.lead_blocks) {        // the first workgroups of the grid carry work of other calls
        if ((int)blockIdx.x < ta.small_lead) {
            if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
                step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)tsm, (int32_t *)tsm + MOA_MAX_TREE);
        } else if ((int)blockIdx.x - ta.small_lead < ta.red_blocks) {
            splitk_reduce_block(ta.red, (int)blockIdx.x - ta.small_lead, (int)threadIdx.x);
        }
        return;
    }
    const int bx = (int)blockIdx.x - ta.lead_blocks;
    // Workgroups are handed to the 8 XCDs round-robin (id % 8), and each XCD has its own L2.  Give every
    // XCD a contiguous group of feature tiles for all row tiles: its slice of W then stays in its L2 and
    // each activation tile is fetched once per XCD instead of once per workgroup.
    const int xcd = bx & 7, j = bx >> 3;
    const int ftile = xcd * ta.tiles_per_xcd + j % ta.tiles_per_xcd;
    if (ftile >= ta.tile_begin[a.nseg]) return;
    int s = 0;
    while (s + 1 < a.nseg && ftile >= ta.tile_begin[s + 1]) ++s;
    const int n0 = (ftile - ta.tile_begin[s]) * BN;
    const int64_t r0 = (int64_t)(j / ta.tiles_per_xcd) * BM;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int wf0 = (wave & 1) * (32 * WF);   // feature offset of this wave inside the tile
    const int wr0 = (wave >> 1) * (32 * WR);  // row offset
    const int K = a.K;
    const bf16_t *W = (const bf16_t *)a.seg[s].W;
    const bf16_t *X = (const bf16_t *)(a.seg[s].X ? a.seg[s].X : a.X);
    const int64_t ldx = a.seg[s].X ? a.seg[s].ldx : a.ldx;

    // wave w moves tile rows (BN/4) w .. of W and (BM/4) w .. of X, eight rows per instruction
    const int lrow = lane >> 3, lpos = lane & 7;
    const bf16_t *wsrc[NWI], *xsrc[NXI];
#pragma unroll
    for (int i = 0; i < NWI; ++i) {
        const int row = (BN / 4) * wave + 8 * i + lrow;
        wsrc[i] = W + (int64_t)(n0 + row) * K + 8 * (lpos ^ ((row >> 1) & 7));
    }
#pragma unroll
    for (int i = 0; i < NXI; ++i) {
        const int row = (BM / 4) * wave + 8 * i + lrow;
        int64_t r = r0 + row;
        if (r > a.R - 1) r = a.R - 1;          // rows past the end repeat the last row; never stored
        xsrc[i] = X + r * ldx + 8 * (lpos ^ ((row >> 1) & 7));
    }
    auto issue = [&](int buf, int kt) {
        bf16_t *wb = tsm + buf * STAGE;
        bf16_t *xb = wb + BN * BK;
#pragma unroll
        for (int i = 0; i < NWI; ++i)
            __builtin_amdgcn_global_load_lds((global_void_t *)(wsrc[i] + (int64_t)kt * BK),
                                             (lds_void_t *)(wb + ((BN / 4) * wave + 8 * i) * BK), 16, 0, 0);
#pragma unroll
        for (int i = 0; i < NXI; ++i)
            __builtin_amdgcn_global_load_lds((global_void_t *)(xsrc[i] + (int64_t)kt * BK),
                                             (lds_void_t *)(xb + ((BM / 4) * wave + 8 * i) * BK), 16, 0, 0);
    };

    f32x16 acc[WF][WR];
#pragma unroll
    for (int i = 0; i < WF; ++i)
#pragma unroll
        for (int jj = 0; jj < WR; ++jj)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][jj][e] = 0.f;

    const int nk = K / BK;
    issue(0, 0);
    __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0): this wave's share of tile 0 has landed in LDS
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) issue(buf ^ 1, kt + 1);   // everyone is past the reads of tile kt-1 (same buffer)
        const bf16_t *wb = tsm + buf * STAGE;
        const bf16_t *xb = wb + BN * BK;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 af[WF], bfr[WR];
#pragma unroll
            for (int i = 0; i < WF; ++i) {
                const int row = wf0 + 32 * i + l32;
                af[i] = *(const bf16x8 *)&wb[row * BK + 8 * ((2 * ks + half) ^ ((row >> 1) & 7))];
            }
#pragma unroll
            for (int i = 0; i < WR; ++i) {
                const int row = wr0 + 32 * i + l32;
                bfr[i] = *(const bf16x8 *)&xb[row * BK + 8 * ((2 * ks + half) ^ ((row >> 1) & 7))];
            }
#pragma unroll
            for (int i = 0; i < WF; ++i)
#pragma unroll
                for (int jj = 0; jj < WR; ++jj)
                    acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[jj], acc[i][jj], 0, 0, 0);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70);    // tile kt+1 of this wave is in LDS
        __syncthreads();
    }

    // acc[i][jj][v]: feature = wf0 + 32 i + 8 (v/4) + 4 half + v%4, row = wr0 + 32 jj + l32
    bf16_t *dst = (bf16_t *)a.seg[s].st.dst;
#pragma unroll
    for (int jj = 0; jj < WR; ++jj) {
        const int64_t r = r0 + wr0 + 32 * jj + l32;
        if (r >= a.R) continue;
        const int64_t rp = store_row_part(a.seg[s].st, r);
        if (rp < 0) continue;
#pragma unroll
        for (int i = 0; i < WF; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wf0 + 32 * i + 8 * q + 4 * half;
                const int64_t off = rp + store_feat_part(a.seg[s].st, n);
                u32x2 pk;
                pk[0] = pack_bf16x2(acc[i][jj][4 * q + 0], acc[i][jj][4 * q + 1]);
                pk[1] = pack_bf16x2(acc[i][jj][4 * q + 2], acc[i][jj][4 * q + 3]);
                *(u32x2 *)(dst + off) = pk;
            }
    }
}

template <int WF, int WR>
static hipError_t launch_tiled(const LinArgs &a, hipStream_t stream)
{
    constexpr int BN = 64 * WF, BM = 64 * WR;
    TiledArgs ta;
    ta.a = a;
    int t = 0;
    for (int s = 0; s < a.nseg; ++s) { ta.tile_begin[s] = t; t += a.seg[s].N / BN; }
    ta.tile_begin[a.nseg] = t;
    ta.tiles_per_xcd = (t + 7) / 8;
    ta.small_lead = (a.rider_units + 7) & ~7;       // multiples of the XCD count: the tile mapping keeps its phase
    ta.red_blocks = 0;
    ta.red = SumArgs{};
    if (a.carry_sum && a.carry_sum->blocks > 0) {
        ta.red = *a.carry_sum;
        ta.red_blocks = a.carry_sum->blocks;
    }
    ta.lead_blocks = ta.small_lead + ((ta.red_blocks + 7) & ~7);
    const dim3 grid((unsigned)(ta.lead_blocks + 8 * ta.tiles_per_xcd * (int)((a.R + BM - 1) / BM)));
    const size_t lds = (size_t)2 * (BN + BM) * 64 * sizeof(bf16_t);
    static bool raised[16] = {};
    hipError_t e = raise_lds_limit_once(raised, (const void *)k_linear_tiled_bf16<WF, WR>, lds);
    if (e != hipSuccess) return e;
    prof_begin(K_LIN_TILED + 64 * (WF * 8 + WR), stream);
    MOA_KLAUNCH((k_linear_tiled_bf16<WF, WR>), grid, dim3(256), lds, stream, ta);
    prof_end(stream);
    return hipGetLastError();
}

// ------------------------------------------------------------------ dispatch
static bool aligned16(const void *p) { return (((uintptr_t)p) & 15) == 0; }

// which kernel a call gets; decided from shapes and alignment alone, so that launch_linear knows beforehand whether
// the launch can carry what LinArgs::carry_sum names
enum LinPath { P_TILED, P_SPLITK, P_SKINNY, P_EACH, P_GENERIC };

static LinPath linear_path(int dtype, const LinArgs &a, int *nq_out)
{
    *nq_out = 0;
    bool own_x = false;
    for (int s = 0; s < a.nseg; ++s) own_x = own_x || a.seg[s].X != nullptr;
    bool fast = dtype == DT_BF16 && a.K % 128 == 0 && a.ldx % 8 == 0 && aligned16(a.X);
    for (int s = 0; s < a.nseg && fast; ++s)
        if (a.seg[s].X) fast = a.seg[s].ldx % 8 == 0 && aligned16(a.seg[s].X);
    for (int s = 0; s < a.nseg && fast; ++s) {
        const StoreSpec &st = a.seg[s].st;
        fast = a.seg[s].N % 32 == 0 && aligned16(a.seg[s].W) && aligned16(st.dst) &&
               (st.mode == StoreSpec::ROW ? st.ld % 8 == 0 : st.dh % 8 == 0);
    }
    if (!fast) return own_x ? P_EACH : P_GENERIC;
    bool all128 = true, all64 = true;
    int ntot = 0;
    for (int s = 0; s < a.nseg; ++s) {
        all128 = all128 && a.seg[s].N % 128 == 0;
        all64 = all64 && a.seg[s].N % 64 == 0;
        ntot += a.seg[s].N;
    }
    const int nq = splitk_plan(a.R, a.K);
    if (!nq && all128) return P_TILED;
    const size_t need = all64 ? linear_workspace_bytes(dtype, a.R, a.K, ntot) : 0;
    if (need && a.ws && a.ws_bytes >= need && (((uintptr_t)a.ws) & 15) == 0) {
        *nq_out = nq;
        return P_SPLITK;
    }
    return own_x ? P_EACH : P_SKINNY;
}

static hipError_t launch_linear_impl(int dtype, const LinArgs &a, hipStream_t stream, bool *rode, bool *fused);

static thread_local bool t_leave_room = false;
LinearLeaveRoom::LinearLeaveRoom() : before(t_leave_room) { t_leave_room = true; }
LinearLeaveRoom::~LinearLeaveRoom() { t_leave_room = before; }

// the pass that adds up the K slices a weight-streaming kernel has left in ka.part: launched, or handed to the caller
static hipError_t finish_splitk(const LinArgs &a, const SplitKArgs &ka, int ntot, hipStream_t stream, bool *fused)
{
    // the residual + norm pass takes rows of at most 8192 values with 16-byte aligned operands, and is never carried
    const bool norm_ok = a.epi != LinArgs::EPI_ADD_NORM ||
                         (ntot <= 256 * 8 * 4 && !a.sum_out && a.norm.x && a.norm.g && a.norm.h && a.norm.n &&
                          ((((uintptr_t)a.norm.x) | ((uintptr_t)a.norm.g) | ((uintptr_t)a.norm.h) | ((uintptr_t)a.norm.n)) & 15) == 0);
    *fused = a.epi != LinArgs::EPI_NONE && norm_ok;
    SumArgs sum = {};
    const int64_t items = a.R * ((a.epi == LinArgs::EPI_SWIGLU ? ntot / 2 : ntot) / 8);
    sum.blocks = (int)((items + 255) / 256);
    sum.R = a.R;
    sum.nseg = a.nseg;
    for (int s = 0; s < a.nseg; ++s) sum.st[s] = a.seg[s].st;
    for (int s = 0; s <= a.nseg; ++s) sum.tile_begin[s] = ka.tile_begin[s];
    sum.splits = ka.splits;
    sum.ntot = ntot;
    sum.part = ka.part;
    sum.epi = norm_ok ? a.epi : (int)LinArgs::EPI_NONE;
    sum.epi_res = a.epi_res;
    sum.epi_out = a.epi_out;
    sum.norm = a.norm;
    if (a.epi == LinArgs::EPI_ROPE) {
        sum.rope = a.rope;
        sum.rope_log_theta = log(a.rope.theta);
    }
    if (a.sum_out) {                         // the caller has it carried by a later launch, or launches it
        *a.sum_out = sum;
        return hipSuccess;
    }
    return launch_splitk_sum(sum, stream);
}

// Grid of the resident-activation kernel for a projection whose K slices are 1024 wide (ka.splits of them): one
// workgroup per compute unit, classes = runs of segments that read the same activations, each class with a share of
// the workgroups in proportion to its features, every wavefront of a workgroup one 16-feature group (or the same
// small number of them).  False when the shape does not fill the chip that way.
static bool plan_xres(const SplitKArgs &ka, XresArgs *xa, int *nw_out)
{
    const LinArgs &a = ka.a;
    const int S = ka.splits;
    if (t_leave_room) return false;              // 132 KB of LDS: nothing else fits beside it
    if (a.R > 64 || a.K % 1024 || S < 1 || S * 1024 != a.K) return false;
    static int cus = 0;
    if (!cus) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
        cus = n;
    }
    const int per_split = cus / S;               // workgroups per K slice
    if (per_split < 1) return false;
    xa->k = ka;
    xa->ncls = 0;
    int groups[4] = {0, 0, 0, 0}, g = 0;
    for (int s = 0; s < a.nseg; ++s) {
        const void *X = a.seg[s].X ? a.seg[s].X : a.X;
        const int64_t ldx = a.seg[s].X ? a.seg[s].ldx : a.ldx;
        if (xa->ncls == 0 || X != xa->X[xa->ncls - 1] || ldx != xa->ldx[xa->ncls - 1]) {
            xa->X[xa->ncls] = X;
            xa->ldx[xa->ncls] = ldx;
            xa->g0[xa->ncls] = g;
            ++xa->ncls;
        }
        groups[xa->ncls - 1] += a.seg[s].N / 16;
        g += a.seg[s].N / 16;
    }
    xa->g0[xa->ncls] = g;
    if (xa->ncls > per_split) return false;
    // workgroups per class and K slice: in proportion to the groups, the remainder to whoever has most groups per workgroup
    int wg[4], left = per_split;
    for (int c = 0; c < xa->ncls; ++c) {
        wg[c] = (int)((int64_t)per_split * groups[c] / g);
        if (wg[c] < 1) wg[c] = 1;
        left -= wg[c];
    }
    if (left < 0) return false;
    for (; left > 0; --left) {
        int best = 0;
        for (int c = 1; c < xa->ncls; ++c)
            if ((int64_t)groups[c] * wg[best] > (int64_t)groups[best] * wg[c]) best = c;
        ++wg[best];
    }
    int most = 0, w0 = 0;
    for (int c = 0; c < xa->ncls; ++c) {
        xa->gpw[c] = (groups[c] + wg[c] - 1) / wg[c];
        wg[c] = (groups[c] + xa->gpw[c] - 1) / xa->gpw[c];      // no workgroup without a group
        xa->wg0[c] = w0;
        w0 += wg[c] * S;
        if (xa->gpw[c] > most) most = xa->gpw[c];
    }
    xa->wg0[xa->ncls] = w0;
    const int per_wave = (most + 15) / 16;
    const int nw = (most + per_wave - 1) / per_wave;
    if (nw < 5) return false;                    // too few wavefronts per compute unit to keep the memory busy (60 x 4096: five at 5120 features 14.7 against 17.3 us chunked, four at 4096 features 13.8 against 12.7)
    *nw_out = nw;
    return true;
}

// kernels without per-segment activation support get one call per segment
static hipError_t launch_linear_each(int dtype, const LinArgs &a, hipStream_t stream)
{
    for (int s = 0; s < a.nseg; ++s) {
        LinArgs one = a;
        one.rider_units = 0;
        one.carry_sum = nullptr;
        one.sum_out = nullptr;
        one.nseg = 1;
        one.seg[0] = a.seg[s];
        if (a.seg[s].X) { one.X = a.seg[s].X; one.ldx = a.seg[s].ldx; }
        one.seg[0].X = nullptr;
        one.epi = LinArgs::EPI_NONE;
        bool rode = false, fused = false;
        hipError_t e = launch_linear_impl(dtype, one, stream, &rode, &fused);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// *rode is set when the launch carried a.rider in its grid, *fused when it applied a.epi.  a.carry_sum is only
// set where the path can carry it (launch_linear sees to that).
static hipError_t launch_linear_impl(int dtype, const LinArgs &a, hipStream_t stream, bool *rode, bool *fused)
{
    *rode = false;
    *fused = false;
    if (a.R <= 0) return hipSuccess;
    int nq = 0;
    const LinPath path = linear_path(dtype, a, &nq);
    if (path == P_TILED) {
        // 2x2 blocks per wave keeps two workgroups per CU; a 4x2 variant halves the LDS traffic per MFMA but drops
        // to one workgroup per CU and measured slower
        *rode = a.rider_units > 0;
        return launch_tiled<2, 2>(a, stream);
    }
    if (path == P_SPLITK) {
        SplitKArgs ka;
        ka.a = a;
        int t = 0, ntot = 0;
        for (int s = 0; s < a.nseg; ++s) { ka.tile_begin[s] = t; t += a.seg[s].N / 64; ntot += a.seg[s].N; }
        ka.tile_begin[a.nseg] = t;
        ka.splits = a.K / (128 * nq);
        ka.ntot = ntot;
        ka.part = (float *)a.ws;
        ka.lead_blocks = (a.rider_units + 7) & ~7;
        *rode = a.rider_units > 0;
        // At most 64 rows and a grid that still gives every CU a workgroup: K is cut into 1024-wide slices walked in
        // four chunks (half the partial sums of the 512-wide single-shot form, three workgroups per CU); measured
        // -4 us per step at C1.
        int ch = 0;                                  // chunks per workgroup; 0 = the single-shot kernel
        if (a.R <= 64) {
            if (a.K % 1024 == 0 && (int64_t)t * (a.K / 1024) >= 256) ch = 4;
            else if (a.K % 512 == 0 && (int64_t)t * (a.K / 512) >= 256) ch = 2;
        }
        if (ch) ka.splits = a.K / (256 * ch);
        if (ch == 4) {
            XresArgs xa;
            int nw = 0;
            if (plan_xres(ka, &xa, &nw)) {
                const size_t xl = (size_t)64 * (1024 + 8) * sizeof(bf16_t);
                static bool raised_x[16] = {};
                hipError_t ex = raise_lds_limit_once(raised_x, (const void *)k_linear_splitk_xres_bf16, xl);
                if (ex != hipSuccess) return ex;
                prof_begin(K_LIN_SPLITK_XRES, stream);
                MOA_KLAUNCH(k_linear_splitk_xres_bf16, dim3((unsigned)(ka.lead_blocks + xa.wg0[xa.ncls])), dim3(64 * nw), xl, stream, xa);
                prof_end(stream);
                ex = hipGetLastError();
                if (ex != hipSuccess) return ex;
                return finish_splitk(a, ka, ntot, stream, fused);
            }
        }
        const dim3 grid((unsigned)(ka.lead_blocks + t * ka.splits));
        const size_t lds = (size_t)64 * (128 * (ch ? 2 : nq) + 8) * sizeof(bf16_t);
        hipError_t e = hipSuccess;
        prof_begin(ch ? K_LIN_SPLITK_CHUNKED + 64 * ch : K_LIN_SPLITK + 64 * nq, stream);
        if (ch == 4) MOA_KLAUNCH(k_linear_splitk_chunked_bf16<4>, grid, dim3(256), lds, stream, ka);
        else if (ch == 2) MOA_KLAUNCH(k_linear_splitk_chunked_bf16<2>, grid, dim3(256), lds, stream, ka);
        else
        switch (nq) {
        case 1: MOA_KLAUNCH(k_linear_splitk_bf16<1>, grid, dim3(256), lds, stream, ka); break;
        case 2: MOA_KLAUNCH(k_linear_splitk_bf16<2>, grid, dim3(256), lds, stream, ka); break;
        case 4: MOA_KLAUNCH(k_linear_splitk_bf16<4>, grid, dim3(256), lds, stream, ka); break;
        default:
            static bool raised8[16] = {};
            e = raise_lds_limit_once(raised8, (const void *)k_linear_splitk_bf16<8>, lds);
            if (e == hipSuccess) MOA_KLAUNCH(k_linear_splitk_bf16<8>, grid, dim3(256), lds, stream, ka);
            break;
        }
        prof_end(stream);
        if (e != hipSuccess) return e;
        e = hipGetLastError();
        if (e != hipSuccess) return e;
        return finish_splitk(a, ka, ntot, stream, fused);
    }
    if (path == P_EACH) return launch_linear_each(dtype, a, stream);
    if (path == P_SKINNY) {
        SkinnyArgs sa;
        sa.a = a;
        int t = 0;
        for (int s = 0; s < a.nseg; ++s) { sa.tile_begin[s] = t; t += a.seg[s].N / 32; }
        sa.tile_begin[a.nseg] = t;
        dim3 grid(t, (unsigned)((a.R + 63) / 64));
        { prof_begin(K_LIN_SKINNY, stream); MOA_KLAUNCH(k_linear_skinny_bf16<2>, grid, dim3(256), 0, stream, sa); prof_end(stream); }
        return hipGetLastError();
    }
    for (int s = 0; s < a.nseg; ++s) {
        dim3 grid((a.seg[s].N + 63) / 64, (unsigned)((a.R + 63) / 64));
        if (dtype == DT_BF16)
            { prof_begin(K_LIN_GENERIC, stream); MOA_KLAUNCH(k_linear_generic<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t *)a.X, a.R, a.K,
                               a.ldx, (const bf16_t *)a.seg[s].W, a.seg[s].N, a.seg[s].st); prof_end(stream); }
        else
            { prof_begin(K_LIN_GENERIC, stream); MOA_KLAUNCH(k_linear_generic<float>, grid, dim3(256), 0, stream, (const float *)a.X, a.R, a.K,
                               a.ldx, (const float *)a.seg[s].W, a.seg[s].N, a.seg[s].st); prof_end(stream); }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_linear(int dtype, const LinArgs &a, hipStream_t stream)
{
    if (a.sum_out) *a.sum_out = SumArgs{};
    if (a.epi == LinArgs::EPI_ADD_F32 && a.nseg != 1) return hipErrorInvalidValue;
    if (a.epi == LinArgs::EPI_SWIGLU && (a.nseg != 2 || a.seg[0].N != a.seg[1].N)) return hipErrorInvalidValue;
    if (a.epi == LinArgs::EPI_ADD_NORM && a.nseg != 1) return hipErrorInvalidValue;
    if (a.epi == LinArgs::EPI_ROPE && (a.nseg != 3 || a.rope.dh % 16 || a.seg[0].N != a.rope.H * a.rope.dh || a.seg[1].N != a.rope.Hkv * a.rope.dh))
        return hipErrorInvalidValue;
    // A carried pass rides in the tiled kernel only: that one keeps several workgroups per CU busy with matrix work,
    // so a few hundred short workgroups in front cost it nothing.  In the weight-streaming kernel (two workgroups per
    // CU, bound by the same memory path the pass uses) riding measured slower than a launch of its own.
    int nq = 0;
    LinArgs b = a;
    if (a.carry_sum && a.carry_sum->blocks > 0 && !(a.R > 0 && linear_path(dtype, a, &nq) == P_TILED)) {
        const hipError_t es = launch_splitk_sum(*a.carry_sum, stream);
        if (es != hipSuccess) return es;
        b.carry_sum = nullptr;
    }
    bool rode = false, fused = false;
    hipError_t e = launch_linear_impl(dtype, b, stream, &rode, &fused);
    if (e != hipSuccess) return e;
    if (a.epi != LinArgs::EPI_NONE && !fused) {     // the projection was stored as its segments say: finish row-wise
        const RopeArgs &ro = a.rope;
        if (a.epi == LinArgs::EPI_SWIGLU) e = launch_swiglu(dtype, a.seg[0].st.dst, a.R, a.seg[0].N, a.epi_out, stream);
        else if (a.epi == LinArgs::EPI_ROPE)
            e = launch_rope(dtype, ro.q, ro.k_draft, ro.prefix_len, ro.depth, ro.B, ro.Mn, ro.M, ro.node0, ro.H, ro.Hkv, ro.dh, ro.theta,
                            ro.P_cap, stream);
        else if (a.epi == LinArgs::EPI_ADD_NORM)
            e = launch_rmsnorm(dtype, a.norm.x, a.seg[0].st.dst, a.R, a.seg[0].N, a.norm.g, a.norm.eps, a.norm.h, a.norm.n, stream);
        else e = launch_add_out(dtype, a.epi_res, a.seg[0].st.dst, a.R * a.seg[0].N, a.epi_out, stream);
        if (e != hipSuccess) return e;
    }
    if (a.rider_units <= 0 || rode) return hipSuccess;
    return launch_step_small(a.rider, stream);      // the kernel that ran has no spare workgroups for it
}

}  // namespace moa

// ------------------------------------------------------------------ identity "projection"
// A NULL weight means the input is already projected; rows still have to reach the layout the
// store spec describes (e.g. [B, Hkv, M, dh] slabs).
namespace moa {

template <typename T>
__global__ void k_scatter_copy(const T *__restrict__ X, int64_t R, int N, int64_t ldx, StoreSpec stp)
{
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= R * N) return;
    const int64_t r = idx / N;
    const int n = (int)(idx - r * N);
    const int64_t off = store_offset(stp, r, n);
    if (off >= 0) ((T *)stp.dst)[off] = X[r * ldx + n];
}

hipError_t launch_scatter_copy(int dtype, const void *X, int64_t R, int N, int64_t ldx, const StoreSpec &st,
                               hipStream_t stream)
{
    if (R <= 0) return hipSuccess;
    const int64_t total = R * N;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (dtype == DT_BF16)
        { prof_begin(K_SCATTER, stream); MOA_KLAUNCH(k_scatter_copy<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t *)X, R, N, ldx, st); prof_end(stream); }
    else
        { prof_begin(K_SCATTER, stream); MOA_KLAUNCH(k_scatter_copy<float>, grid, dim3(256), 0, stream, (const float *)X, R, N, ldx, st); prof_end(stream); }
    return hipGetLastError();
}

}  // namespace moa
