// Layer Self-Attention with mean aggregation in ONE kernel (paper Sec. 3.1.1; Alg. 1, LSA_layer_with_mean):
// Q/K/V projection of a token's L layer rows, attention over the layer axis, and the mean over the layers, with the
// projected Q, K, V never leaving the compute unit.  Every token is independent of the others (Sec. 3.1.1), so a
// workgroup that owns whole tokens needs nothing from any other workgroup.
//
// A workgroup of eight wavefronts owns TT tokens (all their layer rows: RB = 32 NB TT rows, NB = ceil(L/32)) and the
// features of one KV head's group that one attention needs: two query heads, the key head and the value head, 4 dh
// features.  (A group of more than two query heads is cut into parts of two; each part recomputes K and V.)
//
//  projection  [RB x d_in] x [4 dh x d_in]^T on MFMA 32x32x16, walked along d_in in tiles of 64.  Wavefront w owns
//              the features w dh/2 .. and ALL rows, so its slice of the weight tile is its own: it fetches it itself
//              (global memory straight into LDS, 128-byte rows, XOR-swizzled against bank conflicts) into a private
//              two-stage ring and needs no barrier for it, only its own load counter.  As soon as a wavefront has
//              read its fragments of tile kt it requests tile kt+2 into the same place, so one whole tile and most of
//              another are in flight per compute unit while a tile is being multiplied.  The activation tile (RB rows,
//              shared by all wavefronts, an eighth of the weight tile) goes through a small ring of its own with one
//              barrier per tile.
//              Three things cost about the same per tile -- the weight tile's way from the L2 into LDS (64 KB per
//              64 of d_in, all workgroups of an XCD asking for the same lines at once), the operand reads from LDS
//              and the matrix work -- and they overlap only in part; the lever that is left is rows per workgroup
//              (2, 3 or 4 tokens at one 32-layer block each), chosen from the token count on the host.
//  attention   the accumulators are rounded to the storage type and parked in LDS as a [RB x 4 dh] tile (the ring
//              memory is reused); one wavefront per (token, query head): S^T = K Q^T by MFMA, fp32 softmax in
//              registers, column means of P summed over the 32 query lanes (DPP moves, one shuffle), then
//              abar = sum_j pbar_j V_j  (mean_i(P V) = (1^T P / L) V, exact in real arithmetic).  The output
//              projection follows in another launch on one row per token.
//
// Three kernels share that second half: k_lsa_fused (plain weights, as above), k_lsa_fused_pk (weights packed once
// into MFMA-operand order and read straight into registers; the form a step runs when it is given the packed copy)
// and k_lsa_fused_pk_lean (the same held to a third of a SIMD's registers, for the two-stream schedule).
//
// Arithmetic is that of the three-kernel form (same MFMA order along d_in, Q/K/V rounded once to the storage type,
// the same order of additions in the column sums), so all give the same bits.
#include "moa_common.h"
#include "moa_sum_device.h"
#include "moa_tree_device.h"

#include <math.h>
#include <type_traits>
#include <utility>

namespace moa {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void global_void_t;

struct LsaFusedArgs {
    const bf16_t *hs;              // [T, L, d_in]
    const bf16_t *wq, *wk, *wv;    // [Hq*dh, d_in], [Hkv*dh, d_in] x 2
    const bf16_t *wpk;             // the same weights in MFMA-operand order (k_lsa_pack_weights), or NULL
    bf16_t *abar;                  // [T, Hq*dh]
    int64_t T;
    int L, d_in, Hq, Hkv;
    int parts;                     // Hq / Hkv / 2: workgroups per KV head
    int units;                     // Hkv * parts
    int units_per_xcd;
    int lead_blocks, small_lead, red_blocks;   // workgroups in front of the kernel's own: integer work of a step, a carried summing pass
    int pf_lead;                               // the last of them (a multiple of the XCD count) only read ahead: see lsa_warm_block
    int rider_units;
    StepSmallArgs rider;
    SumArgs red;
};

template <int DH, int NB, int TT>
struct LsaFusedGeom {
    static constexpr int NF = 4 * DH;            // features per workgroup
    static constexpr int FW = NF / 8;            // per wavefront
    static constexpr int RB = 32 * NB * TT;      // rows per workgroup
    static constexpr int BK = 64;
    static constexpr int XS = RB <= 64 ? 3 : 2;  // stages of the activation ring
    static constexpr size_t w_bytes = (size_t)8 * 2 * FW * BK * sizeof(bf16_t);
    static constexpr size_t x_bytes = (size_t)XS * RB * BK * sizeof(bf16_t);
    static constexpr int TLD = NF + 8;           // row of the parked Q/K/V tile: 16-byte reads of 8 rows hit all banks
    static constexpr size_t tile_bytes = (size_t)RB * TLD * sizeof(bf16_t);
    static constexpr size_t pbar_bytes = (size_t)8 * 32 * NB * sizeof(float);
    static constexpr size_t loop_bytes = w_bytes + x_bytes;
    static constexpr size_t epi_bytes = tile_bytes + pbar_bytes;
    static constexpr size_t bytes = loop_bytes > epi_bytes ? loop_bytes : epi_bytes;
    // the form that takes packed weights keeps them in registers: only a two-stage activation ring is left in LDS
    static constexpr int WS = 2;                 // weight tiles held in registers per wavefront: with the requests spread between the MFMAs two do as well as four
    static constexpr int UN = 8;                 // tile steps per trip of the tile loop (a multiple of WS)
    static constexpr size_t pk_loop_bytes = (size_t)2 * RB * BK * sizeof(bf16_t);
    static constexpr size_t pk_bytes = pk_loop_bytes > epi_bytes ? pk_loop_bytes : epi_bytes;
};

// Second half of both kernels below: the accumulators of a workgroup's [RB x 4 dh] projection tile (acc[i][j][v]:
// feature wave FW + 32 i + 8 (v / 4) + 4 half + v % 4, row 32 j + lane % 32) are rounded to the storage type and
// parked in LDS, then one wavefront per (token of the tile, query head) runs the attention over the layer axis and the
// mean.  Called by all 512 threads; `sm` is the workgroup's whole LDS, free to reuse after the barrier in here.
template <int DH, int NB, int TT, typename Acc>
__device__ __forceinline__ void lsa_fused_epilogue(Acc &acc, const LsaFusedArgs &a, bf16_t *sm, int64_t tile, int g, int part)
{
    using Gm = LsaFusedGeom<DH, NB, TT>;
    constexpr int FW = Gm::FW, RB = Gm::RB, TLD = Gm::TLD;
    constexpr int WFB = FW / 32, NRB = RB / 32;
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int G = a.Hq / a.Hkv, L = a.L;

    // park Q | Q' | K | V of the RB rows in LDS, rounded to the storage type
    __syncthreads();                             // every wavefront is done with the rings
    bf16_t *tile_s = sm;
    float *pbar_s = (float *)((char *)sm + Gm::tile_bytes) + wave * 32 * NB;
    // acc[i][j][v]: feature = f0 + 32 i + 8 (v / 4) + 4 half + v % 4, row = 32 j + l32
    const int f0 = wave * FW;
    {
#pragma unroll
        for (int i = 0; i < WFB; ++i)
#pragma unroll
            for (int j = 0; j < NRB; ++j)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    u32x2 pk;
                    pk[0] = pack_bf16x2(acc[i][j][4 * q + 0], acc[i][j][4 * q + 1]);
                    pk[1] = pack_bf16x2(acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    *(u32x2 *)&tile_s[(32 * j + l32) * TLD + f0 + 32 * i + 8 * q + 4 * half] = pk;
                }
    }
    __syncthreads();

    // attention over the layer axis: one wavefront per (token of the tile, query head); spare wavefronts redo a
    // unit and store nothing, so that the barriers below are reached by all
    constexpr int NU = 2 * TT;
    constexpr int NKS = DH / 16;
    const bool live_wave = wave < NU;
    const int u = wave % NU, tt = u >> 1, hq = u & 1;
    const int64_t tok = tile * TT + tt;
    const bf16_t *trow = tile_s + (size_t)tt * 32 * NB * TLD;
    const float sc = 1.4426950408889634f / sqrtf((float)DH);      // log2 domain

    // column sums of P in the S^T register layout: csum[jb][v] belongs to key 32 jb + 8 (v/4) + 4 half + v%4
    float csum[NB][16];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int e = 0; e < 16; ++e) csum[jb][e] = 0.f;
#pragma unroll
    for (int ib = 0; ib < NB; ++ib) {
        const bool qvalid = 32 * ib + l32 < L;
        bf16x8 qf[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8 *)&trow[(32 * ib + l32) * TLD + hq * DH + 16 * ks + 8 * half];
        f32x16 s[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[jb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {        // key fragments straight from the parked tile: nothing to keep across blocks
                const bf16x8 kf = *(const bf16x8 *)&trow[(32 * jb + l32) * TLD + 2 * DH + 16 * ks + 8 * half];
                s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[jb], 0, 0, 0);
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int key = 32 * jb + 8 * (e >> 2) + 4 * half + (e & 3);
                const float x = key < L ? s[jb][e] * sc : -INFINITY;
                s[jb][e] = x;
                mx = fmaxf(mx, x);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        float sum = 0.f;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) { const float p = exp2f(s[jb][e] - mx); s[jb][e] = p; sum += p; }
        sum += __shfl_xor(sum, 32);
        const float inv = qvalid ? 1.0f / sum : 0.f;              // padded query columns contribute nothing
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) csum[jb][e] += s[jb][e] * inv;
    }
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            csum[jb][e] = sum_over_lanes32(csum[jb][e]);
        }
    if (l32 == 0) {
        const float invL = 1.0f / (float)L;
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) pbar_s[32 * jb + 8 * (e >> 2) + 4 * half + (e & 3)] = csum[jb][e] * invL;
    }
    __syncthreads();

    // abar[c] = sum_j pbar[j] V[j][c]: a lane weights 8 components of its rows, then the row groups are added up
    constexpr int CPR = DH / 8;                  // 16-byte pieces per V row
    constexpr int RPI = 64 / CPR;                // rows per instruction
    constexpr int NVI = 32 / RPI;
    const int vrow0 = lane / CPR, vpiece = lane % CPR;
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int i = 0; i < NVI; ++i) {
            const int row = 32 * jb + RPI * i + vrow0;
            const float pj = row < L ? pbar_s[row] : 0.f;
            const u32x4 vv = *(const u32x4 *)&trow[row * TLD + 3 * DH + 8 * vpiece];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                o[2 * w] = fmaf(pj, __uint_as_float(vv[w] << 16), o[2 * w]);
                o[2 * w + 1] = fmaf(pj, __uint_as_float(vv[w] & 0xffff0000u), o[2 * w + 1]);
            }
        }
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int off = CPR; off < 64; off <<= 1) o[c] += __shfl_xor(o[c], off);
    if (live_wave && tok < a.T && lane < CPR) {
        u32x4 pk;
#pragma unroll
        for (int w = 0; w < 4; ++w) pk[w] = pack_bf16x2(o[2 * w], o[2 * w + 1]);
        *(u32x4 *)(a.abar + tok * (int64_t)a.Hq * DH + (int64_t)(g * G + 2 * part + hq) * DH + 8 * lane) = pk;
    }
}

template <int DH, int NB, int TT>
__global__ __launch_bounds__(512) void k_lsa_fused(LsaFusedArgs a)
{
    using Gm = LsaFusedGeom<DH, NB, TT>;
    constexpr int FW = Gm::FW, RB = Gm::RB, BK = Gm::BK, XS = Gm::XS;
    constexpr int WFB = FW / 32;                 // 32-feature blocks per wavefront
    constexpr int NRB = RB / 32;                 // 32-row blocks
    constexpr int NWI = FW / 8;                  // weight-tile load instructions per wavefront (8 rows of 128 B each)
    constexpr int NXI = (RB / 8 + 7) / 8;        // activation-tile load instructions per wavefront
    constexpr int XD = XS - 1;                   // activation tiles requested ahead
    extern __shared__ __attribute__((aligned(16))) bf16_t sm[];

    if ((int)blockIdx.x < a.lead_blocks) {       // the first workgroups of the grid carry work of other calls
        if ((int)blockIdx.x < a.small_lead) {
            if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
                step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)sm, (int32_t *)sm + MOA_MAX_TREE);
        } else {
            const int blk = 2 * ((int)blockIdx.x - a.small_lead) + (int)(threadIdx.x >> 8);
            if (blk < a.red_blocks) splitk_reduce_block(a.red, blk, (int)(threadIdx.x & 255));
        }
        return;
    }
    // Workgroups are dealt round-robin to the 8 XCDs, each with its own L2: an XCD keeps the weight slices of its
    // units (2 MB each at the Llama-3-8B shape) and every token tile's activations pass through it once.
    const int bx = (int)blockIdx.x - a.lead_blocks;
    const int xcd = bx & 7, slot = bx >> 3;
    const int unit = xcd * a.units_per_xcd + slot % a.units_per_xcd;
    const int64_t tile = slot / a.units_per_xcd;
    if (unit >= a.units) return;                 // the whole workgroup leaves before any barrier
    const int g = unit / a.parts, part = unit - g * a.parts;
    const int G = a.Hq / a.Hkv, L = a.L, K = a.d_in;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int lrow = lane >> 3, lpos = lane & 7;

    f32x16 acc[WFB][NRB];
#pragma unroll
    for (int i = 0; i < WFB; ++i)
#pragma unroll
        for (int j = 0; j < NRB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int nk = K / BK;                       // >= 2 (checked on the host)

    // this wavefront's FW feature rows of the weight tile: inside one of Wq (two heads), Wk, Wv
    const int which = wave * FW / DH;
    const bf16_t *wm = which < 2 ? a.wq + (int64_t)((g * G + 2 * part + which) * DH + wave * FW % DH) * K
                                 : (which == 2 ? a.wk : a.wv) + (int64_t)(g * DH + wave * FW % DH) * K;
    const bf16_t *wsrc[NWI];
#pragma unroll
    for (int i = 0; i < NWI; ++i) {
        const int row = 8 * i + lrow;
        wsrc[i] = wm + (int64_t)row * K + 8 * (lpos ^ ((row >> 1) & 7));
    }
    // its share of the activation tile: instruction xi covers tile rows 8 xi .. 8 xi + 7 (a row past the tokens or the
    // layers repeats a valid one; such rows are masked as keys and dropped as queries)
    const bf16_t *xsrc[NXI];
    int xrow0[NXI];
#pragma unroll
    for (int n = 0; n < NXI; ++n) {
        int xi = wave + 8 * n;
        if (xi > RB / 8 - 1) xi = RB / 8 - 1;    // a spare instruction repeats the last one (same bytes to the same place)
        xrow0[n] = 8 * xi;
        const int s = 8 * xi + lrow;
        int64_t tok = tile * TT + s / (32 * NB);
        int lay = s % (32 * NB);
        if (tok > a.T - 1) tok = a.T - 1;
        if (lay > L - 1) lay = L - 1;
        xsrc[n] = a.hs + (tok * L + lay) * (int64_t)K + 8 * (lpos ^ ((s >> 1) & 7));
    }
    bf16_t *wl = sm + (size_t)wave * 2 * FW * BK;                 // this wavefront's ring: [2][FW][BK]
    bf16_t *xl = sm + (size_t)8 * 2 * FW * BK;                    // [XS][RB][BK]
    auto issue_w = [&](int kt) {
        bf16_t *dst = wl + (kt & 1) * FW * BK;
#pragma unroll
        for (int i = 0; i < NWI; ++i)
            __builtin_amdgcn_global_load_lds((global_void_t *)(wsrc[i] + (int64_t)kt * BK), (lds_void_t *)(dst + 8 * i * BK), 16, 0, 0);
    };
    auto issue_x = [&](int kt) {
        bf16_t *dst = xl + (kt % XS) * RB * BK;
#pragma unroll
        for (int n = 0; n < NXI; ++n)
            __builtin_amdgcn_global_load_lds((global_void_t *)(xsrc[n] + (int64_t)kt * BK), (lds_void_t *)(dst + xrow0[n] * BK), 16, 0, 0);
    };

    // Requests are issued in the order X(0) W(0) X(1) W(1) (W(0) X(0) W(1) with a two-stage activation ring), then per
    // tile kt: X(kt+XD) W(kt+2), and complete in that order (all of them go straight to LDS).  At the top of tile kt,
    // X(kt) and W(kt) must have landed; what was requested after the later of the two is X(kt+1) W(kt+1) (only
    // W(kt+1) with the two-stage ring), and nothing in the last round.
    if (XD >= 2) issue_x(0);
    issue_w(0);
    issue_x(XD >= 2 ? 1 : 0);
    issue_w(1);
    constexpr int PENDING = XD >= 2 ? NXI + NWI : NWI;
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) asm volatile("s_waitcnt vmcnt(%0)\n\ts_barrier" ::"n"(PENDING) : "memory");
        else asm volatile("s_waitcnt vmcnt(0)\n\ts_barrier" ::: "memory");
        const bf16_t *wb = wl + (kt & 1) * FW * BK;
        const bf16_t *xb = xl + (kt % XS) * RB * BK;
        // The four k-steps of a tile are software-pipelined: the fragments of step ks+1 are requested from LDS before
        // the MFMAs of step ks are issued, so LDS reads and matrix work of one wavefront overlap.  Once the last
        // step's fragments have been read, the ring places this tile occupied are free and are refilled.
        auto read_frags = [&](int ks, bf16x8 (&fa)[WFB], bf16x8 (&fb)[NRB]) {
#pragma unroll
            for (int i = 0; i < WFB; ++i) {
                const int row = 32 * i + l32;
                fa[i] = *(const bf16x8 *)&wb[row * BK + 8 * ((2 * ks + half) ^ ((row >> 1) & 7))];
            }
#pragma unroll
            for (int j = 0; j < NRB; ++j) {
                const int row = 32 * j + l32;
                fb[j] = *(const bf16x8 *)&xb[row * BK + 8 * ((2 * ks + half) ^ ((row >> 1) & 7))];
            }
        };
        bf16x8 af[2][WFB], bfr[2][NRB];
        read_frags(0, af[0], bfr[0]);
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            if (ks + 1 < BK / 16) read_frags(ks + 1, af[(ks + 1) & 1], bfr[(ks + 1) & 1]);
            if (ks == BK / 16 - 1) {
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                if (kt + XD < nk) issue_x(kt + XD);
                if (kt + 2 < nk) issue_w(kt + 2);
            }
#pragma unroll
            for (int i = 0; i < WFB; ++i)
#pragma unroll
                for (int j = 0; j < NRB; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
        }
    }

    lsa_fused_epilogue<DH, NB, TT>(acc, a, sm, tile, g, part);
}

// f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{}): a loop whose index is a constant
// expression in the body (register arrays indexed by it stay in registers)
template <int... I, typename F>
__device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_impl(std::make_integer_sequence<int, N>{}, f);
}

// Helper workgroup `h` of `a.pf_lead` (packed form).  A cold weight tile is first touched by all of an XCD's
// workgroups at once (they walk the k tiles in step), so all of them wait for HBM together, tile after tile; from the
// L2 they do not.  At decode sizes the kernel's own workgroups leave sixteen compute units idle: two helpers per XCD
// read that XCD's units' packed weights once, tile by tile and in turn, ahead of the workgroups that multiply them,
// and throw them away.  (One compute unit pulls about 50 GB/s of misses however many requests it keeps in flight, so
// sixteen helpers move 0.8 TB/s: the 16 MiB of weights in the kernel's first half.  Reading further operands of the
// step's later launches ahead in the same way -- caches, output-projection weights, here or from the compute units
// the attention cores leave idle -- was measured too: what the later launches gained, the carrying launch lost.)
template <int DH, int NB, int TT>
__device__ __forceinline__ void lsa_warm_block(const LsaFusedArgs &a, int h, bf16_t *sm)
{
    constexpr int NWP = 4 * (LsaFusedGeom<DH, NB, TT>::FW / 32);
    static_assert(NWP * 64 == 512, "one piece per thread and (wavefront, k tile) block");
    const int tid = threadIdx.x, nk = a.d_in / 64;
    const int xcd = h & 7, turn = h >> 3, turns = a.pf_lead >> 3;
    u32x4 acc = {0u, 0u, 0u, 0u};
    for (int uu = 0; uu < a.units_per_xcd; ++uu) {
        const int unit = xcd * a.units_per_xcd + uu;
        if (unit >= a.units) break;
        // [unit][wavefront][k tile] blocks of NWP * 64 pieces: one piece per thread and block
        const u32x4 *base = (const u32x4 *)a.wpk + (int64_t)unit * 8 * nk * (NWP * 64) + tid;
        for (int kt = 2 * turn; kt < nk; kt += 2 * turns) {          // two tiles per round: sixteen requests in flight
            const int kt1 = kt + 1 < nk ? kt + 1 : kt;
            u32x4 v[16];
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                v[w] = base[(int64_t)(w * nk + kt) * (NWP * 64)];
                v[8 + w] = base[(int64_t)(w * nk + kt1) * (NWP * 64)];
            }
#pragma unroll
            for (int w = 0; w < 16; ++w) acc ^= v[w];
        }
    }
    ((u32x4 *)sm)[tid] = acc;                    // into LDS nobody reads: what keeps the loads from being dropped
}

// The same kernel for weights that the caller has packed once into MFMA-operand order (k_lsa_pack_weights).  A
// wavefront's slice of the weight tile is used by that wavefront alone, so with the operands already in lane order it
// has no business in LDS: every 16-byte operand piece is loaded straight into the register that the MFMA reads, 1 KB
// contiguous per instruction.  That takes the weight tile (8/9 of the bytes) out of the LDS traffic -- reads and
// writes of the unpacked form add up to the LDS bandwidth of the whole tile time -- and lets WS - 1 whole tiles be in
// flight per wavefront in registers, which the 160 KB of LDS could not hold.  The activation tile goes through
// registers into a two-stage LDS ring (one bare barrier per tile); all loads are ordinary loads, so the waits are the
// compiler's.  Same MFMA order along d_in as the unpacked form: same bits.
template <int DH, int NB, int TT, int WS, bool SPREAD>
__device__ __forceinline__ void lsa_fused_pk_body(const LsaFusedArgs &a)
{
    using Gm = LsaFusedGeom<DH, NB, TT>;
    constexpr int FW = Gm::FW, RB = Gm::RB, BK = Gm::BK;
    constexpr int WFB = FW / 32;                 // 32-feature blocks per wavefront
    constexpr int NRB = RB / 32;                 // 32-row blocks
    constexpr int NWP = 4 * WFB;                 // operand pieces per lane and weight tile
    constexpr int NXI = (RB / 8 + 7) / 8;        // activation-tile load instructions per wavefront
    extern __shared__ __attribute__((aligned(16))) bf16_t sm[];

    if ((int)blockIdx.x < a.lead_blocks) {       // the first workgroups of the grid carry work of other calls
        if ((int)blockIdx.x >= a.lead_blocks - a.pf_lead) {
            lsa_warm_block<DH, NB, TT>(a, (int)blockIdx.x - (a.lead_blocks - a.pf_lead), sm);
            return;
        }
        if ((int)blockIdx.x < a.small_lead) {
            if ((int)blockIdx.x < a.rider_units && threadIdx.x < 64)
                step_small_unit(a.rider, (int)blockIdx.x, (int32_t *)sm, (int32_t *)sm + MOA_MAX_TREE);
        } else {
            const int blk = 2 * ((int)blockIdx.x - a.small_lead) + (int)(threadIdx.x >> 8);
            if (blk < a.red_blocks) splitk_reduce_block(a.red, blk, (int)(threadIdx.x & 255));
        }
        return;
    }
    const int bx = (int)blockIdx.x - a.lead_blocks;
    const int xcd = bx & 7, slot = bx >> 3;
    const int unit = xcd * a.units_per_xcd + slot % a.units_per_xcd;
    const int64_t tile = slot / a.units_per_xcd;
    if (unit >= a.units) return;                 // the whole workgroup leaves before any barrier
    const int g = unit / a.parts, part = unit - g * a.parts;
    const int L = a.L, K = a.d_in;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, half = lane >> 5;
    const int lrow = lane >> 3, lpos = lane & 7;

    f32x16 acc[WFB][NRB];
#pragma unroll
    for (int i = 0; i < WFB; ++i)
#pragma unroll
        for (int j = 0; j < NRB; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
    const int nk = K / BK;

    // packed weights: [unit][wavefront][k tile][k step][feature block][lane] pieces of 8 elements
    const bf16x8 *wp = (const bf16x8 *)a.wpk + ((int64_t)(unit * 8 + wave) * nk) * (NWP * 64) + lane;
    // activation rows as in the unpacked form: instruction n covers tile rows xrow0[n] .. + 7, the piece a lane fetches
    // is the one whose swizzled place in LDS is the lane's own
    const bf16_t *xsrc[NXI];
    int xrow0[NXI];
#pragma unroll
    for (int n = 0; n < NXI; ++n) {
        int xi = wave + 8 * n;
        if (xi > RB / 8 - 1) xi = RB / 8 - 1;
        xrow0[n] = 8 * xi;
        const int s = 8 * xi + lrow;
        int64_t tok = tile * TT + s / (32 * NB);
        int lay = s % (32 * NB);
        if (tok > a.T - 1) tok = a.T - 1;
        if (lay > L - 1) lay = L - 1;
        xsrc[n] = a.hs + (tok * L + lay) * (int64_t)K + 8 * (lpos ^ ((s >> 1) & 7));
    }
    bf16_t *xl = sm;                             // [2][RB][BK]

    // both operands are requested WS - 1 tiles ahead into register rings (a weight stage is refilled as soon as its
    // tile has been multiplied, an activation stage as soon as it has been copied to LDS)
    bf16x8 wr[WS][NWP];
    bf16x8 xr[WS][NXI];
    auto load_w = [&](int kt, bf16x8 (&dst)[NWP]) {
#pragma unroll
        for (int b = 0; b < NWP; ++b) dst[b] = wp[((int64_t)kt * NWP + b) * 64];
    };
    auto load_x = [&](int kt, bf16x8 (&dst)[NXI]) {
#pragma unroll
        for (int n = 0; n < NXI; ++n) dst[n] = *(const bf16x8 *)(xsrc[n] + (int64_t)kt * BK);
    };
#pragma unroll
    for (int s = 0; s < WS; ++s) {               // a tile past the last repeats the last (nk >= 2)
        if (s < WS - 1) load_x(s < nk ? s : nk - 1, xr[s]);
        load_w(s < nk ? s : nk - 1, wr[s]);
    }

    // One tile step on register stage S.  The activation tile of this step goes to LDS (the place was last read two
    // tiles ago, before the previous barrier) and the one WS - 1 ahead is requested into the registers it leaves.
    // Inside the step the weight requests are spread between the MFMAs: as soon as a k-step's MFMAs have been issued
    // its weight registers are refilled with the same k-step of the tile WS ahead.  Issued in one burst at the top of
    // a step, the requests of all eight wavefronts queue up at the compute unit's one address unit while the matrix
    // cores wait (measured on a cut-down loop: 0.99 us per tile in a burst, 0.78 us spread out).  The scheduling
    // barriers keep the compiler from regrouping them.  No branch surrounds a load: the compiler's load counter then
    // stays exact (partial waits), where a conditional request makes it wait for everything in flight; requests past
    // the last tile repeat the last tile.  GUARDED steps (the few behind the last whole trip) may lie past the last
    // tile and then skip their arithmetic; they refill in one go behind it, and so do the forms without SPREAD (128-row
    // tiles and the lean form: the spread-out order costs registers they do not have).
    auto tile_step = [&](auto stage_c, auto guarded_c, int kt) {
        constexpr int S = decltype(stage_c)::value;
        constexpr bool GUARDED = decltype(guarded_c)::value;
        const bf16_t *xb = xl + (kt & 1) * RB * BK;
        {
            bf16_t *xw = xl + (kt & 1) * RB * BK;
#pragma unroll
            for (int n = 0; n < NXI; ++n) *(bf16x8 *)&xw[xrow0[n] * BK + 8 * lane] = xr[S][n];
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        load_x(kt + WS - 1 < nk ? kt + WS - 1 : nk - 1, xr[(S + WS - 1) % WS]);
        const int kw = kt + WS < nk ? kt + WS : nk - 1;
        const bf16x8 *wnext = wp + (int64_t)kw * NWP * 64;
        auto read_frags = [&](int ks, bf16x8 (&fb)[NRB]) {
#pragma unroll
            for (int j = 0; j < NRB; ++j) {
                const int row = 32 * j + l32;
                fb[j] = *(const bf16x8 *)&xb[row * BK + 8 * ((2 * ks + half) ^ ((row >> 1) & 7))];
            }
        };
        if constexpr (GUARDED || !SPREAD) {
            if (!GUARDED || kt < nk) {
                bf16x8 bfr[2][NRB];
                read_frags(0, bfr[0]);
#pragma unroll
                for (int ks = 0; ks < BK / 16; ++ks) {
                    if (ks + 1 < BK / 16) read_frags(ks + 1, bfr[(ks + 1) & 1]);
#pragma unroll
                    for (int i = 0; i < WFB; ++i)
#pragma unroll
                        for (int j = 0; j < NRB; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[S][ks * WFB + i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
                }
            }
            load_w(kw, wr[S]);
        } else {
            // operand fragments of the next k-step are read ahead where the registers allow (64-row tiles)
            constexpr int NBUF = NRB <= 2 ? 2 : 1;
            bf16x8 bfr[NBUF][NRB];
            read_frags(0, bfr[0]);
#pragma unroll
            for (int ks = 0; ks < BK / 16; ++ks) {
                if (NBUF == 2 && ks + 1 < BK / 16) read_frags(ks + 1, bfr[(ks + 1) & 1]);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < WFB; ++i)
#pragma unroll
                    for (int j = 0; j < NRB; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[S][ks * WFB + i], bfr[ks % NBUF][j], acc[i][j], 0, 0, 0);
                if (NBUF == 1 && ks + 1 < BK / 16) read_frags(ks + 1, bfr[0]);
#pragma unroll
                for (int i = 0; i < WFB; ++i) wr[S][ks * WFB + i] = wnext[(ks * WFB + i) * 64];
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // whole trips of UN steps (at the top of a trip the compiler's wait is a conservative one, so trips are long), then
    // the remaining steps in rounds of WS
    constexpr int UN = Gm::UN;
    static_assert(UN % WS == 0, "a trip of the tile loop is a whole number of register-ring rounds");
    const int nk_main = nk / UN * UN;
#pragma unroll 1
    for (int kt0 = 0; kt0 < nk_main; kt0 += UN)
        static_for<UN>([&](auto u) { tile_step(std::integral_constant<int, decltype(u)::value % WS>{}, std::false_type{}, kt0 + decltype(u)::value); });
    const int nk_end = nk_main + (nk - nk_main + WS - 1) / WS * WS;
#pragma unroll 1
    for (int kt0 = nk_main; kt0 < nk_end; kt0 += WS)
        static_for<WS>([&](auto u) { tile_step(u, std::true_type{}, kt0 + decltype(u)::value); });
    lsa_fused_epilogue<DH, NB, TT>(acc, a, sm, tile, g, part);
}

template <int DH, int NB, int TT>
__global__ __launch_bounds__(512) void k_lsa_fused_pk(LsaFusedArgs a)
{
    lsa_fused_pk_body<DH, NB, TT, LsaFusedGeom<DH, NB, TT>::WS, true>(a);
}

// The same with two register stages and the compiler held to a third of a SIMD's registers per wavefront (168): beside
// a workgroup of this kernel a compute unit still has registers and LDS for a workgroup of the weight-streaming
// projection kernel, so a step that runs its two independent branches on two streams gets them side by side on the same
// compute units.  (64-row tiles only: larger tiles need the registers for their accumulators.)
template <int DH, int NB, int TT>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(3, 3))) void k_lsa_fused_pk_lean(LsaFusedArgs a)
{
    lsa_fused_pk_body<DH, NB, TT, 2, false>(a);
}

// Packs Wq / Wk / Wv for k_lsa_fused_pk: piece (unit, wavefront, k tile, k step, feature block, lane) holds the 8
// elements that lane supplies as the A operand of that MFMA, i.e. row  f(unit, wavefront) + 32 block + lane % 32  of
// the wavefront's matrix at columns  64 tile + 16 step + 8 (lane / 32) ..  One thread per piece.
template <int DH>
__global__ __launch_bounds__(256) void k_lsa_pack_weights(const bf16_t *wq, const bf16_t *wk, const bf16_t *wv, bf16_t *out,
                                                          int d_in, int Hq, int Hkv, int64_t pieces)
{
    constexpr int FW = 4 * DH / 8, WFB = FW / 32;
    const int64_t p = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (p >= pieces) return;
    const int nk = d_in / 64, G = Hq / Hkv, parts = G / 2;
    int64_t r = p;
    const int lane = (int)(r % 64); r /= 64;
    const int i = (int)(r % WFB); r /= WFB;
    const int ks = (int)(r % 4); r /= 4;
    const int kt = (int)(r % nk); r /= nk;
    const int wave = (int)(r % 8); r /= 8;
    const int unit = (int)r;
    const int g = unit / parts, part = unit - g * parts;
    const int which = wave * FW / DH;
    const int frow = wave * FW % DH + 32 * i + (lane & 31);
    const bf16_t *src = which < 2 ? wq + (int64_t)((g * G + 2 * part + which) * DH + frow) * d_in
                                  : (which == 2 ? wk : wv) + (int64_t)(g * DH + frow) * d_in;
    *(u32x4 *)(out + p * 8) = *(const u32x4 *)(src + 64 * kt + 16 * ks + 8 * (lane >> 5));
}

// ------------------------------------------------------------------ host side
bool lsa_fused_ok(int dtype, int L, int d_in, int Hq, int Hkv, int dh, const void *hs, const void *wq, const void *wk,
                  const void *wv, const void *abar)
{
    auto al = [](const void *p) { return p && (((uintptr_t)p) & 15) == 0; };
    if (!lsa_fused_shape_ok(dtype, L, d_in, Hq, Hkv, dh)) return false;
    return al(hs) && al(wq) && al(wk) && al(wv) && al(abar);
}

bool lsa_fused_shape_ok(int dtype, int L, int d_in, int Hq, int Hkv, int dh)
{
    if (dtype != DT_BF16 || dh != 128) return false;
    if (L < 1 || L > 96 || d_in < 128 || d_in % 64) return false;
    if (Hkv < 1 || Hq % Hkv || (Hq / Hkv) % 2) return false;
    return true;
}

// LDS a workgroup may ask for on the current device (looked up once per device; 0 if the query fails)
static size_t lds_limit()
{
    static size_t limit[16] = {};
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return 0;
    if (!limit[dev]) {
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || v <= 0) return 0;
        limit[dev] = (size_t)v;
    }
    return limit[dev];
}

template <int NB, int TT>
static hipError_t launch_lsa_fused_as(LsaFusedArgs &fa, hipStream_t stream, bool lean = false)
{
    using Gm = LsaFusedGeom<128, NB, TT>;
    const int64_t tiles = (fa.T + TT - 1) / TT;
    // Two helper workgroups per XCD (lsa_warm_block), where they cost nothing and can do their job: the kernel's own
    // workgroups leave that many compute units idle (decode sizes), and an XCD's share of the weights fits its L2
    // beside the activations streaming through.  Otherwise they take compute units and L2 from the workgroups they
    // are meant to help (measured: first cycle 536 -> 559 us, d_in 4096 191 -> 197 us with helpers everywhere).
    if (fa.pf_lead) {
        static int cus = 0;
        if (!cus) {
            int dev = 0, n = 0;
            if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) n = 256;
            cus = n;
        }
        const int64_t own = 8 * (int64_t)fa.units_per_xcd * tiles;
        const size_t w_per_xcd = (size_t)fa.units_per_xcd * (size_t)(fa.d_in / 64) * 65536;
        if (lean || own + fa.pf_lead > cus || w_per_xcd > ((size_t)3 << 20)) fa.pf_lead = 0;
        fa.lead_blocks += fa.pf_lead;
    }
    const int64_t grid = fa.lead_blocks + 8 * (int64_t)fa.units_per_xcd * tiles;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    if constexpr (Gm::RB <= 64) {
        if (fa.wpk && lean) {
            static bool raised[16] = {};
            hipError_t e = raise_lds_limit_once(raised, (const void *)k_lsa_fused_pk_lean<128, NB, TT>, Gm::pk_bytes);
            if (e != hipSuccess) return e;
            prof_begin(K_LSA_FUSED_PK_LEAN + 64 * (NB * 8 + TT), stream);
            MOA_KLAUNCH((k_lsa_fused_pk_lean<128, NB, TT>), dim3((unsigned)grid), dim3(512), Gm::pk_bytes, stream, fa);
            prof_end(stream);
            return hipGetLastError();
        }
    }
    if (fa.wpk) {
        static bool raised[16] = {};
        hipError_t e = raise_lds_limit_once(raised, (const void *)k_lsa_fused_pk<128, NB, TT>, Gm::pk_bytes);
        if (e != hipSuccess) return e;
        prof_begin(K_LSA_FUSED_PK + 64 * (NB * 8 + TT), stream);
        MOA_KLAUNCH((k_lsa_fused_pk<128, NB, TT>), dim3((unsigned)grid), dim3(512), Gm::pk_bytes, stream, fa);
    } else {
        static bool raised[16] = {};
        hipError_t e = raise_lds_limit_once(raised, (const void *)k_lsa_fused<128, NB, TT>, Gm::bytes);
        if (e != hipSuccess) return e;
        prof_begin(K_LSA_FUSED + 64 * (NB * 8 + TT), stream);
        MOA_KLAUNCH((k_lsa_fused<128, NB, TT>), dim3((unsigned)grid), dim3(512), Gm::bytes, stream, fa);
    }
    prof_end(stream);
    return hipGetLastError();
}

size_t lsa_packed_weight_bytes(int d_in, int Hq, int Hkv, int dh)
{
    // a workgroup's unit is two query heads with their key and value head: 4 dh rows; a group of more than two query
    // heads repeats its K and V rows in each of its units
    return (size_t)(Hq / 2) * 4 * dh * d_in * sizeof(bf16_t);
}

hipError_t launch_lsa_pack_weights(const void *wq, const void *wk, const void *wv, void *out, int d_in, int Hq, int Hkv,
                                   hipStream_t stream)
{
    const int64_t pieces = (int64_t)(Hq / 2) * 4 * 128 * d_in / 8;
    const int64_t grid = (pieces + 255) / 256;
    if (grid > 0x7fffffff) return hipErrorInvalidValue;
    prof_begin(K_LSA_PACK, stream);
    MOA_KLAUNCH((k_lsa_pack_weights<128>), dim3((unsigned)grid), dim3(256), 0, stream, (const bf16_t *)wq, (const bf16_t *)wk,
                (const bf16_t *)wv, (bf16_t *)out, d_in, Hq, Hkv, pieces);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_lsa_fused(const LsaFusedCall &c, hipStream_t stream)
{
    if (c.T <= 0) return hipSuccess;
    LsaFusedArgs fa = {};
    fa.hs = (const bf16_t *)c.hs;
    fa.wq = (const bf16_t *)c.wq;
    fa.wk = (const bf16_t *)c.wk;
    fa.wv = (const bf16_t *)c.wv;
    fa.wpk = (const bf16_t *)c.w_packed;
    fa.abar = (bf16_t *)c.abar;
    fa.T = c.T;
    fa.L = c.L;
    fa.d_in = c.d_in;
    fa.Hq = c.Hq;
    fa.Hkv = c.Hkv;
    fa.parts = c.Hq / c.Hkv / 2;
    fa.units = c.Hkv * fa.parts;
    fa.units_per_xcd = (fa.units + 7) / 8;
    fa.rider_units = c.rider_units;
    if (c.rider_units > 0) fa.rider = c.rider;
    fa.small_lead = (c.rider_units + 7) & ~7;    // multiples of the XCD count: the unit mapping keeps its phase
    fa.red_blocks = 0;
    if (c.carry_sum && c.carry_sum->blocks > 0) {
        fa.red = *c.carry_sum;
        fa.red_blocks = c.carry_sum->blocks;
    }
    fa.lead_blocks = fa.small_lead + ((((fa.red_blocks + 1) / 2) + 7) & ~7);   // a lead workgroup of 512 threads does two blocks of the pass
    fa.pf_lead = (c.w_packed && !c.leave_room) ? 16 : 0;     // wanted; launch_lsa_fused_as decides when it knows the grid
    // Rows per workgroup.  Measured at the Llama-3-8B shape (d_in 2048), a workgroup takes about 31 + 9 (rows / 32)
    // microseconds from plain weights and 10 + 11.7 (rows / 32) from packed ones, whatever else runs (it is bound by
    // its own chain of tile fetches from the L2 and its matrix work), and the chip runs 256 of them at a time: few
    // tokens want small tiles (every compute unit busy), many tokens large ones (fewer passes over the weights).  Pick
    // the tile that minimises rounds x time per round.
    const int nb = (c.L + 31) / 32;
    const bool big_ok = lds_limit() >= LsaFusedGeom<128, 1, 4>::bytes;      // the 128-row tiles fill the LDS to the last byte
    const double fixed = fa.wpk ? 10.0 : 31.0, per_block = fa.wpk ? 11.7 : 9.0;
    auto cost = [&](int tt) {
        const double wgs = (double)fa.units * (double)((c.T + tt - 1) / tt);
        return ceil(wgs / 256.0) * (fixed + per_block * nb * tt);    // one workgroup per compute unit, all equally long: whole rounds
    };
    // leave_room: another stream's kernels are meant to run beside this launch.  From packed weights that is the
    // 64-row tile in its lean form, which shares a compute unit with them; from plain weights (LDS full either way) the
    // largest tile, which leaves whole compute units empty.
    const bool lean = c.leave_room && fa.wpk;
    if (nb == 1) {
        int best = 2;
        if (!lean) {
            if (cost(3) < cost(best)) best = 3;
            if (big_ok && (cost(4) < cost(best) || c.leave_room)) best = 4;
        }
        if (best == 4) return launch_lsa_fused_as<1, 4>(fa, stream);
        if (best == 3) return launch_lsa_fused_as<1, 3>(fa, stream);
        return launch_lsa_fused_as<1, 2>(fa, stream, lean);
    }
    if (nb == 2) {
        if (!lean && big_ok && (cost(2) < cost(1) || c.leave_room)) return launch_lsa_fused_as<2, 2>(fa, stream);
        return launch_lsa_fused_as<2, 1>(fa, stream, lean);
    }
    return launch_lsa_fused_as<3, 1>(fa, stream);
}

}  // namespace moa
