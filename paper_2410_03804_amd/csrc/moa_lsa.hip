// Layer Self-Attention core (paper Sec. 3.1.1): for one token and one head, full attention over the
// L layer rows, with the mean aggregation folded in:
//     mean_i ( sum_j P[i][j] V[j] ) = sum_j ( (1/L) sum_i P[i][j] ) V[j]
// so only the column means of the L x L probability matrix are applied to V, and the output
// projection runs afterwards on one row per token instead of L (both are exact identities).
//
//   k_lsa_attn       any dtype / size: one workgroup per (token, head), Q/K rows and the L x L scores in
//                    LDS, fp32 FMA.
//   k_lsa_attn_mfma  bf16, head_dim 64/128, L <= 96: one wavefront per (token, head).  Scores are computed
//                    transposed (S^T = K Q^T, MFMA 32x32x16 fed straight from global memory: both
//                    operands are head_dim-contiguous rows), so a lane owns one query column: the row
//                    softmax is an in-register reduction plus one exchange with lane^32, and the column
//                    means are a 32-lane butterfly.  The L means then weight the V rows with plain
//                    vector loads (HBM/L2-bound part, no matrix shape left).
#include "moa_common.h"

#include <math.h>

namespace moa {

template <typename T>
__global__ __launch_bounds__(256) void k_lsa_attn(LsaAttnArgs a)
{
    extern __shared__ float smem[];
    const int L = a.L, dh = a.dh, ldr = dh + 1, lds = L + 1;
    float *Qs = smem;                 // [L][dh+1]
    float *Ks = Qs + (size_t)L * ldr; // [L][dh+1]
    float *S = Ks + (size_t)L * ldr;  // [L][L+1]
    float *pbar = S + (size_t)L * lds;

    const int tid = threadIdx.x;
    const int64_t t = blockIdx.x / a.Hq;
    const int h = blockIdx.x % a.Hq, g = h / (a.Hq / a.Hkv);
    const T *q = (const T *)a.q + t * L * a.ldq + (int64_t)h * dh;
    const T *k = (const T *)a.k + t * L * a.ldk + (int64_t)g * dh;
    const T *v = (const T *)a.v + t * L * a.ldv + (int64_t)g * dh;
    const float scale = 1.0f / sqrtf((float)dh);

    for (int idx = tid; idx < L * dh; idx += 256) {
        const int l = idx / dh, c = idx - l * dh;
        Qs[l * ldr + c] = ld<T>(q + (int64_t)l * a.ldq + c);
        Ks[l * ldr + c] = ld<T>(k + (int64_t)l * a.ldk + c);
    }
    __syncthreads();
    for (int idx = tid; idx < L * L; idx += 256) {
        const int i = idx / L, j = idx - i * L;
        float d = 0.f;
        for (int c = 0; c < dh; ++c) d = fmaf(Qs[i * ldr + c], Ks[j * ldr + c], d);
        S[i * lds + j] = d * scale;
    }
    __syncthreads();
    for (int i = tid; i < L; i += 256) {     // row softmax, full mask over the layer axis
        float mx = -INFINITY;
        for (int j = 0; j < L; ++j) mx = fmaxf(mx, S[i * lds + j]);
        float sum = 0.f;
        for (int j = 0; j < L; ++j) { const float e = expf(S[i * lds + j] - mx); S[i * lds + j] = e; sum += e; }
        const float inv = 1.0f / sum;
        for (int j = 0; j < L; ++j) S[i * lds + j] *= inv;
    }
    __syncthreads();
    for (int j = tid; j < L; j += 256) {     // column means = the mean aggregation over layers
        float s = 0.f;
        for (int i = 0; i < L; ++i) s += S[i * lds + j];
        pbar[j] = s / (float)L;
    }
    __syncthreads();
    T *o = (T *)a.abar + t * (int64_t)a.Hq * dh + (int64_t)h * dh;
    for (int c = tid; c < dh; c += 256) {
        float acc = 0.f;
        for (int j = 0; j < L; ++j) acc = fmaf(pbar[j], ld<T>(v + (int64_t)j * a.ldv + c), acc);
        st<T>(o + c, acc);
    }
}

// ------------------------------------------------------------------ MFMA, one wavefront per (token, head)
template <int DH, int NB>   // NB = ceil(L / 32) blocks of 32 layers
__global__ __launch_bounds__(256) void k_lsa_attn_mfma(LsaAttnArgs a)
{
    constexpr int NKS = DH / 16;
    __shared__ float pbar_s[4][32 * NB];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, l32 = lane & 31, half = lane >> 5;
    const int64_t unit = (int64_t)blockIdx.x * 4 + wave;       // (token, head)
    const bool live = unit < a.T * a.Hq;
    const int64_t u = live ? unit : a.T * a.Hq - 1;             // idle waves redo the last unit, store nothing
    const int64_t t = u / a.Hq;
    const int h = (int)(u - t * a.Hq), g = h / (a.Hq / a.Hkv);
    const int L = a.L;
    const bf16_t *q = (const bf16_t *)a.q + t * L * a.ldq + (int64_t)h * DH;
    const bf16_t *k = (const bf16_t *)a.k + t * L * a.ldk + (int64_t)g * DH;
    const bf16_t *v = (const bf16_t *)a.v + t * L * a.ldv + (int64_t)g * DH;
    const float sc = 1.4426950408889634f / sqrtf((float)DH);    // log2 domain

    // K fragments (A operand): row = key layer, 8 head_dim values per lane; rows past L repeat row L-1
    bf16x8 kf[NB][NKS];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb) {
        int row = 32 * jb + l32;
        if (row > L - 1) row = L - 1;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) kf[jb][ks] = *(const bf16x8 *)(k + (int64_t)row * a.ldk + 16 * ks + 8 * half);
    }

    // V rows, requested now so that they arrive behind the score computation: 16 lanes cover one 256-byte
    // row piece (8 head_dim values per lane), instruction i of block jb holds row 32 jb + 4 i + lane / 16
    constexpr int CPR = DH / 8;            // 16-byte pieces per V row
    constexpr int RPI = 64 / CPR;          // rows per load instruction
    constexpr int NVI = 32 / RPI;          // load instructions per block of 32 rows
    const int vrow0 = lane / CPR, vpiece = lane % CPR;
    u32x4 vreg[NB][NVI];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int i = 0; i < NVI; ++i) {
            int row = 32 * jb + RPI * i + vrow0;
            if (row > L - 1) row = L - 1;      // weight 0 below
            vreg[jb][i] = *(const u32x4 *)(v + (int64_t)row * a.ldv + 8 * vpiece);
        }

    // column sums of P, kept in the S^T register layout: csum[jb][v] belongs to key 32 jb + 8 (v/4) + 4 half + v%4
    float csum[NB][16];
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int e = 0; e < 16; ++e) csum[jb][e] = 0.f;

#pragma unroll
    for (int ib = 0; ib < NB; ++ib) {
        int qrow = 32 * ib + l32;
        const bool qvalid = qrow < L;
        if (qrow > L - 1) qrow = L - 1;
        bf16x8 qf[NKS];
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) qf[ks] = *(const bf16x8 *)(q + (int64_t)qrow * a.ldq + 16 * ks + 8 * half);
        f32x16 s[NB];
#pragma unroll
        for (int jb = 0; jb < NB; ++jb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) s[jb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
                s[jb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[jb][ks], qf[ks], s[jb], 0, 0, 0);
        }
        // softmax over the keys of this lane's query
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
        const float inv = qvalid ? 1.0f / sum : 0.f;      // padded query columns contribute nothing
#pragma unroll
        for (int jb = 0; jb < NB; ++jb)
#pragma unroll
            for (int e = 0; e < 16; ++e) csum[jb][e] += s[jb][e] * inv;
    }

    // sum over the 32 query lanes of each half, then publish the L column means
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
            for (int e = 0; e < 16; ++e) pbar_s[wave][32 * jb + 8 * (e >> 2) + 4 * half + (e & 3)] = csum[jb][e] * invL;
    }
    __syncthreads();

    // abar[c] = sum_j pbar[j] V[j][c]: each lane weights its rows' 8 components, then the RPI row groups of
    // the wavefront are added up (lanes that differ in lane / CPR)
    float o[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) o[c] = 0.f;
#pragma unroll
    for (int jb = 0; jb < NB; ++jb)
#pragma unroll
        for (int i = 0; i < NVI; ++i) {
            const int row = 32 * jb + RPI * i + vrow0;
            const float pj = row < L ? pbar_s[wave][row] : 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t x = vreg[jb][i][w];
                o[2 * w] = fmaf(pj, __uint_as_float(x << 16), o[2 * w]);
                o[2 * w + 1] = fmaf(pj, __uint_as_float(x & 0xffff0000u), o[2 * w + 1]);
            }
        }
#pragma unroll
    for (int c = 0; c < 8; ++c)
#pragma unroll
        for (int off = CPR; off < 64; off <<= 1) o[c] += __shfl_xor(o[c], off);
    if (live && lane < CPR) {
        u32x4 pk;
#pragma unroll
        for (int w = 0; w < 4; ++w) pk[w] = pack_bf16x2(o[2 * w], o[2 * w + 1]);
        *(u32x4 *)((bf16_t *)a.abar + t * (int64_t)a.Hq * DH + (int64_t)h * DH + 8 * lane) = pk;
    }
}

constexpr size_t LSA_MAX_LDS = 150 * 1024;   // what the host-side argument check admits

size_t lsa_attn_lds_bytes(int /*dtype*/, int L, int dh)
{
    return sizeof(float) * ((size_t)2 * L * (dh + 1) + (size_t)L * (L + 1) + L);
}

static bool lsa_mfma_ok(const LsaAttnArgs &a)
{
    auto al = [](const void *p) { return (((uintptr_t)p) & 15) == 0; };
    return a.dtype == DT_BF16 && (a.dh == 64 || a.dh == 128) && a.L <= 96 && al(a.q) && al(a.k) && al(a.v) &&
           al(a.abar) && a.ldq % 8 == 0 && a.ldk % 8 == 0 && a.ldv % 8 == 0;
}

hipError_t launch_lsa_attn(const LsaAttnArgs &a, hipStream_t stream)
{
    if (a.T <= 0) return hipSuccess;
    if (lsa_mfma_ok(a)) {
        const dim3 grid((unsigned)((a.T * a.Hq + 3) / 4));
        const int nb = (a.L + 31) / 32;
        prof_begin(K_LSA_ATTN_MFMA + 64 * (a.dh * 8 + nb), stream);
#define MOA_LSA_CASE(DH, NBV) MOA_KLAUNCH((k_lsa_attn_mfma<DH, NBV>), grid, dim3(256), 0, stream, a)
        if (a.dh == 128) { if (nb == 1) MOA_LSA_CASE(128, 1); else if (nb == 2) MOA_LSA_CASE(128, 2); else MOA_LSA_CASE(128, 3); }
        else { if (nb == 1) MOA_LSA_CASE(64, 1); else if (nb == 2) MOA_LSA_CASE(64, 2); else MOA_LSA_CASE(64, 3); }
#undef MOA_LSA_CASE
        prof_end(stream);
        return hipGetLastError();
    }
    const size_t lds = lsa_attn_lds_bytes(a.dtype, a.L, a.dh);
    if (lds > LSA_MAX_LDS) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(a.T * a.Hq));
    hipError_t e;
    static bool raised[2][16] = {};          // the limit is raised once, to the most any accepted call needs
    if (a.dtype == DT_BF16) {
        e = raise_lds_limit_once(raised[0], (const void *)k_lsa_attn<bf16_t>, LSA_MAX_LDS);
        if (e != hipSuccess) return e;
        { prof_begin(K_LSA_ATTN, stream); MOA_KLAUNCH(k_lsa_attn<bf16_t>, grid, dim3(256), lds, stream, a); prof_end(stream); }
    } else {
        e = raise_lds_limit_once(raised[1], (const void *)k_lsa_attn<float>, LSA_MAX_LDS);
        if (e != hipSuccess) return e;
        { prof_begin(K_LSA_ATTN, stream); MOA_KLAUNCH(k_lsa_attn<float>, grid, dim3(256), lds, stream, a); prof_end(stream); }
    }
    return hipGetLastError();
}

}  // namespace moa
