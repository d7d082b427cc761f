// Layer Self-Attention core (paper Sec. 3.1.1): for one token and one head, full attention over the
// L layer rows, with the mean aggregation folded in:
//     mean_i ( sum_j P[i][j] V[j] ) = sum_j ( (1/L) sum_i P[i][j] ) V[j]
// so only the column means of the L x L probability matrix are applied to V, and the output
// projection runs afterwards on one row per token instead of L (both are exact identities).
// One workgroup per (token, head); the token's Q and K rows of that head are staged in LDS,
// the L x L scores live in LDS, softmax is fp32.
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

size_t lsa_attn_lds_bytes(int /*dtype*/, int L, int dh)
{
    return sizeof(float) * ((size_t)2 * L * (dh + 1) + (size_t)L * (L + 1) + L);
}

hipError_t launch_lsa_attn(const LsaAttnArgs &a, hipStream_t stream)
{
    if (a.T <= 0) return hipSuccess;
    const size_t lds = lsa_attn_lds_bytes(a.dtype, a.L, a.dh);
    const dim3 grid((unsigned)(a.T * a.Hq));
    hipError_t e;
    if (a.dtype == DT_BF16) {
        e = hipFuncSetAttribute((const void *)k_lsa_attn<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        { prof_begin(K_LSA_ATTN, stream); hipLaunchKernelGGL(k_lsa_attn<bf16_t>, grid, dim3(256), lds, stream, a); prof_end(stream); }
    } else {
        e = hipFuncSetAttribute((const void *)k_lsa_attn<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        { prof_begin(K_LSA_ATTN, stream); hipLaunchKernelGGL(k_lsa_attn<float>, grid, dim3(256), lds, stream, a); prof_end(stream); }
    }
    return hipGetLastError();
}

}  // namespace moa
