// Row-wise pieces of a reused LLM decoder layer (Target Layer Inference, Sec. 3.2): RMS normalisation with the
// residual add folded in, rotary positions for the projected queries / keys of the tree nodes, the gated
// activation of the MLP, and the final residual add.  All are a few hundred KB of traffic at decode sizes:
// launch latency, not bandwidth, is what they cost, so each does as much per launch as the data flow allows.
#include "moa_common.h"

namespace moa {

// h = x (+ res); n = h / sqrt(mean(h^2) + eps) * g.  One workgroup per row; h is kept in fp32 when asked for
// (the residual stream is rounded to the storage type only once, at the end of the layer).
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const T *__restrict__ x, const T *__restrict__ res, int d,
                                                 const T *__restrict__ g, float eps, float *__restrict__ h_out,
                                                 T *__restrict__ n_out)
{
    __shared__ float part[4];
    const int64_t r = blockIdx.x;
    const T *xr = x + r * d;
    const T *rr = res ? res + r * d : nullptr;
    float ss = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) {
        const float v = ld<T>(xr + c) + (rr ? ld<T>(rr + c) : 0.f);
        ss += v * v;
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    for (int c = threadIdx.x; c < d; c += 256) {
        const float v = ld<T>(xr + c) + (rr ? ld<T>(rr + c) : 0.f);
        if (h_out) h_out[r * d + c] = v;
        st<T>(n_out + r * d + c, v * inv * ld<T>(g + c));
    }
}

// bf16 rows of up to 256 * 8 * NCH values (d a multiple of 8, 16-byte aligned rows): every lane requests its
// 16-byte pieces up front and keeps them in registers for both passes.
template <int NCH>
__global__ __launch_bounds__(256) void k_rmsnorm_bf16v(const bf16_t *__restrict__ x, const bf16_t *__restrict__ res, int d,
                                                      const bf16_t *__restrict__ g, float eps, float *__restrict__ h_out,
                                                      bf16_t *__restrict__ n_out)
{
    __shared__ float part[4];
    const int64_t r = blockIdx.x;
    const int nch = d >> 3;
    u32x4 xv[NCH], rv[NCH], gv[NCH];
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const int c = threadIdx.x + 256 * i;
        const int cc = c < nch ? c : 0;
        xv[i] = *(const u32x4 *)(x + r * d + 8 * cc);
        rv[i] = res ? *(const u32x4 *)(res + r * d + 8 * cc) : u32x4{0u, 0u, 0u, 0u};
        gv[i] = *(const u32x4 *)(g + 8 * cc);
    }
    float v[NCH][8];
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
        const bool live = threadIdx.x + 256 * i < nch;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float lo = __uint_as_float(xv[i][e] << 16) + __uint_as_float(rv[i][e] << 16);
            const float hi = __uint_as_float(xv[i][e] & 0xffff0000u) + __uint_as_float(rv[i][e] & 0xffff0000u);
            v[i][2 * e] = lo;
            v[i][2 * e + 1] = hi;
            if (live) ss += lo * lo + hi * hi;
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) ss += __shfl_xor(ss, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = (part[0] + part[1]) + (part[2] + part[3]);
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
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
        *(u32x4 *)(n_out + r * d + 8 * c) = o;
        if (h_out) {
            *(f32x4 *)(h_out + r * d + 8 * c) = f32x4{v[i][0], v[i][1], v[i][2], v[i][3]};
            *(f32x4 *)(h_out + r * d + 8 * c + 4) = f32x4{v[i][4], v[i][5], v[i][6], v[i][7]};
        }
    }
}

// Rotary positions, pairs (c, c + dh/2), angle = pos * theta^(-2c/dh), pos = prefix_len[b] + depth[b][node]:
// the place the drafted token would take in its own sequence.  Queries [B*Mn, H*dh] and the new rows of the
// draft key slabs [B, Hkv, M, dh] in place.  The angle is formed in double precision: at position 32768 a
// single-precision angle is only good to 4e-3 rad, which would be the largest error of the whole layer.
template <typename T>
__global__ __launch_bounds__(256) void k_rope(T *__restrict__ q, T *__restrict__ k_draft, const int32_t *__restrict__ prefix_len,
                                              const int32_t *__restrict__ depth, int B, int Mn, int M, int node0, int H,
                                              int Hkv, int dh, double log_theta, int P_cap)
{
    const int half = dh >> 1;
    const int64_t per_row = (int64_t)(H + Hkv) * half;
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (int64_t)B * Mn * per_row) return;
    const int64_t r = idx / per_row;
    const int e = (int)(idx - r * per_row), hh = e / half, c = e - hh * half;
    const int b = (int)(r / Mn), i = node0 + (int)(r - (int64_t)b * Mn);
    int plen = prefix_len[b];
    plen = plen < 0 ? 0 : (plen > P_cap ? P_cap : plen);           // the attention core flags a bad length
    const double pos = (double)plen + (double)depth[(int64_t)b * M + i];
    const double ang = pos * exp(-2.0 * (double)c / (double)dh * log_theta);
    double sn, cs;
    sincos(ang, &sn, &cs);
    T *v = hh < H ? q + (r * H + hh) * dh : k_draft + (((int64_t)b * Hkv + (hh - H)) * M + i) * dh;
    const float a = ld<T>(v + c), bb = ld<T>(v + c + half);
    st<T>(v + c, (float)((double)a * cs - (double)bb * sn));
    st<T>(v + c + half, (float)((double)bb * cs + (double)a * sn));
}

// act[r, j] = silu(gu[r, j]) * gu[r, d_ff + j]   (gate and up projections side by side in one row)
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const T *__restrict__ gu, int64_t R, int d_ff, T *__restrict__ act)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= R * d_ff) return;
    const int64_t r = idx / d_ff;
    const int j = (int)(idx - r * d_ff);
    const float gt = ld<T>(gu + r * 2 * d_ff + j), up = ld<T>(gu + r * 2 * d_ff + d_ff + j);
    st<T>(act + idx, gt / (1.0f + __expf(-gt)) * up);
}

// out = h (fp32 residual stream) + t
template <typename T>
__global__ __launch_bounds__(256) void k_add_out(const float *__restrict__ h, const T *__restrict__ t, int64_t n, T *__restrict__ out)
{
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (idx < n) st<T>(out + idx, h[idx] + ld<T>(t + idx));
}

// out[n, k] = sum_j a[n, j] b[j, k]: the product of two projection matrices applied one after the other.  Run once
// per pair of weights, so a plain LDS-tiled kernel with fp32 accumulation.
template <typename T>
__global__ __launch_bounds__(256) void k_fold_weights(const T *__restrict__ a, const T *__restrict__ b, int N, int J, int K,
                                                      T *__restrict__ out)
{
    __shared__ float as[16][17], bs[16][17];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int n = blockIdx.y * 16 + ty, k = blockIdx.x * 16 + tx;
    float acc = 0.f;
    for (int j0 = 0; j0 < J; j0 += 16) {
        as[ty][tx] = (n < N && j0 + tx < J) ? ld<T>(a + (int64_t)n * J + j0 + tx) : 0.f;
        bs[ty][tx] = (j0 + ty < J && k < K) ? ld<T>(b + (int64_t)(j0 + ty) * K + k) : 0.f;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < 16; ++j) acc += as[ty][j] * bs[j][tx];
        __syncthreads();
    }
    if (n < N && k < K) st<T>(out + (int64_t)n * K + k, acc);
}

hipError_t launch_fold_weights(int dtype, const void *a, const void *b, int N, int J, int K, void *out, hipStream_t stream)
{
    const dim3 grid((unsigned)((K + 15) / 16), (unsigned)((N + 15) / 16));
    if (dtype == DT_BF16) hipLaunchKernelGGL(k_fold_weights<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t *)a, (const bf16_t *)b, N, J, K, (bf16_t *)out);
    else hipLaunchKernelGGL(k_fold_weights<float>, grid, dim3(256), 0, stream, (const float *)a, (const float *)b, N, J, K, (float *)out);
    return hipGetLastError();
}

hipError_t launch_rmsnorm(int dtype, const void *x, const void *res, int64_t R, int d, const void *g, float eps,
                          float *h_out, void *n_out, hipStream_t stream)
{
    if (R <= 0) return hipSuccess;
    prof_begin(K_RMSNORM, stream);
    const bool vec = dtype == DT_BF16 && d % 8 == 0 && d <= 256 * 8 * 4 &&
                     ((((uintptr_t)x) | ((uintptr_t)res) | ((uintptr_t)g) | ((uintptr_t)n_out) | ((uintptr_t)h_out)) & 15) == 0;
    if (vec && d <= 256 * 8 * 2)
        MOA_KLAUNCH(k_rmsnorm_bf16v<2>, dim3((unsigned)R), dim3(256), 0, stream, (const bf16_t *)x, (const bf16_t *)res, d,
                    (const bf16_t *)g, eps, h_out, (bf16_t *)n_out);
    else if (vec)
        MOA_KLAUNCH(k_rmsnorm_bf16v<4>, dim3((unsigned)R), dim3(256), 0, stream, (const bf16_t *)x, (const bf16_t *)res, d,
                    (const bf16_t *)g, eps, h_out, (bf16_t *)n_out);
    else if (dtype == DT_BF16)
        MOA_KLAUNCH(k_rmsnorm<bf16_t>, dim3((unsigned)R), dim3(256), 0, stream, (const bf16_t *)x, (const bf16_t *)res, d,
                    (const bf16_t *)g, eps, h_out, (bf16_t *)n_out);
    else
        MOA_KLAUNCH(k_rmsnorm<float>, dim3((unsigned)R), dim3(256), 0, stream, (const float *)x, (const float *)res, d,
                    (const float *)g, eps, h_out, (float *)n_out);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_rope(int dtype, void *q, void *k_draft, const int32_t *prefix_len, const int32_t *depth, int B, int Mn,
                       int M, int node0, int H, int Hkv, int dh, double theta, int P_cap, hipStream_t stream)
{
    const int64_t n = (int64_t)B * Mn * (H + Hkv) * (dh / 2);
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256));
    const double lt = log(theta);
    prof_begin(K_ROPE, stream);
    if (dtype == DT_BF16)
        MOA_KLAUNCH(k_rope<bf16_t>, grid, dim3(256), 0, stream, (bf16_t *)q, (bf16_t *)k_draft, prefix_len, depth, B, Mn, M,
                    node0, H, Hkv, dh, lt, P_cap);
    else
        MOA_KLAUNCH(k_rope<float>, grid, dim3(256), 0, stream, (float *)q, (float *)k_draft, prefix_len, depth, B, Mn, M,
                    node0, H, Hkv, dh, lt, P_cap);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_swiglu(int dtype, const void *gu, int64_t R, int d_ff, void *act, hipStream_t stream)
{
    const int64_t n = R * d_ff;
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256));
    prof_begin(K_SWIGLU, stream);
    if (dtype == DT_BF16) MOA_KLAUNCH(k_swiglu<bf16_t>, grid, dim3(256), 0, stream, (const bf16_t *)gu, R, d_ff, (bf16_t *)act);
    else MOA_KLAUNCH(k_swiglu<float>, grid, dim3(256), 0, stream, (const float *)gu, R, d_ff, (float *)act);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_add_out(int dtype, const float *h, const void *t, int64_t n, void *out, hipStream_t stream)
{
    if (n <= 0) return hipSuccess;
    const dim3 grid((unsigned)((n + 255) / 256));
    prof_begin(K_ADD_OUT, stream);
    if (dtype == DT_BF16) MOA_KLAUNCH(k_add_out<bf16_t>, grid, dim3(256), 0, stream, h, (const bf16_t *)t, n, (bf16_t *)out);
    else MOA_KLAUNCH(k_add_out<float>, grid, dim3(256), 0, stream, h, (const float *)t, n, (float *)out);
    prof_end(stream);
    return hipGetLastError();
}

}  // namespace moa
