// Client-server messages (Sec. 4.2; appendix table of message lengths): the draft tree as 4 bytes per node, the
// server's answer as 3 bytes per accepted token plus its activations quantised to 8 bits per value.
// Byte work of a few KB to a few hundred KB: one launch each, every byte written by a vector store of the
// thread that owns it.  All quantiser arithmetic is single precision in the order the header states, so codes
// are a pure function of the inputs.
#include "moa_common.h"
#include "../../include/moa.h"

namespace moa {

__global__ __launch_bounds__(256) void k_msg_pack_tree(const int32_t *__restrict__ tok, const int32_t *__restrict__ parent,
                                                       int64_t n, uint32_t *__restrict__ msg, int32_t *dev_status)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const int32_t t = tok[i], p = parent[i];
    if ((t < 0 || t >= (1 << 24) || p < -1 || p >= 255) && dev_status) atomicOr(dev_status, MOA_DEV_BAD_MESSAGE);
    msg[i] = ((uint32_t)t & 0xffffffu) | ((p < 0 ? 0xffu : (uint32_t)p & 0xffu) << 24);      // little-endian: id, then position
}

__global__ __launch_bounds__(256) void k_msg_unpack_tree(const uint32_t *__restrict__ msg, int64_t n, int32_t *__restrict__ tok,
                                                         int32_t *__restrict__ parent)
{
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n) return;
    const uint32_t w = msg[i];
    tok[i] = (int32_t)(w & 0xffffffu);
    parent[i] = (w >> 24) == 0xffu ? -1 : (int32_t)(w >> 24);
}

// one workgroup per (token, vector); token 0's workgroup of a token also writes the 3-byte id
template <typename T>
__global__ __launch_bounds__(256) void k_msg_pack_accept(const int32_t *__restrict__ tok, const T *__restrict__ x, int n_vec, int n,
                                                         uint8_t *__restrict__ msg, int32_t *dev_status)
{
    __shared__ float part[4];
    const int a = blockIdx.x / n_vec, v = blockIdx.x - a * n_vec, t = threadIdx.x;
    const int64_t per = 3 + (int64_t)n_vec * (4 + n);
    uint8_t *m = msg + a * per;
    const T *xv = x + ((int64_t)a * n_vec + v) * n;
    float amax = 0.f;
    for (int c = t; c < n; c += 256) amax = fmaxf(amax, fabsf(ld<T>(xv + c)));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) amax = fmaxf(amax, __shfl_xor(amax, o));
    if ((t & 63) == 0) part[t >> 6] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(part[0], part[1]), fmaxf(part[2], part[3]));
    const float scale = amax / 127.0f;
    uint8_t *mv = m + 3 + (int64_t)v * (4 + n);
    if (t < 4) mv[t] = (uint8_t)(__float_as_uint(scale) >> (8 * t));
    if (v == 0 && t >= 4 && t < 7) {
        const int32_t id = tok[a];
        if (t == 4 && (id < 0 || id >= (1 << 24)) && dev_status) atomicOr(dev_status, MOA_DEV_BAD_MESSAGE);
        m[t - 4] = (uint8_t)((uint32_t)id >> (8 * (t - 4)));
    }
    for (int c = t; c < n; c += 256) {
        float q = scale > 0.f ? rintf(ld<T>(xv + c) / scale) : 0.f;
        q = fminf(fmaxf(q, -127.f), 127.f);
        mv[4 + c] = (uint8_t)(int8_t)q;
    }
}

__global__ __launch_bounds__(256) void k_msg_unpack_accept(const uint8_t *__restrict__ msg, int n_vec, int n, int32_t *__restrict__ tok,
                                                           float *__restrict__ x)
{
    const int a = blockIdx.x / n_vec, v = blockIdx.x - a * n_vec, t = threadIdx.x;
    const int64_t per = 3 + (int64_t)n_vec * (4 + n);
    const uint8_t *m = msg + a * per;
    const uint8_t *mv = m + 3 + (int64_t)v * (4 + n);
    const float scale = __uint_as_float((uint32_t)mv[0] | ((uint32_t)mv[1] << 8) | ((uint32_t)mv[2] << 16) | ((uint32_t)mv[3] << 24));
    if (v == 0 && t == 0) tok[a] = (int32_t)m[0] | ((int32_t)m[1] << 8) | ((int32_t)m[2] << 16);
    float *xv = x + ((int64_t)a * n_vec + v) * n;
    for (int c = t; c < n; c += 256) xv[c] = (float)(int8_t)mv[4 + c] * scale;
}

}  // namespace moa

using namespace moa;

extern "C" {

int32_t moa_msg_pack_tree(const int32_t *tok, const int32_t *parent, int32_t B, int32_t M, void *msg, int32_t *dev_status,
                          void *stream)
{
    if (!tok || !parent || !msg) return api_fail(MOA_ERR_NULL, "msg_pack_tree: NULL pointer");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE) return api_fail(MOA_ERR_SHAPE, "msg_pack_tree: B >= 1, 1 <= M <= 256");
    if (((uintptr_t)msg) & 3) return api_fail(MOA_ERR_SHAPE, "msg_pack_tree: msg must be 4-byte aligned");
    const int64_t n = (int64_t)B * M;
    prof_set_site(S_MSG);
    prof_begin(K_MSG_TREE, (hipStream_t)stream);
    MOA_KLAUNCH(k_msg_pack_tree, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, tok, parent, n, (uint32_t *)msg, dev_status);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : api_fail(MOA_ERR_HIP, "msg_pack_tree: launch failed");
}

int32_t moa_msg_unpack_tree(const void *msg, int32_t B, int32_t M, int32_t *tok, int32_t *parent, void *stream)
{
    if (!tok || !parent || !msg) return api_fail(MOA_ERR_NULL, "msg_unpack_tree: NULL pointer");
    if (B < 1 || M < 1 || M > MOA_MAX_TREE) return api_fail(MOA_ERR_SHAPE, "msg_unpack_tree: B >= 1, 1 <= M <= 256");
    if (((uintptr_t)msg) & 3) return api_fail(MOA_ERR_SHAPE, "msg_unpack_tree: msg must be 4-byte aligned");
    const int64_t n = (int64_t)B * M;
    prof_set_site(S_MSG);
    prof_begin(K_MSG_TREE, (hipStream_t)stream);
    MOA_KLAUNCH(k_msg_unpack_tree, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, (hipStream_t)stream, (const uint32_t *)msg, n, tok, parent);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : api_fail(MOA_ERR_HIP, "msg_unpack_tree: launch failed");
}

int32_t moa_msg_accept_bytes(int32_t A, int32_t n_vec, int32_t n, size_t *bytes_host)
{
    if (!bytes_host) return api_fail(MOA_ERR_NULL, "msg_accept_bytes: bytes_host is NULL");
    if (A < 0 || n_vec < 0 || n < 1) return api_fail(MOA_ERR_SHAPE, "msg_accept_bytes: A >= 0, n_vec >= 0, n >= 1");
    *bytes_host = (size_t)A * (3 + (size_t)n_vec * (4 + (size_t)n));
    return MOA_OK;
}

int32_t moa_msg_pack_accept(int32_t dtype, const int32_t *tok, const void *x, int32_t A, int32_t n_vec, int32_t n, void *msg,
                            int32_t *dev_status, void *stream)
{
    if (!tok || !x || !msg) return api_fail(MOA_ERR_NULL, "msg_pack_accept: NULL pointer");
    if (dtype != MOA_F32 && dtype != MOA_BF16) return api_fail(MOA_ERR_DTYPE, "msg_pack_accept: dtype");
    if (A < 0 || n_vec < 1 || n < 1) return api_fail(MOA_ERR_SHAPE, "msg_pack_accept: A >= 0, n_vec >= 1, n >= 1");
    if (A == 0) return MOA_OK;
    prof_set_site(S_MSG);
    prof_begin(K_MSG_ACCEPT, (hipStream_t)stream);
    const dim3 grid((unsigned)((int64_t)A * n_vec));
    if (dtype == MOA_BF16) MOA_KLAUNCH(k_msg_pack_accept<bf16_t>, grid, dim3(256), 0, (hipStream_t)stream, tok, (const bf16_t *)x, n_vec, n, (uint8_t *)msg, dev_status);
    else MOA_KLAUNCH(k_msg_pack_accept<float>, grid, dim3(256), 0, (hipStream_t)stream, tok, (const float *)x, n_vec, n, (uint8_t *)msg, dev_status);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : api_fail(MOA_ERR_HIP, "msg_pack_accept: launch failed");
}

int32_t moa_msg_unpack_accept(const void *msg, int32_t A, int32_t n_vec, int32_t n, int32_t *tok, float *x, void *stream)
{
    if (!tok || !x || !msg) return api_fail(MOA_ERR_NULL, "msg_unpack_accept: NULL pointer");
    if (A < 0 || n_vec < 1 || n < 1) return api_fail(MOA_ERR_SHAPE, "msg_unpack_accept: A >= 0, n_vec >= 1, n >= 1");
    if (A == 0) return MOA_OK;
    prof_set_site(S_MSG);
    prof_begin(K_MSG_ACCEPT, (hipStream_t)stream);
    MOA_KLAUNCH(k_msg_unpack_accept, dim3((unsigned)((int64_t)A * n_vec)), dim3(256), 0, (hipStream_t)stream, (const uint8_t *)msg, n_vec, n, tok, x);
    prof_end((hipStream_t)stream);
    return hipGetLastError() == hipSuccess ? MOA_OK : api_fail(MOA_ERR_HIP, "msg_unpack_accept: launch failed");
}

}  // extern "C"
