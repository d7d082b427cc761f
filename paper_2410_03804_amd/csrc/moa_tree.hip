// Draft-tree integer kernels: ancestor bitsets + depths, greedy accept walk, cache length update.
// One 64-lane wavefront per sequence; a mask row is at most 4 x 64-bit words (M <= 256).
#include "moa_common.h"
#include "moa_tree_device.h"
#include "../../include/moa.h"

namespace moa {

__global__ __launch_bounds__(64) void k_tree_build(const int32_t *__restrict__ parent, int M,
                                                   uint64_t *__restrict__ mask, int32_t *__restrict__ depth,
                                                   int32_t *dev_status)
{
    __shared__ int32_t par[MOA_MAX_TREE];
    tree_build_block(blockIdx.x, parent, M, mask, depth, dev_status, par);
}

__global__ __launch_bounds__(64) void k_tree_accept(const int32_t *__restrict__ parent,
                                                    const int32_t *__restrict__ tok,
                                                    const int32_t *__restrict__ tgt, int M,
                                                    int32_t *__restrict__ path, int32_t *__restrict__ n_path,
                                                    int32_t *__restrict__ bonus)
{
    __shared__ int32_t par[MOA_MAX_TREE], tk[MOA_MAX_TREE];
    tree_accept_block(blockIdx.x, parent, tok, tgt, M, path, n_path, bonus, par, tk);
}

__global__ void k_append_lengths(const int32_t *__restrict__ tok_off, int B, int32_t *ca_len, int cap,
                                 int32_t *dev_status)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < B) append_length_one(b, tok_off, ca_len, cap, nullptr, dev_status);
}

// The three integer pieces of a step in one launch (one unit per 64-lane workgroup)
__global__ __launch_bounds__(64) void k_step_small(StepSmallArgs a)
{
    __shared__ int32_t par[MOA_MAX_TREE], tk[MOA_MAX_TREE];
    step_small_unit(a, blockIdx.x, par, tk);
}

hipError_t launch_tree_build(const int32_t *parent, int B, int M, uint64_t *mask, int32_t *depth,
                             int32_t *dev_status, hipStream_t stream)
{
    { prof_begin(K_TREE_BUILD, stream); MOA_KLAUNCH(k_tree_build, dim3(B), dim3(64), 0, stream, parent, M, mask, depth, dev_status); prof_end(stream); }
    return hipGetLastError();
}

hipError_t launch_tree_accept(const int32_t *parent, const int32_t *tok, const int32_t *tgt, int B, int M,
                              int32_t *path, int32_t *n_path, int32_t *bonus, hipStream_t stream)
{
    { prof_begin(K_TREE_ACCEPT, stream); MOA_KLAUNCH(k_tree_accept, dim3(B), dim3(64), 0, stream, parent, tok, tgt, M, path, n_path, bonus); prof_end(stream); }
    return hipGetLastError();
}

hipError_t launch_step_small(const StepSmallArgs &a, hipStream_t stream)
{
    prof_begin(K_STEP_SMALL, stream);
    MOA_KLAUNCH(k_step_small, dim3(2 * a.B + 1), dim3(64), 0, stream, a);
    prof_end(stream);
    return hipGetLastError();
}

hipError_t launch_append_lengths(const int32_t *tok_off, int B, int32_t *ca_len, int cap, int32_t *dev_status,
                                 hipStream_t stream)
{
    { prof_begin(K_APPEND_LEN, stream); MOA_KLAUNCH(k_append_lengths, dim3((B + 63) / 64), dim3(64), 0, stream, tok_off, B, ca_len, cap,
                       dev_status); prof_end(stream); }
    return hipGetLastError();
}

}  // namespace moa
