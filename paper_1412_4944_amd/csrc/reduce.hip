// Total squared representation error sum_i err_i of one coding pass (numerator of the
// RMSE of Section 4), as a fixed-order two-level sum in double precision.
#include "sbo_internal.h"

namespace sbo {

namespace {

// ids == nullptr: all m entries; otherwise the m entries err[ids[0..m)]
__global__ __launch_bounds__(256) void sq_partial_kernel(const float* __restrict__ err,
                                                         const int32_t* __restrict__ ids, int64_t m,
                                                         double* __restrict__ part) {
    __shared__ double red[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < m; i += (int64_t)gridDim.x * 256)
        s += (double)err[ids ? ids[i] : i];
    red[threadIdx.x] = s;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) part[blockIdx.x] = red[0];
}

__global__ __launch_bounds__(256) void sq_final_kernel(const double* __restrict__ part, int n,
                                                       double* __restrict__ out) {
    __shared__ double red[256];
    red[threadIdx.x] = (int)threadIdx.x < n ? part[threadIdx.x] : 0.0;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = red[0];
}


__global__ __launch_bounds__(256) void single_block_kernel(const int32_t* __restrict__ ids, int32_t n,
                                                           int32_t m, int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets) {
    const int q = blockIdx.x * 256 + threadIdx.x;
    if (q < n) perm[q] = min(max(ids[q], 0), m - 1);
    if (q == 0) {
        counts[0] = n;
        offsets[0] = 0;
        offsets[1] = n;
    }
}

}  // namespace

// A signal set as one block for the grouped kernels: perm = the ids (clamped to valid
// signal indices, so that a bad id cannot become a bad address), counts = {n}, offsets = {0, n}.
hipError_t launch_single_block(const int32_t* ids, int64_t n, int64_t m, const Workspace& ws,
                               hipStream_t st) {
    hipLaunchKernelGGL(single_block_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, ids,
                       (int32_t)n, (int32_t)m, ws.perm, ws.counts, ws.offsets);
    return hipGetLastError();
}

namespace {

__global__ __launch_bounds__(256) void equal_blocks_kernel(const int32_t* __restrict__ ids, int32_t n_blocks,
                                                           int32_t per_block, int32_t m,
                                                           int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ counts,
                                                           int32_t* __restrict__ offsets) {
    const int64_t q = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (q < (int64_t)n_blocks * per_block) perm[q] = min(max(ids[q], 0), m - 1);
    if (q < n_blocks) counts[q] = per_block;
    if (q <= n_blocks) offsets[q] = (int32_t)(q * per_block);
}

}  // namespace

// n_blocks signal sets of per_block signals each (ids[n_blocks][per_block]) as the grouping of
// n_blocks blocks: perm = the ids (clamped), counts[j] = per_block, offsets[j] = j * per_block.
hipError_t launch_equal_blocks(const int32_t* ids, int n_blocks, int64_t per_block, int64_t m,
                               const Workspace& ws, hipStream_t st) {
    const int64_t n = (int64_t)n_blocks * per_block;
    const int64_t threads = n > n_blocks + 1 ? n : n_blocks + 1;   // offsets has n_blocks + 1 entries
    hipLaunchKernelGGL(equal_blocks_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, ids,
                       n_blocks, (int32_t)per_block, (int32_t)m, ws.perm, ws.counts, ws.offsets);
    return hipGetLastError();
}


// Sum of err over all m signals (ids == nullptr) or over the m listed signals.
hipError_t launch_sqerr(const float* err, const int32_t* ids, int64_t m, const Workspace& ws,
                        double* out, hipStream_t st) {
    hipLaunchKernelGGL(sq_partial_kernel, dim3(kSqBlocks), dim3(256), 0, st, err, ids, m,
                       ws.sq_partial);
    hipLaunchKernelGGL(sq_final_kernel, dim3(1), dim3(256), 0, st, ws.sq_partial, kSqBlocks, out);
    return hipGetLastError();
}

}  // namespace sbo
