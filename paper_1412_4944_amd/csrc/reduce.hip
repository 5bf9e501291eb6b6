// Total squared representation error sum_i err_i of one coding pass (numerator of the
// RMSE of Section 4), as a fixed-order two-level sum in double precision.
#include "sbo_internal.h"

namespace sbo {

namespace {

__global__ __launch_bounds__(256) void sq_partial_kernel(const float* __restrict__ err, int64_t m,
                                                         double* __restrict__ part) {
    __shared__ double red[256];
    double s = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < m; i += (int64_t)gridDim.x * 256)
        s += (double)err[i];
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

}  // namespace

hipError_t launch_sqerr(const float* err, int64_t m, const Workspace& ws, double* out,
                        hipStream_t st) {
    hipLaunchKernelGGL(sq_partial_kernel, dim3(kSqBlocks), dim3(256), 0, st, err, m, ws.sq_partial);
    hipLaunchKernelGGL(sq_final_kernel, dim3(1), dim3(256), 0, st, ws.sq_partial, kSqBlocks, out);
    return hipGetLastError();
}

}  // namespace sbo
