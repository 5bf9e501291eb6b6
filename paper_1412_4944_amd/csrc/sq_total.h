// Total squared representation error sum_i err[i] (numerator of the RMSE of Section 4) formed
// by `nb` workgroups that ride along in another kernel's launch: workgroup b sums a contiguous
// share in a fixed order, and the one that finishes last adds the shares in index order (it is
// identified by an integer counter, which it sets back to zero; nobody waits for anybody).
// Fixed order, double precision: the result does not depend on scheduling.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbo {

// Every thread of a workgroup of NTH threads calls this for share b of nb (nb <= 256).
// lds: NTH doubles + one int.  sq_counter must be zero when the launch starts.
template <int NTH>
__device__ __forceinline__ void sq_total_part(const float* __restrict__ err, int64_t m, int b, int nb,
                                              double* sq_part, int* sq_counter, double* __restrict__ sq_out,
                                              double* lds) {
    double* red = lds;
    int* is_last = reinterpret_cast<int*>(lds + NTH);
    const int tid = threadIdx.x;
    const int64_t per = (m + nb - 1) / nb;
    const int64_t beg = b * per, end = beg + per < m ? beg + per : m;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;       // four loads in flight per thread
    int64_t i = beg + tid;
    for (; i + 3 * NTH < end; i += 4 * NTH) {
        const float a = err[i], b2 = err[i + NTH], c2 = err[i + 2 * NTH], d2 = err[i + 3 * NTH];
        s0 += (double)a;
        s1 += (double)b2;
        s2 += (double)c2;
        s3 += (double)d2;
    }
    for (; i < end; i += NTH) s0 += (double)err[i];
    red[tid] = (s0 + s1) + (s2 + s3);
    __syncthreads();
    for (int o = NTH / 2; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (tid == 0) {
        __hip_atomic_store(&sq_part[b], red[0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __threadfence();
        *is_last = atomicAdd(sq_counter, 1) == nb - 1;
    }
    __syncthreads();
    if (!*is_last) return;
    __threadfence();
    double t = 0.0;                                      // shares in index order, NTH at a time
    for (int k = tid; k < nb; k += NTH)
        t += __hip_atomic_load(&sq_part[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    red[tid] = t;
    __syncthreads();
    for (int o = NTH / 2; o > 0; o >>= 1) {
        if (tid < o) red[tid] += red[tid + o];
        __syncthreads();
    }
    if (tid == 0) {
        *sq_out = red[0];
        *sq_counter = 0;
    }
}

}  // namespace sbo
