// Batched SVD update Q_j = U V^T (Algorithm 1, steps 6-7) by a one-sided Jacobi SVD, one
// workgroup per block (the routine itself is in jacobi_block.h), and the dispatch between this
// kernel and the Newton-Schulz kernels (launch_polar).  This kernel runs in eigen mode
// (symmetric input, eigenvectors wanted) and for every block when SBO_SVD_JACOBI is set; for the
// blocks on which Newton-Schulz does not converge (rank-deficient or very ill-conditioned P_j)
// the Newton-Schulz kernel calls the same routine itself.
#include "sbo_internal.h"
#include "device_utils.h"
#include "jacobi_block.h"

namespace sbo {

namespace {

template <int P, int TPP>
__global__ __launch_bounds__((P / 2) * TPP) void polar_kernel(const float* __restrict__ M,
                                                             const int32_t* __restrict__ counts,
                                                             float* __restrict__ D,
                                                             float* __restrict__ eig_sv, float done,
                                                             float* __restrict__ dsw,
                                                             unsigned* __restrict__ dsb, int dsb_kind,
                                                             int32_t* __restrict__ sweeps_out,
                                                             const int32_t* __restrict__ only) {
    __shared__ __attribute__((aligned(16))) float lds[jacobi_lds_floats<P>()];
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    if (only != nullptr && only[j] == 0) return;        // uniform: another kernel has done this block
    if (counts != nullptr && counts[j] == 0) {          // uniform: block keeps its basis
        if (sweeps_out != nullptr && tid == 0) sweeps_out[j] = 0;
        return;
    }
    const BlockMatrixSource src = {M + (int64_t)j * P * P, nullptr, 0, 0, P * P};
    jacobi_block<P, TPP>(src, D + (int64_t)j * P * P, eig_sv ? eig_sv + (int64_t)j * P : nullptr, done, dsw,
                         dsb, dsb_kind, j, sweeps_out ? sweeps_out + j : nullptr, lds);
}

}  // namespace

// TPP = 16 lanes per column pair (4 and 8 were measured slower at every p).
static hipError_t launch_jacobi(int p, int K, const float* M, const int32_t* counts, float* D,
                                float* eig_sv, float* dsw, unsigned* dsb, int dsb_kind, int32_t* sweeps,
                                const int32_t* only, hipStream_t st) {
    constexpr int TPP = 16;
    const float done = kPolarDone;
    switch (p) {
        case 16: hipLaunchKernelGGL((polar_kernel<16, TPP>), dim3(K), dim3(8 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, dsb_kind, sweeps, only); break;
        case 32: hipLaunchKernelGGL((polar_kernel<32, TPP>), dim3(K), dim3(16 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, dsb_kind, sweeps, only); break;
        case 64: hipLaunchKernelGGL((polar_kernel<64, TPP>), dim3(K), dim3(32 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, dsb_kind, sweeps, only); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_polar(int p, int K, const float* M, const int32_t* counts, float* D,
                        const Workspace& ws, int jacobi_only, float* eig_sv, int write_ops,
                        hipStream_t st) {
    const bool ns = eig_sv == nullptr && !jacobi_only;
    if (p == 256) {
        if (write_ops) return hipErrorInvalidValue;   // p = 256 rewrites the operand order itself
        if (!ns)
            return launch_polar_wide(K, M, counts, D, ws.vwork, ws.jac_a, eig_sv, ws.sweeps, nullptr,
                                     ws.raised, st);
        hipError_t e = launch_polar_wide_ns(K, M, counts, D, ws.jac_a, ws.ns_fallback, ws.sweeps,
                                            ws.raised, st);
        if (e != hipSuccess) return e;
        return launch_polar_wide(K, M, counts, D, ws.vwork, ws.jac_a, nullptr, ws.sweeps,
                                 ws.ns_fallback, ws.raised, st);
    }
    float* dsw = write_ops == 1 ? ws.dsw : nullptr;
    unsigned* dsb = write_ops >= 2 ? ws.dsb : nullptr;
    if (!ns) return launch_jacobi(p, K, M, counts, D, eig_sv, dsw, dsb, write_ops, ws.sweeps, nullptr, st);
    // Newton-Schulz for every block; a block on which it does not converge gets the Jacobi SVD in
    // the same workgroup.
    return launch_polar_ns(p, K, M, nullptr, nullptr, 0, counts, D, dsw, dsb, write_ops, ws.ns_fallback, ws.sweeps,
                           SqTotalArgs{}, ws.raised, st);
}

hipError_t launch_polar_from_pieces(int p, int K, int64_t m, float* D, const Workspace& ws, int write_ops,
                                    const float* err, double* sq_out, hipStream_t st) {
    if (p > 64) return hipErrorInvalidValue;
    SqTotalArgs sq;
    if (err != nullptr && sq_out != nullptr) {
        sq.err = err;
        sq.m = m;
        sq.part = ws.sq_partial;
        sq.counter = ws.sq_counter;
        sq.out = sq_out;
        sq.nb = 128;                           // <= kSqBlocks shares of err
    }
    return launch_polar_ns(p, K, nullptr, ws.partial, ws.offsets, accum_piece(m, K, p), ws.counts, D,
                           write_ops == 1 ? ws.dsw : nullptr, write_ops >= 2 ? ws.dsb : nullptr, write_ops,
                           ws.ns_fallback, ws.sweeps, sq, ws.raised, st);
}

}  // namespace sbo
