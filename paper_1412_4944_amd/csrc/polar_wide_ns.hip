// Orthogonal polar factor Q_j = U V^T of P_j (Algorithm 1, steps 6-7) for p = 256 by the
// Newton-Schulz iteration X <- X (3 I - X^T X) / 2 (see polar_ns.hip), spread over the whole
// chip: a 256 x 256 matrix does not fit the LDS of a CU, but every product of the iteration
// splits into 64 independent 32 x 32 output tiles per block, so each step is two launches
// (G = X^T X, then the update) over all tiles of all blocks, with X ping-ponging between two
// global buffers (L2-resident: 256 KiB per block).
//
// No launch depends on the host: the deviation d_k = max |X^T X - I| of every step is kept
// per block (integer atomic maximum on the bit pattern of a non-negative float, so the
// result does not depend on the order), and every workgroup derives from that history
// whether its block is still active; workgroups of finished blocks return at once.  A block
// that has not converged within the launched steps is flagged for the Jacobi SVD.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int P = 256;
constexpr int kTiles = P / 32;                 // 8 tiles per side
constexpr int kHist = 32;                      // deviation history entries per block
constexpr float kLast = 2e-4f;                 // below this deviation the step that follows is the last
constexpr float kFail = 4.f;                   // at or above (or NaN): diverging, leave it to the fallback

struct NsScratch {
    float* Xa;        // [K][P][P]
    float* Xb;        // [K][P][P]
    float* G;         // [K][P][P]
    unsigned* dmax;   // [K][kHist] bit patterns of the deviations
    float* s2;        // [K] bound on sigma_max^2 of the input
};
__host__ __device__ inline NsScratch ns_carve(float* base, int K) {
    NsScratch s;
    const size_t pp = (size_t)P * P;
    s.Xa = base;
    s.Xb = base + (size_t)K * pp;
    s.G = base + 2 * (size_t)K * pp;
    s.dmax = reinterpret_cast<unsigned*>(base + 3 * (size_t)K * pp);
    s.s2 = base + 3 * (size_t)K * pp + (size_t)K * kHist;
    return s;
}

// State of block j before step `it` (steps are numbered from 0; step 0 always runs):
// 0 = active, 1 = finished (converged at an earlier step), 2 = failed.
__device__ __forceinline__ int block_state(const NsScratch& ns, int j, int it) {
    const float s2 = ns.s2[j];
    if (it >= 1 && !(s2 > 0.f && s2 < 3e38f)) return 2;
    for (int i = 1; i < it; ++i) {
        const float d = __uint_as_float(ns.dmax[j * kHist + i]);
        if (!(d < kFail)) return 2;
        if (d < kLast) return 1;
    }
    return 0;
}

// G = X^T X for the X before step `it`; for it >= 1 also the deviation of the step.
__global__ __launch_bounds__(256) void wide_ns_gram_kernel(const float* __restrict__ M,
                                                           const int32_t* __restrict__ counts,
                                                           float* scratch, int K, int it) {
    const NsScratch ns = ns_carve(scratch, K);
    const int j = blockIdx.y;
    if (counts != nullptr && counts[j] == 0) return;       // uniform
    const int tid = threadIdx.x;
    if (it == 0) {
        if (blockIdx.x == 0 && tid < kHist) ns.dmax[j * kHist + tid] = 0u;
    } else if (block_state(ns, j, it) != 0) {
        return;                                            // uniform
    }
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;
    // a workgroup owns a 64 x 64 part of G, a wavefront one 32 x 32 tile of it
    const int ta = 2 * (blockIdx.x / (kTiles / 2)) + (wave >> 1);
    const int tb = 2 * (blockIdx.x % (kTiles / 2)) + (wave & 1);
    const float* X = (it == 0 ? M : ((it & 1) ? ns.Xb : ns.Xa)) + (int64_t)j * P * P;

    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    // 32 steps (64 loads) in flight per wavefront: with one wavefront per SIMD the loads are
    // what the kernel waits on
#pragma unroll 1
    for (int s0 = 0; s0 < P / 2; s0 += 32) {
        float a[32], b[32];
#pragma unroll
        for (int u = 0; u < 32; ++u) {
            a[u] = X[(2 * (s0 + u) + h) * P + ta * 32 + n];
            b[u] = X[(2 * (s0 + u) + h) * P + tb * 32 + n];
        }
#pragma unroll
        for (int u = 0; u < 32; ++u) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u], b[u], acc, 0, 0, 0);
    }
    float* Gj = ns.G + (int64_t)j * P * P;
    float dev = 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int row = ta * 32 + (q >> 2) * 8 + h * 4 + (q & 3), col = tb * 32 + n;
        Gj[row * P + col] = acc[q];
        dev = fmaxf(dev, fabsf(acc[q] - (row == col ? 1.f : 0.f)));
    }
    if (it >= 1) {
        if (!(dev == dev)) dev = __uint_as_float(0x7f800000u);   // NaN -> +inf keeps the maximum monotone
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) dev = fmaxf(dev, __shfl_xor(dev, o, 64));
        if (lane == 0) atomicMax(&ns.dmax[j * kHist + it], __float_as_uint(dev));
    }
}

// s2[j] ~ sigma_max^2 of the input = largest eigenvalue of G: Rayleigh quotient after a few
// power-iteration steps from the vector of absolute row sums, times 1.08 (see polar_ns.hip;
// G is symmetric, so rows are read as columns, coalesced).
__global__ __launch_bounds__(256) void wide_ns_scale_kernel(const int32_t* __restrict__ counts,
                                                            float* scratch, int K) {
    __shared__ float vec[P], wec[P];
    const NsScratch ns = ns_carve(scratch, K);
    const int j = blockIdx.x;
    if (counts != nullptr && counts[j] == 0) return;
    const int tid = threadIdx.x;
    const float* Gj = ns.G + (int64_t)j * P * P;
    float rs = 0.f;
    for (int b = 0; b < P; ++b) rs += fabsf(Gj[b * P + tid]);
    vec[tid] = rs;
    __syncthreads();
    float s2 = 0.f;
    for (int round = 0; round < 4; ++round) {
        float w = 0.f;
        for (int b = 0; b < P; ++b) w += Gj[b * P + tid] * vec[b];
        wec[tid] = w;
        __syncthreads();
        float vv = 0.f, vw = 0.f, wmax = 0.f;  // every thread, same order: same values
        for (int a = 0; a < P; ++a) {
            vv += vec[a] * vec[a];
            vw += vec[a] * wec[a];
            wmax = fmaxf(wmax, fabsf(wec[a]));
        }
        s2 = 1.08f * vw / vv;                  // NaN for a zero matrix: the update kernel checks
        __syncthreads();
        vec[tid] = wec[tid] / wmax;
        __syncthreads();
    }
    if (tid == 0) ns.s2[j] = s2;
}

// Step `it`: X_out = c1 X_in - c2 X_in G (c1 = 3/2, c2 = 1/2; step 0 folds the scaling in).
__global__ __launch_bounds__(256) void wide_ns_update_kernel(const float* __restrict__ M,
                                                             const int32_t* __restrict__ counts,
                                                             float* scratch, int K, int it) {
    const NsScratch ns = ns_carve(scratch, K);
    const int j = blockIdx.y;
    if (counts != nullptr && counts[j] == 0) return;       // uniform
    if (block_state(ns, j, it) != 0) return;               // uniform
    float c1 = 1.5f, c2 = 0.5f;
    if (it == 0) {
        const float s2 = ns.s2[j];
        if (!(s2 > 0.f && s2 < 3e38f)) return;             // uniform: zero, infinite or NaN input
        const float inv = __builtin_amdgcn_rsqf(s2);
        c1 = 1.5f * inv;
        c2 = 0.5f * inv * inv * inv;
    } else {
        const float d = __uint_as_float(ns.dmax[j * kHist + it]);
        if (!(d < kFail)) return;                          // uniform: diverging
    }
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;
    const int tr = 2 * (blockIdx.x / (kTiles / 2)) + (wave >> 1);
    const int tb = 2 * (blockIdx.x % (kTiles / 2)) + (wave & 1);
    const float* Xin = (it == 0 ? M : ((it & 1) ? ns.Xb : ns.Xa)) + (int64_t)j * P * P;
    float* Xout = ((it & 1) ? ns.Xa : ns.Xb) + (int64_t)j * P * P;
    const float* Gj = ns.G + (int64_t)j * P * P;

    // tile (tr, tb) of X G: rows r = tr*32 + n of X (16 bytes of a row feed two steps),
    // contraction over a, columns tb*32 + n of G
    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    const f32x4* xrow = reinterpret_cast<const f32x4*>(Xin + (tr * 32 + n) * P);
#pragma unroll 1
    for (int q0 = 0; q0 < P / 4; q0 += 16) {
        f32x4 v[16];
        float b0[16], b1[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            v[u] = xrow[q0 + u];
            b0[u] = Gj[(4 * (q0 + u) + h) * P + tb * 32 + n];
            b1[u] = Gj[(4 * (q0 + u) + 2 + h) * P + tb * 32 + n];
        }
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? v[u].y : v[u].x, b0[u], acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? v[u].w : v[u].z, b1[u], acc, 0, 0, 0);
        }
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int row = tr * 32 + (q >> 2) * 8 + h * 4 + (q & 3), col = tb * 32 + n;
        Xout[row * P + col] = c1 * Xin[row * P + col] - c2 * acc[q];
    }
}

// Converged blocks: D[j] = X; every block: fallback flag and step count.
__global__ __launch_bounds__(256) void wide_ns_finish_kernel(const int32_t* __restrict__ counts,
                                                             float* __restrict__ D, float* scratch,
                                                             int K, int steps_launched,
                                                             int32_t* __restrict__ fallback,
                                                             int32_t* __restrict__ iters_out) {
    const NsScratch ns = ns_carve(scratch, K);
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    if (counts != nullptr && counts[j] == 0) {             // uniform: block keeps its basis
        if (tid == 0) {
            fallback[j] = 0;
            if (iters_out != nullptr) iters_out[j] = 0;
        }
        return;
    }
    // the step whose deviation was below kLast is the last one that ran
    int n_steps = 0;
    const float s2 = ns.s2[j];
    if (s2 > 0.f && s2 < 3e38f) {
        for (int i = 1; i < steps_launched; ++i) {
            const float d = __uint_as_float(ns.dmax[j * kHist + i]);
            if (!(d < kFail)) break;
            if (d < kLast) {
                n_steps = i + 1;
                break;
            }
        }
    }
    if (tid == 0) {
        fallback[j] = n_steps == 0;
        if (iters_out != nullptr) iters_out[j] = -n_steps;
    }
    if (n_steps == 0) return;                              // uniform
    const f32x4* X = reinterpret_cast<const f32x4*>(((n_steps & 1) ? ns.Xb : ns.Xa) + (int64_t)j * P * P);
    f32x4* Dj = reinterpret_cast<f32x4*>(D + (int64_t)j * P * P);
    for (int e = tid; e < P * P / 4; e += 256) Dj[e] = X[e];
}

}  // namespace

size_t polar_wide_ns_scratch_bytes(int K) {
    return (3 * (size_t)K * P * P + (size_t)K * kHist + (size_t)K) * sizeof(float);
}

// Newton-Schulz for all K blocks; fallback[j] = 1 for every block left to the Jacobi SVD.
hipError_t launch_polar_wide_ns(int K, const float* M, const int32_t* counts, float* D, float* scratch,
                                int32_t* fallback, int32_t* iters, hipStream_t st) {
    constexpr int kSteps = 20;                 // < kHist
    const dim3 grid((kTiles / 2) * (kTiles / 2), K);
    for (int it = 0; it < kSteps; ++it) {
        hipLaunchKernelGGL(wide_ns_gram_kernel, grid, dim3(256), 0, st, M, counts, scratch, K, it);
        if (it == 0) hipLaunchKernelGGL(wide_ns_scale_kernel, dim3(K), dim3(256), 0, st, counts, scratch, K);
        hipLaunchKernelGGL(wide_ns_update_kernel, grid, dim3(256), 0, st, M, counts, scratch, K, it);
    }
    hipLaunchKernelGGL(wide_ns_finish_kernel, dim3(K), dim3(256), 0, st, counts, D, scratch, K, kSteps,
                       fallback, iters);
    return hipGetLastError();
}

}  // namespace sbo
