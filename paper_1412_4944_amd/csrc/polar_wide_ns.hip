// Orthogonal polar factor Q_j = U V^T of P_j (Algorithm 1, steps 6-7) for p = 256 by the
// Newton-Schulz iteration X <- X (3 I - X^T X) / 2 (see polar_ns.hip), spread over the whole
// chip: a 256 x 256 matrix does not fit the LDS of a CU, but every product of the iteration
// splits into 64 independent 32 x 32 output tiles per block, so each step is two launches
// (G = X^T X, then the update) over all tiles of all blocks, with X ping-ponging between two
// global buffers (L2-resident: 256 KiB per block); a workgroup computes a 64 x 64 part of the
// result from two operand panels that it first copies into LDS.
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

constexpr int kPanelLd = 64 + 4;               // leading dimension of a 256 x 64 panel in LDS
constexpr int kRowLd = P + 4;                  // leading dimension of a 64 x 256 panel in LDS

// Copies of operand panels into LDS: every thread issues all its 16-byte loads before the
// first store, so a workgroup has its whole 64 KiB panel in flight at once (with one wavefront
// per SIMD, loads issued a few at a time next to the MFMAs were what these kernels waited on).
// cols: src[r][c0 .. c0+63], r < 256  ->  dst[r][0..63]
__device__ __forceinline__ void load_col_panel(const float* __restrict__ src, int c0, float* dst,
                                               int tid) {
    f32x4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = tid + 256 * u;           // 4096 units of 16 bytes: row e / 16, unit e % 16
        v[u] = *reinterpret_cast<const f32x4*>(src + (e >> 4) * P + c0 + 4 * (e & 15));
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = tid + 256 * u;
        *reinterpret_cast<f32x4*>(dst + (e >> 4) * kPanelLd + 4 * (e & 15)) = v[u];
    }
}
// rows: src[r0 .. r0+63][c], c < 256  ->  dst[0..63][c]
__device__ __forceinline__ void load_row_panel(const float* __restrict__ src, int r0, float* dst,
                                               int tid) {
    f32x4 v[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = tid + 256 * u;           // row e / 64, unit e % 64
        v[u] = *reinterpret_cast<const f32x4*>(src + (r0 + (e >> 6)) * P + 4 * (e & 63));
    }
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        const int e = tid + 256 * u;
        *reinterpret_cast<f32x4*>(dst + (e >> 6) * kRowLd + 4 * (e & 63)) = v[u];
    }
}

// G = X^T X for the X before step `it`; for it >= 1 also the deviation of the step.
// A workgroup owns a 64 x 64 part of G (a wavefront one 32 x 32 tile of it) and stages the two
// 256 x 64 column panels of X it needs in LDS.
__global__ __launch_bounds__(256) void wide_ns_gram_kernel(const float* __restrict__ M,
                                                           const int32_t* __restrict__ counts,
                                                           float* scratch, int K, int it) {
    extern __shared__ float panels[];          // [2][256][kPanelLd]
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
    const int sa = blockIdx.x / (kTiles / 2), sb = blockIdx.x % (kTiles / 2);
    const int ta = 2 * sa + (wave >> 1), tb = 2 * sb + (wave & 1);
    const float* X = (it == 0 ? M : ((it & 1) ? ns.Xb : ns.Xa)) + (int64_t)j * P * P;

    float* pa = panels;
    float* pb = sa == sb ? panels : panels + P * kPanelLd;
    load_col_panel(X, 64 * sa, pa, tid);
    if (sa != sb) load_col_panel(X, 64 * sb, pb, tid);     // uniform
    __syncthreads();

    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    const float* ca = pa + (wave >> 1) * 32 + n;
    const float* cb = pb + (wave & 1) * 32 + n;
#pragma unroll 16
    for (int s = 0; s < P / 2; ++s)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(ca[(2 * s + h) * kPanelLd], cb[(2 * s + h) * kPanelLd],
                                                   acc, 0, 0, 0);
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

// s2[j] = the scale of the input: the larger of 1.08 x a Rayleigh quotient after a few
// power-iteration steps from the vector of absolute row sums (a usually tight lower estimate of
// the largest eigenvalue of G = sigma_max^2) and the largest absolute row sum / 2.9 (a guaranteed
// upper bound / 2.9, which keeps every scaled sigma^2 below 3: see polar_ns.hip; G is symmetric,
// so rows are read as columns, coalesced).
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
    float rsmax = 0.f;                         // every thread, same order: same value
    for (int a = 0; a < P; ++a) rsmax = fmaxf(rsmax, vec[a]);
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
    // a zero, infinite or NaN quotient stays that way (the update kernel then leaves the block
    // to the fallback); otherwise the guaranteed bound applies
    if (s2 > 0.f && s2 < 3e38f) s2 = fmaxf(s2, rsmax * (1.f / 2.9f));
    if (tid == 0) ns.s2[j] = s2;
}

// Step `it`: X_out = c1 X_in - c2 X_in G (c1 = 3/2, c2 = 1/2; step 0 folds the scaling in).
// A workgroup owns a 64 x 64 part of X_out and stages the 64 x 256 row panel of X_in and the
// 256 x 64 column panel of G in LDS.
__global__ __launch_bounds__(256) void wide_ns_update_kernel(const float* __restrict__ M,
                                                             const int32_t* __restrict__ counts,
                                                             float* scratch, int K, int it) {
    extern __shared__ float panels[];          // xrows[64][kRowLd] | gcols[256][kPanelLd]
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
    const int sr = blockIdx.x / (kTiles / 2), sb = blockIdx.x % (kTiles / 2);
    const float* Xin = (it == 0 ? M : ((it & 1) ? ns.Xb : ns.Xa)) + (int64_t)j * P * P;
    float* Xout = ((it & 1) ? ns.Xa : ns.Xb) + (int64_t)j * P * P;
    const float* Gj = ns.G + (int64_t)j * P * P;

    float* xrows = panels;
    float* gcols = panels + 64 * kRowLd;
    load_row_panel(Xin, 64 * sr, xrows, tid);
    load_col_panel(Gj, 64 * sb, gcols, tid);
    __syncthreads();

    // tile of X G: rows (wave>>1)*32 + n of the row panel (16 bytes of a row feed two steps),
    // contraction over a, columns (wave&1)*32 + n of the column panel
    f32x16 acc;
#pragma unroll
    for (int q = 0; q < 16; ++q) acc[q] = 0.f;
    const f32x4* xrow = reinterpret_cast<const f32x4*>(xrows + ((wave >> 1) * 32 + n) * kRowLd);
    const float* gc = gcols + (wave & 1) * 32 + n;
#pragma unroll 8
    for (int q = 0; q < P / 4; ++q) {
        const f32x4 v = xrow[q];
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? v.y : v.x, gc[(4 * q + h) * kPanelLd], acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? v.w : v.z, gc[(4 * q + 2 + h) * kPanelLd], acc, 0, 0, 0);
    }
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int lr = (wave >> 1) * 32 + (q >> 2) * 8 + h * 4 + (q & 3), lc = (wave & 1) * 32 + n;
        Xout[(64 * sr + lr) * P + 64 * sb + lc] = c1 * xrows[lr * kRowLd + 64 * sb + lc] - c2 * acc[q];
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
                                int32_t* fallback, int32_t* iters, LdsRaised* raised, hipStream_t st) {
    constexpr int kSteps = 20;                 // < kHist
    const size_t lds_gram = (size_t)2 * P * kPanelLd * sizeof(float);
    const size_t lds_upd = ((size_t)64 * kRowLd + (size_t)P * kPanelLd) * sizeof(float);
    if (raised == nullptr) return hipErrorInvalidValue;
    hipError_t e = raised->ensure(reinterpret_cast<const void*>(&wide_ns_gram_kernel), lds_gram);
    if (e == hipSuccess) e = raised->ensure(reinterpret_cast<const void*>(&wide_ns_update_kernel), lds_upd);
    if (e != hipSuccess) return e;
    const dim3 grid((kTiles / 2) * (kTiles / 2), K);
    for (int it = 0; it < kSteps; ++it) {
        hipLaunchKernelGGL(wide_ns_gram_kernel, grid, dim3(256), lds_gram, st, M, counts, scratch, K, it);
        if (it == 0) hipLaunchKernelGGL(wide_ns_scale_kernel, dim3(K), dim3(256), 0, st, counts, scratch, K);
        hipLaunchKernelGGL(wide_ns_update_kernel, grid, dim3(256), lds_upd, st, M, counts, scratch, K, it);
    }
    hipLaunchKernelGGL(wide_ns_finish_kernel, dim3(K), dim3(256), 0, st, counts, D, scratch, K, kSteps,
                       fallback, iters);
    return hipGetLastError();
}

}  // namespace sbo
