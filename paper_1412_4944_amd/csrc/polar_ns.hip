// Orthogonal polar factor Q_j = U V^T of P_j (Algorithm 1, steps 6-7) for p <= 64 by the
// Newton-Schulz iteration X <- X (3 I - X^T X) / 2 on the matrix cores.
//
// U V^T is the orthogonal polar factor of P_j, and for a matrix scaled to singular values in
// (0, 1] the iteration converges to it quadratically; each step is two p x p x p products,
// which are dense contractions (fp32 MFMA), where the Jacobi SVD is p - 1 dependent rounds
// of plain ALU work per sweep.  The block matrices P_j = Y_j X_j^T of this method are well
// conditioned (condition numbers of 3 to 60 on the benchmark workloads), so 8 to 15 steps
// reach fp32 accuracy (|Q - Q_exact| of a few 1e-7; still 4e-6 at a condition number of 3000).
// A block that has not converged after max_iters steps (rank-deficient or nearly so) is left
// untouched and flagged; the Jacobi SVD kernel then handles exactly the flagged blocks,
// including the orthonormal completion that a vanishing singular value needs.
//
// The stored matrix is atom-major (the transpose of P_j); the polar factor of the transpose is
// the transpose of the polar factor, so iterating on the stored matrix yields D[j] directly.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

template <int P>
__global__ __launch_bounds__(P == 64 ? 256 : 64) void polar_ns_kernel(
    const float* __restrict__ M, const int32_t* __restrict__ counts, float* __restrict__ D,
    float* __restrict__ dsw, int32_t* __restrict__ fallback, int32_t* __restrict__ iters_out,
    int max_iters) {
    constexpr int T = P == 64 ? 2 : 1;         // 32-wide tiles per side
    constexpr int NTH = T * T * 64;
    constexpr int PAD = T * 32;                // padded dimension (p = 16 sits in one tile)
    constexpr int LD = PAD + 1;
    __shared__ float X[PAD * LD];
    __shared__ float G[PAD * LD];
    __shared__ float red[8];

    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;
    const int ta = wave / T, tb = wave % T;    // this wavefront's output tile
    if (counts != nullptr && counts[j] == 0) { // uniform: block keeps its basis
        if (tid == 0) {
            fallback[j] = 0;
            if (iters_out != nullptr) iters_out[j] = 0;
        }
        return;
    }

    const float* Mj = M + (int64_t)j * P * P;
    for (int e = tid; e < PAD * LD; e += NTH) {
        const int r = e / LD, c = e % LD;
        X[e] = (r < P && c < P) ? Mj[r * P + c] : 0.f;
    }
    __syncthreads();

    // acc = (X^T X) tile (ta, tb): rows a = ta*32 + .., columns b = tb*32 + n; contraction over
    // the rows r = 2s + h of X.  Register q of lane (h, n) is row (q/4)*8 + h*4 + q%4 of the tile.
    auto gram_tile = [&]() {
        f32x16 acc;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll 8
        for (int s = 0; s < P / 2; ++s) {
            const float a = X[(2 * s + h) * LD + ta * 32 + n];
            const float b = X[(2 * s + h) * LD + tb * 32 + n];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        return acc;
    };
    auto store_tile = [&](float* dst, const f32x16& acc, float scale) {
#pragma unroll
        for (int q = 0; q < 16; ++q)
            dst[(ta * 32 + (q >> 2) * 8 + h * 4 + (q & 3)) * LD + tb * 32 + n] = acc[q] * scale;
    };
    // maximum over the workgroup of a per-thread value (ends with a barrier)
    auto wg_max = [&](float v) {
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
        __syncthreads();                       // red may still be read from the previous use
        if (lane == 0) red[wave] = v;
        __syncthreads();
        float r = red[0];
#pragma unroll
        for (int w = 1; w < T * T; ++w) r = fmaxf(r, red[w]);
        return r;
    };

    // Scale so that every singular value is at most one: sigma_max^2 <= max row sum of |X^T X|.
    store_tile(G, gram_tile(), 1.f);
    __syncthreads();
    float rs = 0.f;
    if (tid < P)
        for (int b = 0; b < P; ++b) rs += fabsf(G[tid * LD + b]);
    const float s2 = wg_max(rs);
    bool ok = s2 > 0.f && s2 < 3e38f;          // zero, infinite or NaN input: not for this kernel
    const float inv = ok ? __builtin_amdgcn_rsqf(s2) : 0.f;
    for (int e = tid; e < PAD * LD; e += NTH) {
        X[e] *= inv;
        G[e] *= inv * inv;
    }
    __syncthreads();

    int it = 0;
    bool converged = false;
    while (ok) {
        // d = max |X^T X - I|; below 2e-4 the step that follows is the last (quadratic
        // convergence leaves about d^2 behind)
        float dev = 0.f;
        for (int e = tid; e < P * P; e += NTH) {
            const int a = e / P, b = e % P;
            dev = fmaxf(dev, fabsf(G[a * LD + b] - (a == b ? 1.f : 0.f)));
        }
        const float d = wg_max(dev);
        const bool last = d < 2e-4f;
        if (!(d < 4.f)) break;                 // NaN or diverging: leave it to the fallback

        // X <- 1.5 X - 0.5 X G: tile (ta, tb) of X G, rows r = ta*32 + n, contraction over a
        f32x16 acc;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] = 0.f;
#pragma unroll 8
        for (int s = 0; s < P / 2; ++s) {
            const float a = X[(ta * 32 + n) * LD + 2 * s + h];
            const float b = G[(2 * s + h) * LD + tb * 32 + n];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0);
        }
        __syncthreads();                       // every wavefront has read the old X
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            float* x = &X[(ta * 32 + (q >> 2) * 8 + h * 4 + (q & 3)) * LD + tb * 32 + n];
            *x = 1.5f * *x - 0.5f * acc[q];
        }
        __syncthreads();
        ++it;
        if (last) {
            converged = true;
            break;
        }
        if (it >= max_iters) break;
        store_tile(G, gram_tile(), 1.f);
        __syncthreads();
    }

    if (!converged) {                          // uniform
        if (tid == 0) {
            fallback[j] = 1;
            if (iters_out != nullptr) iters_out[j] = 0;
        }
        return;
    }
    if (tid == 0) {
        fallback[j] = 0;
        if (iters_out != nullptr) iters_out[j] = -it;   // negative: Newton-Schulz steps, not sweeps
    }

    // D[j][k][:] = row k of X; the same 16-byte units in the coding kernel's operand order
    // (see dict_swizzle_kernel: stage of 64 dictionary rows, unit (mt*QN + q)*64 + hh*32 + nn)
    float* Dj = D + (int64_t)j * P * P;
    for (int u = tid; u < P * P / 4; u += NTH) {
        const int k = u / (P / 4), d4 = u % (P / 4);
        const f32x4 row = {X[k * LD + 4 * d4], X[k * LD + 4 * d4 + 1], X[k * LD + 4 * d4 + 2],
                           X[k * LD + 4 * d4 + 3]};
        *reinterpret_cast<f32x4*>(&Dj[k * P + 4 * d4]) = row;
        if (dsw != nullptr) {
            constexpr int QN = P / 8;
            const int grow = j * P + k;
            const int st = grow >> 6, mt = (grow >> 5) & 1, nn = grow & 31;
            const int hh = d4 / QN, q = d4 % QN;
            reinterpret_cast<f32x4*>(dsw)[(int64_t)st * (2 * QN * 64) + (mt * QN + q) * 64 + hh * 32 + nn] = row;
        }
    }
}

}  // namespace

// fallback[j] = 1 for every block this kernel leaves to the Jacobi SVD, 0 otherwise.
hipError_t launch_polar_ns(int p, int K, const float* M, const int32_t* counts, float* D, float* dsw,
                           int32_t* fallback, int32_t* iters, hipStream_t st) {
    constexpr int kMaxIters = 26;
    switch (p) {
        case 16: hipLaunchKernelGGL((polar_ns_kernel<16>), dim3(K), dim3(64), 0, st, M, counts, D, dsw, fallback, iters, kMaxIters); break;
        case 32: hipLaunchKernelGGL((polar_ns_kernel<32>), dim3(K), dim3(64), 0, st, M, counts, D, dsw, fallback, iters, kMaxIters); break;
        case 64: hipLaunchKernelGGL((polar_ns_kernel<64>), dim3(K), dim3(256), 0, st, M, counts, D, dsw, fallback, iters, kMaxIters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sbo
