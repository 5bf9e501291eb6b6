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
    float* __restrict__ dsw, unsigned* __restrict__ dsb, int32_t* __restrict__ fallback,
    int32_t* __restrict__ iters_out, int max_iters) {
    constexpr int T = P == 64 ? 2 : 1;         // 32-wide tiles per side
    constexpr int NTH = T * T * 64;
    constexpr int PAD = T * 32;                // padded dimension (p = 16 sits in one tile)
    constexpr int LD = PAD + 4;                // rows stay 16-byte aligned
    // X, its transpose Xt and G = X^T X (symmetric), all row-major: every MFMA operand is then
    // four consecutive floats of one row (one 16-byte LDS read feeds two MFMA steps).
    __shared__ __attribute__((aligned(16))) float X[PAD * LD];
    __shared__ __attribute__((aligned(16))) float Xt[PAD * LD];
    __shared__ __attribute__((aligned(16))) float G[PAD * LD];
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
    for (int e = tid; e < PAD * PAD; e += NTH) {
        const int r = e / PAD, c = e % PAD;
        const float v = (r < P && c < P) ? Mj[r * P + c] : 0.f;
        X[r * LD + c] = v;
        Xt[c * LD + r] = v;
    }
    __syncthreads();

    // sum over k of A[ra][k] * B[rb][k] for the rows ra = ta*32 + n of A and rb = tb*32 + n of B
    // (both row-major in LDS): the tile (ta, tb) of A B^T.  Register q of lane (h, n) is row
    // (q/4)*8 + h*4 + q%4, column n of the tile.
    auto abt_tile = [&](const float* A, const float* B) {
        f32x16 acc;
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[q] = 0.f;
        const f32x4* ar = reinterpret_cast<const f32x4*>(A + (ta * 32 + n) * LD);
        const f32x4* br = reinterpret_cast<const f32x4*>(B + (tb * 32 + n) * LD);
#pragma unroll
        for (int q = 0; q < P / 4; ++q) {
            const f32x4 a = ar[q], b = br[q];
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? a.y : a.x, h ? b.y : b.x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x2f32(h ? a.w : a.z, h ? b.w : b.z, acc, 0, 0, 0);
        }
        return acc;
    };
    // G tile (ta, tb) -> LDS; returns the lane's max |G - I| (after scaling)
    auto store_gram = [&](const f32x16& acc, float scale) {
        float dev = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int row = ta * 32 + (q >> 2) * 8 + h * 4 + (q & 3), col = tb * 32 + n;
            const float g = acc[q] * scale;
            G[row * LD + col] = g;
            if (row < P && col < P) dev = fmaxf(dev, fabsf(g - (row == col ? 1.f : 0.f)));
        }
        return dev;
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

    // Scale so that the largest singular value is about one.  sigma_max^2 is the largest
    // eigenvalue of G = X^T X.  The iteration sends every singular value in (0, sqrt(3)) to +1,
    // one in (sqrt(3), sqrt(5)) to -1 (an orthogonal matrix that is NOT U V^T, and which the
    // deviation test cannot tell apart), so the scale must be a guaranteed bound: the largest
    // absolute row sum of G is at least its largest eigenvalue, and dividing G by that sum / 2.9
    // keeps every scaled sigma^2 at or below 2.9.  That bound alone is often two to three times
    // too large, which costs iterations; a Rayleigh quotient after a few power-iteration steps
    // from the vector of absolute row sums is a lower estimate that is usually tight, so the
    // scale is the larger of (1.08 x that quotient) and (row-sum bound / 2.9).
    // (X^T X = Xt Xt^T: both operands are rows of Xt.)
    __shared__ float vec[PAD], wec[PAD];
    f32x16 g0 = abt_tile(Xt, Xt);
    store_gram(g0, 1.f);
    __syncthreads();
    if (tid < P) {
        float rs = 0.f;
        for (int b = 0; b < P; ++b) rs += fabsf(G[tid * LD + b]);
        vec[tid] = rs;
    }
    __syncthreads();
    float rsmax = 0.f;                         // every thread, same order: same value
    for (int a = 0; a < P; ++a) rsmax = fmaxf(rsmax, vec[a]);
    float s2 = 0.f;
    for (int round = 0; round < 4; ++round) {
        if (tid < P) {
            float w = 0.f;
            for (int b = 0; b < P; ++b) w += G[tid * LD + b] * vec[b];
            wec[tid] = w;
        }
        __syncthreads();
        float vv = 0.f, vw = 0.f, wmax = 0.f;  // every thread, same order: same values
        for (int a = 0; a < P; ++a) {
            vv += vec[a] * vec[a];
            vw += vec[a] * wec[a];
            wmax = fmaxf(wmax, fabsf(wec[a]));
        }
        s2 = 1.08f * vw / vv;                  // NaN for a zero matrix: caught below
        __syncthreads();
        if (tid < P) vec[tid] = wec[tid] / wmax;
        __syncthreads();
    }
    const bool rq_ok = s2 > 0.f && s2 < 3e38f; // zero, infinite or NaN input: not for this kernel
    s2 = fmaxf(s2, rsmax * (1.f / 2.9f));
    const bool ok = rq_ok && s2 < 3e38f;
    const float inv = ok ? __builtin_amdgcn_rsqf(s2) : 0.f;
    for (int e = tid; e < PAD * LD; e += NTH) {
        X[e] *= inv;
        Xt[e] *= inv;
    }
    float dev = store_gram(g0, inv * inv);     // same tile, scaled (nobody reads G in between)
    int it = 0;
    bool converged = false;
    while (ok) {
        // d = max |X^T X - I|; below 2e-4 the step that follows is the last (quadratic
        // convergence leaves about d^2 behind).  The barriers inside also publish G, X, Xt.
        const float d = wg_max(dev);
        const bool last = d < 2e-4f;
        if (!(d < 4.f)) break;                 // NaN or diverging: leave it to the fallback

        // X <- 1.5 X - 0.5 X G; (X G)[r][b] = sum_a X[r][a] G[b][a] (G symmetric)
        const f32x16 acc = abt_tile(X, G);
        __syncthreads();                       // every wavefront has read the old X
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int row0 = ta * 32 + q4 * 8 + h * 4, col = tb * 32 + n;
            f32x4* xt4 = reinterpret_cast<f32x4*>(&Xt[col * LD + row0]);
            const f32x4 old = *xt4;
            const f32x4 nw = {1.5f * old.x - 0.5f * acc[4 * q4], 1.5f * old.y - 0.5f * acc[4 * q4 + 1],
                              1.5f * old.z - 0.5f * acc[4 * q4 + 2], 1.5f * old.w - 0.5f * acc[4 * q4 + 3]};
            *xt4 = nw;
            X[(row0 + 0) * LD + col] = nw.x;
            X[(row0 + 1) * LD + col] = nw.y;
            X[(row0 + 2) * LD + col] = nw.z;
            X[(row0 + 3) * LD + col] = nw.w;
        }
        __syncthreads();
        ++it;
        if (last) {
            converged = true;
            break;
        }
        if (it >= max_iters) break;
        dev = store_gram(abt_tile(Xt, Xt), 1.f);
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

    // D[j][k][:] = row k of X; the same values in the coding kernel's operand orders
    float* Dj = D + (int64_t)j * P * P;
    for (int u = tid; u < P * P / 4; u += NTH) {
        const int k = u / (P / 4), d4 = u % (P / 4);
        const f32x4 row = {X[k * LD + 4 * d4], X[k * LD + 4 * d4 + 1], X[k * LD + 4 * d4 + 2],
                           X[k * LD + 4 * d4 + 3]};
        *reinterpret_cast<f32x4*>(&Dj[k * P + 4 * d4]) = row;
        if (dsw != nullptr) store_operand_f32<P>(dsw, j * P + k, d4, row);
        if (dsb != nullptr) store_operand_split<P>(dsb, j * P + k, d4, row);
    }
}

}  // namespace

// fallback[j] = 1 for every block this kernel leaves to the Jacobi SVD, 0 otherwise.
hipError_t launch_polar_ns(int p, int K, const float* M, const int32_t* counts, float* D, float* dsw,
                           unsigned* dsb, int32_t* fallback, int32_t* iters, hipStream_t st) {
    constexpr int kMaxIters = 26;
    switch (p) {
        case 16: hipLaunchKernelGGL((polar_ns_kernel<16>), dim3(K), dim3(64), 0, st, M, counts, D, dsw, dsb, fallback, iters, kMaxIters); break;
        case 32: hipLaunchKernelGGL((polar_ns_kernel<32>), dim3(K), dim3(64), 0, st, M, counts, D, dsw, dsb, fallback, iters, kMaxIters); break;
        case 64: hipLaunchKernelGGL((polar_ns_kernel<64>), dim3(K), dim3(256), 0, st, M, counts, D, dsw, dsb, fallback, iters, kMaxIters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace sbo
