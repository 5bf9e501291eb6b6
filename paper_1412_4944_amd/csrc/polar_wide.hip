// Batched SVD update Q_j = U V^T (Algorithm 1, steps 6-7) for p = 256.
//
// The same one-sided Jacobi as for p <= 64 (round-robin tournament, p/2 disjoint column
// pairs per round, eight lanes per pair, DPP dot-product reductions), but A = P_j and V
// (2 x 256 KiB per block) do not fit the LDS of one CU: they live in global memory, where
// they stay resident in the L2 of the block's XCD, and every round streams each column
// pair through registers.  One workgroup of 1024 threads per block; rounds are separated
// by workgroup barriers, which order the global accesses of the workgroup.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int kMaxSweeps = 40;
constexpr float kTol = 1e-6f;     // rotate while |a_i . a_j| > kTol |a_i| |a_j|
constexpr float kDone = 1e-4f;    // a sweep whose cosines were all below this is the last

__global__ __launch_bounds__(1024) void polar_wide_kernel(const float* __restrict__ M,
                                                          const int32_t* __restrict__ counts,
                                                          float* __restrict__ D, float* Vst,
                                                          int warm, float* Aw) {
    constexpr int P = 256;
    constexpr int NT = 1024;
    constexpr int TPP = 8;
    constexpr int RPT = P / TPP;               // 32 contiguous rows per lane
    __shared__ float sig[P];
    __shared__ float coefs[P];
    __shared__ float vec[P];
    __shared__ int isbad[P];
    __shared__ int shared_i[2];

    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    float* A = Aw + (int64_t)j * P * P;        // column c = A[c*P .. c*P+P)
    float* V = Vst + (int64_t)j * P * P;
    if (counts != nullptr && counts[j] == 0) { // uniform: block keeps its basis
        if (!warm)
            for (int e = tid; e < P * P; e += NT) V[e] = (e / P == e % P) ? 1.f : 0.f;
        return;
    }

    const float* Mj = M + (int64_t)j * P * P;
    float mx = 0.f;
    for (int e = tid; e < P * P; e += NT) mx = fmaxf(mx, fabsf(Mj[e]));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((tid & 63) == 0) vec[tid >> 6] = mx;
    __syncthreads();
    mx = 0.f;
    for (int w = 0; w < NT / 64; ++w) mx = fmaxf(mx, vec[w]);
    const float scale = mx > 0.f ? 1.f / mx : 0.f;
    __syncthreads();

    if (!warm) {
        for (int e = tid; e < P * P; e += NT) {
            A[e] = Mj[e] * scale;
            V[e] = (e / P == e % P) ? 1.f : 0.f;
        }
    } else {
        // A = (scale P_j) V with the V kept from this block's previous decomposition
        for (int o = tid; o < P * P / 4; o += NT) {
            const int c = o / (P / 4), r4 = (o % (P / 4)) * 4;
            f32x4 s4 = {0.f, 0.f, 0.f, 0.f};
            for (int k = 0; k < P; ++k) {
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(&Mj[k * P + r4]);
                s4 += b4 * V[c * P + k];
            }
            *reinterpret_cast<f32x4*>(&A[c * P + r4]) = s4 * scale;
        }
    }
    __threadfence_block();
    __syncthreads();

    const int pi = tid / TPP, sub = tid % TPP;
    const int r0 = sub * RPT;
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        int rotated = 0;
        int ca = pi == 0 ? P - 1 : pi;
        int cb = pi == 0 ? 0 : P - 1 - pi;
        for (int step = 0; step < P - 1; ++step) {
            const int ci = min(ca, cb), cj = max(ca, cb);
            float* ai = A + ci * P + r0;
            float* aj = A + cj * P + r0;
            float* vi = V + ci * P + r0;
            float* vj = V + cj * P + r0;
            float x[RPT], y[RPT];
#pragma unroll
            for (int t = 0; t < RPT; t += 4) {
                const f32x4 a4 = *reinterpret_cast<const f32x4*>(ai + t);
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(aj + t);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[t + e] = a4[e];
                    y[t + e] = b4[e];
                }
            }
            float alpha = 0.f, beta = 0.f, gamma = 0.f;
#pragma unroll
            for (int t = 0; t < RPT; ++t) {
                alpha += x[t] * x[t];
                beta += y[t] * y[t];
                gamma += x[t] * y[t];
            }
            alpha = group_sum<TPP>(alpha);
            beta = group_sum<TPP>(beta);
            gamma = group_sum<TPP>(gamma);
            const float d = beta - alpha, g2 = 2.f * gamma;
            const float hh = d * d + g2 * g2;
            const float g2ab = gamma * gamma, ab = alpha * beta;
            if (g2ab > (kDone * kDone) * ab) rotated = 1;
            if (g2ab > (kTol * kTol) * ab && hh > 1e-36f) {
                // cos(2 theta) = |d| / hypot(d, 2 gamma), |theta| <= pi/4
                const float r = __builtin_amdgcn_rsqf(hh);
                const float w = 0.5f + 0.5f * (fabsf(d) * r);
                const float rc = __builtin_amdgcn_rsqf(w);
                const float cs = w * rc;
                const float sn = copysignf(0.5f * rc * r, d) * g2;
#pragma unroll
                for (int t = 0; t < RPT; t += 4) {
                    f32x4 na, nb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        na[e] = cs * x[t + e] - sn * y[t + e];
                        nb[e] = sn * x[t + e] + cs * y[t + e];
                    }
                    *reinterpret_cast<f32x4*>(ai + t) = na;
                    *reinterpret_cast<f32x4*>(aj + t) = nb;
                }
#pragma unroll
                for (int t = 0; t < RPT; t += 4) {
                    const f32x4 p4 = *reinterpret_cast<const f32x4*>(vi + t);
                    const f32x4 q4 = *reinterpret_cast<const f32x4*>(vj + t);
                    *reinterpret_cast<f32x4*>(vi + t) = p4 * cs - q4 * sn;
                    *reinterpret_cast<f32x4*>(vj + t) = p4 * sn + q4 * cs;
                }
            }
            if (pi == 0) {
                cb = cb + 1;
            } else {
                ca = ca + 1 == P - 1 ? 0 : ca + 1;
                cb = cb + 1 == P - 1 ? 0 : cb + 1;
            }
            __threadfence_block();
            __syncthreads();
        }
        if (!__syncthreads_or(rotated)) break;
    }

    // sigma = column norms, U = A / sigma, V columns renormalised
    if (tid < P) {
        float s = 0.f, v = 0.f;
        for (int r = 0; r < P; ++r) {
            s += A[tid * P + r] * A[tid * P + r];
            v += V[tid * P + r] * V[tid * P + r];
        }
        sig[tid] = sqrtf(s);
        vec[tid] = 1.f / sqrtf(v);
    }
    __syncthreads();
    if (tid == 0) {
        float smax = 0.f;
        for (int c = 0; c < P; ++c) smax = fmaxf(smax, sig[c]);
        int nb = 0;
        const float thr = smax * 1e-6f;
        for (int c = 0; c < P; ++c) {
            isbad[c] = !(sig[c] > thr);
            nb += isbad[c];
        }
        shared_i[0] = nb;
    }
    __syncthreads();
    for (int e = tid; e < P * P; e += NT) {
        const int c = e / P;
        A[e] = isbad[c] ? 0.f : A[e] / sig[c];
        V[e] *= vec[c];
    }
    __threadfence_block();
    __syncthreads();

    if (shared_i[0] > 0) {                     // uniform: complete the vanished columns
        for (int c = 0; c < P; ++c) {
            if (!isbad[c]) continue;           // uniform
            if (tid < P) {
                float s = 0.f;
                for (int cc = 0; cc < P; ++cc) s += A[cc * P + tid] * A[cc * P + tid];
                vec[tid] = s;
            }
            __syncthreads();
            if (tid == 0) {
                int best = 0;
                for (int r = 1; r < P; ++r)
                    if (vec[r] < vec[best]) best = r;
                shared_i[1] = best;
            }
            __syncthreads();
            const int rs = shared_i[1];
            float w = 0.f;
            if (tid < P) {
                float s = (tid == rs) ? 1.f : 0.f;
                for (int cc = 0; cc < P; ++cc) s -= A[cc * P + rs] * A[cc * P + tid];
                w = s;
                vec[tid] = s;
            }
            __syncthreads();
            if (tid < P) {
                float dsum = 0.f;
                for (int r = 0; r < P; ++r) dsum += A[tid * P + r] * vec[r];
                coefs[tid] = dsum;
            }
            __syncthreads();
            if (tid < P) {
                for (int cc = 0; cc < P; ++cc) w -= coefs[cc] * A[cc * P + tid];
            }
            __syncthreads();
            if (tid < P) vec[tid] = w;
            __syncthreads();
            if (tid < P) {
                float nrm = 0.f;
                for (int r = 0; r < P; ++r) nrm += vec[r] * vec[r];
                A[c * P + tid] = w / sqrtf(nrm);
            }
            __threadfence_block();
            __syncthreads();
        }
    }

    // Q = U V^T, atom-major: D[j][k][r] = sum_c U[r][c] V[k][c]
    float* Dj = D + (int64_t)j * P * P;
    for (int tile = tid; tile < (P / 4) * (P / 4); tile += NT) {
        const int q0 = 4 * (tile % (P / 4)), k0 = 4 * (tile / (P / 4));
        float o[4][4] = {};
        for (int c = 0; c < P; ++c) {
            const f32x4 u = *reinterpret_cast<const f32x4*>(&A[c * P + q0]);
            const f32x4 v = *reinterpret_cast<const f32x4*>(&V[c * P + k0]);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) o[a][b] += v[a] * u[b];
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 row = {o[a][0], o[a][1], o[a][2], o[a][3]};
            *reinterpret_cast<f32x4*>(&Dj[(k0 + a) * P + q0]) = row;
        }
    }
}

}  // namespace

hipError_t launch_polar_wide(int K, const float* M, const int32_t* counts, float* D, float* vstate,
                             int warm, float* jac_a, hipStream_t st) {
    if (vstate == nullptr || jac_a == nullptr) return hipErrorInvalidValue;
    hipLaunchKernelGGL(polar_wide_kernel, dim3(K), dim3(1024), 0, st, M, counts, D, vstate, warm,
                       jac_a);
    return hipGetLastError();
}

}  // namespace sbo
