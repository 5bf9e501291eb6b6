// Batched SVD update Q_j = U V^T (Algorithm 1, steps 6-7) for p = 256.
//
// The same one-sided Jacobi as for p <= 64 (round-robin tournament, p/2 disjoint column
// pairs per round, eight lanes per pair, DPP dot-product reductions), but A = P_j and V
// (2 x 256 KiB per block) do not fit the LDS of one CU.  The work is therefore split:
//
//   1. wide_jacobi_kernel, one workgroup of 1024 threads per block, orthogonalises the
//      columns of A only.  Rows 0..127 of A live in LDS (132 KiB), rows 128..255 in global
//      memory (L2); every round streams each column pair through registers.  The rotation
//      (cos, sin) of every pair and round is appended to a log.
//   2. wide_replay_kernel applies the logged rotations to V.  Rows of V are independent,
//      so this spreads over the whole chip: a wavefront keeps four rows in LDS and walks
//      the log.
//   3. wide_finish_kernel: sigma = column norms, U = A / sigma, completion of vanished
//      columns, Q = U V^T.
//
// Keeping V out of the tournament halves the data each round has to move through one CU,
// which is what bounds step 1.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int P = 256;
constexpr int kPairs = P / 2;
constexpr int kSteps = P - 1;
constexpr int kMaxSweeps = 24;    // rounds logged per block: kMaxSweeps * kSteps
constexpr float kTol = 1e-6f;     // rotate while |a_i . a_j| > kTol |a_i| |a_j|
constexpr int LDA = 132;          // LDS leading dimension of the 128 on-chip rows
constexpr int kRowsLds = 128;

constexpr size_t kLogFloatsPerBlock = (size_t)kMaxSweeps * kSteps * kPairs * 2;

// Scratch layout per launch: A[K][P][P] | log[K][kLogFloatsPerBlock] | nsweeps[K] (ints)
struct WideScratch {
    float* A;
    float* log;
    int* nsweeps;
};
__host__ __device__ inline WideScratch carve(float* base, int K) {
    WideScratch s;
    s.A = base;
    s.log = base + (size_t)K * P * P;
    s.nsweeps = reinterpret_cast<int*>(s.log + (size_t)K * kLogFloatsPerBlock);
    return s;
}

// Tournament schedule: player P-1 stays, the others advance by one (mod P-1) per round.
__device__ __forceinline__ void pair_init(int pi, int& ca, int& cb) {
    ca = pi == 0 ? P - 1 : pi;
    cb = pi == 0 ? 0 : P - 1 - pi;
}
__device__ __forceinline__ void pair_next(int pi, int& ca, int& cb) {
    if (pi == 0) {
        cb = cb + 1;
    } else {
        ca = ca + 1 == P - 1 ? 0 : ca + 1;
        cb = cb + 1 == P - 1 ? 0 : cb + 1;
    }
}

__global__ __launch_bounds__(1024) void wide_jacobi_kernel(const float* __restrict__ M,
                                                           const int32_t* __restrict__ counts,
                                                           float* scratch, int K, float done,
                                                           int32_t* __restrict__ sweeps_out,
                                                           const int32_t* __restrict__ only) {
    constexpr int NT = 1024;
    constexpr int TPP = 8;
    constexpr int RPT = P / TPP;               // 32 rows per lane: 16 on chip, 16 in global memory
    constexpr int HALF = RPT / 2;
    static_assert(HALF * TPP == kRowsLds, "row split");
    extern __shared__ float AL[];              // [P][LDA]: rows 0..127 of every column
    __shared__ float red[NT / 64];

    const WideScratch ws = carve(scratch, K);
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    if (only != nullptr && only[j] == 0) return;   // uniform: another kernel has done this block
    if (counts != nullptr && counts[j] == 0) { // uniform: block keeps its basis
        if (tid == 0) {
            ws.nsweeps[j] = 0;
            if (sweeps_out != nullptr) sweeps_out[j] = 0;
        }
        return;
    }
    float* A = ws.A + (int64_t)j * P * P;      // column c = A[c*P .. c*P+P); rows >= 128 used here
    float* log = ws.log + (int64_t)j * kLogFloatsPerBlock;

    // scale by 1 / max|entry| (the orthogonal factor does not depend on scale)
    const float* Mj = M + (int64_t)j * P * P;
    float mx = 0.f;
    for (int e = tid; e < P * P; e += NT) mx = fmaxf(mx, fabsf(Mj[e]));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    mx = 0.f;
    for (int w = 0; w < NT / 64; ++w) mx = fmaxf(mx, red[w]);
    const float scale = mx > 0.f ? 1.f / mx : 0.f;

    // A = scale * P_j
    for (int o = tid; o < P * P / 4; o += NT) {
        const int c = o / (P / 4), r4 = (o % (P / 4)) * 4;
        f32x4 s4 = *reinterpret_cast<const f32x4*>(&Mj[c * P + r4]);
        s4 *= scale;
        if (r4 < kRowsLds) *reinterpret_cast<f32x4*>(&AL[c * LDA + r4]) = s4;
        else *reinterpret_cast<f32x4*>(&A[c * P + r4]) = s4;
    }
    __threadfence_block();
    __syncthreads();

    // lane `sub` of a pair owns rows sub*16..+15 (LDS) and 128 + sub*16..+15 (global), so
    // every lane has both kinds of access in flight at once
    const int pi = tid / TPP, sub = tid % TPP;
    const int rl = sub * HALF;                 // first on-chip row
    const int rg = kRowsLds + sub * HALF;      // first global row
    int sweeps_done = 0;
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        int rotated = 0;
        int ca, cb;
        pair_init(pi, ca, cb);
        float* lg = log + ((size_t)sweep * kSteps * kPairs + pi) * 2;
        for (int step = 0; step < kSteps; ++step, lg += kPairs * 2) {
            const int ci = min(ca, cb), cj = max(ca, cb);
            float* gi = A + ci * P + rg;
            float* gj = A + cj * P + rg;
            float* li = AL + ci * LDA + rl;
            float* lj = AL + cj * LDA + rl;
            float x[RPT], y[RPT];
#pragma unroll
            for (int t = 0; t < HALF; t += 4) {
                const f32x4 a4 = *reinterpret_cast<const f32x4*>(gi + t);
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(gj + t);
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    x[HALF + t + e] = a4[e];
                    y[HALF + t + e] = b4[e];
                }
            }
#pragma unroll
            for (int t = 0; t < HALF; t += 4) {
                const f32x4 a4 = *reinterpret_cast<const f32x4*>(li + t);
                const f32x4 b4 = *reinterpret_cast<const f32x4*>(lj + t);
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
            if (g2ab > (done * done) * ab) rotated = 1;
            float cs = 1.f, sn = 0.f;
            if (g2ab > (kTol * kTol) * ab && hh > 1e-36f) {
                // cos(2 theta) = |d| / hypot(d, 2 gamma), |theta| <= pi/4
                const float r = __builtin_amdgcn_rsqf(hh);
                const float w = 0.5f + 0.5f * (fabsf(d) * r);
                const float rc = __builtin_amdgcn_rsqf(w);
                cs = w * rc;
                sn = copysignf(0.5f * rc * r, d) * g2;
#pragma unroll
                for (int t = 0; t < HALF; t += 4) {
                    f32x4 na, nb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        na[e] = cs * x[HALF + t + e] - sn * y[HALF + t + e];
                        nb[e] = sn * x[HALF + t + e] + cs * y[HALF + t + e];
                    }
                    *reinterpret_cast<f32x4*>(gi + t) = na;
                    *reinterpret_cast<f32x4*>(gj + t) = nb;
                }
#pragma unroll
                for (int t = 0; t < HALF; t += 4) {
                    f32x4 na, nb;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        na[e] = cs * x[t + e] - sn * y[t + e];
                        nb[e] = sn * x[t + e] + cs * y[t + e];
                    }
                    *reinterpret_cast<f32x4*>(li + t) = na;
                    *reinterpret_cast<f32x4*>(lj + t) = nb;
                }
            }
            if (sub == 0) {                    // (ci, cj) of a round follow from the schedule
                lg[0] = cs;
                lg[1] = sn;
            }
            pair_next(pi, ca, cb);
            __threadfence_block();
            __syncthreads();
        }
        sweeps_done = sweep + 1;
        if (!__syncthreads_or(rotated)) break;
    }
    if (tid == 0) {
        ws.nsweeps[j] = sweeps_done;
        if (sweeps_out != nullptr) sweeps_out[j] = sweeps_done;
    }

    // the on-chip rows go back next to the others for the finishing kernel
    for (int o = tid; o < P * kRowsLds / 4; o += NT) {
        const int c = o / (kRowsLds / 4), r4 = (o % (kRowsLds / 4)) * 4;
        *reinterpret_cast<f32x4*>(&A[c * P + r4]) = *reinterpret_cast<const f32x4*>(&AL[c * LDA + r4]);
    }
}

// V <- I * (logged rotations), four rows per wavefront.
constexpr int kReplayRows = 4;

__global__ __launch_bounds__(256) void wide_replay_kernel(const int32_t* __restrict__ counts,
                                                          float* Vst,
                                                          const float* scratch, int K,
                                                          const int32_t* __restrict__ only) {
    __shared__ float rows_all[4][kReplayRows][P];
    const WideScratch ws = carve(const_cast<float*>(scratch), K);
    const int j = blockIdx.x;
    if (only != nullptr && only[j] == 0) return;   // uniform
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = (blockIdx.y * 4 + wave) * kReplayRows;
    float* V = Vst + (int64_t)j * P * P;       // column-major: V[c*P + r]
    float(*rows)[P] = rows_all[wave];

    if (counts != nullptr && counts[j] == 0) return;   // uniform: block keeps its basis, V unused
#pragma unroll
    for (int rr = 0; rr < kReplayRows; ++rr)
        for (int c = lane; c < P; c += 64) rows[rr][c] = c == row0 + rr ? 1.f : 0.f;
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();

    const int ns = ws.nsweeps[j];
    const float* log = ws.log + (int64_t)j * kLogFloatsPerBlock;
    const int p0 = lane, p1 = lane + 64;       // this lane's pairs (neighbouring lanes touch
                                               // neighbouring columns: no bank conflicts)
    for (int sweep = 0; sweep < ns; ++sweep) {
        int ca0, cb0, ca1, cb1;
        pair_init(p0, ca0, cb0);
        pair_init(p1, ca1, cb1);
        const float2* lg = reinterpret_cast<const float2*>(log + (size_t)sweep * kSteps * kPairs * 2);
        float2 n0 = lg[p0], n1 = lg[p1];
        for (int step = 0; step < kSteps; ++step) {
            const float2 r0 = n0, r1 = n1;     // (cos, sin) of this lane's two pairs
            if (step + 1 < kSteps) {
                n0 = lg[(size_t)(step + 1) * kPairs + p0];
                n1 = lg[(size_t)(step + 1) * kPairs + p1];
            }
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            {
                const int ci = min(ca0, cb0), cj = max(ca0, cb0);
#pragma unroll
                for (int rr = 0; rr < kReplayRows; ++rr) {
                    const float pv = rows[rr][ci], qv = rows[rr][cj];
                    rows[rr][ci] = r0.x * pv - r0.y * qv;
                    rows[rr][cj] = r0.y * pv + r0.x * qv;
                }
            }
            {
                const int ci = min(ca1, cb1), cj = max(ca1, cb1);
#pragma unroll
                for (int rr = 0; rr < kReplayRows; ++rr) {
                    const float pv = rows[rr][ci], qv = rows[rr][cj];
                    rows[rr][ci] = r1.x * pv - r1.y * qv;
                    rows[rr][cj] = r1.y * pv + r1.x * qv;
                }
            }
            pair_next(p0, ca0, cb0);
            pair_next(p1, ca1, cb1);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the next round pairs other columns
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int rr = 0; rr < kReplayRows; ++rr)
        for (int c = lane; c < P; c += 64) V[c * P + row0 + rr] = rows[rr][c];
}

__global__ __launch_bounds__(1024) void wide_finish_kernel(const float* __restrict__ M,
                                                           const int32_t* __restrict__ counts,
                                                           float* __restrict__ D, float* Vst,
                                                           float* scratch, int K,
                                                           float* __restrict__ eig_sv,
                                                           const int32_t* __restrict__ only) {
    constexpr int NT = 1024;
    __shared__ float sig[P];
    __shared__ float coefs[P];
    __shared__ float vec[P];
    __shared__ int isbad[P];
    __shared__ int shared_i[2];

    const WideScratch ws = carve(scratch, K);
    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    if (only != nullptr && only[j] == 0) return;       // uniform
    if (counts != nullptr && counts[j] == 0) return;   // uniform: block keeps its basis
    float* A = ws.A + (int64_t)j * P * P;
    float* V = Vst + (int64_t)j * P * P;

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

    // Eigen mode (see polar_kernel): atoms = eigenvectors (columns of V) by descending
    // eigenvalue, eig_sv = square roots of the eigenvalues.  The scale the Jacobi kernel
    // applied (1 / max|entry| of P_j) is recomputed here.
    if (eig_sv != nullptr) {
        const float* Mj = M + (int64_t)j * P * P;
        float mx = 0.f;
        for (int e = tid; e < P * P; e += NT) mx = fmaxf(mx, fabsf(Mj[e]));
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        if ((tid & 63) == 0) coefs[tid >> 6] = mx;
        __syncthreads();
        mx = 0.f;
        for (int w = 0; w < NT / 64; ++w) mx = fmaxf(mx, coefs[w]);
        __syncthreads();
        if (tid < P) {
            int rank = 0;
            for (int c = 0; c < P; ++c) rank += sig[c] > sig[tid] || (sig[c] == sig[tid] && c < tid);
            isbad[tid] = rank;
            eig_sv[(int64_t)j * P + rank] = sqrtf(sig[tid] * vec[tid] * mx);   // |A_c| / |V_c|, rescaled
        }
        __syncthreads();
        float* Dj = D + (int64_t)j * P * P;
        for (int e = tid; e < P * P; e += NT) Dj[isbad[e / P] * P + (e % P)] = V[e];
        return;                                // uniform
    }

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

size_t polar_wide_scratch_bytes(int K) {
    return ((size_t)K * P * P + (size_t)K * kLogFloatsPerBlock) * sizeof(float) + (size_t)K * sizeof(int);
}

hipError_t launch_polar_wide(int K, const float* M, const int32_t* counts, float* D, float* vwork,
                             float* jac_a, float* eig_sv, int32_t* sweeps, const int32_t* only,
                             LdsRaised* raised, hipStream_t st) {
    if (vwork == nullptr || jac_a == nullptr || raised == nullptr) return hipErrorInvalidValue;
    const size_t lds = (size_t)P * LDA * sizeof(float);
    hipError_t e = raised->ensure(reinterpret_cast<const void*>(&wide_jacobi_kernel), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(wide_jacobi_kernel, dim3(K), dim3(1024), lds, st, M, counts, jac_a, K, kPolarDone,
                       sweeps, only);
    hipLaunchKernelGGL(wide_replay_kernel, dim3(K, P / (4 * kReplayRows)), dim3(256), 0, st, counts,
                       vwork, jac_a, K, only);
    hipLaunchKernelGGL(wide_finish_kernel, dim3(K), dim3(1024), 0, st, M, counts, D, vwork, jac_a, K,
                       eig_sv, only);
    return hipGetLastError();
}

}  // namespace sbo
