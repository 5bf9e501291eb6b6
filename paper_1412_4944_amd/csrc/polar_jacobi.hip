// Batched SVD update Q_j = U V^T (Algorithm 1, steps 6-7) by a Jacobi SVD, one workgroup per
// block, and the dispatch between this kernel and the Newton-Schulz kernels (launch_polar):
// the SVD runs for the blocks the Newton-Schulz iteration leaves flagged (rank-deficient or
// very ill-conditioned P_j), in eigen mode (symmetric input, eigenvectors wanted), and for
// every block when Newton-Schulz is switched off.
//
// One-sided (Hestenes) Jacobi: plane rotations applied from the right to the columns
// of A = P_j and to V (starting at I) until all columns of A are mutually orthogonal;
// then A = U diag(sigma) and P_j = U diag(sigma) V^T, so Q_j = sum_c (A_c / sigma_c) V_c^T.
// A and V live in LDS for the whole decomposition.  p/2 disjoint column pairs (round-
// robin tournament) are rotated concurrently, TPP (default 16) lanes per pair, with one barrier
// per tournament round.  Columns whose norm vanishes (rank-deficient P_j) are replaced
// by an orthonormal completion, which is a valid choice of U there.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int kMaxSweeps = 30;
// A pair is rotated while |a_i . a_j| > kTol |a_i| |a_j|.  Convergence is quadratic: a
// sweep in which every pair already had a cosine below `done` (kPolarDone) leaves cosines of
// the order of done^2 behind, so it is the last one and no sweep is spent on verifying.
constexpr float kTol = 1e-6f;

template <int P, int TPP>
__global__ __launch_bounds__((P / 2) * TPP) void polar_kernel(const float* __restrict__ M,
                                                             const int32_t* __restrict__ counts,
                                                             float* __restrict__ D,
                                                             float* __restrict__ eig_sv, float done,
                                                             float* __restrict__ dsw,
                                                             unsigned* __restrict__ dsb,
                                                             int32_t* __restrict__ sweeps_out,
                                                             const int32_t* __restrict__ only) {
    constexpr int LD = P + 4;
    constexpr int NT = (P / 2) * TPP;          // threads: TPP lanes per column pair
    constexpr int RPT = P / TPP;               // contiguous rows per lane in a rotation
    static_assert(TPP == 4 || TPP == 8 || TPP == 16, "lanes per pair");
    static_assert(RPT >= 1 && P % TPP == 0, "rows per lane");
    __shared__ __attribute__((aligned(16))) float A[P * LD];
    __shared__ __attribute__((aligned(16))) float V[P * LD];
    __shared__ float sig[P];
    __shared__ float coefs[P];
    __shared__ float vec[P];
    __shared__ int isbad[P];
    __shared__ int shared_i[2];

    const int j = blockIdx.x;
    const int tid = threadIdx.x;
    if (only != nullptr && only[j] == 0) return;        // uniform: another kernel has done this block
    if (counts != nullptr && counts[j] == 0) {          // uniform: block keeps its basis
        if (sweeps_out != nullptr && tid == 0) sweeps_out[j] = 0;
        return;
    }

    // Load P_j scaled by 1 / max|entry| (the orthogonal factor does not depend on scale;
    // this keeps the squared norms below well inside the fp32 range).
    const float* Mj = M + (int64_t)j * P * P;
    float mx = 0.f;
    for (int e = tid; e < P * P; e += NT) mx = fmaxf(mx, fabsf(Mj[e]));
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
    if ((tid & 63) == 0) vec[tid >> 6] = mx;
    __syncthreads();
    mx = 0.f;
    for (int w = 0; w < (NT + 63) / 64; ++w) mx = fmaxf(mx, vec[w]);
    const float scale = mx > 0.f ? 1.f / mx : 0.f;
    __syncthreads();
    for (int e = tid; e < P * P; e += NT) {
        const int c = e / P, r = e % P;
        A[c * LD + r] = Mj[e] * scale;
        V[c * LD + r] = (c == r) ? 1.f : 0.f;
    }
    __syncthreads();

    // Round-robin tournament on P players: player P-1 stays, the others rotate; group pi
    // meets columns ca, cb, which advance by one (mod P-1) every round.
    const int pi = tid / TPP, sub = tid % TPP;
    const int r0 = sub * RPT;
    int sweeps_done = 0;
    for (int sweep = 0; sweep < kMaxSweeps; ++sweep) {
        int rotated = 0;
        // columns as LDS offsets (column * LD), advanced by additions only
        constexpr int WRAP = (P - 1) * LD;
        int oa = (pi == 0 ? P - 1 : pi) * LD;
        int ob = (pi == 0 ? 0 : P - 1 - pi) * LD;
        for (int step = 0; step < P - 1; ++step) {
            const int oi = min(oa, ob), oj = max(oa, ob);
            float* ai = A + oi + r0;
            float* aj = A + oj + r0;
            float* vi = V + oi + r0;
            float* vj = V + oj + r0;
            float x[RPT], y[RPT], vx[RPT], vy[RPT];
            if constexpr (RPT % 4 == 0) {
#pragma unroll
                for (int t = 0; t < RPT; t += 4) {
                    const f32x4 a4 = *reinterpret_cast<const f32x4*>(ai + t);
                    const f32x4 b4 = *reinterpret_cast<const f32x4*>(aj + t);
                    const f32x4 c4 = *reinterpret_cast<const f32x4*>(vi + t);
                    const f32x4 d4 = *reinterpret_cast<const f32x4*>(vj + t);
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        x[t + e] = a4[e];
                        y[t + e] = b4[e];
                        vx[t + e] = c4[e];
                        vy[t + e] = d4[e];
                    }
                }
            } else {
#pragma unroll
                for (int t = 0; t < RPT; ++t) {
                    x[t] = ai[t];
                    y[t] = aj[t];
                    vx[t] = vi[t];
                    vy[t] = vj[t];
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
            // Rotation by theta with tan(2 theta) = 2 gamma / (beta - alpha), |theta| <= pi/4,
            // from cos(2 theta) = |d| / hypot(d, 2 gamma).  One-ulp reciprocal square roots
            // suffice: the iteration corrects itself.
            const float d = beta - alpha, g2 = 2.f * gamma;
            const float hh = d * d + g2 * g2;
            // keep the V loads issued together with the A loads, ahead of the decision
#pragma unroll
            for (int t = 0; t < RPT; ++t) asm volatile("" : "+v"(vx[t]), "+v"(vy[t]));
            const float g2ab = gamma * gamma, ab = alpha * beta;
            if (g2ab > (done * done) * ab) rotated = 1;          // another sweep is needed
            if (g2ab > (kTol * kTol) * ab && hh > 1e-36f) {
                const float r = __builtin_amdgcn_rsqf(hh);
                const float w = 0.5f + 0.5f * (fabsf(d) * r);
                const float rc = __builtin_amdgcn_rsqf(w);
                const float cs = w * rc;
                const float sn = copysignf(0.5f * rc * r, d) * g2;
                float nx[RPT], ny[RPT], nvx[RPT], nvy[RPT];
#pragma unroll
                for (int t2 = 0; t2 < RPT; ++t2) {
                    nx[t2] = cs * x[t2] - sn * y[t2];
                    ny[t2] = sn * x[t2] + cs * y[t2];
                    nvx[t2] = cs * vx[t2] - sn * vy[t2];
                    nvy[t2] = sn * vx[t2] + cs * vy[t2];
                }
                if constexpr (RPT % 4 == 0) {
#pragma unroll
                    for (int t = 0; t < RPT; t += 4) {
                        *reinterpret_cast<f32x4*>(ai + t) = f32x4{nx[t], nx[t + 1], nx[t + 2], nx[t + 3]};
                        *reinterpret_cast<f32x4*>(aj + t) = f32x4{ny[t], ny[t + 1], ny[t + 2], ny[t + 3]};
                        *reinterpret_cast<f32x4*>(vi + t) = f32x4{nvx[t], nvx[t + 1], nvx[t + 2], nvx[t + 3]};
                        *reinterpret_cast<f32x4*>(vj + t) = f32x4{nvy[t], nvy[t + 1], nvy[t + 2], nvy[t + 3]};
                    }
                } else {
#pragma unroll
                    for (int t2 = 0; t2 < RPT; ++t2) {
                        ai[t2] = nx[t2];
                        aj[t2] = ny[t2];
                        vi[t2] = nvx[t2];
                        vj[t2] = nvy[t2];
                    }
                }
            }
            {
                const int na = oa + LD, nb = ob + LD;
                oa = pi == 0 ? oa : (na == WRAP ? 0 : na);        // player P-1 stays
                ob = (pi == 0 || nb != WRAP) ? nb : 0;            // pi == 0: 0, 1, ..., P-2
            }
            __syncthreads();
        }
        sweeps_done = sweep + 1;
        if (!__syncthreads_or(rotated)) break;
    }
    if (sweeps_out != nullptr && tid == 0) sweeps_out[j] = sweeps_done;

    // Singular values = column norms; U = A diag(1/sigma).
    // The accumulated rotations leave V orthogonal but let its column norms drift by a few
    // ulps per rotation; they are reset to one here.
    if (tid < P) {
        float s = 0.f, v = 0.f;
        for (int r = 0; r < P; ++r) {
            s += A[tid * LD + r] * A[tid * LD + r];
            v += V[tid * LD + r] * V[tid * LD + r];
        }
        sig[tid] = sqrtf(s);
        vec[tid] = 1.f / sqrtf(v);
    }
    __syncthreads();
    if (tid == 0) {
        float mx = 0.f;
        for (int c = 0; c < P; ++c) mx = fmaxf(mx, sig[c]);
        int nb = 0;
        const float thr = mx * (1e-6f);
        for (int c = 0; c < P; ++c) {
            isbad[c] = !(sig[c] > thr);
            nb += isbad[c];
        }
        shared_i[0] = nb;
    }
    __syncthreads();
    for (int e = tid; e < P * P; e += NT) {
        const int c = e / P, r = e % P;
        A[c * LD + r] = isbad[c] ? 0.f : A[c * LD + r] / sig[c];
        V[c * LD + r] *= vec[c];
    }
    __syncthreads();

    // Eigen mode (P_j symmetric positive semidefinite, e.g. a Gram matrix sum y y^T): the
    // columns of V are its eigenvectors and the column norms of A its eigenvalues.  Output:
    // atom k = eigenvector of the k-th largest eigenvalue (equal values: lower column first),
    // eig_sv[k] = its square root, i.e. the k-th singular value of the underlying signal matrix.
    if (eig_sv != nullptr) {
        if (tid < P) {
            int rank = 0;
            for (int c = 0; c < P; ++c) rank += sig[c] > sig[tid] || (sig[c] == sig[tid] && c < tid);
            isbad[tid] = rank;
            // A_c = P_j V_c holds exactly (both received the same rotations), so the drift of
            // the column norms over many rotations cancels in |A_c| / |V_c|
            eig_sv[(int64_t)j * P + rank] = scale > 0.f ? sqrtf(sig[tid] * vec[tid] / scale) : 0.f;
        }
        __syncthreads();
        float* Dj = D + (int64_t)j * P * P;
        for (int e = tid; e < P * P; e += NT) Dj[isbad[e / P] * P + (e % P)] = V[(e / P) * LD + (e % P)];
        return;                                // uniform
    }

    if (shared_i[0] > 0) {                     // uniform
        for (int c = 0; c < P; ++c) {
            if (!isbad[c]) continue;           // uniform
            // the coordinate axis least covered by the columns accepted so far
            if (tid < P) {
                float s = 0.f;
                for (int cc = 0; cc < P; ++cc) s += A[cc * LD + tid] * A[cc * LD + tid];
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
            // two Gram-Schmidt passes of e_rs against the accepted columns
            float w = 0.f;
            if (tid < P) {
                float s = (tid == rs) ? 1.f : 0.f;
                for (int cc = 0; cc < P; ++cc) s -= A[cc * LD + rs] * A[cc * LD + tid];
                w = s;
                vec[tid] = s;
            }
            __syncthreads();
            if (tid < P) {
                float dsum = 0.f;
                for (int r = 0; r < P; ++r) dsum += A[tid * LD + r] * vec[r];
                coefs[tid] = dsum;
            }
            __syncthreads();
            if (tid < P) {
                for (int cc = 0; cc < P; ++cc) w -= coefs[cc] * A[cc * LD + tid];
            }
            __syncthreads();
            if (tid < P) vec[tid] = w;
            __syncthreads();
            if (tid < P) {
                float nrm = 0.f;
                for (int r = 0; r < P; ++r) nrm += vec[r] * vec[r];
                A[c * LD + tid] = w / sqrtf(nrm);
            }
            __syncthreads();
        }
    }

    // Q = U V^T, written atom-major: D[j][k][r] = sum_c U[r][c] V[k][c].
    constexpr int TILES = (P / 4) * (P / 4);
    float* Dj = D + (int64_t)j * P * P;
    for (int tile = tid; tile < TILES; tile += NT) {
        const int q0 = 4 * (tile % (P / 4)), k0 = 4 * (tile / (P / 4));
        float o[4][4] = {};
        for (int c = 0; c < P; ++c) {
            const f32x4 u = *reinterpret_cast<const f32x4*>(&A[c * LD + q0]);
            const f32x4 v = *reinterpret_cast<const f32x4*>(&V[c * LD + k0]);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) o[a][b] += v[a] * u[b];
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            f32x4 row = {o[a][0], o[a][1], o[a][2], o[a][3]};
            *reinterpret_cast<f32x4*>(&Dj[(k0 + a) * P + q0]) = row;
            // the same four values in the coding kernel's operand orders
            if (dsw != nullptr) store_operand_f32<P>(dsw, j * P + k0 + a, q0 >> 2, row);
            if (dsb != nullptr) store_operand_split<P>(dsb, j * P + k0 + a, q0 >> 2, row);
        }
    }
}

}  // namespace

// TPP = 16 lanes per column pair (4 and 8 were measured slower at every p).
static hipError_t launch_jacobi(int p, int K, const float* M, const int32_t* counts, float* D,
                                float* eig_sv, float* dsw, unsigned* dsb, int32_t* sweeps,
                                const int32_t* only, hipStream_t st) {
    constexpr int TPP = 16;
    const float done = kPolarDone;
    switch (p) {
        case 16: hipLaunchKernelGGL((polar_kernel<16, TPP>), dim3(K), dim3(8 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, sweeps, only); break;
        case 32: hipLaunchKernelGGL((polar_kernel<32, TPP>), dim3(K), dim3(16 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, sweeps, only); break;
        case 64: hipLaunchKernelGGL((polar_kernel<64, TPP>), dim3(K), dim3(32 * TPP), 0, st, M, counts, D, eig_sv, done, dsw, dsb, sweeps, only); break;
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
    unsigned* dsb = write_ops == 2 ? ws.dsb : nullptr;
    if (!ns) return launch_jacobi(p, K, M, counts, D, eig_sv, dsw, dsb, ws.sweeps, nullptr, st);
    // Newton-Schulz for every block; the Jacobi SVD only for the ones it flags.
    hipError_t e = launch_polar_ns(p, K, M, counts, D, dsw, dsb, ws.ns_fallback, ws.sweeps, st);
    if (e != hipSuccess) return e;
    return launch_jacobi(p, K, M, counts, D, nullptr, dsw, dsb, ws.sweeps, ws.ns_fallback, st);
}

}  // namespace sbo
