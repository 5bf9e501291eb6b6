// One-sided (Hestenes) Jacobi SVD of one p x p matrix held in LDS, with the U V^T epilogue:
// the body of the batched SVD update Q_j = U V^T (Algorithm 1, steps 6-7), shared by the
// stand-alone kernel (one workgroup per block, polar_jacobi.hip) and by the Newton-Schulz kernel,
// whose workgroup continues here for a block on which the iteration does not converge
// (polar_ns.hip).
//
// Plane rotations are applied from the right to the columns of A = P_j and to V (starting at I)
// until all columns of A are mutually orthogonal; then A = U diag(sigma) and
// P_j = U diag(sigma) V^T, so Q_j = sum_c (A_c / sigma_c) V_c^T.  p/2 disjoint column pairs
// (round-robin tournament) are rotated concurrently, TPP lanes per pair, one barrier per
// tournament round.  Columns whose norm vanishes (rank-deficient P_j) are replaced by an
// orthonormal completion, which is a valid choice of U there.
#pragma once

#include "device_utils.h"

namespace sbo {

constexpr int kJacobiMaxSweeps = 30;
// A pair is rotated while |a_i . a_j| > kJacobiTol |a_i| |a_j|.  Convergence is quadratic: a
// sweep in which every pair already had a cosine below `done` leaves cosines of the order of
// done^2 behind, so it is the last one and no sweep is spent on verifying.
constexpr float kJacobiTol = 1e-6f;

// Where the entries of the p x p input come from: a finished matrix (M, atom-major), or the
// per-piece partial matrices of the block, summed in piece order (the same order and therefore
// the same bits as accum_reduce_kernel).
struct BlockMatrixSource {
    const float* M;         // finished matrix of this block, or nullptr
    const float* partial;   // [pieces][p*p]
    int pc_beg, pc_end;     // this block's pieces
    int pp;                 // p * p
    __device__ __forceinline__ float get(int e) const {
        if (M != nullptr) return M[e];
        float s = 0.f;
        for (int pc = pc_beg; pc < pc_end; ++pc) s += partial[(int64_t)pc * pp + e];
        return s;
    }
};

// LDS the routine needs, in floats (A and V with leading dimension p + 4, five small arrays).
template <int P>
constexpr int jacobi_lds_floats() {
    return 2 * P * (P + 4) + 5 * P + 4;
}

// Every thread of a workgroup of (P / 2) * TPP threads must call this with the same arguments.
// lds: jacobi_lds_floats<P>() floats, 16-byte aligned.  Dj: this block's atoms (written).
// eig_sv != nullptr: eigen mode (see below), eig_sv[0..P) receives the singular values.
template <int P, int TPP>
__device__ __forceinline__ void jacobi_block(const BlockMatrixSource& src, float* __restrict__ Dj,
                                             float* __restrict__ eig_sv, float done,
                                             float* __restrict__ dsw, unsigned* __restrict__ dsb, int dsb_kind, int j,
                                             int32_t* __restrict__ sweeps_out, float* lds) {
    constexpr int LD = P + 4;
    constexpr int NT = (P / 2) * TPP;          // threads: TPP lanes per column pair
    constexpr int RPT = P / TPP;               // contiguous rows per lane in a rotation
    constexpr int kMaxSweeps = kJacobiMaxSweeps;
    constexpr float kTol = kJacobiTol;
    static_assert(TPP == 4 || TPP == 8 || TPP == 16, "lanes per pair");
    static_assert(RPT >= 1 && P % TPP == 0, "rows per lane");
    float* A = lds;
    float* V = A + P * LD;
    float* sig = V + P * LD;
    float* coefs = sig + P;
    float* vec = coefs + P;
    int* isbad = reinterpret_cast<int*>(vec + P);
    int* shared_i = isbad + P;                 // 2 ints (+ P spare)
    const int tid = threadIdx.x;

    // Load P_j scaled by 1 / max|entry| (the orthogonal factor does not depend on scale;
    // this keeps the squared norms below well inside the fp32 range).
    float mx = 0.f;
    for (int e = tid; e < P * P; e += NT) mx = fmaxf(mx, fabsf(src.get(e)));
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
        A[c * LD + r] = src.get(e) * scale;
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
    if (sweeps_out != nullptr && tid == 0) *sweeps_out = sweeps_done;

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
            eig_sv[rank] = scale > 0.f ? sqrtf(sig[tid] * vec[tid] / scale) : 0.f;
        }
        __syncthreads();
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
            if (dsb != nullptr) store_operand_parts<P>(dsb, dsb_kind, j * P + k0 + a, q0 >> 2, row);
        }
    }
}

}  // namespace sbo
