// Orthogonal polar factor Q_j = U V^T of P_j (Algorithm 1, steps 6-7) for p <= 64 by the
// Newton-Schulz iteration X <- X (3 I - X^T X) / 2 on the matrix cores, one workgroup per block.
//
// U V^T is the orthogonal polar factor of P_j, and for a matrix scaled to singular values in
// (0, sqrt(3)) the iteration converges to it quadratically; each step is two p x p x p products,
// which are dense contractions, where the Jacobi SVD is p - 1 dependent rounds of plain ALU
// work per sweep.  The block matrices P_j = Y_j X_j^T of this method are well conditioned
// (condition numbers of 3 to 60 on the benchmark workloads), so 4 to 9 steps reach fp32
// accuracy.  A block that has not converged after max_iters steps (rank-deficient or nearly
// so, zero, NaN) is handed, in the same workgroup, to the one-sided Jacobi SVD (jacobi_block.h),
// which also supplies the orthonormal completion a vanishing singular value needs.
//
// The products run on the bf16 matrix cores at fp32 accuracy: X, its transpose and G = X^T X
// are kept in LDS as three bf16 parts per entry (their exact sum is the fp32 value, see
// device_utils.h), row-major, so that every MFMA operand is one 16-byte LDS read, and the six
// partial products above 2^-24 are accumulated in fp32 (v_mfma_f32_32x32x16_bf16).  Every
// wavefront owns one 32 x 32 tile of X in fp32 registers.
//
// The same launch can (a) sum the per-piece partial matrices of the fused select + accumulate
// kernel on the way in, in piece order, which saves the separate reduction launch, and (b) form
// the total squared error of the coding pass in extra workgroups.
//
// The stored matrix is atom-major (the transpose of P_j); the polar factor of the transpose is
// the transpose of the polar factor, so iterating on the stored matrix yields D[j] directly.
#include "sbo_internal.h"
#include "device_utils.h"
#include "jacobi_block.h"
#include "sq_total.h"

namespace sbo {

namespace {

// upper half of a -> low half of the result, upper half of b -> high half
__device__ __forceinline__ unsigned pack_upper(unsigned a, unsigned b) {
    return __builtin_amdgcn_perm(b, a, 0x07060302u);
}

struct NsArgs {
    const float* M;            // [K][p][p] finished matrices, or nullptr: sum the pieces
    const float* partial;      // [pieces][p][p] (M == nullptr)
    const int32_t* offsets;    // [K+1] (M == nullptr): the grouping the pieces were cut from
    int piece;                 // signals per piece
    const int32_t* counts;     // [K] or nullptr
    float* D;
    float* dsw;
    unsigned* dsb;
    int dsb_kind;              // 2 = three bf16 parts, 3 = two fp16 parts (device_utils.h)
    int32_t* fallback;         // [K] 1 = the block went to the Jacobi SVD
    int32_t* iters_out;        // [K] minus the Newton-Schulz steps, or the Jacobi sweeps
    int max_iters;
    int K;
    // total squared error (extra workgroups), or sq_out == nullptr
    const float* err;
    int64_t m;
    double* sq_part;
    int* sq_counter;
    double* sq_out;
    int nb;
};

template <int P>
constexpr int ns_threads() {
    return P == 64 ? 256 : 64;
}
template <int P>
constexpr int ns_pad() {
    return P == 64 ? 64 : 32;
}
// dynamic LDS: nine bf16 planes [PAD][PAD + 8] (the Jacobi routine reuses this part) | fp32
// scratch [PAD][PAD + 4] | vec, wec [PAD] | red[8]
template <int P>
constexpr size_t ns_front_bytes() {
    constexpr int PAD = ns_pad<P>();
    const size_t planes = (size_t)9 * PAD * (PAD + 8) * 2;
    const size_t jac = (size_t)jacobi_lds_floats<P>() * 4;
    return ((planes > jac ? planes : jac) + 15) / 16 * 16;
}
template <int P>
constexpr size_t ns_lds_bytes() {
    constexpr int PAD = ns_pad<P>();
    return ns_front_bytes<P>() + (size_t)PAD * (PAD + 4) * 4 + (size_t)2 * PAD * 4 + 8 * 4;
}

template <int P>
__global__ __launch_bounds__(ns_threads<P>()) void polar_ns_kernel(NsArgs g) {
    constexpr int T = P == 64 ? 2 : 1;         // 32-wide tiles per side
    constexpr int NTH = ns_threads<P>();
    constexpr int PAD = ns_pad<P>();           // padded dimension (p = 16 sits in one tile)
    constexpr int LDB = PAD + 8;               // row stride of a bf16 plane (rows stay 16-byte aligned,
                                               // eight consecutive rows cover all LDS banks)
    constexpr int LDF = PAD + 4;               // row stride of the fp32 scratch
    constexpr int KS16 = PAD / 16;
    constexpr int PLANE = PAD * LDB;           // bf16 elements per plane
    constexpr int TPP_FALLBACK = NTH / (P / 2);          // the Jacobi routine with this workgroup's threads
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    unsigned short* Xp = reinterpret_cast<unsigned short*>(lds_raw);      // [3][PAD][LDB]
    unsigned short* Xtp = Xp + 3 * PLANE;
    unsigned short* Gp = Xtp + 3 * PLANE;                                 // holds G^T
    float* F = reinterpret_cast<float*>(lds_raw + ns_front_bytes<P>());   // [PAD][LDF]
    float* vec = F + PAD * LDF;
    float* wec = vec + PAD;
    float* red = wec + PAD;

    const int tid = threadIdx.x;
    if ((int)blockIdx.x >= g.K) {              // uniform: the workgroups of the squared-error total
        const int b = (int)blockIdx.x - g.K;
        if (g.sq_out != nullptr && b < g.nb)
            sq_total_part<NTH>(g.err, g.m, b, g.nb, g.sq_part, g.sq_counter, g.sq_out,
                               reinterpret_cast<double*>(lds_raw));
        return;
    }
    const int j = blockIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;
    const int ta = wave / T, tb = wave % T;    // this wavefront's tile of X
    if (g.counts != nullptr && g.counts[j] == 0) {       // uniform: block keeps its basis
        if (tid == 0) {
            g.fallback[j] = 0;
            if (g.iters_out != nullptr) g.iters_out[j] = 0;
        }
        return;
    }

    // Where P_j comes from.  Pieces: block j' has ceil(n_j' / piece) of them, in block order.
    BlockMatrixSource src = {nullptr, g.partial, 0, 0, P * P};
    if (g.M != nullptr) {
        src.M = g.M + (int64_t)j * P * P;
    } else {
        int before = 0;
        for (int jj = tid; jj < j; jj += NTH) before += (g.offsets[jj + 1] - g.offsets[jj] + g.piece - 1) / g.piece;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) before += __shfl_xor(before, o, 64);
        if (lane == 0) red[wave] = __builtin_bit_cast(float, before);
        __syncthreads();
        before = 0;
        for (int w = 0; w < T * T; ++w) before += __builtin_bit_cast(int, red[w]);
        __syncthreads();
        src.pc_beg = before;
        src.pc_end = before + (g.offsets[j + 1] - g.offsets[j] + g.piece - 1) / g.piece;
    }

    // P_j -> the fp32 scratch, summed over the block's pieces in piece order (the order, and so
    // the bits, of accum_reduce_kernel; a finished matrix is a single piece).  16-byte loads,
    // those of kInFlight pieces in flight at a time: one workgroup has to pull a few hundred KiB
    // that other CUs have just written, and each round of loads is a trip to memory.
    {
        constexpr int U = (P * P / 4 + NTH - 1) / NTH;     // 16-byte units per thread
        constexpr int kInFlight = 8;
        const f32x4* base = reinterpret_cast<const f32x4*>(src.M != nullptr ? src.M : src.partial);
        const int pc_beg = src.M != nullptr ? 0 : src.pc_beg, pc_end = src.M != nullptr ? 1 : src.pc_end;
        f32x4 sum[U];
#pragma unroll
        for (int u = 0; u < U; ++u) sum[u] = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int pc = pc_beg; pc < pc_end; pc += kInFlight) {
            f32x4 v[kInFlight][U];
#pragma unroll
            for (int k = 0; k < kInFlight; ++k)
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int e4 = tid + NTH * u;
                    const int pcc = min(pc + k, pc_end - 1);      // clamped loads are not added
                    v[k][u] = e4 < P * P / 4 ? base[(int64_t)pcc * (P * P / 4) + e4] : f32x4{0.f, 0.f, 0.f, 0.f};
                }
#pragma unroll
            for (int k = 0; k < kInFlight; ++k)
                if (pc + k < pc_end) {                            // uniform
#pragma unroll
                    for (int u = 0; u < U; ++u) sum[u] += v[k][u];
                }
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int e4 = tid + NTH * u;
            if (e4 < P * P / 4) *reinterpret_cast<f32x4*>(&F[(e4 / (P / 4)) * LDF + 4 * (e4 % (P / 4))]) = sum[u];
        }
        __syncthreads();
    }
    // Register q of lane (h, n) of tile (ta, tb) is row ta*32 + (q/4)*8 + h*4 + q%4, column
    // tb*32 + n (the accumulator layout of the 32 x 32 matrix instructions).
    auto row_of = [&](int q) { return ta * 32 + (q >> 2) * 8 + h * 4 + (q & 3); };
    const int col = tb * 32 + n;
    float xr[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        const int row = row_of(q);
        xr[q] = (row < P && col < P) ? F[row * LDF + col] : 0.f;
    }
    __syncthreads();                           // F is rewritten below

    // tile -> three bf16 planes, transposed: dst[c][r] = v[r][c]; four consecutive rows of a
    // lane's column are 8 bytes of a plane row
    auto store_transposed = [&](unsigned short* dst, const float (&v)[16]) {
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const TriWord a = split_trunc(v[4 * q4]), b = split_trunc(v[4 * q4 + 1]);
            const TriWord c = split_trunc(v[4 * q4 + 2]), d = split_trunc(v[4 * q4 + 3]);
            const int at = col * LDB + ta * 32 + q4 * 8 + h * 4;
            *reinterpret_cast<u32x2*>(dst + at) = u32x2{pack_upper(a.hi, b.hi), pack_upper(c.hi, d.hi)};
            *reinterpret_cast<u32x2*>(dst + PLANE + at) = u32x2{pack_upper(a.mid, b.mid), pack_upper(c.mid, d.mid)};
            *reinterpret_cast<u32x2*>(dst + 2 * PLANE + at) = u32x2{pack_upper(a.lo, b.lo), pack_upper(c.lo, d.lo)};
        }
    };
    // tile -> three bf16 planes, row-major: dst[r][c] = v[r][c]; neighbouring lanes hold
    // neighbouring columns, so a lane pair exchanges half of its values and each lane writes
    // (column pair) words of every other row
    auto store_rowmajor = [&](unsigned short* dst, const float (&v)[16]) {
        const bool odd = n & 1;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float e = v[2 * k], o = v[2 * k + 1];
            const float got = dpp_f<kDppXor1>(odd ? e : o);
            const TriWord lo = split_trunc(odd ? got : e), hi = split_trunc(odd ? o : got);
            const int at = row_of(2 * k + (odd ? 1 : 0)) * LDB + tb * 32 + (n & ~1);
            *reinterpret_cast<unsigned*>(dst + at) = pack_upper(lo.hi, hi.hi);
            *reinterpret_cast<unsigned*>(dst + PLANE + at) = pack_upper(lo.mid, hi.mid);
            *reinterpret_cast<unsigned*>(dst + 2 * PLANE + at) = pack_upper(lo.lo, hi.lo);
        }
    };
    // tile (ta, tb) of A B^T for row-major planes A, B: sum over k of A[ta*32 + n][k] B[tb*32 + n][k],
    // six partial products per 16 dims, smallest first, two accumulators alternating
    auto abt_tile = [&](const unsigned short* A, const unsigned short* B, float (&out)[16]) {
        constexpr int TA[6] = {2, 0, 1, 1, 0, 0};
        constexpr int TB[6] = {0, 2, 1, 0, 1, 0};
        f32x16 acc[2];
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            acc[0][q] = 0.f;
            acc[1][q] = 0.f;
        }
        const unsigned short* ar = A + (ta * 32 + n) * LDB + h * 8;
        const unsigned short* br = B + (tb * 32 + n) * LDB + h * 8;
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            u32x4 a[3], b[3];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) {
                a[pl] = *reinterpret_cast<const u32x4*>(ar + pl * PLANE + ks * 16);
                b[pl] = *reinterpret_cast<const u32x4*>(br + pl * PLANE + ks * 16);
            }
#pragma unroll
            for (int t = 0; t < 6; ++t)
                acc[ks & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[TA[t]]),
                                                                      __builtin_bit_cast(bf16x8, b[TB[t]]),
                                                                      acc[ks & 1], 0, 0, 0);
        }
#pragma unroll
        for (int q = 0; q < 16; ++q) out[q] = KS16 > 1 ? acc[0][q] + acc[1][q] : acc[0][q];
    };
    // largest |v - I| over the valid part of the tile
    auto deviation = [&](const float (&v)[16]) {
        float dev = 0.f;
#pragma unroll
        for (int q = 0; q < 16; ++q) {
            const int row = row_of(q);
            if (row < P && col < P) dev = fmaxf(dev, fabsf(v[q] - (row == col ? 1.f : 0.f)));
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

    // G0 = X^T X of the unscaled input (X^T X = Xt Xt^T: both operands are rows of Xt), in fp32
    // in F for the scale estimate.
    store_transposed(Xtp, xr);
    __syncthreads();
    float gt[16];
    abt_tile(Xtp, Xtp, gt);
#pragma unroll
    for (int q = 0; q < 16; ++q) F[row_of(q) * LDF + col] = gt[q];
    __syncthreads();

    // Scale so that the largest singular value is about one.  sigma_max^2 is the largest
    // eigenvalue of G = X^T X.  The iteration sends every singular value in (0, sqrt(3)) to +1,
    // one in (sqrt(3), sqrt(5)) to -1 (an orthogonal matrix that is NOT U V^T, and which the
    // deviation test cannot tell apart), so the scale must be a guaranteed bound: the largest
    // absolute row sum of G is at least its largest eigenvalue, and dividing G by that sum / 2.9
    // keeps every scaled sigma^2 at or below 2.9.  That bound alone is often two to three times
    // too large, which costs iterations; a Rayleigh quotient after a few power-iteration steps
    // from the vector of absolute row sums is a lower estimate that is usually tight, so the
    // scale is the larger of (1.08 x that quotient) and (row-sum bound / 2.9).
    if (tid < P) {
        float rs = 0.f;
        for (int b = 0; b < P; ++b) rs += fabsf(F[tid * LDF + b]);
        vec[tid] = rs;
    }
    __syncthreads();
    float rsmax = 0.f;                         // every thread, same order: same value
    for (int a = 0; a < P; ++a) rsmax = fmaxf(rsmax, vec[a]);
    float s2 = 0.f;
    for (int round = 0; round < 4; ++round) {
        if (tid < P) {
            float w = 0.f;
            for (int b = 0; b < P; ++b) w += F[tid * LDF + b] * vec[b];
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
    const bool rq_ok = s2 > 0.f && s2 < 3e38f; // zero, infinite or NaN input: not for this iteration
    s2 = fmaxf(s2, rsmax * (1.f / 2.9f));
    const bool ok = rq_ok && s2 < 3e38f;
    const float inv = ok ? __builtin_amdgcn_rsqf(s2) : 0.f;
#pragma unroll
    for (int q = 0; q < 16; ++q) {
        xr[q] *= inv;
        gt[q] *= inv * inv;
    }
    store_rowmajor(Xp, xr);
    store_transposed(Xtp, xr);                 // (every wavefront has finished reading the unscaled Xt)
    store_transposed(Gp, gt);
    float dev = deviation(gt);
    int it = 0;
    bool converged = false;
    while (ok) {
        // d = max |X^T X - I|; below 2e-4 the step that follows is the last (quadratic
        // convergence leaves about d^2 behind).  The barriers inside also publish the planes.
        const float d = wg_max(dev);
        const bool last = d < 2e-4f;
        if (!(d < 4.f)) break;                 // NaN or diverging: leave it to the Jacobi SVD

        // X <- 1.5 X - 0.5 X G; X G = X (G^T)^T: rows of X against rows of the stored G^T
        float xg[16];
        abt_tile(Xp, Gp, xg);
#pragma unroll
        for (int q = 0; q < 16; ++q) xr[q] = 1.5f * xr[q] - 0.5f * xg[q];
        __syncthreads();                       // every wavefront has read the old planes
        ++it;
        if (last) {
            converged = true;
            break;
        }
        if (it >= g.max_iters) break;
        store_rowmajor(Xp, xr);
        store_transposed(Xtp, xr);
        __syncthreads();
        abt_tile(Xtp, Xtp, gt);
        store_transposed(Gp, gt);              // G was last read before the barrier above
        dev = deviation(gt);
    }

    if (!converged) {                          // uniform: the Jacobi SVD of this block, right here
        __syncthreads();
        if (tid == 0) g.fallback[j] = 1;
        jacobi_block<P, TPP_FALLBACK>(src, g.D + (int64_t)j * P * P, nullptr, kPolarDone, g.dsw, g.dsb, g.dsb_kind, j,
                                      g.iters_out ? g.iters_out + j : nullptr,
                                      reinterpret_cast<float*>(lds_raw));
        return;
    }
    if (tid == 0) {
        g.fallback[j] = 0;
        if (g.iters_out != nullptr) g.iters_out[j] = -it;   // negative: Newton-Schulz steps, not sweeps
    }

    // D[j][k][:] = row k of X, through the fp32 scratch so that a thread holds four consecutive
    // dims of a row; the same values in the coding kernels' operand orders
#pragma unroll
    for (int q = 0; q < 16; ++q) F[row_of(q) * LDF + col] = xr[q];
    __syncthreads();
    float* Dj = g.D + (int64_t)j * P * P;
    for (int u = tid; u < P * P / 4; u += NTH) {
        const int k = u / (P / 4), d4 = u % (P / 4);
        const f32x4 row = *reinterpret_cast<const f32x4*>(&F[k * LDF + 4 * d4]);
        *reinterpret_cast<f32x4*>(&Dj[k * P + 4 * d4]) = row;
        if (g.dsw != nullptr) store_operand_f32<P>(g.dsw, j * P + k, d4, row);
        if (g.dsb != nullptr) store_operand_parts<P>(g.dsb, g.dsb_kind, j * P + k, d4, row);
    }
}

template <int P>
hipError_t launch_ns_p(const NsArgs& a, LdsRaised* raised, hipStream_t st) {
    constexpr size_t lds = ns_lds_bytes<P>();
    if (lds > 64 * 1024) {
        if (raised == nullptr) return hipErrorInvalidValue;
        if (hipError_t e = raised->ensure(reinterpret_cast<const void*>(&polar_ns_kernel<P>), lds); e != hipSuccess)
            return e;
    }
    hipLaunchKernelGGL((polar_ns_kernel<P>), dim3(a.K + (a.sq_out ? a.nb : 0)), dim3(ns_threads<P>()), lds, st, a);
    return hipGetLastError();
}

}  // namespace

// Newton-Schulz (Jacobi SVD in the same workgroup for a block that does not converge) for all K
// blocks.  fallback[j] = 1 for every block that went to the Jacobi SVD.
// M == nullptr: P_j = the sum of block j's pieces in partial (cut from offsets with `piece`
// signals per piece).  sq.out != nullptr: extra workgroups form *sq.out = sum of sq.err[0..m).
hipError_t launch_polar_ns(int p, int K, const float* M, const float* partial, const int32_t* offsets,
                           int piece, const int32_t* counts, float* D, float* dsw, unsigned* dsb, int dsb_kind,
                           int32_t* fallback, int32_t* iters, const SqTotalArgs& sq, LdsRaised* raised,
                           hipStream_t st) {
    constexpr int kMaxIters = 26;
    NsArgs a;
    a.M = M;
    a.partial = partial;
    a.offsets = offsets;
    a.piece = piece;
    a.counts = counts;
    a.D = D;
    a.dsw = dsw;
    a.dsb = dsb;
    a.dsb_kind = dsb_kind;
    a.fallback = fallback;
    a.iters_out = iters;
    a.max_iters = kMaxIters;
    a.K = K;
    a.err = sq.err;
    a.m = sq.m;
    a.sq_part = sq.part;
    a.sq_counter = sq.counter;
    a.sq_out = sq.out;
    a.nb = sq.out != nullptr ? sq.nb : 0;
    if (M == nullptr && (partial == nullptr || offsets == nullptr || piece < 1)) return hipErrorInvalidValue;
    switch (p) {
        case 16: return launch_ns_p<16>(a, raised, st);
        case 32: return launch_ns_p<32>(a, raised, st);
        case 64: return launch_ns_p<64>(a, raised, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
