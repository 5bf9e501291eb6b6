// Sparse-coding stage 1: for every signal, the kept energy in every orthobase and
// the block where it is largest (Section 2, eq. (4); Section 3.1).
//
// c = Q_j^T y is a dense contraction for the matrix cores: 32 x 32 MFMA tiles with atoms
// on the M axis and signals on the N axis, so that the accumulator tile leaves every
// signal's coefficients in just two lanes (l and l^32).  The s0 largest magnitudes
// are then found in registers by compare-exchange networks, merged across the lane
// pair, squared and summed, and compared against the running best block.  The K*p x m
// projection never leaves the register file.
//
// Dictionary rows (atom k of block j = row j*p + k) are streamed through LDS in stages of
// 64 (p = 256: 32) rows, double-buffered, in the exact per-lane order the MFMA A operand
// wants, so every LDS read is one conflict-free 16-byte load per lane.  A small kernel
// first rewrites D into that order (zero-padded to whole stages), which makes the
// per-stage copy global -> registers -> LDS linear on both sides.
//
// Three arithmetics, chosen per context (SBO_OPT_CODING_ARITH), each with its own kernels:
//   energy_kernel                          the fp32 matrix instruction (32x32x2);
//   energy_split_kernel MODE 0 / 1 / 2,    every fp32 operand as three bf16 parts, six (screening:
//   energy_split_wide_kernel<false>        three) partial products on the bf16 matrix cores;
//   energy_split_kernel MODE 3,            every (scaled) fp32 operand as two fp16 parts, three
//   energy_split_wide_kernel<true>         partial products on the fp16 matrix cores (the default).
#include "sbo_internal.h"
#include "device_utils.h"

#include <type_traits>

namespace sbo {

namespace {

// Both halves of a register pair after v_permlane32_swap(x, z):
//   first  = [x.lo, z.lo]   second = [x.hi, z.hi]   (lo/hi = lanes 0-31 / 32-63)
struct SwapPair {
    float first, second;
};
__device__ __forceinline__ SwapPair swap32(float x, float z) {
    auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, x),
                                              __builtin_bit_cast(unsigned, z), false, false);
    const unsigned u0 = r[0], u1 = r[1];   // copy out first: a bit_cast applied to a vector
                                           // element expression reads element 0 for both
    return {__builtin_bit_cast(float, u0), __builtin_bit_cast(float, u1)};
}

// Sum of squares of the N largest magnitudes of the union of two sorted (descending)
// lists, one per lane of a lane pair, of which the first N <= S entries are used (the N
// largest of the union lie among the N largest of either list); valid and bitwise equal in
// both lanes.  The N largest of the union are max(a_i(lo), a_{N-1-i}(hi)); the high lane
// reverses its list so that both operands of one maximum sit in the same register, and one
// swap serves two maxima.
template <int S, int N>
__device__ __forceinline__ float pair_fold_energy(const float (&a)[S], bool hi) {
    static_assert(N >= 1 && N <= S, "fold width");
    if constexpr (N == 1) {
        SwapPair t = swap32(a[0], a[0]);
        const float m = fmaxf(t.first, t.second);
        return m * m;
    } else {
        // r_i = hi ? a_{N-1-i} : a_i as one bit-select per element (written with integer
        // masks so that it is not rewritten into a lane-dependent index into a[])
        const unsigned msk = hi ? 0xffffffffu : 0u;
        float r[N];
#pragma unroll
        for (int i = 0; i < N; ++i) {
            const unsigned fwd = __builtin_bit_cast(unsigned, a[i]);
            const unsigned rev = __builtin_bit_cast(unsigned, a[N - 1 - i]);
            r[i] = __builtin_bit_cast(float, (rev & msk) | (fwd & ~msk));
        }
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i + 1 < N; i += 2) {
            SwapPair t = swap32(r[i], r[i + 1]);
            const float m = fmaxf(t.first, t.second);   // low lanes: maximum i, high: i+1
            sum = fmaf(m, m, sum);
        }
        if constexpr (N % 2 == 1) {            // the middle maximum: the same in both lanes, counted once
            SwapPair t = swap32(r[N - 1], r[N - 1]);
            const float m = fmaxf(t.first, t.second);
            sum = fmaf(hi ? 0.f : m, m, sum);
        }
        SwapPair t = swap32(sum, sum);
        return t.first + t.second;
    }
}

// Energy (sum of squares) of the s0 largest magnitudes in the union of two sorted
// (descending) S-lists of magnitudes, one per lane of a lane pair.  SX = s0 when it is known
// at compile time (S/2 < SX <= S), 0 otherwise.
template <int S, int SX>
__device__ __forceinline__ float pair_list_energy(const float (&a)[S], int s0, bool hi) {
    if constexpr (SX > 0) {
        return pair_fold_energy<S, SX>(a, hi);
    } else {
        float b[S], c[S];
#pragma unroll
        for (int i = 0; i < S; ++i) b[i] = other_half(a[i]);
#pragma unroll
        for (int i = 0; i < S; ++i) c[i] = fmaxf(a[i], b[S - 1 - i]);
        bitonic_merge_desc<S>(c);
        float e = 0.f;
#pragma unroll
        for (int t = 0; t < S; ++t) e += (t < s0) ? c[t] * c[t] : 0.f;
        return e;
    }
}

// The same for the NV magnitudes x held by this lane and the NV held by its partner
// (one block's coefficients of one signal).  S = power of two >= s0, S <= 2 * NV.
template <int NV, int S, int SX>
__device__ __forceinline__ float pair_top_energy(const float (&x)[NV], int s0, bool hi) {
    constexpr int L = S < NV ? S : NV;
    float a[L];
    top_sorted<NV, L>(x, a);
    if constexpr (L == S) {
        return pair_list_energy<S, SX>(a, s0, hi);
    } else {
        static_assert(2 * L == S, "sort width exceeds the coefficients of a lane pair");
        float c[S];
#pragma unroll
        for (int i = 0; i < L; ++i) {
            c[i] = a[i];
            c[S - 1 - i] = other_half(a[i]);
        }
        bitonic_merge_desc<S>(c);
        float e = 0.f;
#pragma unroll
        for (int t = 0; t < S; ++t) e += (t < s0) ? c[t] * c[t] : 0.f;
        return e;
    }
}

// Dsw[stage][(mt*QN + q)*64 + hh*32 + nn] = dims hh*P/2 + 4q .. +3 of row stage*64 + mt*32 + nn
// (rows past K*P are zero): the order in which a wavefront's lanes consume the A operand.
template <int P>
__global__ __launch_bounds__(256) void dict_swizzle_kernel(const float* __restrict__ D, int K,
                                                           f32x4* __restrict__ Dsw) {
    constexpr int QN = P / 8;
    constexpr int STAGE_F4 = 2 * QN * 64;
    const f32x4* D4 = reinterpret_cast<const f32x4*>(D);
    const int rows = K * P;
    const int s = blockIdx.x;
    for (int f = threadIdx.x; f < STAGE_F4; f += 256) {
        const int nn = f & 31, hh = (f >> 5) & 1, mq = f >> 6;
        const int q = mq % QN, mt = mq / QN;
        const int grow = s * 64 + mt * 32 + nn;
        const int d4 = hh * QN + q;
        Dsw[(int64_t)s * STAGE_F4 + f] =
            grow < rows ? D4[(int64_t)grow * (P / 4) + d4] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
}

// The same dictionary in the split operand order (see device_utils.h): every entry as three
// bf16 parts, 8 consecutive dims of a row per 16-byte unit and part.
template <int P, int NPL>
__global__ __launch_bounds__(256) void dict_swizzle_split_kernel(const float* __restrict__ D, int K,
                                                                 u32x4* __restrict__ Dsb) {
    constexpr int KS16 = P / 16;
    constexpr int STAGE_U = 2 * KS16 * NPL * 64;
    const f32x4* D4 = reinterpret_cast<const f32x4*>(D);
    const int rows = K * P;
    const int s = blockIdx.x;
    for (int g = threadIdx.x; g < 2 * KS16 * 64; g += 256) {       // (mt, ks, lane)
        const int lane = g & 63, mk = g >> 6;
        const int nn = lane & 31, hh = lane >> 5, ks = mk % KS16, mt = mk / KS16;
        const int grow = s * 64 + mt * 32 + nn;
        f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
        if (grow < rows) {
            v0 = D4[(int64_t)grow * (P / 4) + ks * 4 + hh * 2];
            v1 = D4[(int64_t)grow * (P / 4) + ks * 4 + hh * 2 + 1];
        }
        u32x4* out = Dsb + (int64_t)s * STAGE_U + (mk * NPL) * 64 + lane;
        if constexpr (NPL == 3) {
            const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
            const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
            out[0] = u32x4{a.hi, b.hi, c.hi, d.hi};
            out[64] = u32x4{a.mid, b.mid, c.mid, d.mid};
            out[128] = u32x4{a.lo, b.lo, c.lo, d.lo};
        } else {
            constexpr float sc = kF16DictScale;
            const F16x2Pair a = split_f16x2(v0.x * sc, v0.y * sc), b = split_f16x2(v0.z * sc, v0.w * sc);
            const F16x2Pair c = split_f16x2(v1.x * sc, v1.y * sc), d = split_f16x2(v1.z * sc, v1.w * sc);
            out[0] = u32x4{a.hi, b.hi, c.hi, d.hi};
            out[64] = u32x4{a.lo, b.lo, c.lo, d.lo};
        }
    }
}

template <int P, int S, int NT, int SX>
__global__ __launch_bounds__(256) void energy_kernel(const float* __restrict__ Y, int m,
                                                     const f32x4* __restrict__ Dsw, int K, int s0,
                                                     int32_t* __restrict__ blk,
                                                     float* __restrict__ energy,
                                                     int32_t* __restrict__ chunk_count, int chunk,
                                                     int units_per_y) {
    constexpr int KS = P / 2;            // contraction steps (each lane half covers P/2 dims)
    constexpr int QN = P / 8;            // 16-byte groups of steps per 32-row tile
    constexpr int NB = P <= 64 ? 64 / P : 1;   // blocks per 64-row stage (p <= 64)
    constexpr int SPB = P <= 64 ? 1 : P / 64;  // 64-row stages per block (p > 64)
    constexpr int NV = P <= 64 ? P / 2 : 32;   // coefficients per lane per block and stage
    constexpr int STAGE_F4 = 2 * QN * 64;
    constexpr int FPT = STAGE_F4 / 256;  // 16-byte pieces each thread moves per stage
    static_assert(P == 16 || P == 32 || P == 64 || P == 256, "unsupported p");
    static_assert(P <= 64 || S <= 32, "sort width");

    extern __shared__ f32x4 Qs_raw[];    // [2][STAGE_F4]
    f32x4(*Qs)[STAGE_F4] = reinterpret_cast<f32x4(*)[STAGE_F4]>(Qs_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;
    const int64_t sig0 = ((int64_t)blockIdx.x * 4 + wave) * (32 * NT);

    // B operand: this lane's half of the dims of NT signals, kept for the whole kernel.
    float yb[NT][KS];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int64_t i = sig0 + nt * 32 + n;
        if (i < m) {
            const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + h * KS);
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                f32x4 v = src[q];
                yb[nt][4 * q + 0] = v.x;
                yb[nt][4 * q + 1] = v.y;
                yb[nt][4 * q + 2] = v.z;
                yb[nt][4 * q + 3] = v.w;
            }
        } else {
#pragma unroll
            for (int t = 0; t < KS; ++t) yb[nt][t] = 0.f;
        }
    }

    // Small m: the blocks are split over blockIdx.y (units_per_y > 0: that many stages, for
    // p > 64 that many blocks, per workgroup row), so that the chip is filled; every row then
    // writes its own best (energy, block) per signal at offset blockIdx.y * m and
    // energy_merge_kernel picks the winner.
    const int n_stage = (K * P + 63) / 64;
    int s_beg = 0, s_end = n_stage;
    if (units_per_y > 0) {
        s_beg = min(n_stage, (int)blockIdx.y * units_per_y * SPB);
        s_end = min(n_stage, s_beg + units_per_y * SPB);
        blk += (int64_t)blockIdx.y * m;
        energy += (int64_t)blockIdx.y * m;
    }

    f32x4 pre[FPT];
    auto fetch = [&](int s) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) pre[r] = Dsw[(int64_t)s * STAGE_F4 + tid + 256 * r];
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) Qs[buf][tid + 256 * r] = pre[r];
    };

    if (s_beg < s_end) {                 // uniform
        fetch(s_beg);
        stash(0);
    }
    __syncthreads();

    int best[NT];
    float bestE[NT];
    float run[NT][S];                    // p > 64: lane's top-S magnitudes of the current block
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        best[nt] = 0;
        bestE[nt] = -1.f;
#pragma unroll
        for (int i = 0; i < S; ++i) run[nt][i] = 0.f;
    }

    for (int s = s_beg; s < s_end; ++s) {
        const int cur = (s - s_beg) & 1;
        if (s + 1 < s_end) fetch(s + 1);

        f32x16 acc[NT][2];
        const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                             0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            f32x4 a[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) a[mt] = Qs[cur][(mt * QN + q) * 64 + lane];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            a[mt][kk], yb[nt][4 * q + kk], (q == 0 && kk == 0) ? zero : acc[nt][mt],
                            0, 0, 0);
        }

        if (s + 1 < s_end) stash(cur ^ 1);

        if constexpr (P <= 64) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    float x[NV];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int f = b * NV + v;      // flattened (tile, register)
                        x[v] = fabsf(acc[nt][f >> 4][f & 15]);
                    }
                    const float e = pair_top_energy<NV, S, SX>(x, s0, h != 0);
                    const int j = s * NB + b;
                    if (j < K && e > bestE[nt]) {
                        bestE[nt] = e;
                        best[nt] = j;
                    }
                }
            }
        } else {
            // A block spans SPB stages: keep the lane's sorted top-S across them and
            // combine the lane pair after the block's last stage.
            const int part = s % SPB;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                float x[32], a[S];
#pragma unroll
                for (int f = 0; f < 32; ++f) x[f] = fabsf(acc[nt][f >> 4][f & 15]);
                top_sorted<32, S>(x, a);
                if (part == 0) {
#pragma unroll
                    for (int i = 0; i < S; ++i) run[nt][i] = a[i];
                } else {
#pragma unroll
                    for (int i = 0; i < S; ++i) run[nt][i] = fmaxf(run[nt][i], a[S - 1 - i]);
                    bitonic_merge_desc<S>(run[nt]);
                }
                if (part == SPB - 1) {
                    const float e = pair_list_energy<S, SX>(run[nt], s0, h != 0);
                    const int j = s / SPB;
                    if (j < K && e > bestE[nt]) {
                        bestE[nt] = e;
                        best[nt] = j;
                    }
                }
            }
        }
        __syncthreads();
    }

    if (h == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const int64_t i = sig0 + nt * 32 + n;
            if (i < m) {
                blk[i] = best[nt];
                energy[i] = bestE[nt];
            }
        }
    }

    // First step of the grouping (Section 3.3), folded in here: chunk_count[c][j] += number of
    // this workgroup's signals that chose block j, c = the chunk of consecutive signals the
    // workgroup lies in (chunk is a multiple of the signals per workgroup; the array is zero
    // on entry).  Integer atomics only: the sums do not depend on the order.
    if (chunk_count != nullptr) {        // uniform
        int* lh = reinterpret_cast<int*>(Qs_raw);          // the stage buffers are dead (>= 8 KiB)
        for (int j = tid; j < K; j += 256) lh[j] = 0;
        __syncthreads();
        if (h == 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (sig0 + nt * 32 + n < m) atomicAdd(&lh[best[nt]], 1);
        }
        __syncthreads();
        const int64_t c = ((int64_t)blockIdx.x * (4 * 32 * NT)) / chunk;
        for (int j = tid; j < K; j += 256)
            if (lh[j] != 0) atomicAdd(&chunk_count[c * K + j], lh[j]);
    }
}

// The same kernel with the projection on the bf16 matrix cores: every fp32 operand entry is
// the exact sum of three bf16 parts (device_utils.h), and the six partial products that matter
// at fp32 accuracy are accumulated in fp32 by v_mfma_f32_32x32x16_bf16.  Per 32 x 32 x 16 step
// that is six matrix instructions of 8 passes each where the fp32 instruction needs 8 x 16
// passes for the same 16 dims, and, unlike the fp32 matrix instruction, they run beside the
// vector ALU.  The signals' three parts stay in registers for the whole kernel (B operand, 8
// bf16 per lane and step); the dictionary arrives pre-split (Dsb) and is staged through LDS,
// double-buffered, one barrier per stage.
// A stage is 64 dictionary rows (24 KiB at p = 64), a wavefront owns 64 signals, and a
// workgroup is two teams of four wavefronts, one wavefront of each team per SIMD, half a stage
// apart: while team 0 multiplies stage s, team 1 runs the selection networks on its stage s - 1
// results, then the roles swap; both read the same LDS stage.  (p = 256: energy_split_wide_kernel.)
//
// MODE 0: as described, for every signal.
// MODE 1 (screening): only the three largest partial products (hi*hi, hi*mid, mid*hi) are formed.
//   With round-to-nearest parts |mid| <= 2^-8 |a| and |lo| <= 2^-16 |a|, so the dropped terms are
//   below 3.01 * 2^-16 |a||b|, a coefficient is off by at most kScreenCoef * ||y|| (Cauchy-Schwarz
//   over the unit atom), and a block's kept energy by at most eps = (2 sqrt(s0) kScreenCoef +
//   s0 kScreenCoef^2) ||y||^2.  A block whose screened energy lies more than 2 eps below the best
//   screened energy cannot be the true winner, so a signal whose two best screened energies are
//   more than 2 eps apart has its block decided; every other signal is appended to a list
//   (flag_ids, flag_count) and left out of the chunk histograms.
// MODE 2 (resolution): MODE 0 for the signals of that list only (ids, *count read from device
//   memory; workgroups past the end return at once): the full six products over all K blocks.  The
//   list is short, so the stages are always split over blockIdx.y (as for small m); row y leaves
//   its best (energy, block) of list entry t at blk / energy [y * m + t], and
//   energy_resolve_merge_kernel picks the winners, writes them at the listed signals and
//   completes the chunk histograms.
// Half the matrix work for all signals and the full work for the few undecided ones give the same
// blocks as the full work for all.
//
// MODE 3 (two fp16 parts, device_utils.h): the signals are scaled by a power of two each (largest
//   magnitude into [2^13, 2^14)), the dictionary by kF16DictScale, both split into hi + lo in fp16,
//   and the three products hi*lo, lo*hi, hi*hi run on v_mfma_f32_32x32x16_f16 into the one fp32
//   accumulator: half the matrix work and two thirds of the operand traffic of MODE 0, with a
//   per-term error of 3 * 2^-22 |a b| (an fp32 dot product of p terms guarantees p * 2^-24 sum |a b|).
//   The choice of the block does not see the scales (common to all blocks of a signal); the
//   energy written out is scaled back.
// Winners of the resolution pass (energy_split_kernel MODE 2): entry t of the list has one
// (energy, block) per row at part_* [y * m + t], rows in ascending block order; the winner goes to
// blk / energy of signal ids[t] and into the grouping's chunk histograms.
__global__ __launch_bounds__(256) void energy_resolve_merge_kernel(
    const float* __restrict__ part_E, const int32_t* __restrict__ part_j, int rows, int m, int K,
    const int32_t* __restrict__ ids, const int32_t* __restrict__ count, int32_t* __restrict__ blk,
    float* __restrict__ energy, int32_t* __restrict__ chunk_count, int chunk) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= min(m, *count)) return;
    int best = 0;
    float bestE = -1.f;
    for (int y = 0; y < rows; ++y) {
        const float e = part_E[(int64_t)y * m + t];
        if (e > bestE) {
            bestE = e;
            best = part_j[(int64_t)y * m + t];
        }
    }
    const int i = ids[t];
    blk[i] = best;
    energy[i] = bestE;
    if (chunk_count != nullptr) atomicAdd(&chunk_count[(int64_t)(i / chunk) * K + best], 1);
}

// Bound on a screened coefficient's error relative to ||y||: the three dropped partial products
// (3.01 * 2^-16) plus the fp32 accumulation of up to 256 terms.
constexpr float kScreenCoef = 3.01f / 65536.f + 2e-6f;

constexpr int kSplitWgWaves = 8;

template <int P, int NPL = 3>
struct SplitGeom {
    static constexpr int MTS = 2;                        // 32-row tiles per stage
    static constexpr int NT = 2;                         // 32-signal tile columns per wavefront
    static constexpr int WAVES = kSplitWgWaves;
    static constexpr bool TEAMS = true;
    static constexpr int KS16 = P / 16;                  // contraction steps of 16 dims
    static constexpr int STAGE_ROWS = 32 * MTS;
    static constexpr int STAGE_U = MTS * KS16 * NPL * 64;   // 16-byte units per stage
    static constexpr size_t LDS = (size_t)2 * STAGE_U * 16;
};

template <int P, int S, int SX, int MODE>
__global__ __launch_bounds__(64 * kSplitWgWaves) void energy_split_kernel(
    const float* __restrict__ Y, int m, const u32x4* __restrict__ Dsb, int K, int s0,
    int32_t* __restrict__ blk, float* __restrict__ energy, int32_t* __restrict__ chunk_count, int chunk,
    int units_per_y, int32_t* __restrict__ flag_ids, int32_t* __restrict__ flag_count, float margin_rel) {
    constexpr bool F16 = MODE == 3;
    constexpr int NPL = F16 ? 2 : 3;           // operand parts
    using G = SplitGeom<P, NPL>;
    constexpr int MTS = G::MTS, NT = G::NT, KS16 = G::KS16, STAGE_U = G::STAGE_U;
    constexpr int NTH = 64 * G::WAVES;
    constexpr int NB = 64 / P;                 // blocks per stage
    constexpr int SPB = 1;
    constexpr int NV = P / 2;                  // coefficients per lane per block and stage
    constexpr int FPT = (STAGE_U + NTH - 1) / NTH;         // 16-byte units each thread moves per stage
    constexpr bool kWhole = STAGE_U % NTH == 0;
    static_assert(P == 16 || P == 32 || P == 64, "unsupported p");

    extern __shared__ u32x4 Qb_raw[];    // [2][STAGE_U]
    u32x4(*Qs)[STAGE_U] = reinterpret_cast<u32x4(*)[STAGE_U]>(Qb_raw);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int team = G::TEAMS ? wave >> 2 : 0;           // wavefronts w and w + 4 share a SIMD
    const int h = lane >> 5, n = lane & 31;
    const int64_t sig0 = ((int64_t)blockIdx.x * G::WAVES + wave) * (32 * NT);
    const int m_all = m;
    if constexpr (MODE == 2) {
        m = min(m, *flag_count);                           // the listed signals only
        if ((int64_t)blockIdx.x * (G::WAVES * 32 * NT) >= m) return;   // uniform over the workgroup
    }

    // B operand: the parts of this lane's dims (ks*16 + h*8 .. +7) of NT signals.
    u32x4 yq[NT][KS16][NPL];
    int64_t sig[NT];                     // the signal of this lane in tile column nt (-1: none)
    int64_t tpos[NT];                    // where its result goes (MODE 2: its place in the list)
    float yn2[NT];                       // MODE 1: this lane's share of ||y||^2
    float unscale[NT];                   // MODE 3: 1 / (scale of the signal * scale of the dictionary)^2
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int64_t t = sig0 + nt * 32 + n;
        sig[nt] = t < m ? (MODE == 2 ? (int64_t)flag_ids[t] : t) : -1;
        tpos[nt] = t;
        const int64_t i = sig[nt];
        yn2[nt] = 0.f;
        unscale[nt] = 1.f;
        f32x4 raw[KS16][2];
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            raw[ks][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            raw[ks][1] = raw[ks][0];
            if (i >= 0) {
                const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + ks * 16 + h * 8);
                raw[ks][0] = src[0];
                raw[ks][1] = src[1];
            }
        }
        float scale = 1.f;
        if constexpr (F16) {
            float vmax = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS16; ++ks)
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    vmax = fmaxf(fmaxf(fmaxf(vmax, fabsf(raw[ks][e].x)), fmaxf(fabsf(raw[ks][e].y), fabsf(raw[ks][e].z))),
                                 fabsf(raw[ks][e].w));
            vmax = fmaxf(vmax, other_half(vmax));
            scale = f16_signal_scale(vmax);
            const float inv = 1.f / (scale * kF16DictScale);       // a power of two: exact
            unscale[nt] = inv * inv;
        }
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            const f32x4 v0 = raw[ks][0], v1 = raw[ks][1];
            if constexpr (MODE == 1)
                yn2[nt] += v0.x * v0.x + v0.y * v0.y + v0.z * v0.z + v0.w * v0.w + v1.x * v1.x + v1.y * v1.y +
                           v1.z * v1.z + v1.w * v1.w;
            if constexpr (F16) {
                const F16x2Pair a = split_f16x2(v0.x * scale, v0.y * scale), b = split_f16x2(v0.z * scale, v0.w * scale);
                const F16x2Pair c = split_f16x2(v1.x * scale, v1.y * scale), d = split_f16x2(v1.z * scale, v1.w * scale);
                yq[nt][ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
                yq[nt][ks][1] = u32x4{a.lo, b.lo, c.lo, d.lo};
            } else {
                const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
                const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
                yq[nt][ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
                yq[nt][ks][1] = u32x4{a.mid, b.mid, c.mid, d.mid};
                yq[nt][ks][2] = u32x4{a.lo, b.lo, c.lo, d.lo};
            }
        }
    }

    // Small m: the stages are split over blockIdx.y exactly as in energy_kernel.
    const int n_stage = (K * P + G::STAGE_ROWS - 1) / G::STAGE_ROWS;
    int s_beg = 0, s_end = n_stage;
    if (units_per_y > 0) {
        s_beg = min(n_stage, (int)blockIdx.y * units_per_y * SPB);
        s_end = min(n_stage, s_beg + units_per_y * SPB);
        blk += (int64_t)blockIdx.y * m_all;
        energy += (int64_t)blockIdx.y * m_all;
    }

    u32x4 pre[FPT];
    auto fetch = [&](int s) {
#pragma unroll
        for (int r = 0; r < FPT; ++r)
            if (kWhole || tid + NTH * r < STAGE_U) pre[r] = Dsb[(int64_t)s * STAGE_U + tid + NTH * r];
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int r = 0; r < FPT; ++r)
            if (kWhole || tid + NTH * r < STAGE_U) Qs[buf][tid + NTH * r] = pre[r];
    };

    int best[NT];
    float bestE[NT], secondE[NT];        // secondE (MODE 1): the second-best screened energy
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        best[nt] = 0;
        bestE[nt] = -1.f;
        secondE[nt] = -1.f;
    }

    // the partial products, smallest first: (A part, B part); screening forms the last three of
    // the bf16 list, the fp16 parts have three in all
    constexpr int TA[6] = {F16 ? 0 : 2, F16 ? 1 : 0, F16 ? 0 : 1, 1, 0, 0};
    constexpr int TB[6] = {F16 ? 1 : 0, F16 ? 0 : 2, F16 ? 0 : 1, 0, 1, 0};
    constexpr int T0 = MODE == 1 ? 3 : 0;
    constexpr int T1 = F16 ? 3 : 6;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[NT][MTS];

    // Projection of the wavefront's signals onto the rows staged in buffer buf:
    // NT x MTS x KS16 x 6 matrix instructions into acc.
    auto project = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            u32x4 a[MTS][NPL];
#pragma unroll
            for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
                for (int pl = 0; pl < NPL; ++pl) a[mt][pl] = Qs[buf][((mt * KS16 + ks) * NPL + pl) * 64 + lane];
#pragma unroll
            for (int t = T0; t < T1; ++t)
#pragma unroll
                for (int mt = 0; mt < MTS; ++mt)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt) {
                        const f32x16 c_in = (ks == 0 && t == T0) ? zero : acc[nt][mt];
                        if constexpr (F16)
                            acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(
                                __builtin_bit_cast(f16x8, a[mt][TA[t]]), __builtin_bit_cast(f16x8, yq[nt][ks][TB[t]]),
                                c_in, 0, 0, 0);
                        else
                            acc[nt][mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                                __builtin_bit_cast(bf16x8, a[mt][TA[t]]),
                                __builtin_bit_cast(bf16x8, yq[nt][ks][TB[t]]), c_in, 0, 0, 0);
                    }
        }
    };
    // Kept energy of the wavefront's signals in the blocks of stage s (from acc) against the
    // running best.
    auto select = [&](int s) {
        {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    float x[NV];
#pragma unroll
                    for (int v = 0; v < NV; ++v) {
                        const int f = b * NV + v;      // flattened (tile, register)
                        x[v] = fabsf(acc[nt][f >> 4][f & 15]);
                    }
                    const float e = pair_top_energy<NV, S, SX>(x, s0, h != 0);
                    const int j = s * NB + b;
                    if constexpr (MODE == 1) {
                        if (j < K) secondE[nt] = fmaxf(secondE[nt], fminf(e, bestE[nt]));
                    }
                    if (j < K && e > bestE[nt]) {
                        bestE[nt] = e;
                        best[nt] = j;
                    }
                }
            }
        }
    };

    if (s_beg < s_end) {                 // uniform
        fetch(s_beg);
        stash(0);
    }
    __syncthreads();
    for (int s = s_beg; s < s_end; ++s) {
        const int cur = (s - s_beg) & 1;
        if (s + 1 < s_end) fetch(s + 1);
        if (team == 0) {                 // uniform over the wavefront
            project(cur);
            select(s);
        } else {
            if (s > s_beg) select(s - 1);
            project(cur);
        }
        if (s + 1 < s_end) stash(cur ^ 1);
        __syncthreads();
    }
    if (team == 1 && s_beg < s_end) select(s_end - 1);

    bool undecided[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        undecided[nt] = false;
        if constexpr (MODE == 1) {
            const float y2 = yn2[nt] + other_half(yn2[nt]);
            undecided[nt] = !(bestE[nt] - secondE[nt] > margin_rel * y2);       // also for NaN
        }
    }
    if (h == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            if (sig[nt] >= 0) {
                blk[tpos[nt]] = best[nt];
                energy[tpos[nt]] = bestE[nt] * unscale[nt];
            }
        }
    }
    if constexpr (MODE == 1) {
        // The undecided signals of the workgroup -> the list: one reservation per workgroup (a
        // returning atomic per wavefront on the one counter would serialise thousands of them).
        // The stage buffers are dead; the words used here lie beyond the histogram below.
        int* fl = reinterpret_cast<int*>(Qb_raw) + 2048;   // [2 * WAVES] counts | [1] base
        unsigned long long mask[NT];
        bool put[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            put[nt] = h == 0 && sig[nt] >= 0 && undecided[nt];
            mask[nt] = __ballot(put[nt]);
            if (lane == 0) fl[wave * NT + nt] = __popcll(mask[nt]);
        }
        __syncthreads();
        if (tid == 0) {
            int total = 0;
            for (int e = 0; e < G::WAVES * NT; ++e) {
                const int c = fl[e];
                fl[e] = total;
                total += c;
            }
            fl[G::WAVES * NT] = total > 0 ? atomicAdd(flag_count, total) : 0;
        }
        __syncthreads();
        const int base = fl[G::WAVES * NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            if (put[nt])
                flag_ids[base + fl[wave * NT + nt] + __popcll(mask[nt] & ((1ull << lane) - 1ull))] =
                    (int32_t)sig[nt];
    }

    // the grouping's chunk histograms (see energy_kernel); the undecided signals of a screening
    // pass are added by the resolution pass
    if (chunk_count != nullptr) {        // uniform (MODE 2: the merge kernel does this)
        if constexpr (MODE != 2) {
            int* lh = reinterpret_cast<int*>(Qb_raw);      // the stage buffers are dead (>= 12 KiB): the
                                                           // loop's last barrier follows the last read
            for (int j = tid; j < K; j += NTH) lh[j] = 0;
            __syncthreads();
            if (h == 0) {
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    if (sig[nt] >= 0 && !undecided[nt]) atomicAdd(&lh[best[nt]], 1);
            }
            __syncthreads();
            const int64_t c = ((int64_t)blockIdx.x * (G::WAVES * 32 * NT)) / chunk;
            for (int j = tid; j < K; j += NTH)
                if (lh[j] != 0) atomicAdd(&chunk_count[c * K + j], lh[j]);
        }
    }
}

// p = 256 on the bf16 / fp16 matrix cores.  The three bf16 parts of 32 signals take 192 registers
// per lane, too many for two wavefronts per SIMD, and with one wavefront per SIMD the selection
// networks would run while the matrix cores idle.  So the CONTRACTION is halved instead: the
// two wavefronts of a SIMD (w and w + 4) share their signals, each holds one half of the dims and
// multiplies the staged rows (32 atoms a stage, double-buffered) by its half.  With three bf16
// parts (F16 = false) that is one tile of 32 signals per pair (96 registers); with two fp16 parts
// (F16 = true, scaling and products as in energy_split_kernel MODE 3) two tiles (128 registers), so
// that an A operand read from LDS feeds twice as many matrix instructions and a stage is 32 KiB
// instead of 48.  For every block one of the two is the selector (even blocks: the wavefront with
// the lower dims, odd blocks: the other): its partner leaves its partial products in LDS, the
// selector adds them to its own one stage later and runs the selection networks on the sums
// while the partner already multiplies the next stage.  A block spans 8 stages, across which the
// selector keeps the lane's running sorted top-S; the two wavefronts' best blocks are compared
// at the end.
constexpr int kWideWaves = 8;

template <int P, int S, int SX, bool F16>
__global__ __launch_bounds__(64 * kWideWaves) void energy_split_wide_kernel(
    const float* __restrict__ Y, int m, const u32x4* __restrict__ Dsb, int K, int s0,
    int32_t* __restrict__ blk, float* __restrict__ energy, int32_t* __restrict__ chunk_count, int chunk,
    int units_per_y) {
    constexpr int KS16 = P / 16, KH = KS16 / 2;            // contraction steps: all, per wavefront
    constexpr int SPB = P / 32;                            // stages per block
    constexpr int NPL = F16 ? 2 : 3;                       // operand parts
    constexpr int NT = F16 ? 2 : 1;                        // 32-signal tiles per pair of wavefronts
    constexpr int STAGE_U = KS16 * NPL * 64;               // 16-byte units per stage of 32 rows
    constexpr int NTH = 64 * kWideWaves;
    constexpr int FPT = STAGE_U / NTH;
    static_assert(P == 256 && STAGE_U % NTH == 0 && S <= 16, "shape");

    extern __shared__ u32x4 Qw_raw[];    // Qs[2][STAGE_U] | xch[2][4 SIMDs][NT][4][64] (f32x4)
    u32x4(*Qs)[STAGE_U] = reinterpret_cast<u32x4(*)[STAGE_U]>(Qw_raw);
    f32x4* xch = reinterpret_cast<f32x4*>(Qw_raw + 2 * STAGE_U);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int simd = wave & 3, half = wave >> 2;           // wavefronts w and w + 4 share a SIMD
    const int h = lane >> 5, n = lane & 31;
    // B operand: the parts of dims (half*KH + ks)*16 + h*8 .. +7 of this lane's signal in tile nt
    u32x4 yq[NT][KH][NPL];
    int64_t sig[NT];
    float unscale[NT];                   // F16: 1 / (scale of the signal * scale of the dictionary)^2
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int64_t i = (((int64_t)blockIdx.x * 4 + simd) * NT + nt) * 32 + n;
        sig[nt] = i < m ? i : -1;
        unscale[nt] = 1.f;
        f32x4 raw[KH][2];
#pragma unroll
        for (int ks = 0; ks < KH; ++ks) {
            raw[ks][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            raw[ks][1] = raw[ks][0];
            if (i < m) {
                const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + (half * KH + ks) * 16 + h * 8);
                raw[ks][0] = src[0];
                raw[ks][1] = src[1];
            }
        }
        float scale = 1.f;
        if constexpr (F16) {
            // the largest magnitude of the whole signal: this lane's dims, the other lane half's,
            // and the partner wavefront's half of the dims (through LDS, before the stages use it)
            float vmax = 0.f;
#pragma unroll
            for (int ks = 0; ks < KH; ++ks)
#pragma unroll
                for (int e = 0; e < 2; ++e)
                    vmax = fmaxf(fmaxf(fmaxf(vmax, fabsf(raw[ks][e].x)), fmaxf(fabsf(raw[ks][e].y), fabsf(raw[ks][e].z))),
                                 fabsf(raw[ks][e].w));
            vmax = fmaxf(vmax, other_half(vmax));
            float* vx = reinterpret_cast<float*>(Qw_raw);  // [2 halves][4 SIMDs][64]
            vx[(half * 4 + simd) * 64 + lane] = vmax;
            __syncthreads();
            vmax = fmaxf(vmax, vx[((half ^ 1) * 4 + simd) * 64 + lane]);
            __syncthreads();
            scale = f16_signal_scale(vmax);
            const float inv = 1.f / (scale * kF16DictScale);
            unscale[nt] = inv * inv;
        }
#pragma unroll
        for (int ks = 0; ks < KH; ++ks) {
            const f32x4 v0 = raw[ks][0], v1 = raw[ks][1];
            if constexpr (F16) {
                const F16x2Pair a = split_f16x2(v0.x * scale, v0.y * scale), b = split_f16x2(v0.z * scale, v0.w * scale);
                const F16x2Pair c = split_f16x2(v1.x * scale, v1.y * scale), d = split_f16x2(v1.z * scale, v1.w * scale);
                yq[nt][ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
                yq[nt][ks][1] = u32x4{a.lo, b.lo, c.lo, d.lo};
            } else {
                const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
                const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
                yq[nt][ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
                yq[nt][ks][1] = u32x4{a.mid, b.mid, c.mid, d.mid};
                yq[nt][ks][2] = u32x4{a.lo, b.lo, c.lo, d.lo};
            }
        }
    }

    // Small m: the blocks are split over blockIdx.y exactly as in energy_kernel.
    const int n_stage = K * SPB;
    int s_beg = 0, s_end = n_stage;
    if (units_per_y > 0) {
        s_beg = min(n_stage, (int)blockIdx.y * units_per_y * SPB);
        s_end = min(n_stage, s_beg + units_per_y * SPB);
        blk += (int64_t)blockIdx.y * m;
        energy += (int64_t)blockIdx.y * m;
    }

    u32x4 pre[FPT];
    auto fetch = [&](int s) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) pre[r] = Dsb[(int64_t)s * STAGE_U + tid + NTH * r];
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) Qs[buf][tid + NTH * r] = pre[r];
    };

    int best[NT];
    float bestE[NT];
    float run[NT][S];                    // selector: lane's top-S magnitudes of the current block
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        best[nt] = 0;
        bestE[nt] = -1.f;
#pragma unroll
        for (int t = 0; t < S; ++t) run[nt][t] = 0.f;
    }

    // the partial products, smallest first: (A part, B part): six of three bf16 parts, three of
    // two fp16 parts
    constexpr int TA[6] = {F16 ? 0 : 2, F16 ? 1 : 0, F16 ? 0 : 1, 1, 0, 0};
    constexpr int TB[6] = {F16 ? 1 : 0, F16 ? 0 : 2, F16 ? 0 : 1, 0, 1, 0};
    constexpr int T1 = F16 ? 3 : 6;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) acc[nt] = zero;
    auto selects = [&](int s) { return (((s / SPB) & 1) == half); };   // uniform over the wavefront

    // This wavefront's half of the products of the rows staged in buffer buf.
    auto project = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < KH; ++ks) {
            u32x4 a[NPL];
#pragma unroll
            for (int pl = 0; pl < NPL; ++pl) a[pl] = Qs[buf][((half * KH + ks) * NPL + pl) * 64 + lane];
#pragma unroll
            for (int t = 0; t < T1; ++t)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    const f32x16 c_in = (ks == 0 && t == 0) ? zero : acc[nt];
                    if constexpr (F16)
                        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a[TA[t]]),
                                                                         __builtin_bit_cast(f16x8, yq[nt][ks][TB[t]]),
                                                                         c_in, 0, 0, 0);
                    else
                        acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[TA[t]]),
                                                                          __builtin_bit_cast(bf16x8, yq[nt][ks][TB[t]]),
                                                                          c_in, 0, 0, 0);
                }
        }
    };
    // Selector of stage s: own partial (still in acc) + the partner's (exchange buffer buf), then
    // the lane's running top-S and, after the block's last stage, the kept energy of the lane pair.
    auto select = [&](int s, int buf) {
        const int part = s % SPB;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            float x[16], a[S];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 o = xch[(((buf * 4 + simd) * NT + nt) * 4 + q) * 64 + lane];
                x[4 * q + 0] = fabsf(acc[nt][4 * q + 0] + o.x);
                x[4 * q + 1] = fabsf(acc[nt][4 * q + 1] + o.y);
                x[4 * q + 2] = fabsf(acc[nt][4 * q + 2] + o.z);
                x[4 * q + 3] = fabsf(acc[nt][4 * q + 3] + o.w);
            }
            top_sorted<16, S>(x, a);
            if (part == 0) {             // uniform
#pragma unroll
                for (int t = 0; t < S; ++t) run[nt][t] = a[t];
            } else {
#pragma unroll
                for (int t = 0; t < S; ++t) run[nt][t] = fmaxf(run[nt][t], a[S - 1 - t]);
                bitonic_merge_desc<S>(run[nt]);
            }
            if (part == SPB - 1) {       // uniform
                const float e = pair_list_energy<S, SX>(run[nt], s0, h != 0);
                const int j = s / SPB;
                if (e > bestE[nt]) {
                    bestE[nt] = e;
                    best[nt] = j;
                }
            }
        }
    };

    if (s_beg < s_end) {                 // uniform
        fetch(s_beg);
        stash(0);
    }
    __syncthreads();
    for (int s = s_beg; s < s_end; ++s) {
        const int cur = (s - s_beg) & 1;
        if (s + 1 < s_end) fetch(s + 1);
        if (s > s_beg && selects(s - 1)) select(s - 1, cur ^ 1);
        project(cur);
        if (!selects(s)) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    xch[(((cur * 4 + simd) * NT + nt) * 4 + q) * 64 + lane] =
                        f32x4{acc[nt][4 * q + 0], acc[nt][4 * q + 1], acc[nt][4 * q + 2], acc[nt][4 * q + 3]};
        }
        if (s + 1 < s_end) stash(cur ^ 1);
        __syncthreads();
    }
    if (s_beg < s_end && selects(s_end - 1)) select(s_end - 1, (s_end - 1 - s_beg) & 1);

    // the better of the two wavefronts' best blocks (equal energies: the lower block)
    __syncthreads();                     // the exchange buffers are free
    float* mrgE = reinterpret_cast<float*>(xch);           // [4][NT][64]
    int* mrgJ = reinterpret_cast<int*>(xch) + 4 * NT * 64;
    if (half == 1) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            mrgE[(simd * NT + nt) * 64 + lane] = bestE[nt];
            mrgJ[(simd * NT + nt) * 64 + lane] = best[nt];
        }
    }
    __syncthreads();
    if (half == 0) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const float e = mrgE[(simd * NT + nt) * 64 + lane];
            const int j = mrgJ[(simd * NT + nt) * 64 + lane];
            if (e > bestE[nt] || (e == bestE[nt] && j < best[nt])) {
                bestE[nt] = e;
                best[nt] = j;
            }
            if (h == 0 && sig[nt] >= 0) {
                blk[sig[nt]] = best[nt];
                energy[sig[nt]] = bestE[nt] * unscale[nt];
            }
        }
    }

    // the grouping's chunk histograms (see energy_kernel)
    if (chunk_count != nullptr) {        // uniform
        int* lh = reinterpret_cast<int*>(Qw_raw);          // the stage buffers are dead
        for (int j = tid; j < K; j += NTH) lh[j] = 0;
        __syncthreads();
        if (half == 0 && h == 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                if (sig[nt] >= 0) atomicAdd(&lh[best[nt]], 1);
        }
        __syncthreads();
        const int64_t c = ((int64_t)blockIdx.x * (128 * NT)) / chunk;
        for (int j = tid; j < K; j += NTH)
            if (lh[j] != 0) atomicAdd(&chunk_count[c * K + j], lh[j]);
    }
}

// Winner over the rows of a split launch: part_E / part_j hold, per row y, the best energy
// and block of the row's share of the blocks (rows in ascending block order, so the strict
// comparison keeps the lowest block among equal energies).  Also the grouping histogram
// (see energy_kernel).
__global__ __launch_bounds__(256) void energy_merge_kernel(const float* __restrict__ part_E,
                                                           const int32_t* __restrict__ part_j,
                                                           int rows, int m, int K,
                                                           int32_t* __restrict__ blk,
                                                           float* __restrict__ energy,
                                                           int32_t* __restrict__ chunk_count,
                                                           int chunk) {
    extern __shared__ int lh[];          // [K]
    const int tid = threadIdx.x;
    const int i = blockIdx.x * 256 + tid;
    int best = 0;
    float bestE = -1.f;
    if (i < m) {
        for (int y = 0; y < rows; ++y) {
            const float e = part_E[(int64_t)y * m + i];
            if (e > bestE) {
                bestE = e;
                best = part_j[(int64_t)y * m + i];
            }
        }
        blk[i] = best;
        energy[i] = bestE;
    }
    if (chunk_count != nullptr) {        // uniform
        for (int j = tid; j < K; j += 256) lh[j] = 0;
        __syncthreads();
        if (i < m) atomicAdd(&lh[best], 1);
        __syncthreads();
        const int64_t c = ((int64_t)blockIdx.x * 256) / chunk;
        for (int j = tid; j < K; j += 256)
            if (lh[j] != 0) atomicAdd(&chunk_count[c * K + j], lh[j]);
    }
}

// Dsb != nullptr: the projection on the bf16 matrix cores from the split dictionary.
template <int P, int S, int SX>
hipError_t launch_pse(const float* Y, int64_t m, int K, int s0, int32_t* blk, float* energy,
                      const f32x4* Dsw, const u32x4* Dsb, int dsb_kind, int32_t* chunk_count, float* part_E,
                      int32_t* part_j, LdsRaised* raised, const EnergyScreen* scr, hipStream_t st) {
    constexpr int NT = P <= 64 ? 2 : 1;
    constexpr int QN = P / 8;
    constexpr size_t lds = (size_t)2 * (2 * QN * 64) * sizeof(f32x4);
    constexpr bool wide = P > 64;
    using G = SplitGeom<wide ? 64 : P>;
    constexpr size_t lds_f16 = SplitGeom<wide ? 64 : P, 2>::LDS;
    const bool f16 = Dsb != nullptr && dsb_kind == 3;
    // p = 256: two stages of 32 rows + the partial-product exchange (2 x 4 SIMDs x 4 KiB per signal tile)
    constexpr size_t lds_split = wide ? (size_t)2 * (P / 16) * 3 * 64 * 16 + (size_t)2 * 4 * 4 * 64 * 16 : G::LDS;
    constexpr size_t lds_wide16 = (size_t)2 * (P / 16) * 2 * 64 * 16 + (size_t)2 * 2 * 4 * 4 * 64 * 16;
    const bool split = Dsb != nullptr;
    const int per_wg = split ? (wide ? (f16 ? 256 : 128) : G::WAVES * 32 * G::NT) : 4 * 32 * NT;
    dim3 grid((unsigned)((m + per_wg - 1) / per_wg));
    if (raised == nullptr) return hipErrorInvalidValue;
    if (!split && lds > 64 * 1024) {
        if (hipError_t e = raised->ensure(reinterpret_cast<const void*>(&energy_kernel<P, S, NT, SX>), lds);
            e != hipSuccess)
            return e;
    }
    if constexpr (wide) {
        if (split) {
            hipError_t e = f16 ? raised->ensure(reinterpret_cast<const void*>(
                                                    &energy_split_wide_kernel<P, S, SX, true>), lds_wide16)
                               : raised->ensure(reinterpret_cast<const void*>(
                                                    &energy_split_wide_kernel<P, S, SX, false>), lds_split);
            if (e != hipSuccess) return e;
        }
    }
    const int chunk = group_geom(m).chunk;
    if (chunk % per_wg != 0) return hipErrorInvalidValue;
    // Fewer workgroups than CUs: split the blocks over a second grid dimension.
    const int units = P <= 64 ? (K * P + 63) / 64 : K;     // stages (p <= 64) or blocks
    const int rows_wanted = (int)grid.x >= kEnergySplitBelow ? 1
                                                             : (2 * kNumCU + (int)grid.x - 1) / (int)grid.x;
    int rows = rows_wanted < units ? rows_wanted : units;
    if (rows > kEnergySplitRows) rows = kEnergySplitRows;
    const bool by_rows = rows > 1 && part_E != nullptr && part_j != nullptr && m <= kEnergySplitSignals;
    int units_per_y = 0;
    if (by_rows) {
        units_per_y = (units + rows - 1) / rows;
        rows = (units + units_per_y - 1) / units_per_y;
        grid.y = rows;
    }
    int32_t* out_j = by_rows ? part_j : blk;
    float* out_E = by_rows ? part_E : energy;
    int32_t* hist = by_rows ? nullptr : chunk_count;
    if (split) {
        if constexpr (wide) {
            if (f16)
                hipLaunchKernelGGL((energy_split_wide_kernel<P, S, SX, true>), grid, dim3(64 * kWideWaves),
                                   lds_wide16, st, Y, (int)m, Dsb, K, s0, out_j, out_E, hist, chunk, units_per_y);
            else
                hipLaunchKernelGGL((energy_split_wide_kernel<P, S, SX, false>), grid, dim3(64 * kWideWaves),
                                   lds_split, st, Y, (int)m, Dsb, K, s0, out_j, out_E, hist, chunk, units_per_y);
        } else if (scr != nullptr && !f16 && !by_rows && K > 1 && part_E != nullptr && part_j != nullptr) {
            // screening pass over all signals, then the full products for the undecided ones
            const float kc = kScreenCoef;
            const float margin = 2.f * (2.f * sqrtf((float)s0) * kc + (float)s0 * kc * kc) * 1.05f;
            hipLaunchKernelGGL((energy_split_kernel<P, S, SX, 1>), grid, dim3(64 * G::WAVES), lds_split, st, Y,
                               (int)m, Dsb, K, s0, out_j, out_E, hist, chunk, 0, scr->ids, scr->count, margin);
            int r_rows = units < kEnergySplitRows ? units : kEnergySplitRows;
            const int r_upy = (units + r_rows - 1) / r_rows;
            r_rows = (units + r_upy - 1) / r_upy;
            hipLaunchKernelGGL((energy_split_kernel<P, S, SX, 2>), dim3(grid.x, r_rows), dim3(64 * G::WAVES),
                               lds_split, st, Y, (int)m, Dsb, K, s0, part_j, part_E, nullptr, chunk, r_upy,
                               scr->ids, scr->count, 0.f);
            hipLaunchKernelGGL(energy_resolve_merge_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256), 0, st,
                               part_E, part_j, r_rows, (int)m, K, scr->ids, scr->count, blk, energy, chunk_count,
                               chunk);
        } else if (f16) {
            if constexpr (!wide)
                hipLaunchKernelGGL((energy_split_kernel<P, S, SX, 3>), grid, dim3(64 * G::WAVES), lds_f16, st, Y, (int)m, Dsb, K, s0, out_j, out_E, hist, chunk,
                                   units_per_y, nullptr, nullptr, 0.f);
        } else
            hipLaunchKernelGGL((energy_split_kernel<P, S, SX, 0>), grid, dim3(64 * G::WAVES), lds_split, st, Y,
                               (int)m, Dsb, K, s0, out_j, out_E, hist, chunk, units_per_y, nullptr, nullptr,
                               0.f);
    } else {
        hipLaunchKernelGGL((energy_kernel<P, S, NT, SX>), grid, dim3(256), lds, st, Y, (int)m, Dsw, K, s0,
                           out_j, out_E, hist, chunk, units_per_y);
    }
    if (by_rows)
        hipLaunchKernelGGL(energy_merge_kernel, dim3((unsigned)((m + 255) / 256)), dim3(256),
                           (size_t)K * sizeof(int), st, part_E, part_j, rows, (int)m, K, blk, energy,
                           chunk_count, chunk);
    return hipGetLastError();
}

// s0 in (S/2, S] is made a compile-time constant of the kernel (the lane-pair fold then
// needs no sort), except where a lane holds fewer than S coefficients of a block (p = 16,
// s0 > 8), which takes the run-time path.
template <int P, int S>
hipError_t launch_ps(const float* Y, int64_t m, int K, int s0, int32_t* blk, float* energy,
                     const float* dsw, const unsigned* dsb, int dsb_kind, int32_t* chunk_count, float* part_E,
                     int32_t* part_j, LdsRaised* raised, const EnergyScreen* scr, hipStream_t st) {
    const f32x4* Dsw = reinterpret_cast<const f32x4*>(dsw);
    const u32x4* Dsb = reinterpret_cast<const u32x4*>(dsb);
    constexpr int NV = P <= 64 ? P / 2 : 32;
    if constexpr (S > NV) {
        return launch_pse<P, S, 0>(Y, m, K, s0, blk, energy, Dsw, Dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
    } else {
        switch (S - s0) {
#define SBO_CASE(DELTA)                                                                          \
    case DELTA:                                                                                  \
        if constexpr (S - DELTA > S / 2 || S == 1)                                               \
            return launch_pse<P, S, S - DELTA>(Y, m, K, s0, blk, energy, Dsw, Dsb, dsb_kind, chunk_count,  \
                                               part_E, part_j, raised, scr, st);                      \
        break;
            SBO_CASE(0) SBO_CASE(1) SBO_CASE(2) SBO_CASE(3) SBO_CASE(4) SBO_CASE(5) SBO_CASE(6) SBO_CASE(7)
#undef SBO_CASE
            default: break;
        }
        return hipErrorInvalidValue;
    }
}

template <int P>
hipError_t launch_p(int s0, const float* Y, int64_t m, int K, int32_t* blk, float* energy,
                    const float* dsw, const unsigned* dsb, int dsb_kind, int32_t* chunk_count, float* part_E,
                    int32_t* part_j, LdsRaised* raised, const EnergyScreen* scr, hipStream_t st) {
    if (s0 <= 1) return launch_ps<P, 1>(Y, m, K, s0, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
    if (s0 <= 2) return launch_ps<P, 2>(Y, m, K, s0, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
    if (s0 <= 4) return launch_ps<P, 4>(Y, m, K, s0, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
    if (s0 <= 8) return launch_ps<P, 8>(Y, m, K, s0, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
    return launch_ps<P, 16>(Y, m, K, s0, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
}

}  // namespace

hipError_t launch_dict_swizzle(int p, int K, const float* D, float* dsw, hipStream_t st) {
    f32x4* out = reinterpret_cast<f32x4*>(dsw);
    const dim3 grid((K * p + 63) / 64);
    switch (p) {
        case 16: hipLaunchKernelGGL((dict_swizzle_kernel<16>), grid, dim3(256), 0, st, D, K, out); break;
        case 32: hipLaunchKernelGGL((dict_swizzle_kernel<32>), grid, dim3(256), 0, st, D, K, out); break;
        case 64: hipLaunchKernelGGL((dict_swizzle_kernel<64>), grid, dim3(256), 0, st, D, K, out); break;
        case 256: hipLaunchKernelGGL((dict_swizzle_kernel<256>), grid, dim3(256), 0, st, D, K, out); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_dict_swizzle_split(int p, int K, const float* D, unsigned* dsb, int kind, hipStream_t st) {
    u32x4* out = reinterpret_cast<u32x4*>(dsb);
    const dim3 grid((K * p + 63) / 64);
    if (kind == 3) {
        switch (p) {
            case 16: hipLaunchKernelGGL((dict_swizzle_split_kernel<16, 2>), grid, dim3(256), 0, st, D, K, out); break;
            case 32: hipLaunchKernelGGL((dict_swizzle_split_kernel<32, 2>), grid, dim3(256), 0, st, D, K, out); break;
            case 64: hipLaunchKernelGGL((dict_swizzle_split_kernel<64, 2>), grid, dim3(256), 0, st, D, K, out); break;
            case 256: hipLaunchKernelGGL((dict_swizzle_split_kernel<256, 2>), grid, dim3(256), 0, st, D, K, out); break;
            default: return hipErrorInvalidValue;
        }
        return hipGetLastError();
    }
    switch (p) {
        case 16: hipLaunchKernelGGL((dict_swizzle_split_kernel<16, 3>), grid, dim3(256), 0, st, D, K, out); break;
        case 32: hipLaunchKernelGGL((dict_swizzle_split_kernel<32, 3>), grid, dim3(256), 0, st, D, K, out); break;
        case 64: hipLaunchKernelGGL((dict_swizzle_split_kernel<64, 3>), grid, dim3(256), 0, st, D, K, out); break;
        case 256: hipLaunchKernelGGL((dict_swizzle_split_kernel<256, 3>), grid, dim3(256), 0, st, D, K, out); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_energy(int p, int K, int s0, const float* Y, int64_t m, const float* dsw,
                         const unsigned* dsb, int dsb_kind, int32_t* blk, float* energy, int32_t* chunk_count,
                         float* part_E, int32_t* part_j, LdsRaised* raised, const EnergyScreen* scr, hipStream_t st) {
    switch (p) {
        case 16: return launch_p<16>(s0, Y, m, K, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
        case 32: return launch_p<32>(s0, Y, m, K, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
        case 64: return launch_p<64>(s0, Y, m, K, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
        case 256: return launch_p<256>(s0, Y, m, K, blk, energy, dsw, dsb, dsb_kind, chunk_count, part_E, part_j, raised, scr, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
