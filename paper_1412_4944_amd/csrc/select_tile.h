// Per-tile support selection shared by the select kernels.
#pragma once

#include "device_utils.h"

namespace sbo {

// One wavefront holds, in MFMA accumulator layout, the projections c = Q_j^T y of a tile
// of up to 32 signals onto ONE block: register r of tile mt in lane (h, n) is atom
// mt*32 + (r/4)*8 + h*4 + r%4 of signal n.  Finds the s0-th largest magnitude tau of every
// signal with the compare-exchange networks, then writes the support {|c| > tau} plus the
// lowest-index entries equal to tau in ascending atom order, the coefficients and the
// residual (sum of the dropped c^2) of signal i (original index; active = lane has a
// signal).  Exact magnitude ties beyond the trivial one are resolved by a sequential
// per-signal pass through the wave-private LDS tile ct[32][P+1] (p <= 64; for larger p by
// running counts over the registers, and ct is not used: pass nullptr).  The (atom, coefficient)
// rows are first compacted in the wave-private LDS area stage[32][2][16] (words) and then
// written with one or a few wide stores per lane (lane half 0: supp row, half 1: coef row),
// because scattered 4-byte stores to rows in original signal order are what this step
// would otherwise wait on.
// KEEP_X: on return ct[n][atom] holds the sparse code x of every signal of the tile
// (kept coefficients, zeros elsewhere).  Without KEEP_X ct is touched only on the tie path
// (*used_ct is then set).  On return the compacted rows are still in `stage`: entry pos of
// signal n at stage_idx(n, 0, pos) (atom) and stage_idx(n, 1, pos) (coefficient bits).
constexpr int kSelectStageWords = 32 * 2 * 16;

// Word index of entry `pos` (< 16) of signal row n in the stage area; kind 0 = atom, 1 =
// coefficient bits.  A row is 32 words = 8 groups of 4 (groups 0-3 atoms, 4-7 coefficients);
// the group index is XORed with the row number so that lanes writing the same entry of
// different rows do not all land in one LDS bank (a plain [n][32] layout would put them there),
// while the four words of a group stay together for the 16-byte copy out.
__device__ __forceinline__ int stage_idx(int n, int kind, int pos) {
    return n * 32 + ((((kind << 2) | (pos >> 2)) ^ (n & 7)) << 2) + (pos & 3);
}

template <int P, int S, bool KEEP_X>
__device__ __forceinline__ void tile_select(const f32x16* acc, int h, int n, bool active, int64_t i,
                                            int s0, float* ct, int* stage,
                                            int32_t* __restrict__ supp, float* __restrict__ coef,
                                            float* __restrict__ err, bool* used_ct = nullptr) {
    constexpr int MT = P >= 32 ? P / 32 : 1;
    constexpr int NVL = MT * 16;
    constexpr int LDC = P + 1;
    static_assert(S <= NVL, "sort width exceeds the values of one lane");
    float c[NVL], mag[NVL];
#pragma unroll
    for (int f = 0; f < NVL; ++f) {
        const int r = f & 15;
        const int atom = (f >> 4) * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
        c[f] = acc[f >> 4][r];
        mag[f] = atom < P ? fabsf(c[f]) : -1.f;
    }

    // tau = s0-th largest magnitude of the signal.
    float top[S], oth[S], mrg[S];
    top_sorted<NVL, S>(mag, top);
#pragma unroll
    for (int t = 0; t < S; ++t) oth[t] = other_half(top[t]);
#pragma unroll
    for (int t = 0; t < S; ++t) mrg[t] = fmaxf(top[t], oth[S - 1 - t]);
    bitonic_merge_desc<S>(mrg);
    float tau = mrg[0];
#pragma unroll
    for (int t = 1; t < S; ++t) tau = (t == s0 - 1) ? mrg[t] : tau;

    // Entries with |c| >= tau, per group of 4 consecutive atoms (the groups alternate
    // between the two lanes of a signal).  Exactly s0 of them: no tie at tau to break.
    int own[NVL / 4], par[NVL / 4], total = 0;
#pragma unroll
    for (int g = 0; g < NVL / 4; ++g) {
        own[g] = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e) own[g] += mag[4 * g + e] >= tau;
        par[g] = other_half(own[g]);
        total += own[g] + par[g];
    }
    const bool simple = !active || total == s0;

    if (__all(simple)) {
        // Every entry with |c| >= tau is kept.  Emit in ascending atom order.
        int run = 0;
        float dropped = 0.f;
#pragma unroll
        for (int g = 0; g < NVL / 4; ++g) {
            int pos = run + (h ? par[g] : 0);
            run += own[g] + par[g];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int f = 4 * g + e;
                const int atom = (f >> 4) * 32 + ((f & 15) >> 2) * 8 + h * 4 + (f & 3);
                if (mag[f] >= tau) {
                    if (active) {             // (a lane without a signal keeps "everything")
                        stage[stage_idx(n, 0, pos)] = atom;
                        stage[stage_idx(n, 1, pos)] = __builtin_bit_cast(int, c[f]);
                    }
                    ++pos;
                } else if (atom < P) {
                    dropped += c[f] * c[f];
                }
                if constexpr (KEEP_X)
                    if (atom < P) ct[n * LDC + atom] = mag[f] >= tau ? c[f] : 0.f;
            }
        }
        dropped += other_half(dropped);
        if (active && h == 0) err[i] = dropped;
    } else if constexpr (P > 64) {
        // Exact magnitude ties, in registers (a [32][P] scratch tile per wavefront would not fit
        // beside the staged dictionary): entries above tau are kept, entries equal to tau in
        // ascending atom order until s0 are reached.  Atom order = group order, and within a
        // group the lane of half 0 comes first, so the running counts cross the lane pair once
        // per group.
        if (used_ct != nullptr) *used_ct = true;
        int gt = 0;
#pragma unroll
        for (int f = 0; f < NVL; ++f) gt += mag[f] > tau;
        gt += other_half(gt);
        const int need = s0 - gt;              // entries equal to tau still to take (>= 1)
        int run_eq = 0, run_keep = 0;
        float dropped = 0.f;
#pragma unroll
        for (int g = 0; g < NVL / 4; ++g) {
            int eq_own = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) eq_own += mag[4 * g + e] == tau;
            const int eq_par = other_half(eq_own);
            int eq_rank = run_eq + (h ? eq_par : 0);
            run_eq += eq_own + eq_par;
            bool keep[4];
            int keep_own = 0;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bool is_eq = mag[4 * g + e] == tau;
                keep[e] = mag[4 * g + e] > tau || (is_eq && eq_rank < need);
                eq_rank += is_eq;
                keep_own += keep[e];
            }
            const int keep_par = other_half(keep_own);
            int pos = run_keep + (h ? keep_par : 0);
            run_keep += keep_own + keep_par;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int f = 4 * g + e;
                const int atom = (f >> 4) * 32 + ((f & 15) >> 2) * 8 + h * 4 + (f & 3);
                if (keep[e]) {
                    if (active && pos < s0) {
                        stage[stage_idx(n, 0, pos)] = atom;
                        stage[stage_idx(n, 1, pos)] = __builtin_bit_cast(int, c[f]);
                    }
                    ++pos;
                } else if (atom < P) {
                    dropped += c[f] * c[f];
                }
            }
        }
        dropped += other_half(dropped);
        if (active && h == 0) err[i] = dropped;
    } else {
        // Exact magnitude ties: walk each signal's coefficients in atom order.
        if (used_ct != nullptr) *used_ct = true;
#pragma unroll
        for (int f = 0; f < NVL; ++f) {
            const int atom = (f >> 4) * 32 + ((f & 15) >> 2) * 8 + h * 4 + (f & 3);
            if (atom < P) ct[n * LDC + atom] = c[f];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        int gt = 0;
#pragma unroll
        for (int f = 0; f < NVL; ++f) gt += mag[f] > tau;
        gt += other_half(gt);
        const int need = s0 - gt;              // entries equal to tau still to take (>= 1)
        if (active && h == 0) {
            int pos = 0, taken_eq = 0;
            float dropped = 0.f;
            for (int k = 0; k < P; ++k) {
                const float v = ct[n * LDC + k];
                const float a = fabsf(v);
                bool take = a > tau;
                if (!take && a == tau && taken_eq < need) {
                    take = true;
                    ++taken_eq;
                }
                if (take && pos < s0) {
                    stage[stage_idx(n, 0, pos)] = k;
                    stage[stage_idx(n, 1, pos)] = __builtin_bit_cast(int, v);
                    ++pos;
                } else {
                    dropped += v * v;
                    if constexpr (KEEP_X) ct[n * LDC + k] = 0.f;
                }
            }
            err[i] = dropped;
        }
    }

    // compact rows -> global memory
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (active) {
        int* dst = (h ? reinterpret_cast<int*>(coef) : supp) + i * s0;
        typedef int i32x4 __attribute__((ext_vector_type(4)));
        typedef int i32x2 __attribute__((ext_vector_type(2)));
        if ((s0 & 3) == 0) {
            for (int t = 0; t < s0; t += 4)
                *reinterpret_cast<i32x4*>(dst + t) = *reinterpret_cast<const i32x4*>(stage + stage_idx(n, h, t));
        } else if ((s0 & 1) == 0) {
            for (int t = 0; t < s0; t += 2)
                *reinterpret_cast<i32x2*>(dst + t) = *reinterpret_cast<const i32x2*>(stage + stage_idx(n, h, t));
        } else {
            for (int t = 0; t < s0; ++t) dst[t] = stage[stage_idx(n, h, t)];
        }
    }
    __builtin_amdgcn_wave_barrier();           // stage is reused by the caller's next tile

}

}  // namespace sbo
