// Small device helpers shared by the libsbo kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbo {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

// Value held by the lane 32 positions away (the other half of the wavefront).
__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }
__device__ __forceinline__ int other_half(int x) { return __shfl_xor(x, 32, 64); }

// ---- DPP lane exchanges (all lanes active, in-row patterns) ---------------------------
template <int CTRL>
__device__ __forceinline__ float dpp_f(float x) {
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;        // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;        // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141; // lane i <-> 7 - i inside each group of 8
constexpr int kDppRowMirror = 0x140;  // lane i <-> 15 - i inside each row of 16

// Sum over aligned groups of G = 4, 8 or 16 lanes; every lane of the group receives the
// bitwise identical total.
template <int G>
__device__ __forceinline__ float group_sum(float x) {
    x += dpp_f<kDppXor1>(x);
    x += dpp_f<kDppXor2>(x);
    if constexpr (G >= 8) x += dpp_f<kDppHalfMirror>(x);
    if constexpr (G == 16) x += dpp_f<kDppRowMirror>(x);
    return x;
}

// ---- fp32 as a sum of three bf16 -------------------------------------------------------
// v = hi + mid + lo exactly: each part is the bf16 nearest to what the parts before it leave
// (3 x 8 significand bits plus the signs of the remainders cover the 24 bits of fp32; the two
// subtractions are exact).  Two values at a time, packed as the matrix cores take them
// (first value in the low half of the word).  With a = a_hi + a_mid + a_lo and likewise b,
// a * b = hi*hi + (hi*mid + mid*hi) + (hi*lo + mid*mid + lo*hi) + terms below 2^-24 |a b|,
// every product of two bf16 being exact in fp32: six bf16 matrix products with fp32
// accumulation reproduce an fp32 contraction to fp32 accuracy.
struct Bf16x3Pair {
    unsigned hi, mid, lo;
};
__device__ __forceinline__ unsigned pack_bf16(float v0, float v1) {
    const bf16x2 t = {(__bf16)v0, (__bf16)v1};           // v_cvt_pk_bf16_f32: round to nearest even
    return __builtin_bit_cast(unsigned, t);
}
__device__ __forceinline__ Bf16x3Pair split_bf16x3(float v0, float v1) {
    Bf16x3Pair r;
    r.hi = pack_bf16(v0, v1);
    const float a0 = v0 - __builtin_bit_cast(float, r.hi << 16);
    const float a1 = v1 - __builtin_bit_cast(float, r.hi & 0xffff0000u);
    r.mid = pack_bf16(a0, a1);
    const float b0 = a0 - __builtin_bit_cast(float, r.mid << 16);
    const float b1 = a1 - __builtin_bit_cast(float, r.mid & 0xffff0000u);
    r.lo = pack_bf16(b0, b1);
    return r;
}

// The same decomposition by truncation (8 + 8 + 8 significand bits), one value at a time: three
// words whose upper halves are bf16 numbers with hi + mid + lo = v exactly.
struct TriWord {
    unsigned hi, mid, lo;
};
__device__ __forceinline__ TriWord split_trunc(float v) {
    TriWord t;
    t.hi = __builtin_bit_cast(unsigned, v) & 0xffff0000u;
    const float r1 = v - __builtin_bit_cast(float, t.hi);
    t.mid = __builtin_bit_cast(unsigned, r1) & 0xffff0000u;
    const float r2 = r1 - __builtin_bit_cast(float, t.mid);
    t.lo = __builtin_bit_cast(unsigned, r2);             // at most 8 significant bits are left
    return t;
}

// Byte offset of bf16 element (row, col) in a transposed MFMA operand tile [row][16 signals]: rows
// of 32 bytes = two 16-byte units; the unit index is flipped on every other group of four rows so
// that the eight rows a quarter-wavefront reads at once cover all LDS banks.
__device__ __forceinline__ int tr_off(int row, int col) {
    return row * 32 + ((((col >> 3) ^ (row >> 2)) & 1) << 4) + (col & 7) * 2;
}

// ---- fp32 as a sum of two fp16 ------------------------------------------------------------
// For v scaled by a power of two so that |v| < 2^15: v = hi + lo + r with hi the fp16 nearest
// to v, lo the fp16 nearest to v - hi (exact in fp32) and |r| <= 2^-22 |v| (11 + 11 significand
// bits; lo is a normal fp16 unless |v| < 2^-3, where its absolute error 2^-25 is below 2^-39 of
// the largest entry).  a * b = hi*hi + hi*lo + lo*hi + terms below 3 * 2^-22 |a b|, every
// product of two fp16 being exact in fp32: three fp16 matrix products with fp32 accumulation
// give a contraction whose error per term, 3 * 2^-22 |a b|, is below the p * 2^-24 sum |a b|
// that an fp32 dot product of p >= 16 terms guarantees.
struct F16x2Pair {
    unsigned hi, lo;
};
__device__ __forceinline__ unsigned pack_f16(float v0, float v1) {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    const f16x2 t = {(_Float16)v0, (_Float16)v1};        // round to nearest even
    return __builtin_bit_cast(unsigned, t);
}
__device__ __forceinline__ F16x2Pair split_f16x2(float v0, float v1) {
    typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
    F16x2Pair r;
    r.hi = pack_f16(v0, v1);
    const f16x2 h = __builtin_bit_cast(f16x2, r.hi);
    r.lo = pack_f16(v0 - (float)h[0], v1 - (float)h[1]);
    return r;
}
// Dictionary entries (|q| <= 1 for orthonormal atoms; anything below 8 is representable) are
// scaled by this before the split.
constexpr float kF16DictScale = 8192.f;
// Power of two that brings a signal whose largest magnitude is vmax into [2^13, 2^14).  1 for a
// zero or non-finite signal and for one below 2^-63: its energies (squares of its coefficients)
// underflow in fp32 whatever the arithmetic, and all its parts then round to zero.
__device__ __forceinline__ float f16_signal_scale(float vmax) {
    const unsigned e = (__builtin_bit_cast(unsigned, vmax) >> 23) & 0xffu;      // biased exponent
    if (e < 64u || e == 0xffu) return 1.f;
    return __builtin_bit_cast(float, (unsigned)(127 + 13 + 127 - (int)e) << 23);   // 2^(13 - (e - 127))
}

// ---- the dictionary in the coding kernels' operand orders --------------------------------
// Rows = atoms of all blocks (row j*P + k = atom k of Q_j), in stages of 64 rows, each stage a
// run of 16-byte units in exactly the order the lanes of a wavefront consume the MFMA A operand
// (row = stage*64 + mt*32 + nn, lane = hh*32 + nn):
//   fp32 order : unit (mt*(P/8) + q)*64 + lane        = dims hh*P/2 + 4q .. +3 of the row
//   split order: unit ((mt*(P/16) + ks)*3 + pl)*64 + lane = the 8 bf16 of part pl (0 hi, 1 mid,
//                2 lo) of dims ks*16 + hh*8 .. +7 of the row
//   fp16 order : unit ((mt*(P/16) + ks)*2 + pl)*64 + lane = the 8 fp16 of part pl (0 hi, 1 lo) of
//                the same dims, entries scaled by kF16DictScale
// These store the four dims 4*d4 .. 4*d4+3 of row `grow`.
template <int P>
__device__ __forceinline__ void store_operand_f32(float* __restrict__ dsw, int grow, int d4, f32x4 row) {
    constexpr int QN = P / 8;
    const int st = grow >> 6, mt = (grow >> 5) & 1, nn = grow & 31;
    const int hh = d4 / QN, q = d4 % QN;
    reinterpret_cast<f32x4*>(dsw)[(int64_t)st * (2 * QN * 64) + (mt * QN + q) * 64 + hh * 32 + nn] = row;
}
template <int P>
__device__ __forceinline__ void store_operand_split(unsigned* __restrict__ dsb, int grow, int d4, f32x4 row) {
    constexpr int KS16 = P / 16;
    const int st = grow >> 6, mt = (grow >> 5) & 1, nn = grow & 31;
    const int ks = d4 >> 2, hh = (d4 >> 1) & 1, half = d4 & 1;
    const Bf16x3Pair a = split_bf16x3(row.x, row.y), b = split_bf16x3(row.z, row.w);
    u32x2* out = reinterpret_cast<u32x2*>(dsb) +
                 ((int64_t)st * (2 * KS16 * 3 * 64) + (int64_t)((mt * KS16 + ks) * 3) * 64 + hh * 32 + nn) * 2 + half;
    out[0] = u32x2{a.hi, b.hi};
    out[2 * 64] = u32x2{a.mid, b.mid};
    out[4 * 64] = u32x2{a.lo, b.lo};
}

template <int P>
__device__ __forceinline__ void store_operand_f16x2(unsigned* __restrict__ dsb, int grow, int d4, f32x4 row) {
    constexpr int KS16 = P / 16;
    const int st = grow >> 6, mt = (grow >> 5) & 1, nn = grow & 31;
    const int ks = d4 >> 2, hh = (d4 >> 1) & 1, half = d4 & 1;
    const F16x2Pair a = split_f16x2(row.x * kF16DictScale, row.y * kF16DictScale);
    const F16x2Pair b = split_f16x2(row.z * kF16DictScale, row.w * kF16DictScale);
    u32x2* out = reinterpret_cast<u32x2*>(dsb) +
                 ((int64_t)st * (2 * KS16 * 2 * 64) + (int64_t)((mt * KS16 + ks) * 2) * 64 + hh * 32 + nn) * 2 + half;
    out[0] = u32x2{a.hi, b.hi};
    out[2 * 64] = u32x2{a.lo, b.lo};
}
// kind: 2 = the three-bf16 split order, 3 = the two-fp16 order
template <int P>
__device__ __forceinline__ void store_operand_parts(unsigned* __restrict__ dsb, int kind, int grow, int d4,
                                                    f32x4 row) {
    if (kind == 3) store_operand_f16x2<P>(dsb, grow, d4, row);
    else store_operand_split<P>(dsb, grow, d4, row);
}

// Workgroup-wide exclusive scan of n <= 4 * blockDim.x integers produced by f(idx).
// out (LDS) receives n + 1 entries (out[n] = total); tmp (LDS) needs 16 ints.
// Every thread of the workgroup must call this; ends with a barrier.
template <class F>
__device__ __forceinline__ void wg_exclusive_scan4(F f, int n, int* out, int* tmp) {
    const int t = threadIdx.x;
    const int lane = t & 63, wave = t >> 6;
    const int nwaves = (blockDim.x + 63) >> 6;
    int v[4];
    int s = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        int idx = 4 * t + e;
        v[e] = idx < n ? f(idx) : 0;
        s += v[e];
    }
    int incl = s;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        int o = __shfl_up(incl, d, 64);
        if (lane >= d) incl += o;
    }
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    int base = 0, total = 0;
    for (int w = 0; w < nwaves; ++w) {
        int x = tmp[w];
        if (w < wave) base += x;
        total += x;
    }
    int ex = base + incl - s;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        int idx = 4 * t + e;
        if (idx < n) out[idx] = ex;
        ex += v[e];
    }
    if (t == 0) out[n] = total;
    __syncthreads();
}

// Largest j in [0, n) with start[j] <= x, for a non-decreasing start[0..n].
__host__ __device__ __forceinline__ int upper_slot(const int* start, int n, int x) {
    int lo = 0, hi = n;  // invariant: start[lo] <= x, answer in [lo, hi)
    while (hi - lo > 1) {
        int mid = (lo + hi) >> 1;
        if (start[mid] <= x) lo = mid; else hi = mid;
    }
    return lo;
}

// ---- compare-exchange networks on register arrays (descending order) ---------------
__host__ __device__ __forceinline__ void cmpx_desc(float& a, float& b) {
    float hi = fmaxf(a, b), lo = fminf(a, b);
    a = hi;
    b = lo;
}

// v is bitonic -> sorted descending.
template <int N>
__host__ __device__ __forceinline__ void bitonic_merge_desc(float (&v)[N]) {
#pragma unroll
    for (int half = N / 2; half >= 1; half >>= 1) {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            if ((i & half) == 0) cmpx_desc(v[i], v[i + half]);
        }
    }
}

// Full bitonic sorting network, descending.
template <int N>
__host__ __device__ __forceinline__ void bitonic_sort_desc(float (&v)[N]) {
#pragma unroll
    for (int k = 2; k <= N; k <<= 1) {
#pragma unroll
        for (int j = k >> 1; j > 0; j >>= 1) {
#pragma unroll
            for (int i = 0; i < N; ++i) {
                int l = i ^ j;
                if (l > i) {
                    if ((i & k) == 0 || k == N) cmpx_desc(v[i], v[l]);
                    else cmpx_desc(v[l], v[i]);
                }
            }
        }
    }
}

// 19-comparator sorting network for 8 keys (descending).
__host__ __device__ __forceinline__ void sort8_desc(float (&v)[8]) {
    cmpx_desc(v[0], v[2]); cmpx_desc(v[1], v[3]); cmpx_desc(v[4], v[6]); cmpx_desc(v[5], v[7]);
    cmpx_desc(v[0], v[4]); cmpx_desc(v[1], v[5]); cmpx_desc(v[2], v[6]); cmpx_desc(v[3], v[7]);
    cmpx_desc(v[0], v[1]); cmpx_desc(v[2], v[3]); cmpx_desc(v[4], v[5]); cmpx_desc(v[6], v[7]);
    cmpx_desc(v[2], v[4]); cmpx_desc(v[3], v[5]);
    cmpx_desc(v[1], v[4]); cmpx_desc(v[3], v[6]);
    cmpx_desc(v[1], v[2]); cmpx_desc(v[3], v[4]); cmpx_desc(v[5], v[6]);
}

// Median of three (one instruction on the device).
__host__ __device__ __forceinline__ float med3(float a, float b, float c) {
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_fmed3f(a, b, c);
#else
    return fmaxf(fminf(a, b), fminf(fmaxf(a, b), c));
#endif
}

// Insertion sort as a network of three-input operations (descending): inserting d into the
// sorted v[0..n) gives max(v0, d), med3(v[i-1], d, v[i]) for 0 < i < n, min(v[n-1], d): n + 1
// independent instructions.  3 + 4 + ... + N operations in all (33 for 8 keys, against 38 for
// the 19-comparator network; 133 against 160 for 16 keys).
template <int N>
__host__ __device__ __forceinline__ void insertion_sort_desc(float (&v)[N]) {
    if constexpr (N == 2) {
        cmpx_desc(v[0], v[1]);
    } else if constexpr (N >= 3) {
        {
            const float a = v[0], b = v[1], c = v[2];
            v[0] = fmaxf(fmaxf(a, b), c);
            v[1] = med3(a, b, c);
            v[2] = fminf(fminf(a, b), c);
        }
#pragma unroll
        for (int n = 3; n < N; ++n) {
            const float d = v[n];
            float r[N];
            r[0] = fmaxf(v[0], d);
#pragma unroll
            for (int i = 1; i < n; ++i) r[i] = med3(v[i - 1], d, v[i]);
            r[n] = fminf(v[n - 1], d);
#pragma unroll
            for (int i = 0; i <= n; ++i) v[i] = r[i];
        }
    }
}

template <int N>
__host__ __device__ __forceinline__ void sort_desc(float (&v)[N]) {
    if constexpr (N <= 16) insertion_sort_desc<N>(v);
    else bitonic_sort_desc<N>(v);
}

// The L largest of x[0..NV), sorted descending (NV and L powers of two, L <= NV).
template <int NV, int L>
__host__ __device__ __forceinline__ void top_sorted(const float (&x)[NV], float (&out)[L]) {
#pragma unroll
    for (int i = 0; i < L; ++i) out[i] = x[i];
    sort_desc<L>(out);
#pragma unroll
    for (int g = 1; g < NV / L; ++g) {
        float t[L];
#pragma unroll
        for (int i = 0; i < L; ++i) t[i] = x[g * L + i];
        sort_desc<L>(t);
#pragma unroll
        for (int i = 0; i < L; ++i) out[i] = fmaxf(out[i], t[L - 1 - i]);
        bitonic_merge_desc<L>(out);
    }
}

}  // namespace sbo
