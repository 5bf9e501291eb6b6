// Small device helpers shared by the libsbo kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sbo {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

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
