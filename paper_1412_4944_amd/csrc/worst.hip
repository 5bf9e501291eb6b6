// The W worst represented signals (Algorithm 2, step 3): ids of the W largest squared
// residuals, ties towards the lower signal index, listed in ascending signal order.
//
// Most-significant-digit radix select on an order-preserving 32-bit key: four histogram
// passes of 8 bits each narrow the key of the W-th largest value down to all 32 bits
// (threshold T) and the number `need` of entries equal to T that still belong to the set.
// Histograms use integer atomics only, so the result does not depend on scheduling.
// The set {key > T} plus the first `need` entries with key == T is then written in
// ascending signal order by a two-level stable compaction (counts per chunk, scan over
// chunks, scan inside a chunk).
//
// No kernel waits on another workgroup: the digit found by pass k is recomputed from the
// finished histogram of pass k by every workgroup of the next launch (and stored once for
// the launch after that).
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int kBins = 256;
constexpr int kSelThreads = 256;
constexpr int kSelPerThread = kSelChunk / kSelThreads;   // consecutive entries per thread

// ascending key order = ascending float order (negative values and -0 included)
__device__ __forceinline__ uint32_t order_key(float v) {
    const uint32_t b = __float_as_uint(v);
    return b ^ ((b >> 31) ? 0xffffffffu : 0x80000000u);
}

// Digit of pass `q` and the state after it, from the state before it and hist[q]:
// among the keys that share `prefix` in their higher digits, the `remaining`-th largest
// has digit d where (#keys with digit > d) < remaining <= (#keys with digit >= d).
// Every thread of the workgroup (kSelThreads) must call this; result in st[0..1].
__device__ __forceinline__ void resolve_pass(const int* __restrict__ hist_q, uint32_t prefix,
                                             int remaining, int* above, int* tmp, int* st) {
    if (threadIdx.x == 0) {                    // defined even if the state handed in is not
        st[0] = 0;
        st[1] = 1;
    }
    // above[idx] = number of keys with digit > 255 - idx
    wg_exclusive_scan4([&](int idx) { return hist_q[kBins - 1 - idx]; }, kBins, above, tmp);
    const int t = threadIdx.x;
    if (t < kBins) {
        const int d = kBins - 1 - t;
        const int gt = above[t], ge = gt + hist_q[d];
        if (gt < remaining && remaining <= ge) {
            st[0] = (int)((prefix << 8) | (uint32_t)d);
            st[1] = remaining - gt;
        }
    }
    __syncthreads();
}

// State before pass `pass` (prefix of the higher digits, entries still to take inside it).
// state[q] = state after pass q, stored by workgroup 0 of the launch that resolved it.
__device__ __forceinline__ void state_before(int pass, int W, const int* __restrict__ hist,
                                             int* __restrict__ state, int* above, int* tmp,
                                             int* st, uint32_t& prefix, int& remaining) {
    prefix = 0;
    remaining = W;
    if (pass == 0) return;
    if (pass >= 2) {
        prefix = (uint32_t)state[(pass - 2) * 2];
        remaining = state[(pass - 2) * 2 + 1];
    }
    resolve_pass(hist + (pass - 1) * kBins, prefix, remaining, above, tmp, st);
    prefix = (uint32_t)st[0];
    remaining = st[1];
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        state[(pass - 1) * 2] = st[0];
        state[(pass - 1) * 2 + 1] = st[1];
    }
}

__global__ __launch_bounds__(kSelThreads) void worst_clear_kernel(int* __restrict__ hist) {
    for (int e = threadIdx.x; e < 4 * kBins; e += kSelThreads) hist[e] = 0;
}

__global__ __launch_bounds__(kSelThreads) void worst_hist_kernel(const float* __restrict__ err,
                                                                 int m, int W, int pass,
                                                                 int* __restrict__ hist,
                                                                 int* __restrict__ state) {
    __shared__ int lh[kBins];
    __shared__ int above[kBins + 1];
    __shared__ int tmp[16];
    __shared__ int st[2];
    uint32_t prefix;
    int remaining;
    state_before(pass, W, hist, state, above, tmp, st, prefix, remaining);

    const int tid = threadIdx.x;
    lh[tid] = 0;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    for (int i = blockIdx.x * kSelThreads + tid; i < m; i += gridDim.x * kSelThreads) {
        const uint32_t key = order_key(err[i]);
        if (pass == 0 || (key >> (shift + 8)) == prefix) atomicAdd(&lh[(key >> shift) & 255u], 1);
    }
    __syncthreads();
    if (lh[tid] != 0) atomicAdd(&hist[pass * kBins + tid], lh[tid]);
}

// cnt[chunk] = (entries above T, entries equal to T) of the chunk
__global__ __launch_bounds__(kSelThreads) void worst_count_kernel(const float* __restrict__ err,
                                                                  int m, int W,
                                                                  int* __restrict__ hist,
                                                                  int* __restrict__ state,
                                                                  int* __restrict__ cnt) {
    __shared__ int above[kBins + 1];
    __shared__ int tmp[16];
    __shared__ int st[2];
    __shared__ int red[2][kSelThreads / 64];
    uint32_t T;
    int need;
    state_before(4, W, hist, state, above, tmp, st, T, need);

    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kSelChunk + tid * kSelPerThread;
    int gt = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < kSelPerThread; ++e) {
        if (i0 + e < m) {
            const uint32_t key = order_key(err[i0 + e]);
            gt += key > T;
            eq += key == T;
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        gt += __shfl_xor(gt, o, 64);
        eq += __shfl_xor(eq, o, 64);
    }
    if ((tid & 63) == 0) {
        red[0][tid >> 6] = gt;
        red[1][tid >> 6] = eq;
    }
    __syncthreads();
    if (tid == 0) {
        int g = 0, q = 0;
        for (int w = 0; w < kSelThreads / 64; ++w) {
            g += red[0][w];
            q += red[1][w];
        }
        cnt[blockIdx.x * 2] = g;
        cnt[blockIdx.x * 2 + 1] = q;
    }
}

// base[chunk] = exclusive sums of cnt over the chunks before it (one workgroup)
__global__ __launch_bounds__(kSelThreads) void worst_scan_kernel(const int* __restrict__ cnt,
                                                                 int n_chunks,
                                                                 int* __restrict__ base) {
    __shared__ int out[4 * kSelThreads + 1];
    __shared__ int tmp[16];
    for (int which = 0; which < 2; ++which) {
        int carry = 0;
        for (int c0 = 0; c0 < n_chunks; c0 += 4 * kSelThreads) {
            const int n = min(4 * kSelThreads, n_chunks - c0);
            wg_exclusive_scan4([&](int idx) { return cnt[(c0 + idx) * 2 + which]; }, n, out, tmp);
            for (int e = threadIdx.x; e < n; e += kSelThreads) base[(c0 + e) * 2 + which] = carry + out[e];
            carry += out[n];
            __syncthreads();                   // out is rewritten by the next batch
        }
    }
}

__global__ __launch_bounds__(kSelThreads) void worst_emit_kernel(const float* __restrict__ err,
                                                                 int m, int W,
                                                                 const int* __restrict__ state,
                                                                 const int* __restrict__ base,
                                                                 int32_t* __restrict__ ids) {
    __shared__ int cg[kSelThreads], cq[kSelThreads];
    __shared__ int og[kSelThreads + 1], oq[kSelThreads + 1];
    __shared__ int tmp[16];
    const uint32_t T = (uint32_t)state[3 * 2];
    const int need = state[3 * 2 + 1];

    const int tid = threadIdx.x;
    const int i0 = blockIdx.x * kSelChunk + tid * kSelPerThread;
    uint32_t key[kSelPerThread];
    int gt = 0, eq = 0;
#pragma unroll
    for (int e = 0; e < kSelPerThread; ++e) {
        key[e] = i0 + e < m ? order_key(err[i0 + e]) : 0u;
        if (i0 + e < m) {
            gt += key[e] > T;
            eq += key[e] == T;
        }
    }
    cg[tid] = gt;
    cq[tid] = eq;
    __syncthreads();
    wg_exclusive_scan4([&](int idx) { return cg[idx]; }, kSelThreads, og, tmp);
    wg_exclusive_scan4([&](int idx) { return cq[idx]; }, kSelThreads, oq, tmp);
    int g_before = base[blockIdx.x * 2] + og[tid];
    int q_before = base[blockIdx.x * 2 + 1] + oq[tid];
#pragma unroll
    for (int e = 0; e < kSelPerThread; ++e) {
        if (i0 + e >= m) break;
        const bool is_gt = key[e] > T, is_eq = key[e] == T;
        if (is_gt || (is_eq && q_before < need)) {
            const int pos = g_before + min(q_before, need);
            if (pos < W) ids[pos] = i0 + e;    // always true; keeps a wrong state from writing past the list
        }
        g_before += is_gt;
        q_before += is_eq;
    }
}

}  // namespace

hipError_t launch_worst(const float* err, int64_t m, int64_t W, const Workspace& ws, int32_t* ids,
                        hipStream_t st) {
    const int n_chunks = (int)((m + kSelChunk - 1) / kSelChunk);
    const int hist_grid = n_chunks < 1024 ? n_chunks : 1024;
    hipLaunchKernelGGL(worst_clear_kernel, dim3(1), dim3(kSelThreads), 0, st, ws.sel_hist);
    for (int pass = 0; pass < 4; ++pass)
        hipLaunchKernelGGL(worst_hist_kernel, dim3(hist_grid), dim3(kSelThreads), 0, st, err, (int)m,
                           (int)W, pass, ws.sel_hist, ws.sel_state);
    hipLaunchKernelGGL(worst_count_kernel, dim3(n_chunks), dim3(kSelThreads), 0, st, err, (int)m, (int)W,
                       ws.sel_hist, ws.sel_state, ws.sel_cnt);
    hipLaunchKernelGGL(worst_scan_kernel, dim3(1), dim3(kSelThreads), 0, st, ws.sel_cnt, n_chunks,
                       ws.sel_base);
    hipLaunchKernelGGL(worst_emit_kernel, dim3(n_chunks), dim3(kSelThreads), 0, st, err, (int)m, (int)W,
                       ws.sel_state, ws.sel_base, ids);
    return hipGetLastError();
}

}  // namespace sbo
