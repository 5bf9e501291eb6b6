// Grouping of the signals by chosen block (Section 3.3: signal lists per base, built
// before the training step) as a deterministic counting sort, entirely on the device:
//   1. per-chunk histograms      (one wavefront per chunk of consecutive signals)
//   2. per-block scan over chunks (one workgroup per block)
//   3. stable scatter            (one wavefront per chunk; offsets = scan of counts)
// Only integer additions are involved and every destination slot is computed, not
// claimed by an atomic, so perm is the unique stable permutation.
#include "sbo_internal.h"
#include "device_utils.h"

#include <mutex>

namespace sbo {

namespace {

constexpr int kMaxK = 1024;

// Scratch of launch_group_static (the grouping for callers that must not allocate): the
// per-chunk histograms and per-chunk bases, [2][kStaticChunks][kGroupStaticMaxK] ints = 1 MiB
// on every GPU the library runs on, held until the process ends.
constexpr int kStaticChunks = 1024;            // group_geom() never makes more for m <= 2^20
static __device__ __align__(256) int32_t scratch[2 * kStaticChunks * kGroupStaticMaxK];

// Device address of `scratch` on each GPU (every GPU holds its own copy of the array); looked
// up once per device.  In host code the array's name is only a handle for this lookup.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[kMaxDevices] = {};

hipError_t static_scratch(int32_t** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (g_scratch_ptr[dev] == nullptr) {
        int32_t* ptr = nullptr;
        e = hipGetSymbolAddress(reinterpret_cast<void**>(&ptr), HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (ptr == nullptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}

// 1. chunk_count[c][j] = number of signals of chunk c that chose block j.
__global__ __launch_bounds__(256) void group_hist_kernel(const int32_t* __restrict__ blk, int m,
                                                         int K, int chunk, int n_chunks,
                                                         int32_t* __restrict__ chunk_count) {
    extern __shared__ int lds[];           // [4][K]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int* cnt = lds + wave * K;
    for (int j = lane; j < K; j += 64) cnt[j] = 0;
    __syncthreads();
    const int c = blockIdx.x * 4 + wave;
    if (c < n_chunks) {
        const int beg = c * chunk;
        const int end = min(m, beg + chunk);
        for (int i = beg + lane; i < end; i += 64) {
            const int b = blk[i];
            if ((unsigned)b < (unsigned)K) atomicAdd(&cnt[b], 1);   // out-of-range ids are dropped
        }
    }
    __syncthreads();
    if (c < n_chunks)
        for (int j = lane; j < K; j += 64) chunk_count[(int64_t)c * K + j] = cnt[j];
}

// 2. chunk_base[c][j] = number of signals of block j in chunks before c; counts[j] = total.
// The histogram entries are set back to zero once read: the coding kernel, which can
// produce them itself, adds into the array.
__global__ __launch_bounds__(256) void group_scan_kernel(int32_t* __restrict__ chunk_count,
                                                         int K, int n_chunks,
                                                         int32_t* __restrict__ chunk_base,
                                                         int32_t* __restrict__ counts,
                                                         int32_t* __restrict__ clear_word) {
    __shared__ int out[4 * 256 + 1];
    __shared__ int tmp[16];
    const int j = blockIdx.x;
    int carry = 0;
    for (int c0 = 0; c0 < n_chunks; c0 += 1024) {
        const int n = min(1024, n_chunks - c0);
        wg_exclusive_scan4([&](int idx) { return chunk_count[(int64_t)(c0 + idx) * K + j]; }, n,
                           out, tmp);
        for (int idx = threadIdx.x; idx < n; idx += 256) {
            chunk_base[(int64_t)(c0 + idx) * K + j] = carry + out[idx];
            chunk_count[(int64_t)(c0 + idx) * K + j] = 0;
        }
        carry += out[n];
        __syncthreads();
    }
    if (threadIdx.x == 0) counts[j] = carry;
    // the coding kernel's count of undecided signals has been consumed by now
    if (clear_word != nullptr && j == 0 && threadIdx.x == 0) *clear_word = 0;
}

// 3. perm[offsets[j] + chunk_base[c][j] + rank inside the chunk] = signal id.
__global__ __launch_bounds__(256) void group_scatter_kernel(const int32_t* __restrict__ blk, int m,
                                                            int K, int chunk, int n_chunks,
                                                            const int32_t* __restrict__ chunk_base,
                                                            const int32_t* __restrict__ counts,
                                                            int32_t* __restrict__ offsets,
                                                            int32_t* __restrict__ perm) {
    extern __shared__ int lds[];           // off[K+1] | tmp[16] | run[4][K]
    int* off = lds;
    int* tmp = lds + (K + 1);
    int* runs = tmp + 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    wg_exclusive_scan4([&](int idx) { return counts[idx]; }, K, off, tmp);
    if (blockIdx.x == 0)
        for (int j = threadIdx.x; j <= K; j += 256) offsets[j] = off[j];

    const int c = blockIdx.x * 4 + wave;
    if (c >= n_chunks) return;             // no workgroup barrier below this line
    int* run = runs + wave * K;
    for (int j = lane; j < K; j += 64) run[j] = off[j] + chunk_base[(int64_t)c * K + j];
    __builtin_amdgcn_wave_barrier();

    int nbits = 0;
    while ((1 << nbits) < K) ++nbits;
    const int beg = c * chunk;
    const int end = min(m, beg + chunk);
    for (int i0 = beg; i0 < end; i0 += 64) {
        const int i = i0 + lane;
        int b = i < end ? blk[i] : -1;
        const bool valid = (unsigned)b < (unsigned)K;
        if (!valid) b = 0;
        // lanes holding the same block as this lane
        unsigned long long same = __ballot(valid);
        for (int bit = 0; bit < nbits; ++bit) {
            const bool one = (b >> bit) & 1;
            const unsigned long long bal = __ballot(valid && one);
            same &= one ? bal : ~bal;
        }
        const unsigned long long below = same & ((1ull << lane) - 1ull);
        const int rank = __popcll(below);
        int base = 0;
        if (valid) {
            base = run[b];
            perm[base + rank] = i;
        }
        __builtin_amdgcn_wave_barrier();   // every lane has read run[] before a leader updates it
        if (valid && rank == 0) run[b] = base + __popcll(same);
        __builtin_amdgcn_wave_barrier();
    }
}

}  // namespace

// have_hist: ws.chunk_count already holds the per-chunk histograms (written by the coding
// kernel); otherwise they are computed from blk here.
hipError_t launch_group(int K, const int32_t* blk, int64_t m, const Workspace& ws, bool have_hist,
                        hipStream_t st) {
    if (K > kMaxK) return hipErrorInvalidValue;
    const GroupGeom g = group_geom(m);
    const unsigned wgs = (unsigned)((g.n_chunks + 3) / 4);
    if (!have_hist)
        hipLaunchKernelGGL(group_hist_kernel, dim3(wgs), dim3(256), 4 * K * sizeof(int), st, blk,
                           (int)m, K, g.chunk, g.n_chunks, ws.chunk_count);
    hipLaunchKernelGGL(group_scan_kernel, dim3(K), dim3(256), 0, st, ws.chunk_count, K,
                       g.n_chunks, ws.chunk_base, ws.counts, ws.flag_count);
    hipLaunchKernelGGL(group_scatter_kernel, dim3(wgs), dim3(256),
                       (K + 1 + 16 + 4 * K) * sizeof(int), st, blk, (int)m, K, g.chunk, g.n_chunks,
                       ws.chunk_base, ws.counts, ws.offsets, ws.perm);
    return hipGetLastError();
}

// The same three kernels with the chunk arrays in the static device array above instead of
// a context's workspace: no allocation anywhere.  m <= kGroupStaticMaxM, K <= kGroupStaticMaxK
// (checked by the caller).  Nothing in the scratch has to start at zero: the histogram kernel
// writes every entry the later kernels read.
hipError_t launch_group_static(int K, const int32_t* blk, int64_t m, int32_t* counts, int32_t* offsets,
                               int32_t* perm, hipStream_t st) {
    if (K < 1 || K > kGroupStaticMaxK || m < 1 || m > kGroupStaticMaxM) return hipErrorInvalidValue;
    int32_t* base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return e;
    const GroupGeom g = group_geom(m);
    if (g.n_chunks > kStaticChunks) return hipErrorInvalidValue;
    int32_t* chunk_count = base;
    int32_t* chunk_base = base + (size_t)kStaticChunks * kGroupStaticMaxK;
    const unsigned wgs = (unsigned)((g.n_chunks + 3) / 4);
    hipLaunchKernelGGL(group_hist_kernel, dim3(wgs), dim3(256), 4 * K * sizeof(int), st, blk, (int)m, K,
                       g.chunk, g.n_chunks, chunk_count);
    hipLaunchKernelGGL(group_scan_kernel, dim3(K), dim3(256), 0, st, chunk_count, K, g.n_chunks,
                       chunk_base, counts, nullptr);
    hipLaunchKernelGGL(group_scatter_kernel, dim3(wgs), dim3(256), (K + 1 + 16 + 4 * K) * sizeof(int), st,
                       blk, (int)m, K, g.chunk, g.n_chunks, chunk_base, counts, offsets, perm);
    return hipGetLastError();
}

}  // namespace sbo
