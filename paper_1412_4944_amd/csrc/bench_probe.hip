// Measurement aids for the benchmark, NOT part of libsbo (built into a shared library of its
// own, which only bench.py loads): what a bare fp32 MFMA loop and a plain device copy reach on
// this GPU, so that a kernel's rate can be quoted against an achievable peak as well as against
// the published one.
//
//   int bench_probe_mfma(void* hip_stream, int iters, double* tflops)
//       rate of a bare v_mfma_f32_32x32x2_f32 loop (TFLOP/s; 1024 workgroups of 4 wavefronts,
//       each issuing 32 * iters MFMAs: iters = 150 is a launch of about 0.6 ms, iters = 4000
//       one of about 17 ms, long enough for the power limit to show)
//   int bench_probe_mfma_bf16(void* hip_stream, int iters, int random_operands, double* tflops)
//       rate of a bare v_mfma_f32_32x32x16_bf16 loop (the same launch shape); with
//       random_operands != 0 every lane's operands are random bit patterns of moderate
//       magnitude instead of two constants: the matrix cores then draw far more power and the
//       sustained rate drops, which is the rate a kernel working on real data can reach
//   int bench_probe_copy(void* hip_stream, double* gbps)
//       rate of a plain 256 MiB device copy (GB/s, bytes read + bytes written)
//   int bench_probe_overlap(void* hip_stream, int bf16, double* ms3)
//       does matrix work of one wavefront run beside vector-ALU work of another wavefront on the
//       same SIMD?  256 workgroups of 8 wavefronts (two per SIMD: one issues a bare MFMA loop,
//       the other a loop of dependent min/max/multiply); ms3[0] = the MFMA loop alone, ms3[1] = the
//       vector loop alone, ms3[2] = both.  bf16 != 0: v_mfma_f32_32x32x16_bf16, else
//       v_mfma_f32_32x32x2_f32.  both ~ max(alone) means they overlap, both ~ sum means they share
//       the pipe.
// Both allocate and free their own scratch and synchronise the stream; tflops / gbps are host
// pointers; the return value is a hipError_t (0 = success).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// 4 independent accumulator tiles per wavefront, nothing but v_mfma_f32_32x32x2_f32.
__global__ __launch_bounds__(256) void probe_mfma_kernel(float* __restrict__ out, int iters) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const float a = threadIdx.x * 1e-3f, b = blockIdx.x * 1e-3f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

// the same loop on the bf16 matrix cores; eight operand pairs per lane, constant or random
__global__ __launch_bounds__(256) void probe_mfma_bf16_kernel(float* __restrict__ out, int iters, int random_operands) {
    f32x16 acc[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    u32x4 a[8], b[8];
    unsigned x = (blockIdx.x * 256u + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            x = x * 1664525u + 1013904223u;
            const unsigned ra = random_operands ? x : 0u;
            x = x * 1664525u + 1013904223u;
            const unsigned rb = random_operands ? x : 0u;
            // two bf16 per word, sign and mantissa free, exponent kept near 1 (0x3c00..0x3fff)
            a[u][c] = (ra & 0x83ff83ffu) | 0x3c003c00u;
            b[u][c] = (rb & 0x83ff83ffu) | 0x3c003c00u;
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[u]),
                                                                 __builtin_bit_cast(bf16x8, b[(u + i) & 7]), acc[i], 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    out[blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(256) void probe_copy_kernel(const f32x4* __restrict__ src,
                                                         f32x4* __restrict__ dst, int64_t n) {
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (int64_t)gridDim.x * 256)
        dst[i] = src[i];
}

struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    hipError_t init() {
        hipError_t e = hipEventCreate(&a);
        if (e != hipSuccess) return e;
        return hipEventCreate(&b);
    }
    ~EventPair() {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

hipError_t probe_mfma(hipStream_t st, int iters, double* tflops) {
    constexpr int kWgs = 1024;
    const int kIters = iters;
    float* out = nullptr;
    hipError_t e = hipMalloc(&out, (size_t)kWgs * 256 * sizeof(float));
    if (e != hipSuccess) return e;
    EventPair ev;
    e = ev.init();
    float best = 0.f;
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(kWgs), dim3(256), 0, st, out, rep == 0 ? 200 : kIters);
        if (rep == 0) continue;                 // warm-up
        (void)hipEventRecord(ev.a, st);
        hipLaunchKernelGGL(probe_mfma_kernel, dim3(kWgs), dim3(256), 0, st, out, kIters);
        (void)hipEventRecord(ev.b, st);
        e = hipEventSynchronize(ev.b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
        const float rate = (float)((double)kWgs * 4 * kIters * 8 * 4 * 4096.0 / (ms * 1e-3) / 1e12);
        if (rate > best) best = rate;
    }
    (void)hipFree(out);
    *tflops = best;
    return e;
}

hipError_t probe_mfma_bf16(hipStream_t st, int iters, int random_operands, double* tflops) {
    constexpr int kWgs = 1024;
    float* out = nullptr;
    hipError_t e = hipMalloc(&out, (size_t)kWgs * 256 * sizeof(float));
    if (e != hipSuccess) return e;
    EventPair ev;
    e = ev.init();
    float best = 0.f;
    for (int rep = 0; rep < 3 && e == hipSuccess; ++rep) {
        hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(kWgs), dim3(256), 0, st, out, rep == 0 ? 200 : iters,
                           random_operands);
        if (rep == 0) continue;                 // warm-up
        (void)hipEventRecord(ev.a, st);
        hipLaunchKernelGGL(probe_mfma_bf16_kernel, dim3(kWgs), dim3(256), 0, st, out, iters, random_operands);
        (void)hipEventRecord(ev.b, st);
        e = hipEventSynchronize(ev.b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
        const float rate = (float)((double)kWgs * 4 * iters * 8 * 4 * 32768.0 / (ms * 1e-3) / 1e12);
        if (rate > best) best = rate;
    }
    (void)hipFree(out);
    *tflops = best;
    return e;
}

// Wavefronts 0-3 of a workgroup (one per SIMD) issue MFMAs, wavefronts 4-7 (their SIMD
// partners) vector-ALU work.
template <bool BF16>
__global__ __launch_bounds__(512) void probe_overlap_kernel(float* __restrict__ out, int mfma_iters,
                                                            int valu_iters) {
    typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
    float res = 0.f;
    if (threadIdx.x < 256) {
        f32x16 acc[4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
        const float a = threadIdx.x * 1e-3f, b = blockIdx.x * 1e-3f;
        bf16x8 av, bv;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            av[e] = (__bf16)(a + e);
            bv[e] = (__bf16)(b - e);
        }
        for (int it = 0; it < mfma_iters; ++it) {
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    if constexpr (BF16) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc[i], 0, 0, 0);
                    else acc[i] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc[i], 0, 0, 0);
                }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int r = 0; r < 16; ++r) res += acc[i][r];
    } else {
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) x[i] = threadIdx.x * 0.37f + i;
        for (int it = 0; it < valu_iters; ++it) {
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int i = 0; i < 15; ++i) {
                    const float hi = fmaxf(x[i], x[i + 1]), lo = fminf(x[i], x[i + 1]);
                    x[i] = hi;
                    x[i + 1] = lo * 1.0001f;
                }
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) res += x[i];
    }
    out[blockIdx.x * 512 + threadIdx.x] = res;
}

template <bool BF16>
hipError_t probe_overlap(hipStream_t st, double* ms3) {
    // per loop iteration: 32 MFMAs (bf16: 8 passes, fp32: 16 passes of 4 clocks) against 180
    // vector instructions of 4 clocks; the counts make the two loops alone take about the same time
    const int mfma_iters = BF16 ? 6000 : 3000, valu_iters = 8000;
    float* out = nullptr;
    hipError_t e = hipMalloc(&out, (size_t)256 * 512 * sizeof(float));
    if (e != hipSuccess) return e;
    EventPair ev;
    e = ev.init();
    const int mi[3] = {mfma_iters, 0, mfma_iters}, vi[3] = {0, valu_iters, valu_iters};
    hipLaunchKernelGGL((probe_overlap_kernel<BF16>), dim3(256), dim3(512), 0, st, out, 100, 100);   // warm-up
    for (int c = 0; c < 3 && e == hipSuccess; ++c) {
        float best = 1e30f;
        for (int rep = 0; rep < 2 && e == hipSuccess; ++rep) {
            (void)hipEventRecord(ev.a, st);
            hipLaunchKernelGGL((probe_overlap_kernel<BF16>), dim3(256), dim3(512), 0, st, out, mi[c], vi[c]);
            (void)hipEventRecord(ev.b, st);
            e = hipEventSynchronize(ev.b);
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
            if (ms < best) best = ms;
        }
        ms3[c] = best;
    }
    (void)hipFree(out);
    return e;
}

hipError_t probe_copy(hipStream_t st, double* gbps) {
    const int64_t n = (int64_t)16 * 1024 * 1024;               // 16-byte units: 256 MiB each way
    f32x4 *src = nullptr, *dst = nullptr;
    hipError_t e = hipMalloc(&src, (size_t)n * sizeof(f32x4));
    if (e == hipSuccess) e = hipMalloc(&dst, (size_t)n * sizeof(f32x4));
    EventPair ev;
    if (e == hipSuccess) e = ev.init();
    if (e == hipSuccess) e = hipMemsetAsync(src, 0, (size_t)n * sizeof(f32x4), st);
    float best = 0.f;
    for (int rep = 0; rep < 4 && e == hipSuccess; ++rep) {
        (void)hipEventRecord(ev.a, st);
        hipLaunchKernelGGL(probe_copy_kernel, dim3(8192), dim3(256), 0, st, src, dst, n);
        (void)hipEventRecord(ev.b, st);
        e = hipEventSynchronize(ev.b);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.a, ev.b);
        const float rate = (float)(2.0 * (double)n * sizeof(f32x4) / (ms * 1e-3) / 1e9);
        if (rep > 0 && rate > best) best = rate;
    }
    if (src) (void)hipFree(src);
    if (dst) (void)hipFree(dst);
    *gbps = best;
    return e;
}

}  // namespace

extern "C" int bench_probe_mfma(void* hip_stream, int iters, double* tflops) {
    if (!tflops || iters < 1 || iters > 100000) return (int)hipErrorInvalidValue;
    return (int)probe_mfma((hipStream_t)hip_stream, iters, tflops);
}

extern "C" int bench_probe_mfma_bf16(void* hip_stream, int iters, int random_operands, double* tflops) {
    if (!tflops || iters < 1 || iters > 100000) return (int)hipErrorInvalidValue;
    return (int)probe_mfma_bf16((hipStream_t)hip_stream, iters, random_operands, tflops);
}

extern "C" int bench_probe_overlap(void* hip_stream, int bf16, double* ms3) {
    if (!ms3) return (int)hipErrorInvalidValue;
    return (int)(bf16 ? probe_overlap<true>((hipStream_t)hip_stream, ms3)
                      : probe_overlap<false>((hipStream_t)hip_stream, ms3));
}

extern "C" int bench_probe_copy(void* hip_stream, double* gbps) {
    if (!gbps) return (int)hipErrorInvalidValue;
    return (int)probe_copy((hipStream_t)hip_stream, gbps);
}
