// Block accumulation P_j = Y_j X_j^T (Algorithm 1, step 5), atom-major:
// M[j][k][:] = sum over the signals of block j of x_i[k] * y_i.
//
// X is s0-sparse per signal, so this is s0 scaled row additions per signal and the
// stage is bound by reading Y once.  Determinism comes from a two-level reduction with
// a fixed order: the grouped signal list of every block is cut into pieces; one
// workgroup reduces one piece (each wavefront walks its share of the piece in order
// and owns a private p x p accumulator in LDS; the wave accumulators are then added in
// wave order), and a second kernel adds the piece results of a block in piece order.
// No floating-point atomics touch memory shared between wavefronts.
//
// Lane layout inside a wavefront: 64/p signals side by side ("slots"), lane % p = the
// dimension d it owns.  Every 16-lane row also loads the signal's (atom, coefficient)
// pairs, lane % 16 = t, so that the t-th pair reaches all lanes of the row with a DPP
// row broadcast instead of a trip through scalar registers.  Several signals per slot
// are kept in flight to cover HBM latency.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int kInFlight = 8;                   // signals per slot loaded before any is used

// Value of lane (row base + T) for every lane of each 16-lane row.
template <int T>
__device__ __forceinline__ int row_bcast(int v) {
    return __builtin_amdgcn_update_dpp(0, v, 0x150 + T, 0xf, 0xf, true);
}

// acc_d[k_t * P] += c_t * y for the s0 (atom, coefficient) pairs of ONE signal per slot.
// The LDS cells are read, updated and written back in three batches so that the reads
// overlap; this needs the atoms of a signal to be distinct, which a support is.
// (LDS floating-point atomics would also do, but they retire only a few lanes per
// clock on this chip.)
template <int T0>
__device__ __forceinline__ int row_bcast_dyn(int v, int t) {   // t is a compile-time constant after unrolling
    switch (T0 + t) {
        case 0: return row_bcast<0>(v);
        case 1: return row_bcast<1>(v);
        case 2: return row_bcast<2>(v);
        case 3: return row_bcast<3>(v);
        case 4: return row_bcast<4>(v);
        case 5: return row_bcast<5>(v);
        case 6: return row_bcast<6>(v);
        case 7: return row_bcast<7>(v);
        case 8: return row_bcast<8>(v);
        case 9: return row_bcast<9>(v);
        case 10: return row_bcast<10>(v);
        case 11: return row_bcast<11>(v);
        case 12: return row_bcast<12>(v);
        case 13: return row_bcast<13>(v);
        case 14: return row_bcast<14>(v);
        default: return row_bcast<15>(v);
    }
}

template <int T0, int N>
__device__ __forceinline__ void add_rows(float* acc_d, int koff, float cf, float y) {
    int ko[N];
    float c[N], v[N];
#pragma unroll
    for (int t = 0; t < N; ++t) {
        ko[t] = row_bcast_dyn<T0>(koff, t);
        c[t] = __builtin_bit_cast(float, row_bcast_dyn<T0>(__builtin_bit_cast(int, cf), t));
    }
#pragma unroll
    for (int t = 0; t < N; ++t) v[t] = acc_d[ko[t]];
#pragma unroll
    for (int t = 0; t < N; ++t) v[t] = fmaf(c[t], y, v[t]);
#pragma unroll
    for (int t = 0; t < N; ++t) acc_d[ko[t]] = v[t];
}

template <int P, int S0>
__global__ __launch_bounds__(256) void accum_partial_kernel(const float* __restrict__ Y, int K,
                                                            int piece,
                                                            const int32_t* __restrict__ offsets,
                                                            const int32_t* __restrict__ perm,
                                                            const int32_t* __restrict__ supp,
                                                            const float* __restrict__ coef,
                                                            float* __restrict__ partial) {
    constexpr int SLOTS = 64 / P;              // signals one wavefront handles side by side
    constexpr int PP = P * P;
    extern __shared__ int lds[];               // piece_start[K+1] | tmp[16] | acc[4][SLOTS][PP]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    float* accs = reinterpret_cast<float*>(tmp + 16);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sl = lane / P, d = lane % P, t = lane & 15;

    for (int e = tid; e < 4 * SLOTS * PP; e += 256) accs[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    float* acc_d = accs + (wave * SLOTS + sl) * PP + d;
    constexpr int STRIDE = 4 * SLOTS;          // signals consumed per step by the workgroup
    for (int q0 = 0; q0 < cnt; q0 += STRIDE * kInFlight) {
        int64_t i[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const int q = q0 + u * STRIDE + wave * SLOTS + sl;
            i[u] = q < cnt ? perm[pos0 + q] : -1;
        }
        int koff[kInFlight];
        float cf[kInFlight], y[kInFlight];
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            const bool on = i[u] >= 0;
            y[u] = on ? Y[i[u] * P + d] : 0.f;
            int k = 0;
            float c = 0.f;
            if (on && t < S0) {
                k = supp[i[u] * S0 + t];
                c = coef[i[u] * S0 + t];
            }
            if ((unsigned)k >= (unsigned)P) {  // out-of-range atom ids contribute nothing
                k = 0;
                c = 0.f;
            }
            koff[u] = k * P;
            cf[u] = c;
        }
#pragma unroll
        for (int u = 0; u < kInFlight; ++u) {
            constexpr int HEAD = S0 < 8 ? S0 : 8;
            add_rows<0, HEAD>(acc_d, koff[u], cf[u], y[u]);
            if constexpr (S0 > 8) add_rows<8, S0 - 8>(acc_d, koff[u], cf[u], y[u]);
        }
    }
    __syncthreads();
    float* out = partial + (int64_t)id * PP;
    for (int e = tid; e < PP; e += 256) {
        float s = 0.f;
#pragma unroll
        for (int w = 0; w < 4 * SLOTS; ++w) s += accs[w * PP + e];
        out[e] = s;
    }
}

template <int P>
__global__ __launch_bounds__(256) void accum_reduce_kernel(int K, int piece,
                                                           const int32_t* __restrict__ offsets,
                                                           const float* __restrict__ partial,
                                                           float* __restrict__ M) {
    constexpr int PP = P * P;
    extern __shared__ int lds[];               // piece_start[K+1] | tmp[16]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int j = blockIdx.x;
    const int e = blockIdx.y * 256 + threadIdx.x;
    if (e >= PP) return;
    float s = 0.f;
    for (int pc = piece_start[j]; pc < piece_start[j + 1]; ++pc) s += partial[(int64_t)pc * PP + e];
    M[(int64_t)j * PP + e] = s;
}

template <int P, int S0>
hipError_t launch_ps(int K, const float* Y, int64_t m, const int32_t* supp, const float* coef,
                     const Workspace& ws, float* M, hipStream_t st) {
    constexpr int SLOTS = 64 / P;
    const int piece = accum_piece(m);
    const int max_pieces = accum_max_pieces(m, K);
    const size_t lds1 = (K + 1 + 16) * sizeof(int) + (size_t)4 * SLOTS * P * P * sizeof(float);
    static bool raised = false;
    if (!raised) {
        hipError_t e =
            hipFuncSetAttribute(reinterpret_cast<const void*>(&accum_partial_kernel<P, S0>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((accum_partial_kernel<P, S0>), dim3(max_pieces), dim3(256), lds1, st, Y, K,
                       piece, ws.offsets, ws.perm, supp, coef, ws.partial);
    const size_t lds2 = (K + 1 + 16) * sizeof(int);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256), lds2, st,
                       K, piece, ws.offsets, ws.partial, M);
    return hipGetLastError();
}

template <int P>
hipError_t launch_p(int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                    const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    switch (s0) {
#define SBO_CASE(N) \
    case N: return launch_ps<P, N>(K, Y, m, supp, coef, ws, M, st);
        SBO_CASE(1) SBO_CASE(2) SBO_CASE(3) SBO_CASE(4) SBO_CASE(5) SBO_CASE(6) SBO_CASE(7)
        SBO_CASE(8) SBO_CASE(9) SBO_CASE(10) SBO_CASE(11) SBO_CASE(12) SBO_CASE(13)
        SBO_CASE(14) SBO_CASE(15) SBO_CASE(16)
#undef SBO_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_accumulate(int p, int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                             const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    switch (p) {
        case 16: return launch_p<16>(K, s0, Y, m, supp, coef, ws, M, st);
        case 32: return launch_p<32>(K, s0, Y, m, supp, coef, ws, M, st);
        case 64: return launch_p<64>(K, s0, Y, m, supp, coef, ws, M, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
