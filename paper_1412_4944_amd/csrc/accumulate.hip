// Block accumulation P_j = Y_j X_j^T (Algorithm 1, step 5), atom-major:
// M[j][k][:] = sum over the signals of block j of x_i[k] * y_i.
//
// Determinism comes from a two-level reduction with a fixed order: the grouped signal
// list of every block is cut into pieces; one workgroup reduces one piece (each wavefront
// walks its share of the piece in order with private accumulators, which are then added
// in wave order), and a second kernel adds the piece results of a block in piece order.
// No floating-point atomics are used anywhere.
//
// The piece kernel forms the product on the matrix cores: with atoms on the M axis, the
// dimensions on the N axis and the signal index as the contraction index, one fp32 MFMA
// 32x32x2 adds two signals to a 32x32 tile of P_j.  Its A operand is the dense x_i, which
// each signal's s0 (atom, coefficient) pairs are scattered into through a 64-float row of
// wave-private LDS (written, read back as the operand, cleared again); its B operand is
// y_i straight from global memory in the lane order the instruction wants.  Accumulators
// stay in registers, so no read-modify-write traffic exists at all, and the order of
// additions is fixed by the program.
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

constexpr int kPairs = 8;                      // signal pairs per wavefront loaded before use

template <int P, int S0>
__global__ __launch_bounds__(256) void accum_partial_kernel(const float* __restrict__ Y, int K,
                                                            int piece,
                                                            const int32_t* __restrict__ offsets,
                                                            const int32_t* __restrict__ perm,
                                                            const int32_t* __restrict__ supp,
                                                            const float* __restrict__ coef,
                                                            float* __restrict__ partial) {
    constexpr int MT = P >= 32 ? P / 32 : 1;   // 32-wide tiles per side of P_j
    constexpr int PP = P * P;
    extern __shared__ int lds[];   // piece_start[K+1] | tmp[16] | xd[4][kPairs][2][64] | red[PP]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    float* xd_all = reinterpret_cast<float*>(tmp + 16);
    float* red = xd_all + 4 * kPairs * 2 * 64;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;

    for (int e = tid; e < 4 * kPairs * 2 * 64; e += 256) xd_all[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    f32x16 acc[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    float* xd = xd_all + (wave * kPairs * 2 + h) * 64;   // + u * 128 for pair u
    const int n_pairs = (cnt + 1) >> 1;
    for (int g = wave; g < n_pairs; g += 4 * kPairs) {
        int64_t i[kPairs];
#pragma unroll
        for (int u = 0; u < kPairs; ++u) {
            const int q = 2 * (g + 4 * u) + h;           // lane half h takes the pair's h-th signal
            i[u] = q < cnt ? perm[pos0 + q] : -1;
        }
        float yv[kPairs][MT], c[kPairs];
        int k[kPairs];
#pragma unroll
        for (int u = 0; u < kPairs; ++u) {
            const bool on = i[u] >= 0;
#pragma unroll
            for (int nt = 0; nt < MT; ++nt)
                yv[u][nt] = (on && nt * 32 + n < P) ? Y[i[u] * P + nt * 32 + n] : 0.f;
            k[u] = -1;
            c[u] = 0.f;
            if (on && n < S0) {
                k[u] = supp[i[u] * S0 + n];
                c[u] = coef[i[u] * S0 + n];
            }
            if ((unsigned)k[u] >= (unsigned)P) k[u] = -1;   // out-of-range atoms contribute nothing
        }
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
            if (k[u] >= 0) xd[u * 128 + k[u]] = c[u];
        float a[kPairs][MT];
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[u][mt] = xd[u * 128 + mt * 32 + n];
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
            if (k[u] >= 0) xd[u * 128 + k[u]] = 0.f;
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][mt], yv[u][nt],
                                                                       acc[mt][nt], 0, 0, 0);
    }

    // Wave accumulators are added in wave order.  Register r of tile (mt, nt) in lane
    // (h, n) is atom mt*32 + (r/4)*8 + h*4 + r%4, dimension nt*32 + n.
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int atom = mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                        const int dim = nt * 32 + n;
                        if (atom < P && dim < P) {
                            float* cell = red + atom * P + dim;
                            *cell = (w == 0) ? acc[mt][nt][r] : *cell + acc[mt][nt][r];
                        }
                    }
        }
        __syncthreads();
    }
    float* out = partial + (int64_t)id * PP;
    for (int e = tid; e < PP; e += 256) out[e] = red[e];
}

// Variant for p = 256: a p x p accumulator (64 tiles) does not fit one wavefront, so the
// four wavefronts of a workgroup split the ATOMS (64 each = 2 tile rows x 8 tile columns,
// 256 accumulator registers) and every wavefront walks all signals of the piece.  Each
// wavefront densifies only its own 64 atoms of x_i; the wave results are disjoint slabs of
// the piece's partial matrix, so no cross-wave reduction is needed.
constexpr int kWidePairs = 4;

template <int S0>
__global__ __launch_bounds__(256) void accum_wide_kernel(const float* __restrict__ Y, int K,
                                                         int piece,
                                                         const int32_t* __restrict__ offsets,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ supp,
                                                         const float* __restrict__ coef,
                                                         float* __restrict__ partial) {
    constexpr int P = 256;
    constexpr int NTL = 8;                     // 32-wide tiles along the dimensions
    extern __shared__ int lds[];               // piece_start[K+1] | tmp[16] | xd[4][kWidePairs][2][64]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    float* xd_all = reinterpret_cast<float*>(tmp + 16);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;

    for (int e = tid; e < 4 * kWidePairs * 2 * 64; e += 256) xd_all[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    f32x16 acc[2][NTL];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NTL; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int atom0 = 64 * wave;               // this wavefront's atoms: atom0 .. atom0+63
    float* xd = xd_all + (wave * kWidePairs * 2 + h) * 64;
    const int n_pairs = (cnt + 1) >> 1;
    for (int g = 0; g < n_pairs; g += kWidePairs) {
        int64_t i[kWidePairs];
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u) {
            const int q = 2 * (g + u) + h;
            i[u] = q < cnt ? perm[pos0 + q] : -1;
        }
        float yv[kWidePairs][NTL], c[kWidePairs];
        int k[kWidePairs];
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u) {
            const bool on = i[u] >= 0;
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) yv[u][nt] = on ? Y[i[u] * P + nt * 32 + n] : 0.f;
            k[u] = -1;
            c[u] = 0.f;
            if (on && n < S0) {
                k[u] = supp[i[u] * S0 + n] - atom0;
                c[u] = coef[i[u] * S0 + n];
            }
            if ((unsigned)k[u] >= 64u) k[u] = -1;          // another wavefront's atom, or invalid
        }
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u)
            if (k[u] >= 0) xd[u * 128 + k[u]] = c[u];
        float a[kWidePairs][2];
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) a[u][mt] = xd[u * 128 + mt * 32 + n];
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u)
            if (k[u] >= 0) xd[u * 128 + k[u]] = 0.f;
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][mt], yv[u][nt],
                                                                       acc[mt][nt], 0, 0, 0);
    }

    float* out = partial + (int64_t)id * P * P;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int atom = atom0 + mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                out[atom * P + nt * 32 + n] = acc[mt][nt][r];
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
    const int piece = accum_piece(m, P);
    const int max_pieces = accum_max_pieces(m, K, P);
    const size_t lds1 =
        (K + 1 + 16) * sizeof(int) + ((size_t)4 * kPairs * 2 * 64 + (size_t)P * P) * sizeof(float);
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

template <int S0>
hipError_t launch_wide_s(int K, const float* Y, int64_t m, const int32_t* supp, const float* coef,
                         const Workspace& ws, float* M, hipStream_t st) {
    constexpr int P = 256;
    const int piece = accum_piece(m, P);
    const int max_pieces = accum_max_pieces(m, K, P);
    const size_t lds1 = (K + 1 + 16) * sizeof(int) + (size_t)4 * kWidePairs * 2 * 64 * sizeof(float);
    hipLaunchKernelGGL((accum_wide_kernel<S0>), dim3(max_pieces), dim3(256), lds1, st, Y, K, piece,
                       ws.offsets, ws.perm, supp, coef, ws.partial);
    const size_t lds2 = (K + 1 + 16) * sizeof(int);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256), lds2, st,
                       K, piece, ws.offsets, ws.partial, M);
    return hipGetLastError();
}

hipError_t launch_wide(int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                       const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    switch (s0) {
#define SBO_CASE(N) \
    case N: return launch_wide_s<N>(K, Y, m, supp, coef, ws, M, st);
        SBO_CASE(1) SBO_CASE(2) SBO_CASE(3) SBO_CASE(4) SBO_CASE(5) SBO_CASE(6) SBO_CASE(7)
        SBO_CASE(8) SBO_CASE(9) SBO_CASE(10) SBO_CASE(11) SBO_CASE(12) SBO_CASE(13)
        SBO_CASE(14) SBO_CASE(15) SBO_CASE(16)
#undef SBO_CASE
        default: return hipErrorInvalidValue;
    }
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

// M[j] = sum of the piece results of block j in ws.partial, in piece order.
hipError_t launch_accum_reduce(int p, int K, int64_t m, const Workspace& ws, float* M,
                               hipStream_t st) {
    const int piece = accum_piece(m, p);
    const size_t lds = (K + 1 + 16) * sizeof(int);
    const dim3 grid(K, (p * p + 255) / 256);
    switch (p) {
        case 16: hipLaunchKernelGGL((accum_reduce_kernel<16>), grid, dim3(256), lds, st, K, piece, ws.offsets, ws.partial, M); break;
        case 32: hipLaunchKernelGGL((accum_reduce_kernel<32>), grid, dim3(256), lds, st, K, piece, ws.offsets, ws.partial, M); break;
        case 64: hipLaunchKernelGGL((accum_reduce_kernel<64>), grid, dim3(256), lds, st, K, piece, ws.offsets, ws.partial, M); break;
        case 256: hipLaunchKernelGGL((accum_reduce_kernel<256>), grid, dim3(256), lds, st, K, piece, ws.offsets, ws.partial, M); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_accumulate(int p, int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                             const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    switch (p) {
        case 16: return launch_p<16>(K, s0, Y, m, supp, coef, ws, M, st);
        case 32: return launch_p<32>(K, s0, Y, m, supp, coef, ws, M, st);
        case 64: return launch_p<64>(K, s0, Y, m, supp, coef, ws, M, st);
        case 256: return launch_wide(K, s0, Y, m, supp, coef, ws, M, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
