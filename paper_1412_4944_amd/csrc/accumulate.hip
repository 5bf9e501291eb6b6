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
#include "sbo_internal.h"
#include "device_utils.h"

namespace sbo {

namespace {

template <int P>
__global__ __launch_bounds__(256) void accum_partial_kernel(const float* __restrict__ Y, int K,
                                                            int s0, int piece,
                                                            const int32_t* __restrict__ offsets,
                                                            const int32_t* __restrict__ perm,
                                                            const int32_t* __restrict__ supp,
                                                            const float* __restrict__ coef,
                                                            float* __restrict__ partial) {
    constexpr int SLOTS = 64 / P;              // signals one wavefront handles at a time
    constexpr int PP = P * P;
    extern __shared__ int lds[];               // piece_start[K+1] | tmp[16] | acc[4][SLOTS][PP]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    float* accs = reinterpret_cast<float*>(tmp + 16);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int sl = lane / P, d = lane % P;

    for (int e = tid; e < 4 * SLOTS * PP; e += 256) accs[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    float* acc = accs + (wave * SLOTS + sl) * PP;
    for (int q0 = 0; q0 < cnt; q0 += 4 * SLOTS) {
        const int q = q0 + wave * SLOTS + sl;
        if (q < cnt) {
            const int64_t i = perm[pos0 + q];
            const float y = Y[i * P + d];
            for (int t = 0; t < s0; ++t) {
                const int k = supp[i * s0 + t];
                const float cf = coef[i * s0 + t];
                if ((unsigned)k < (unsigned)P) atomicAdd(&acc[k * P + d], cf * y);
            }
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

template <int P>
hipError_t launch_p(int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                    const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    constexpr int SLOTS = 64 / P;
    const int piece = accum_piece(m);
    const int max_pieces = accum_max_pieces(m, K);
    const size_t lds1 = (K + 1 + 16) * sizeof(int) + (size_t)4 * SLOTS * P * P * sizeof(float);
    static bool raised = false;
    if (!raised) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&accum_partial_kernel<P>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e != hipSuccess) return e;
        raised = true;
    }
    hipLaunchKernelGGL((accum_partial_kernel<P>), dim3(max_pieces), dim3(256), lds1, st, Y, K, s0,
                       piece, ws.offsets, ws.perm, supp, coef, ws.partial);
    const size_t lds2 = (K + 1 + 16) * sizeof(int);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256), lds2, st,
                       K, piece, ws.offsets, ws.partial, M);
    return hipGetLastError();
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
