// Fused second half of sparse coding and block accumulation (p <= 64), used by
// sbo_iterate: for the signals of one block, support / coefficients / residual in that
// block (Section 2; Algorithm 1 steps 3-4) and, from the same tile while it is on chip,
// its contribution to P_j = Y_j X_j^T (Algorithm 1 step 5).  Y is read from HBM once for
// both, and the sparse codes feed the product without a trip through memory.
//
// A workgroup owns one piece of one block's grouped signal list, so Q_j is staged once in
// LDS in MFMA operand order.  Each wavefront walks tiles of 32 signals: projection (atoms
// on M, signals on N), selection (select_tile.h), which leaves the tile's sparse codes in a
// wave-private LDS tile [signal][atom]; that tile, read back with atoms on M and the signal
// index as the contraction index, is the A operand of the product; y reaches the B operand's
// lane order through the same LDS tile (written at load time, read back after the
// projection, before the codes overwrite it).  Accumulators stay in registers across
// the tiles of the piece; the four waves are added in wave order, the pieces of a block in
// piece order by accum_reduce_kernel.
#include "sbo_internal.h"
#include "device_utils.h"
#include "select_tile.h"

namespace sbo {

namespace {

template <int P, int S>
__global__ __launch_bounds__(256) void select_accum_kernel(const float* __restrict__ Y,
                                                           const float* __restrict__ D, int K, int s0,
                                                           int piece,
                                                           const int32_t* __restrict__ offsets,
                                                           const int32_t* __restrict__ perm,
                                                           int32_t* __restrict__ supp,
                                                           float* __restrict__ coef,
                                                           float* __restrict__ err,
                                                           float* __restrict__ partial) {
    constexpr int KS = P / 2;
    constexpr int QN = P / 8;
    constexpr int MT = P >= 32 ? P / 32 : 1;
    constexpr int LDC = P + 1;
    constexpr int PP = P * P;
    constexpr int Q_F4 = MT * QN * 64;         // Q_j in operand order, 16-byte units

    constexpr int LDY = P + 4;                 // row stride of the tile while it holds y
    constexpr int TILE_WORDS = 32 * LDY;       // >= 32 * LDC

    extern __shared__ int lds[];  // piece_start[K+1] | tmp[16] | pad | Qs[Q_F4] f32x4 | tile[4][TILE_WORDS] | stage[4][...]
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;  // keep the 16-byte units aligned
    f32x4* Qs = reinterpret_cast<f32x4*>(lds + head);
    float* tile_all = reinterpret_cast<float*>(Qs + Q_F4);
    int* stage_all = reinterpret_cast<int*>(tile_all + 4 * TILE_WORDS);
    float* red = tile_all;                     // reused after the tile loop (PP <= 4*TILE_WORDS)

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;

    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    // Q_j -> LDS: unit (mt*QN + q)*64 + hh*32 + nn = dims hh*P/2 + 4q.. of atom mt*32 + nn
    const f32x4* D4 = reinterpret_cast<const f32x4*>(D + (int64_t)j * PP);
    for (int f = tid; f < Q_F4; f += 256) {
        const int nn = f & 31, hh = (f >> 5) & 1, mq = f >> 6;
        const int q = mq % QN, mt = mq / QN;
        const int atom = mt * 32 + nn;
        Qs[f] = atom < P ? D4[atom * (P / 4) + hh * QN + q] : f32x4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();

    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 accM[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) accM[a][b] = zero;

    float* xt = tile_all + wave * TILE_WORDS;
    int* stage = stage_all + wave * kSelectStageWords;
    const int n_tiles = (cnt + 31) >> 5;
    // Signal ids are fetched two tiles ahead and the rows of Y one tile ahead: the loads of
    // the next tile are issued as soon as the projection has consumed the current rows, and
    // land while the selection and the product run.  The loads are unconditional (lanes past
    // the end of the piece read the row of signal 0 and are zeroed when consumed).
    auto tile_id = [&](int t) -> int {
        return (t < n_tiles && n < min(32, cnt - t * 32)) ? perm[pos0 + t * 32 + n] : -1;
    };
    float yb[KS];
    auto load_rows = [&](int id) {
        const f32x4* src = reinterpret_cast<const f32x4*>(Y + (int64_t)max(id, 0) * P + h * KS);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            const f32x4 v = src[q];
            yb[4 * q + 0] = v.x;
            yb[4 * q + 1] = v.y;
            yb[4 * q + 2] = v.z;
            yb[4 * q + 3] = v.w;
        }
    };
    int i_cur = tile_id(wave), i_next = tile_id(wave + 4);
    load_rows(i_cur);
    for (int tile = wave; tile < n_tiles; tile += 4) {
        const int64_t i = i_cur;
        const bool active = i >= 0;

        // y: this lane's half row, for the projection (registers) and, transposed through
        // LDS, for the product
#pragma unroll
        for (int t = 0; t < KS; ++t) yb[t] = active ? yb[t] : 0.f;
#pragma unroll
        for (int q = 0; q < QN; ++q)
            *reinterpret_cast<f32x4*>(&xt[n * LDY + h * KS + 4 * q]) =
                f32x4{yb[4 * q], yb[4 * q + 1], yb[4 * q + 2], yb[4 * q + 3]};

        // projection c = Q_j^T y
        f32x16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) {
            acc[mt] = zero;
#pragma unroll
            for (int q = 0; q < QN; ++q) {
                const f32x4 a = Qs[(mt * QN + q) * 64 + lane];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], yb[4 * q + kk], acc[mt], 0,
                                                                   0, 0);
            }
        }
        i_cur = i_next;
        i_next = tile_id(tile + 8);
        load_rows(i_cur);                      // rows of the next tile

        // B operand of the product: lane (h, n) takes dimension nt*32 + n of signal 2*sp + h
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float yv[16][MT];
#pragma unroll
        for (int sp = 0; sp < 16; ++sp)
#pragma unroll
            for (int nt = 0; nt < MT; ++nt)
                yv[sp][nt] = nt * 32 + n < P ? xt[(2 * sp + h) * LDY + nt * 32 + n] : 0.f;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();       // y has been read; the tile now receives the codes

        // support, coefficients, residual; sparse codes of the tile left in xt[32][LDC]
        tile_select<P, S, true>(acc, h, n, active, i, s0, xt, stage, supp, coef, err);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

        // P_j += sum over the tile's signals of y x^T; two signals per MFMA (lane half h)
#pragma unroll
        for (int sp = 0; sp < 16; ++sp) {
            float a[MT];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                a[mt] = mt * 32 + n < P ? xt[(2 * sp + h) * LDC + mt * 32 + n] : 0.f;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
                    accM[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[mt], yv[sp][nt],
                                                                       accM[mt][nt], 0, 0, 0);
        }
        __builtin_amdgcn_wave_barrier();       // xt is rewritten by the next tile
    }
    __syncthreads();                           // all tiles done: their LDS becomes `red`

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
                            *cell = (w == 0) ? accM[mt][nt][r] : *cell + accM[mt][nt][r];
                        }
                    }
        }
        __syncthreads();
    }
    float* out = partial + (int64_t)id * PP;
    for (int e = tid; e < PP; e += 256) out[e] = red[e];
}

template <int P, int S>
hipError_t launch_ps(const float* Y, int64_t m, const float* D, int K, int s0, const Workspace& ws,
                     int32_t* supp, float* coef, float* err, hipStream_t st) {
    constexpr int MT = P >= 32 ? P / 32 : 1;
    const int piece = accum_piece(m, K, P);
    const int max_pieces = accum_max_pieces(m, K, P);
    const int head = ((K + 1 + 16) + 3) & ~3;
    const size_t lds = (size_t)head * sizeof(int) + (size_t)MT * (P / 8) * 64 * sizeof(f32x4) +
                       (size_t)4 * 32 * (P + 4) * sizeof(float) +
                       (size_t)4 * kSelectStageWords * sizeof(int);
    if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&select_accum_kernel<P, S>),
                                         96 * 1024);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((select_accum_kernel<P, S>), dim3(max_pieces), dim3(256), lds, st, Y, D, K, s0,
                       piece, ws.offsets, ws.perm, supp, coef, err, ws.partial);
    return hipGetLastError();
}

template <int P>
hipError_t launch_p(int s0, const float* Y, int64_t m, const float* D, int K, const Workspace& ws,
                    int32_t* supp, float* coef, float* err, hipStream_t st) {
    if (s0 <= 1) return launch_ps<P, 1>(Y, m, D, K, s0, ws, supp, coef, err, st);
    if (s0 <= 2) return launch_ps<P, 2>(Y, m, D, K, s0, ws, supp, coef, err, st);
    if (s0 <= 4) return launch_ps<P, 4>(Y, m, D, K, s0, ws, supp, coef, err, st);
    if (s0 <= 8) return launch_ps<P, 8>(Y, m, D, K, s0, ws, supp, coef, err, st);
    return launch_ps<P, 16>(Y, m, D, K, s0, ws, supp, coef, err, st);
}

}  // namespace

// Support/coefficients/residual of the grouped signals AND the per-piece partial P_j in
// ws.partial (to be summed by launch_accum_reduce).  p <= 64 only.
hipError_t launch_select_accum(int p, int K, int s0, const float* Y, int64_t m, const float* D,
                               const Workspace& ws, int32_t* supp, float* coef, float* err,
                               hipStream_t st) {
    switch (p) {
        case 16: return launch_p<16>(s0, Y, m, D, K, ws, supp, coef, err, st);
        case 32: return launch_p<32>(s0, Y, m, D, K, ws, supp, coef, err, st);
        case 64: return launch_p<64>(s0, Y, m, D, K, ws, supp, coef, err, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
