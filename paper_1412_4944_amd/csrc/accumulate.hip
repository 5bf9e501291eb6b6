// Block accumulation P_j = Y_j X_j^T (Algorithm 1, step 5), atom-major:
// M[j][k][:] = sum over the signals of block j of x_i[k] * y_i.
//
// Determinism comes from a two-level reduction with a fixed order: the grouped signal
// list of every block is cut into pieces; one workgroup reduces one piece (each wavefront
// walks its share of the piece in order with private accumulators, which are then added
// pairwise in a fixed order), and a second kernel adds the piece results of a block in piece order.
// No floating-point atomics are used anywhere.
//
// The piece kernel (p <= 64: one workgroup of 8 wavefronts per piece, as few pieces as keep
// every CU busy in one round (accum_tall_piece), each wavefront keeping the operands of several
// steps in flight) forms the product on the matrix cores: with atoms on the M axis, the
// dimensions on the N axis and the signal index as the contraction index, one fp32 MFMA
// 32x32x2 adds two signals to a 32x32 tile of P_j.  Its A operand is the dense x_i, which
// each signal's s0 (atom, coefficient) pairs are scattered into through a 64-float row of
// wave-private LDS (written, read back as the operand, cleared again); its B operand is
// y_i straight from global memory in the lane order the instruction wants.  Accumulators
// stay in registers, so no read-modify-write traffic exists at all, and the order of
// additions is fixed by the program.
#include "sbo_internal.h"
#include "device_utils.h"
#include "sq_total.h"

namespace sbo {

namespace {

constexpr int kTallWaves = 8;                  // wavefronts per workgroup (one workgroup per CU)
constexpr int kPairs = 4;                      // signal pairs per step of a wavefront
constexpr int kDepth = 6;                      // steps whose operands are in flight per wavefront

// GRAM: the A operand is y itself (S0 is not used): the piece's share of sum_i y_i y_i^T.
template <int P, int S0, bool GRAM>
__global__ __launch_bounds__(64 * kTallWaves) void accum_piece_kernel(
    const float* __restrict__ Y, int K, int piece, const int32_t* __restrict__ offsets,
    const int32_t* __restrict__ perm, const int32_t* __restrict__ supp,
    const float* __restrict__ coef, float* __restrict__ partial) {
    constexpr int MT = P >= 32 ? P / 32 : 1;   // 32-wide tiles per side of P_j
    constexpr int PP = P * P;
    constexpr int NW = kTallWaves;
    constexpr int SPS = 2 * kPairs;            // signals per step
    constexpr int ACC_F4 = MT * MT * 4 * 64;   // one wavefront's accumulators, 16-byte units
    // one lane per (signal, support entry) when the sparse codes of a step are fetched
    constexpr int EPS = S0 <= 1 ? 1 : S0 <= 2 ? 2 : S0 <= 4 ? 4 : S0 <= 8 ? 8 : 16;
    constexpr int SPI = 64 / EPS;              // signals covered by one such fetch
    constexpr int NI = (SPS + SPI - 1) / SPI;  // fetches per step
    // piece_start[K+1] | tmp[16] | pad | ids[kTallMaxPiece] | buf: xd[NW][SPS][64] while the
    // piece is walked, then [NW/2][ACC_F4] 16-byte units while the wavefronts are summed
    extern __shared__ int lds[];
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;
    int* ids = lds + head;
    float* buf = reinterpret_cast<float*>(ids + kTallMaxPiece);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, n = lane & 31;

    for (int e = tid; e < NW * SPS * 64; e += 64 * NW) buf[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);   // <= kTallMaxPiece (launcher)

    for (int q = tid; q < cnt; q += 64 * NW) ids[q] = perm[pos0 + q];
    __syncthreads();

    f32x16 acc[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    // Step G covers signals G*SPS .. G*SPS+SPS-1 of the piece; a wavefront takes steps
    // wave, wave + NW, ...  The operands of kDepth steps are in flight at any time: the ring
    // below lives in registers (every index into it is a compile-time constant).
    struct Operands {
        float yv[kPairs][MT];                  // B operand: lane (h, n) holds dim nt*32+n of signal 2u+h
        float c[NI];                           // one (atom, coefficient) of one signal per lane
        int k[NI];
    };
    // Loads are unconditional (positions past the end of the piece are clamped to its last
    // signal, columns past P to the last one): a signal past the end gets no (atom,
    // coefficient) pair in consume(), so whatever y was loaded for it is multiplied by zero,
    // and columns past P are never stored.
    const int ncol = n < P ? n : P - 1;
    const int sl_lane = lane / EPS, t_lane = lane % EPS < S0 ? lane % EPS : S0 - 1;
    auto fetch = [&](Operands& o, int G) {
#pragma unroll
        for (int u = 0; u < kPairs; ++u) {
            const int64_t i = ids[min(G * SPS + 2 * u + h, cnt - 1)];
#pragma unroll
            for (int nt = 0; nt < MT; ++nt) o.yv[u][nt] = Y[i * P + (MT > 1 ? nt * 32 + n : ncol)];
        }
        if constexpr (!GRAM) {
#pragma unroll
            for (int e = 0; e < NI; ++e) {
                const int64_t i = ids[min(G * SPS + e * SPI + sl_lane, cnt - 1)];
                o.k[e] = supp[i * S0 + t_lane];
                o.c[e] = coef[i * S0 + t_lane];
            }
        }
    };

    float* xd = buf + wave * SPS * 64;         // dense x of the step's signals, one 64-float row each
    auto consume = [&](const Operands& o, int G) {
        if constexpr (GRAM) {
#pragma unroll
            for (int u = 0; u < kPairs; ++u) {
                const bool on = G * SPS + 2 * u + h < cnt;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < MT; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(
                            on ? o.yv[u][mt] : 0.f, o.yv[u][nt], acc[mt][nt], 0, 0, 0);
            }
            return;
        }
        int k[NI];
#pragma unroll
        for (int e = 0; e < NI; ++e) {
            const int sl = e * SPI + sl_lane;
            const bool valid = sl < SPS && lane % EPS < S0 && G * SPS + sl < cnt &&
                               (unsigned)o.k[e] < (unsigned)P;   // out-of-range atoms contribute nothing
            k[e] = valid ? sl * 64 + o.k[e] : -1;
        }
#pragma unroll
        for (int e = 0; e < NI; ++e)
            if (k[e] >= 0) xd[k[e]] = o.c[e];
        float a[kPairs][MT];
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt) a[u][mt] = xd[(2 * u + h) * 64 + mt * 32 + n];
#pragma unroll
        for (int e = 0; e < NI; ++e)
            if (k[e] >= 0) xd[k[e]] = 0.f;
#pragma unroll
        for (int u = 0; u < kPairs; ++u)
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][mt], o.yv[u][nt],
                                                                       acc[mt][nt], 0, 0, 0);
    };

    // Full rounds of kDepth steps run without any condition (so that the operands of the
    // other kDepth-1 slots stay in flight while one is consumed); fetches that reach past
    // the end of the piece are clamped and never consumed.
    const int n_steps = (cnt + SPS - 1) / SPS;
    Operands ring[kDepth];
#pragma unroll
    for (int d = 0; d < kDepth; ++d) fetch(ring[d], wave + NW * d);
    int G = wave;
    for (; G + NW * (kDepth - 1) < n_steps; G += NW * kDepth) {
#pragma unroll
        for (int d = 0; d < kDepth; ++d) {
            consume(ring[d], G + NW * d);
            fetch(ring[d], G + NW * (d + kDepth));
        }
    }
#pragma unroll
    for (int d = 0; d < kDepth - 1; ++d)
        if (G + NW * d < n_steps) consume(ring[d], G + NW * d);   // uniform over the wavefront
    __syncthreads();                           // xd is dead; buf becomes the exchange area

    // Pairwise sum over the wavefronts in a fixed order: wavefront w adds w + half.
    f32x4* xch = reinterpret_cast<f32x4*>(buf);
    for (int half = NW / 2; half >= 1; half >>= 1) {
        if (wave >= half && wave < 2 * half) {
            f32x4* dst = xch + (wave - half) * ACC_F4;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4)
                        dst[((mt * MT + nt) * 4 + r4) * 64 + lane] =
                            f32x4{acc[mt][nt][4 * r4], acc[mt][nt][4 * r4 + 1],
                                  acc[mt][nt][4 * r4 + 2], acc[mt][nt][4 * r4 + 3]};
        }
        __syncthreads();
        if (wave < half) {
            const f32x4* src = xch + wave * ACC_F4;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                    for (int r4 = 0; r4 < 4; ++r4) {
                        const f32x4 v = src[((mt * MT + nt) * 4 + r4) * 64 + lane];
                        acc[mt][nt][4 * r4] += v.x;
                        acc[mt][nt][4 * r4 + 1] += v.y;
                        acc[mt][nt][4 * r4 + 2] += v.z;
                        acc[mt][nt][4 * r4 + 3] += v.w;
                    }
        }
        __syncthreads();
    }

    // Register r of tile (mt, nt) in lane (h, n) is atom mt*32 + (r/4)*8 + h*4 + r%4,
    // dimension nt*32 + n.
    if (wave == 0) {
        float* out = partial + (int64_t)id * PP;
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int atom = mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                    const int dim = nt * 32 + n;
                    if (atom < P && dim < P) out[atom * P + dim] = acc[mt][nt][r];
                }
    }
}

// Variant for p = 256: a p x p accumulator (64 tiles) does not fit one wavefront, so the
// four wavefronts of a workgroup split the ATOMS (64 each = 2 tile rows x 8 tile columns,
// 256 accumulator registers) and every wavefront walks all signals of the piece.  Each
// wavefront densifies only its own 64 atoms of x_i; the wave results are disjoint slabs of
// the piece's partial matrix, so no cross-wave reduction is needed.
constexpr int kWidePairs = 4;
constexpr int kWideMaxPiece = 4096;            // accum_piece() never returns more

template <int S0, bool GRAM>
__global__ __launch_bounds__(256) void accum_wide_kernel(const float* __restrict__ Y, int K,
                                                         int piece,
                                                         const int32_t* __restrict__ offsets,
                                                         const int32_t* __restrict__ perm,
                                                         const int32_t* __restrict__ supp,
                                                         const float* __restrict__ coef,
                                                         float* __restrict__ partial) {
    constexpr int P = 256;
    constexpr int NTL = 8;                     // 32-wide tiles along the dimensions
    // piece_start[K+1] | tmp[16] | xd[4][kWidePairs][2][64] | ids[kWideMaxPiece]
    extern __shared__ int lds[];
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    float* xd_all = reinterpret_cast<float*>(tmp + 16);
    int* ids = reinterpret_cast<int*>(xd_all + 4 * kWidePairs * 2 * 64);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, n = lane & 31;

    for (int e = tid; e < 4 * kWidePairs * 2 * 64; e += 256) xd_all[e] = 0.f;
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);   // <= kWideMaxPiece (launcher)
    for (int q = tid; q < cnt; q += 256) ids[q] = perm[pos0 + q];
    __syncthreads();

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

    // Operands of a step (kWidePairs signal pairs; lane half h takes the h-th signal of a pair).
    // Two sets alternate, so that the loads of the next step are in flight while the current
    // one feeds the matrix cores.  Loads are unconditional: positions past the end of the
    // piece are clamped to its last signal and get no (atom, coefficient) pair when consumed.
    struct Operands {
        float yv[kWidePairs][NTL], c[kWidePairs];
        int k[kWidePairs];
    };
    const int t_lane = n < S0 ? n : S0 - 1;
    auto fetch = [&](Operands& o, int g) {
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u) {
            const int64_t i = ids[min(2 * (g + u) + h, cnt - 1)];
#pragma unroll
            for (int nt = 0; nt < NTL; ++nt) o.yv[u][nt] = Y[i * P + nt * 32 + n];
            if constexpr (!GRAM) {
                o.k[u] = supp[i * S0 + t_lane];
                o.c[u] = coef[i * S0 + t_lane];
            }
        }
    };
    auto consume = [&](const Operands& o, int g) {
        float a[kWidePairs][2];
        if constexpr (GRAM) {                              // rows atom0.. of sum_i y_i y_i^T
#pragma unroll
            for (int u = 0; u < kWidePairs; ++u) {
                const bool on = 2 * (g + u) + h < cnt;
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    a[u][mt] = 0.f;
#pragma unroll
                    for (int w = 0; w < 4; ++w)
                        a[u][mt] = (on && wave == w) ? o.yv[u][2 * w + mt] : a[u][mt];
                }
            }
        } else {
            int k[kWidePairs];
#pragma unroll
            for (int u = 0; u < kWidePairs; ++u) {
                const int kk = o.k[u] - atom0;
                const bool valid = 2 * (g + u) + h < cnt && n < S0 &&
                                   (unsigned)kk < 64u;     // another wavefront's atom, or invalid
                k[u] = valid ? u * 128 + kk : -1;
            }
#pragma unroll
            for (int u = 0; u < kWidePairs; ++u)
                if (k[u] >= 0) xd[k[u]] = o.c[u];
#pragma unroll
            for (int u = 0; u < kWidePairs; ++u)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) a[u][mt] = xd[u * 128 + mt * 32 + n];
#pragma unroll
            for (int u = 0; u < kWidePairs; ++u)
                if (k[u] >= 0) xd[k[u]] = 0.f;
        }
#pragma unroll
        for (int u = 0; u < kWidePairs; ++u)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int nt = 0; nt < NTL; ++nt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[u][mt], o.yv[u][nt],
                                                                       acc[mt][nt], 0, 0, 0);
    };

    Operands opA, opB;
    fetch(opA, 0);
    for (int g = 0; g < n_pairs; g += 2 * kWidePairs) {
        fetch(opB, g + kWidePairs);
        consume(opA, g);
        fetch(opA, g + 2 * kWidePairs);
        consume(opB, g + kWidePairs);          // past the end: contributes nothing
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

// p = 256 on the bf16 matrix cores (three-part split of both operands, six partial products,
// fp32 accumulation: device_utils.h).  Same division of the work as accum_wide_kernel (a piece per
// workgroup, 64 atoms per wavefront, 256 accumulator registers), but a step covers 16 signals, the
// contraction length of v_mfma_f32_32x32x16_bf16, and both operands go through LDS tiles with the
// signals along the rows' 32 bytes, built by the whole workgroup while the matrix cores work on
// the previous step's tiles (two sets of tiles):
//   y tile [3 parts][256 dims][16 signals]: thread t loads dim t of the 16 signals (each load of a
//          wavefront is 256 contiguous bytes), splits pairs of signals and stores two 16-byte units;
//   x tile [3 parts][256 atoms + 1][16 signals]: zero-filled, then one thread per (signal, entry)
//          scatters the three parts of a kept coefficient (entries that do not exist go to the
//          extra row, which nobody reads).
// The loads of a step are issued two steps ahead.
constexpr int kAwsSignals = 16;

template <int S0>
__global__ __launch_bounds__(256) void accum_wide_split_kernel(const float* __restrict__ Y, int K, int piece,
                                                               const int32_t* __restrict__ offsets,
                                                               const int32_t* __restrict__ perm,
                                                               const int32_t* __restrict__ supp,
                                                               const float* __restrict__ coef,
                                                               float* __restrict__ partial) {
    constexpr int P = 256;
    constexpr int NTL = 8;                     // 32-wide tiles along the dimensions
    constexpr int G = kAwsSignals;
    constexpr int YPLANE = P * 32;             // bytes of one part of the y tile
    constexpr int XPLANE = (P + 1) * 32;       // bytes of one part of the x tile (+ the extra row)
    constexpr int SET_B = 3 * YPLANE + 3 * XPLANE;
    static_assert(G * S0 <= 256, "one thread per (signal, entry)");
    // piece_start[K+1] | tmp[16] | pad | ids[kWideMaxPiece] | two sets of (y tile, x tile)
    extern __shared__ int lds[];
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;
    int* ids = lds + head;
    unsigned char* sets = reinterpret_cast<unsigned char*>(ids + kWideMaxPiece);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, n = lane & 31;

    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);   // <= kWideMaxPiece (launcher)
    for (int q = tid; q < cnt; q += 256) ids[q] = perm[pos0 + q];
    __syncthreads();

    f32x16 acc[2][NTL];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NTL; ++b)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[a][b][r] = 0.f;

    const int atom0 = 64 * wave;               // this wavefront's atoms: atom0 .. atom0+63
    const int n_steps = (cnt + G - 1) / G;

    // What a thread fetches for a step: dim `tid` of its 16 signals, and one (atom, coefficient)
    // of one signal (threads below 16 * S0).  Positions past the end of the piece are clamped
    // for the loads and masked when the tiles are built.
    struct Fetched {
        float y[G];
        int k;
        float c;
    };
    const int e_sig = tid / S0, e_ent = tid % S0;
    auto fetch = [&](Fetched& f, int g) {
#pragma unroll
        for (int u = 0; u < G; ++u) {
            const int64_t i = ids[min(g * G + u, cnt - 1)];
            f.y[u] = Y[i * P + tid];
        }
        const int64_t i = ids[min(g * G + min(e_sig, G - 1), cnt - 1)];
        f.k = supp[i * S0 + e_ent];
        f.c = coef[i * S0 + e_ent];
    };
    auto zero_x = [&](int set) {
        u32x4* xt = reinterpret_cast<u32x4*>(sets + (size_t)set * SET_B + 3 * YPLANE);
        for (int e = tid; e < 3 * XPLANE / 16; e += 256) xt[e] = u32x4{0u, 0u, 0u, 0u};
    };
    auto build = [&](const Fetched& f, int g, int set) {
        unsigned char* yt = sets + (size_t)set * SET_B;
        unsigned char* xt = yt + 3 * YPLANE;
        const int left = cnt - g * G;          // signals of this step (uniform)
        unsigned w[3][8];
#pragma unroll
        for (int u = 0; u < G; u += 2) {
            const Bf16x3Pair s = split_bf16x3(u < left ? f.y[u] : 0.f, u + 1 < left ? f.y[u + 1] : 0.f);
            w[0][u >> 1] = s.hi;
            w[1][u >> 1] = s.mid;
            w[2][u >> 1] = s.lo;
        }
#pragma unroll
        for (int pl = 0; pl < 3; ++pl) {
            *reinterpret_cast<u32x4*>(yt + pl * YPLANE + tr_off(tid, 0)) = u32x4{w[pl][0], w[pl][1], w[pl][2], w[pl][3]};
            *reinterpret_cast<u32x4*>(yt + pl * YPLANE + tr_off(tid, 8)) = u32x4{w[pl][4], w[pl][5], w[pl][6], w[pl][7]};
        }
        const bool have = tid < G * S0 && e_sig < left && (unsigned)f.k < (unsigned)P;
        const TriWord t = split_trunc(f.c);
        const int at = tr_off(have ? f.k : P, e_sig & (G - 1));
        if (tid < G * S0) {
            *reinterpret_cast<unsigned short*>(xt + at) = (unsigned short)(t.hi >> 16);
            *reinterpret_cast<unsigned short*>(xt + XPLANE + at) = (unsigned short)(t.mid >> 16);
            *reinterpret_cast<unsigned short*>(xt + 2 * XPLANE + at) = (unsigned short)(t.lo >> 16);
        }
    };
    // the six partial products, smallest first: (A part, B part)
    constexpr int TA[6] = {2, 0, 1, 1, 0, 0};
    constexpr int TB[6] = {0, 2, 1, 0, 1, 0};
    auto multiply = [&](int set) {
        const unsigned char* yt = sets + (size_t)set * SET_B;
        const unsigned char* xt = yt + 3 * YPLANE;
        // operands: lane (h, n) takes signals 8h .. 8h+7 of atom resp. dim tile*32 + n
        u32x4 xa[2][3];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                xa[mt][pl] = *reinterpret_cast<const u32x4*>(xt + pl * XPLANE + tr_off(atom0 + mt * 32 + n, 8 * h));
#pragma unroll
        for (int nt = 0; nt < NTL; ++nt) {
            u32x4 yb[3];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl)
                yb[pl] = *reinterpret_cast<const u32x4*>(yt + pl * YPLANE + tr_off(nt * 32 + n, 8 * h));
#pragma unroll
            for (int t = 0; t < 6; ++t)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
                    acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, xa[mt][TA[t]]), __builtin_bit_cast(bf16x8, yb[TB[t]]), acc[mt][nt],
                        0, 0, 0);
        }
    };

    // step g: its tiles are built during the multiplication of step g - 1 and its loads were issued
    // during that of step g - 2
    Fetched fa, fb;
    fetch(fa, 0);
    fetch(fb, 1);
    zero_x(0);
    __syncthreads();
    build(fa, 0, 0);
    fetch(fa, 2);
    __syncthreads();
    for (int g = 0; g < n_steps; g += 2) {
        // even step g from set 0; meanwhile the tiles of step g + 1 in set 1
        zero_x(1);
        __syncthreads();
        build(fb, g + 1, 1);
        fetch(fb, g + 3);
        multiply(0);
        __syncthreads();
        // odd step g + 1 from set 1; meanwhile the tiles of step g + 2 in set 0
        zero_x(0);
        __syncthreads();
        build(fa, g + 2, 0);
        fetch(fa, g + 4);
        multiply(1);                           // past the end: its tiles hold zeros
        __syncthreads();
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

// Besides the sums over pieces (blockIdx.x < K), nb workgroups in the grid columns from K on form
// the total squared error sum_i err[i] (sq_out != nullptr; see sq_total.h).
template <int P>
__global__ __launch_bounds__(256) void accum_reduce_kernel(int K, int piece,
                                                           const int32_t* __restrict__ offsets,
                                                           const float* __restrict__ partial,
                                                           float* __restrict__ M,
                                                           const float* __restrict__ err, int64_t m,
                                                           double* sq_part, int* sq_counter,
                                                           double* __restrict__ sq_out, int nb) {
    constexpr int PP = P * P;
    extern __shared__ int lds[];               // piece_start[K+1] | tmp[16]
    if ((int)blockIdx.x >= K) {                // uniform over the workgroup
        // the nb workgroups of the squared-error sum occupy the grid columns from K on
        const int b = ((int)blockIdx.x - K) * (int)gridDim.y + (int)blockIdx.y;
        if (sq_out == nullptr || b >= nb) return;
        __shared__ double sq_lds[256 + 1];
        sq_total_part<256>(err, m, b, nb, sq_part, sq_counter, sq_out, sq_lds);
        return;
    }
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
    constexpr int MT = P >= 32 ? P / 32 : 1;
    const int piece = accum_tall_piece(m, K);
    const int max_pieces = (int)((m + piece - 1) / piece) + K;
    const size_t head = ((size_t)(K + 1 + 16) + 3) & ~(size_t)3;
    const size_t walk = (size_t)kTallWaves * 2 * kPairs * 64;
    const size_t xch = (size_t)(kTallWaves / 2) * MT * MT * 16 * 64;
    const size_t lds1 = (head + kTallMaxPiece + (walk > xch ? walk : xch)) * 4;
    if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&accum_piece_kernel<P, S0, false>),
                                         144 * 1024);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((accum_piece_kernel<P, S0, false>), dim3(max_pieces), dim3(64 * kTallWaves), lds1, st,
                       Y, K, piece, ws.offsets, ws.perm, supp, coef, ws.partial);
    const size_t lds2 = (K + 1 + 16) * sizeof(int);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256), lds2, st,
                       K, piece, ws.offsets, ws.partial, M, nullptr, (int64_t)0, nullptr, nullptr, nullptr, 0);
    return hipGetLastError();
}

template <int S0>
hipError_t launch_wide_s(int K, const float* Y, int64_t m, const int32_t* supp, const float* coef,
                         const Workspace& ws, float* M, bool split, hipStream_t st) {
    constexpr int P = 256;
    const int piece = accum_piece(m, K, P);
    const int max_pieces = accum_max_pieces(m, K, P);
    const size_t lds1 = (K + 1 + 16 + kWideMaxPiece) * sizeof(int) + (size_t)4 * kWidePairs * 2 * 64 * sizeof(float);
    if (split) {
        const int head = ((K + 1 + 16) + 3) & ~3;
        const size_t lds = (size_t)(head + kWideMaxPiece) * sizeof(int) +
                           (size_t)2 * (3 * P * 32 + 3 * (P + 1) * 32);
        if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&accum_wide_split_kernel<S0>), lds);
            e != hipSuccess)
            return e;
        hipLaunchKernelGGL((accum_wide_split_kernel<S0>), dim3(max_pieces), dim3(256), lds, st, Y, K, piece,
                           ws.offsets, ws.perm, supp, coef, ws.partial);
    } else {
        hipLaunchKernelGGL((accum_wide_kernel<S0, false>), dim3(max_pieces), dim3(256), lds1, st, Y, K, piece,
                           ws.offsets, ws.perm, supp, coef, ws.partial);
    }
    const size_t lds2 = (K + 1 + 16) * sizeof(int);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256), lds2, st,
                       K, piece, ws.offsets, ws.partial, M, nullptr, (int64_t)0, nullptr, nullptr, nullptr, 0);
    return hipGetLastError();
}

hipError_t launch_wide(int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                       const float* coef, const Workspace& ws, float* M, bool split, hipStream_t st) {
    switch (s0) {
#define SBO_CASE(N) \
    case N: return launch_wide_s<N>(K, Y, m, supp, coef, ws, M, split, st);
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

// G[j] = sum over the signals of block j (ws.perm / ws.offsets, n signals in all) of y y^T.
template <int P>
hipError_t launch_gram_p(int K, const float* Y, int64_t n, const Workspace& ws, float* G,
                         hipStream_t st) {
    constexpr int MT = P >= 32 ? P / 32 : 1;
    const int piece = accum_tall_piece(n, K);
    const int max_pieces = (int)((n + piece - 1) / piece) + K;
    const size_t head = ((size_t)(K + 1 + 16) + 3) & ~(size_t)3;
    const size_t walk = (size_t)kTallWaves * 2 * kPairs * 64;
    const size_t xch = (size_t)(kTallWaves / 2) * MT * MT * 16 * 64;
    const size_t lds1 = (head + kTallMaxPiece + (walk > xch ? walk : xch)) * 4;
    if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&accum_piece_kernel<P, 1, true>),
                                         144 * 1024);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((accum_piece_kernel<P, 1, true>), dim3(max_pieces), dim3(64 * kTallWaves), lds1, st,
                       Y, K, piece, ws.offsets, ws.perm, nullptr, nullptr, ws.partial);
    hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256),
                       (K + 1 + 16) * sizeof(int), st, K, piece, ws.offsets, ws.partial, G, nullptr,
                       (int64_t)0, nullptr, nullptr, nullptr, 0);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gram(int p, int K, const float* Y, int64_t n, const Workspace& ws, float* G,
                       hipStream_t st) {
    switch (p) {
        case 16: return launch_gram_p<16>(K, Y, n, ws, G, st);
        case 32: return launch_gram_p<32>(K, Y, n, ws, G, st);
        case 64: return launch_gram_p<64>(K, Y, n, ws, G, st);
        case 256: {
            constexpr int P = 256;
            const int piece = accum_piece(n, K, P);
            const int max_pieces = (int)((n + piece - 1) / piece) + K;
            const size_t lds1 = (K + 1 + 16 + kWideMaxPiece) * sizeof(int) + (size_t)4 * kWidePairs * 2 * 64 * sizeof(float);
            hipLaunchKernelGGL((accum_wide_kernel<1, true>), dim3(max_pieces), dim3(256), lds1, st, Y, K,
                               piece, ws.offsets, ws.perm, nullptr, nullptr, ws.partial);
            hipLaunchKernelGGL((accum_reduce_kernel<P>), dim3(K, (P * P + 255) / 256), dim3(256),
                               (K + 1 + 16) * sizeof(int), st, K, piece, ws.offsets, ws.partial, G, nullptr,
                               (int64_t)0, nullptr, nullptr, nullptr, 0);
            return hipGetLastError();
        }
        default: return hipErrorInvalidValue;
    }
}

// M[j] = sum of the piece results of block j in ws.partial, in piece order; with sq_out also
// *sq_out = sum of err[0..m) (same launch, extra workgroups).
hipError_t launch_accum_reduce(int p, int K, int64_t m, const Workspace& ws, float* M,
                               const float* err, double* sq_out, hipStream_t st) {
    const int piece = accum_piece(m, K, p);
    const size_t lds = (K + 1 + 16) * sizeof(int);
    const int gy = (p * p + 255) / 256;
    const bool sq = err != nullptr && sq_out != nullptr;
    const int nb = sq ? 128 : 0;               // <= kSqBlocks shares of err
    const dim3 grid(K + (nb + gy - 1) / gy, gy);
    double* so = sq ? sq_out : nullptr;
#define SBO_CASE(N)                                                                              \
    case N:                                                                                      \
        hipLaunchKernelGGL((accum_reduce_kernel<N>), grid, dim3(256), lds, st, K, piece, ws.offsets, \
                           ws.partial, M, err, m, ws.sq_partial, ws.sq_counter, so, nb);         \
        break;
    switch (p) {
        SBO_CASE(16) SBO_CASE(32) SBO_CASE(64) SBO_CASE(256)
        default: return hipErrorInvalidValue;
    }
#undef SBO_CASE
    return hipGetLastError();
}

hipError_t launch_accumulate(int p, int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                             const float* coef, const Workspace& ws, float* M, hipStream_t st) {
    switch (p) {
        case 16: return launch_p<16>(K, s0, Y, m, supp, coef, ws, M, st);
        case 32: return launch_p<32>(K, s0, Y, m, supp, coef, ws, M, st);
        case 64: return launch_p<64>(K, s0, Y, m, supp, coef, ws, M, st);
        case 256: return launch_wide(K, s0, Y, m, supp, coef, ws, M, ws.parts_accum, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
