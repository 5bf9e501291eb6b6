// Fused second half of sparse coding and block accumulation (p <= 64), used by
// sbo_iterate, sbo_train_rounds and sbo_new_base: for the signals of one block, support /
// coefficients / residual in that block (Section 2; Algorithm 1 steps 3-4) and, from the same
// tile while it is on chip, its contribution to P_j = Y_j X_j^T (Algorithm 1 step 5).  Y is
// read from HBM once for both, and the sparse codes feed the product without a trip through
// memory.
//
// A workgroup (8 wavefronts, one workgroup per CU) owns one piece of one block's grouped signal
// list.  Both contractions run on the bf16 matrix cores at fp32 accuracy: every fp32 operand
// entry is the exact sum of three bf16 parts and the six partial products above 2^-24 are
// accumulated in fp32 (device_utils.h).  Q_j is split once per workgroup into LDS in MFMA
// operand order.  Each wavefront walks tiles of 32 signals:
//   projection  c = Q_j^T y : atoms on M, signals on N, dims contracted; y is split in registers
//                             (a lane holds its own signal's dims);
//   selection   (select_tile.h) from the accumulators;
//   product     P_j += x y^T: atoms on M, dims on N, SIGNALS contracted, so both operands are
//                             needed with eight consecutive signals per lane: the split parts of
//                             y go through a wave-private LDS tile [dim][signal] (lane pairs
//                             exchange halves so that every write is a whole word), the s0 kept
//                             coefficients of every signal are scattered into a zeroed tile
//                             [atom][signal] and wiped again after use; 16 signals at a time.
// Accumulators stay in registers across the tiles of the piece; the wavefronts are added in
// wavefront order, the pieces of a block in piece order by the kernel that consumes them.
#include "sbo_internal.h"
#include "device_utils.h"
#include "select_tile.h"

namespace sbo {

namespace {

constexpr int kSaWaves = 8;


template <int P, int S>
__global__ __launch_bounds__(64 * kSaWaves) void select_accum_kernel(
    const float* __restrict__ Y, const float* __restrict__ D, int K, int s0, int piece,
    const int32_t* __restrict__ offsets, const int32_t* __restrict__ perm, int32_t* __restrict__ supp,
    float* __restrict__ coef, float* __restrict__ err, float* __restrict__ partial) {
    constexpr int NW = kSaWaves, NTH = 64 * NW;
    constexpr int KS16 = P / 16;               // projection: steps of 16 dims
    constexpr int MT = P >= 32 ? P / 32 : 1;   // 32-wide tiles per side of P_j
    constexpr int ROWS = MT * 32;              // operand tile rows (atoms resp. dims; rows >= P are not used)
    constexpr int PP = P * P;
    constexpr int Q_U = MT * KS16 * 3 * 64;    // Q_j in split operand order, 16-byte units
    constexpr int PLANE_B = (ROWS + 1) * 32;   // bytes of one part of a transposed operand tile (+ a dummy row)
    constexpr int CT_B = 32 * (P + 1) * 4;     // tie-breaking scratch of tile_select
    constexpr int OPS_B = 6 * PLANE_B;         // x tile (3 parts) + y tile (3 parts)
    constexpr int REGION_B = (OPS_B > CT_B ? OPS_B : CT_B);
    constexpr int WAVE_B = kSelectStageWords * 4 + REGION_B;

    // piece_start[K+1] | tmp[16] | pad | Qs[Q_U] | per wavefront: stage | region
    extern __shared__ int lds[];
    int* piece_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;  // keep the 16-byte units aligned
    u32x4* Qs = reinterpret_cast<u32x4*>(lds + head);
    unsigned char* waves_base = reinterpret_cast<unsigned char*>(Qs + Q_U);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, n = lane & 31;

    // pieces per block, as every kernel that walks the pieces counts them (K <= 4 * NTH)
    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + piece - 1) / piece; }, K,
                       piece_start, tmp);
    const int id = blockIdx.x;
    if (id >= piece_start[K]) return;          // uniform over the workgroup

    const int j = upper_slot(piece_start, K, id);
    const int pos0 = offsets[j] + (id - piece_start[j]) * piece;
    const int cnt = min(piece, offsets[j + 1] - pos0);

    // Q_j -> LDS, split: unit ((mt*KS16 + ks)*3 + part)*64 + hh*32 + nn = the 8 bf16 of that part
    // of dims ks*16 + hh*8 .. +7 of atom mt*32 + nn (atoms >= P: zeros)
    {
        const f32x4* D4 = reinterpret_cast<const f32x4*>(D + (int64_t)j * PP);
        for (int g = tid; g < MT * KS16 * 64; g += NTH) {
            const int ln = g & 63, mk = g >> 6;
            const int nn = ln & 31, hh = ln >> 5, ks = mk % KS16, mt = mk / KS16;
            const int atom = mt * 32 + nn;
            f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
            if (atom < P) {
                v0 = D4[atom * (P / 4) + ks * 4 + hh * 2];
                v1 = D4[atom * (P / 4) + ks * 4 + hh * 2 + 1];
            }
            const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
            const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
            u32x4* out = Qs + (mk * 3) * 64 + ln;
            out[0] = u32x4{a.hi, b.hi, c.hi, d.hi};
            out[64] = u32x4{a.mid, b.mid, c.mid, d.mid};
            out[128] = u32x4{a.lo, b.lo, c.lo, d.lo};
        }
    }
    int* stage = reinterpret_cast<int*>(waves_base + (size_t)wave * WAVE_B);
    unsigned char* region = reinterpret_cast<unsigned char*>(stage + kSelectStageWords);
    unsigned char* xt = region;                // [3 parts][ROWS atoms][16 signals] bf16
    unsigned char* yt = region + 3 * PLANE_B;  // [3 parts][ROWS dims][16 signals] bf16
    // the x tile starts out zero (and is left zero by every tile)
    for (int e = lane; e < 3 * PLANE_B / 16; e += 64) reinterpret_cast<u32x4*>(xt)[e] = u32x4{0u, 0u, 0u, 0u};
    __syncthreads();

    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 accM[MT][MT];
#pragma unroll
    for (int a = 0; a < MT; ++a)
#pragma unroll
        for (int b = 0; b < MT; ++b) accM[a][b] = zero;
    // the six partial products, smallest first: (A part, B part)
    constexpr int TA[6] = {2, 0, 1, 1, 0, 0};
    constexpr int TB[6] = {0, 2, 1, 0, 1, 0};

    const int n_tiles = (cnt + 31) >> 5;
    // Signal ids are fetched two tiles ahead and the rows of Y one tile ahead: the loads of
    // the next tile are issued as soon as the current rows have been split, and land while
    // the matrix work and the selection run.  The loads are unconditional (lanes past the end
    // of the piece read the row of signal 0 and are zeroed when consumed).
    auto tile_id = [&](int t) -> int {
        return (t < n_tiles && n < min(32, cnt - t * 32)) ? perm[pos0 + t * 32 + n] : -1;
    };
    f32x4 raw[KS16][2];                        // this lane's dims ks*16 + h*8 .. +7 of its signal
    auto load_rows = [&](int sid) {
        const f32x4* src = reinterpret_cast<const f32x4*>(Y + (int64_t)max(sid, 0) * P + h * 8);
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            raw[ks][0] = src[ks * 4];
            raw[ks][1] = src[ks * 4 + 1];
        }
    };
    int i_cur = tile_id(wave), i_next = tile_id(wave + NW);
    load_rows(i_cur);
    for (int tile = wave; tile < n_tiles; tile += NW) {
        const int64_t i = i_cur;
        const bool active = i >= 0;
        const int cnt_t = min(32, cnt - tile * 32);        // signals in this tile (uniform)

        // y in three bf16 parts (B operand of the projection)
        u32x4 yq[KS16][3];
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            f32x4 v0 = raw[ks][0], v1 = raw[ks][1];
            if (!active) {
                v0 = f32x4{0.f, 0.f, 0.f, 0.f};
                v1 = v0;
            }
            const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
            const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
            yq[ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
            yq[ks][1] = u32x4{a.mid, b.mid, c.mid, d.mid};
            yq[ks][2] = u32x4{a.lo, b.lo, c.lo, d.lo};
        }
        i_cur = i_next;
        i_next = tile_id(tile + 2 * NW);
        load_rows(i_cur);                      // rows of the next tile

        // projection c = Q_j^T y
        f32x16 acc[MT];
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[mt] = zero;
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            u32x4 a[MT][3];
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) a[mt][pl] = Qs[((mt * KS16 + ks) * 3 + pl) * 64 + lane];
#pragma unroll
            for (int t = 0; t < 6; ++t)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
                    acc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[mt][TA[t]]),
                                                                      __builtin_bit_cast(bf16x8, yq[ks][TB[t]]),
                                                                      acc[mt], 0, 0, 0);
        }

        // support, coefficients, residual; the (atom, coefficient) rows stay in `stage` for the
        // product below.
        // The tie-breaking scratch is the operand region: the x tile is zeroed again if it was used.
        bool ties = false;
        tile_select<P, S, false>(acc, h, n, active, i, s0, reinterpret_cast<float*>(region), stage, supp, coef,
                                 err, &ties);
        if (ties) {                            // uniform (rare): the scratch overwrote the zeroed x tile
            for (int e = lane; e < 3 * PLANE_B / 16; e += 64)
                reinterpret_cast<u32x4*>(xt)[e] = u32x4{0u, 0u, 0u, 0u};
        }

        // P_j += sum over the tile's signals of x y^T, 16 signals at a time
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            if (cnt_t <= 16 * half) break;     // uniform: no signal in this half
            const bool mine = (n >> 4) == half;
            const int sc = n & 15;             // this lane's signal inside the half
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // y parts -> [dim][signal]: a lane holds (dim pair, own signal) words; the lanes of
            // neighbouring signals swap halves, so that the even one writes (signal pair, even dim)
            // and the odd one (signal pair, odd dim)
            {
                const bool odd = n & 1;
                const unsigned sel = odd ? 0x03020706u : 0x05040100u;
#pragma unroll
                for (int ks = 0; ks < KS16; ++ks)
#pragma unroll
                    for (int pl = 0; pl < 3; ++pl)
#pragma unroll
                        for (int c = 0; c < 4; ++c) {
                            const unsigned own = yq[ks][pl][c];
                            const unsigned oth =
                                (unsigned)__builtin_amdgcn_update_dpp(0, (int)own, kDppXor1, 0xf, 0xf, true);
                            const unsigned w = __builtin_amdgcn_perm(oth, own, sel);
                            const int dim = ks * 16 + h * 8 + 2 * c + (odd ? 1 : 0);
                            if (mine) *reinterpret_cast<unsigned*>(yt + pl * PLANE_B + tr_off(dim, sc & ~1)) = w;
                        }
            }
            // kept coefficients -> [atom][signal]; the two lanes of a signal share its entries
            // (entries that do not exist go to the dummy row instead of a branch)
            int at_[(S + 1) / 2];
#pragma unroll
            for (int t = 0; t < (S + 1) / 2; ++t) {
                const int pos = 2 * t + h;
                const bool have = mine && active && pos < s0;
                const int atom = stage[stage_idx(n, 0, have ? pos : 0)];
                const TriWord w = split_trunc(__builtin_bit_cast(float, stage[stage_idx(n, 1, have ? pos : 0)]));
                at_[t] = tr_off(have ? (atom & (ROWS - 1)) : ROWS, sc);   // row ROWS: nobody reads it
                *reinterpret_cast<unsigned short*>(xt + at_[t]) = (unsigned short)(w.hi >> 16);
                *reinterpret_cast<unsigned short*>(xt + PLANE_B + at_[t]) = (unsigned short)(w.mid >> 16);
                *reinterpret_cast<unsigned short*>(xt + 2 * PLANE_B + at_[t]) = (unsigned short)(w.lo >> 16);
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            // operands: lane (h, n) takes signals 8h .. 8h+7 of atom resp. dim t*32 + n
            u32x4 xa[MT][3], yb[MT][3];
#pragma unroll
            for (int t = 0; t < MT; ++t)
#pragma unroll
                for (int pl = 0; pl < 3; ++pl) {
                    xa[t][pl] = *reinterpret_cast<const u32x4*>(xt + pl * PLANE_B + tr_off(t * 32 + n, 8 * h));
                    yb[t][pl] = *reinterpret_cast<const u32x4*>(yt + pl * PLANE_B + tr_off(t * 32 + n, 8 * h));
                }
#pragma unroll
            for (int t = 0; t < 6; ++t)
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int nt = 0; nt < MT; ++nt)
                        accM[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, xa[mt][TA[t]]), __builtin_bit_cast(bf16x8, yb[nt][TB[t]]),
                            accM[mt][nt], 0, 0, 0);
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();   // the operands have been read: wipe the x entries again
#pragma unroll
            for (int t = 0; t < (S + 1) / 2; ++t) {
                *reinterpret_cast<unsigned short*>(xt + at_[t]) = 0;
                *reinterpret_cast<unsigned short*>(xt + PLANE_B + at_[t]) = 0;
                *reinterpret_cast<unsigned short*>(xt + 2 * PLANE_B + at_[t]) = 0;
            }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();       // stage and the region are rewritten by the next tile
    }
    __syncthreads();                           // all tiles done: their LDS becomes the exchange area

    // The wavefronts' accumulators are added in wavefront order: every wavefront stores its own
    // copy atom-major (register r of tile (mt, nt) in lane (h, n) is atom mt*32 + (r/4)*8 + h*4 +
    // r%4, dimension nt*32 + n), then every thread adds the NW copies of four consecutive entries
    // and writes them to the piece result.
    static_assert((size_t)PP * 4 <= (size_t)WAVE_B, "a copy fits the wave's own area");
    {
        float* mine = reinterpret_cast<float*>(waves_base + (size_t)wave * WAVE_B);
#pragma unroll
        for (int mt = 0; mt < MT; ++mt)
#pragma unroll
            for (int nt = 0; nt < MT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int atom = mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
                    const int dim = nt * 32 + n;
                    if (atom < P && dim < P) mine[atom * P + dim] = accM[mt][nt][r];
                }
    }
    __syncthreads();
    f32x4* out = reinterpret_cast<f32x4*>(partial + (int64_t)id * PP);
    for (int e4 = tid; e4 < PP / 4; e4 += NTH) {
        f32x4 sum = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int w = 0; w < NW; ++w)
            sum += reinterpret_cast<const f32x4*>(waves_base + (size_t)w * WAVE_B)[e4];
        out[e4] = sum;
    }
}

template <int P, int S>
hipError_t launch_ps(const float* Y, int64_t m, const float* D, int K, int s0, const Workspace& ws,
                     int32_t* supp, float* coef, float* err, hipStream_t st) {
    constexpr int MT = P >= 32 ? P / 32 : 1;
    constexpr int ROWS = MT * 32;
    constexpr size_t ct_b = (size_t)32 * (P + 1) * 4, ops_b = (size_t)6 * (ROWS + 1) * 32;
    constexpr size_t wave_b = (size_t)kSelectStageWords * 4 + (ops_b > ct_b ? ops_b : ct_b);
    const int piece = accum_piece(m, K, P);
    const int max_pieces = accum_max_pieces(m, K, P);
    const int head = ((K + 1 + 16) + 3) & ~3;
    const size_t lds = (size_t)head * sizeof(int) + (size_t)MT * (P / 16) * 3 * 64 * sizeof(u32x4) + kSaWaves * wave_b;
    if (lds > 160 * 1024) return hipErrorInvalidValue;
    if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&select_accum_kernel<P, S>), 160 * 1024);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((select_accum_kernel<P, S>), dim3(max_pieces), dim3(64 * kSaWaves), lds, st, Y, D, K, s0,
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
// ws.partial (summed in piece order by launch_polar_from_pieces or launch_accum_reduce).
// p <= 64 only.
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
