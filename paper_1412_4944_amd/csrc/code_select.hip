// Sparse-coding stage 2: support, coefficients and residual of every signal in the
// block that won the energy comparison (Section 2: x = Q_j^T y hard-thresholded to the
// s0 entries of largest magnitude; Algorithm 1, steps 3-4).
//
// Signals arrive grouped by block (perm/offsets).  One wavefront takes a tile of up to
// 32 signals of ONE block, so the projection is again one fp32 MFMA tile product with
// atoms on M and signals on N; every signal's p coefficients then sit in two lanes.
// The s0-th largest magnitude tau is found with the same compare-exchange networks as
// in stage 1, and the support {|c| > tau} plus the lowest-index entries equal to tau is
// written in ascending atom order.  Exact ties in magnitude beyond the trivial one are
// resolved by a sequential per-signal pass (rare).
#include "sbo_internal.h"
#include "device_utils.h"
#include "select_tile.h"

namespace sbo {

namespace {

template <int P, int S>
__global__ __launch_bounds__(256) void select_kernel(const float* __restrict__ Y,
                                                     const float* __restrict__ D, int K, int s0,
                                                     const int32_t* __restrict__ offsets,
                                                     const int32_t* __restrict__ perm,
                                                     int32_t* __restrict__ supp,
                                                     float* __restrict__ coef,
                                                     float* __restrict__ err) {
    constexpr int KS = P / 2;
    constexpr int QN = P / 8;
    constexpr int MT = P >= 32 ? P / 32 : 1;   // 32-row tiles per block
    constexpr int NVL = MT * 16;               // accumulator values per lane
    constexpr int LDC = P + 1;
    static_assert(S <= NVL, "sort width exceeds the values of one lane");

    extern __shared__ int lds[];   // tile_start[K+1] | tmp[16] | pad | stage[4][...] | ctile[4][32][LDC]
    int* tile_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;
    int* stage_all = lds + head;
    float* ctile_all = reinterpret_cast<float*>(stage_all + 4 * kSelectStageWords);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;

    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + 31) >> 5; }, K,
                       tile_start, tmp);
    const int wt = blockIdx.x * 4 + wave;
    if (wt >= tile_start[K]) return;           // no workgroup barrier below this line

    const int j = upper_slot(tile_start, K, wt);
    const int pos0 = offsets[j] + (wt - tile_start[j]) * 32;
    const int cnt = min(32, offsets[j + 1] - pos0);
    const bool active = n < cnt;
    const int64_t i = active ? perm[pos0 + n] : -1;

    // B operand: this lane's half of the dims of signal i.
    float yb[KS];
    if (active) {
        const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + h * KS);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            f32x4 v = src[q];
            yb[4 * q + 0] = v.x;
            yb[4 * q + 1] = v.y;
            yb[4 * q + 2] = v.z;
            yb[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < KS; ++t) yb[t] = 0.f;
    }

    // Projection c = Q_j^T y for the tile.
    f32x16 acc[MT];
#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[mt][r] = 0.f;
        const int row = mt * 32 + n;           // atom fed by this lane into the A operand
        const f32x4* arow =
            reinterpret_cast<const f32x4*>(D + ((int64_t)j * P + (row < P ? row : 0)) * P + h * KS);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            f32x4 a = arow[q];
            if (row >= P) a = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                acc[mt] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[kk], yb[4 * q + kk], acc[mt], 0, 0, 0);
        }
    }

    tile_select<P, S, false>(acc, h, n, active, i, s0, ctile_all + wave * 32 * LDC,
                             stage_all + wave * kSelectStageWords, supp, coef, err);
}

// Variant for p > 64.  The p coefficients of a signal no longer fit the registers of a
// lane pair next to the signal itself, so the projection is produced 32 atoms at a time,
// written to a wave-private LDS tile [signal][atom] while the lane keeps a running sorted
// top-S of the magnitudes; the support is then emitted from the tile, each lane of a pair
// walking one half of the atoms in index order (which resolves magnitude ties directly).
template <int P, int S>
__global__ __launch_bounds__(256) void select_wide_kernel(const float* __restrict__ Y,
                                                          const f32x4* __restrict__ Dsw, int K, int s0,
                                                          const int32_t* __restrict__ offsets,
                                                          const int32_t* __restrict__ perm,
                                                          int32_t* __restrict__ supp,
                                                          float* __restrict__ coef,
                                                          float* __restrict__ err) {
    constexpr int KS = P / 2;
    constexpr int QN = P / 8;
    constexpr int MT = P / 32;
    constexpr int LDC = P + 1;
    constexpr int QCH = 8;                     // operand groups loaded ahead of their MFMAs
    static_assert(S <= 16 && QN % QCH == 0, "shape");

    extern __shared__ int lds[];               // tile_start[K+1] | tmp[16] | ctile[4][32][LDC]
    int* tile_start = lds;
    int* tmp = lds + (K + 1);
    float* ctile_all = reinterpret_cast<float*>(tmp + 16);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int h = lane >> 5, n = lane & 31;

    wg_exclusive_scan4([&](int j) { return (offsets[j + 1] - offsets[j] + 31) >> 5; }, K,
                       tile_start, tmp);
    const int wt = blockIdx.x * 4 + wave;
    if (wt >= tile_start[K]) return;           // no workgroup barrier below this line

    const int j = upper_slot(tile_start, K, wt);
    const int pos0 = offsets[j] + (wt - tile_start[j]) * 32;
    const int cnt = min(32, offsets[j + 1] - pos0);
    const bool active = n < cnt;
    const int64_t i = active ? perm[pos0 + n] : -1;

    float yb[KS];
    if (active) {
        const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + h * KS);
#pragma unroll
        for (int q = 0; q < QN; ++q) {
            f32x4 v = src[q];
            yb[4 * q + 0] = v.x;
            yb[4 * q + 1] = v.y;
            yb[4 * q + 2] = v.z;
            yb[4 * q + 3] = v.w;
        }
    } else {
#pragma unroll
        for (int t = 0; t < KS; ++t) yb[t] = 0.f;
    }

    float* ct = ctile_all + wave * 32 * LDC + n * LDC;     // this lane's signal row
    float run[S];
#pragma unroll
    for (int t = 0; t < S; ++t) run[t] = 0.f;
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // A operand = rows of Q_j straight from L2, QCH 16-byte groups per chunk; the next chunk is
    // requested before the MFMAs of the current one (a wavefront has its SIMD to itself here,
    // so nothing else would cover the load latency).
    // Dsw is Q in the coding kernel's operand order (dict_swizzle_kernel): stage of 64 rows,
    // unit (mt2*QN + q)*64 + lane = dims h*P/2 + 4q.. of row stage*64 + mt2*32 + n, so a
    // wavefront's load is 1 KiB contiguous and the four wavefronts of a workgroup (tiles of the
    // same block, in step) ask for the same lines.
    auto load_chunk = [&](f32x4 (&a)[QCH], int mt, int q0) {
        const f32x4* src = Dsw + ((int64_t)j * (P / 64) + (mt >> 1)) * (2 * QN * 64) +
                           ((mt & 1) * QN + q0) * 64 + lane;
#pragma unroll
        for (int q = 0; q < QCH; ++q) a[q] = src[q * 64];
    };
    constexpr int NCH = QN / QCH;              // chunks per tile row of atoms
    static_assert(NCH == 4, "the operand ring below has four slots, one per chunk of a row");
    // chunk t (t = mt * NCH + cc) lives in slot cc; it is requested two chunks ahead
    f32x4 abuf[NCH][QCH];
    load_chunk(abuf[0], 0, 0);
    load_chunk(abuf[1], 0, QCH);
#pragma unroll 1
    for (int mt = 0; mt < MT; ++mt) {
        f32x16 acc = zero;
#pragma unroll
        for (int cc = 0; cc < NCH; ++cc) {
            // the last two requests of all re-read a valid row and are not used
            const int nmt = cc + 2 < NCH ? mt : min(mt + 1, MT - 1);
            load_chunk(abuf[(cc + 2) % NCH], nmt, ((cc + 2) % NCH) * QCH);
#pragma unroll
            for (int q = 0; q < QCH; ++q)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(abuf[cc][q][kk],
                                                               yb[4 * (cc * QCH + q) + kk], acc, 0, 0, 0);
        }
        float x[16], top[S];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int atom = mt * 32 + (r >> 2) * 8 + h * 4 + (r & 3);
            ct[atom] = acc[r];
            x[r] = fabsf(acc[r]);
        }
        top_sorted<16, S>(x, top);
        if (mt == 0) {
#pragma unroll
            for (int t = 0; t < S; ++t) run[t] = top[t];
        } else {
#pragma unroll
            for (int t = 0; t < S; ++t) run[t] = fmaxf(run[t], top[S - 1 - t]);
            bitonic_merge_desc<S>(run);
        }
    }

    // tau = s0-th largest magnitude of the signal
    float oth[S], mrg[S];
#pragma unroll
    for (int t = 0; t < S; ++t) oth[t] = other_half(run[t]);
#pragma unroll
    for (int t = 0; t < S; ++t) mrg[t] = fmaxf(run[t], oth[S - 1 - t]);
    bitonic_merge_desc<S>(mrg);
    float tau = mrg[0];
#pragma unroll
    for (int t = 1; t < S; ++t) tau = (t == s0 - 1) ? mrg[t] : tau;

    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    // lane h of a pair owns atoms [h*P/2, (h+1)*P/2) of its signal
    const float* mine = ct + h * (P / 2);
    int gt_own = 0, eq_own = 0;
#pragma unroll 16
    for (int k = 0; k < P / 2; ++k) {
        const float a = fabsf(mine[k]);
        gt_own += a > tau;
        eq_own += a == tau;
    }
    const int gt_oth = other_half(gt_own), eq_oth = other_half(eq_own);
    const int need = s0 - (gt_own + gt_oth);   // entries equal to tau to take, lowest index first
    const int gt_lo = h ? gt_oth : gt_own, eq_lo = h ? eq_oth : eq_own;
    const int eq_lo_taken = min(eq_lo, need);
    int pos = h ? gt_lo + eq_lo_taken : 0;
    int eq_taken = h ? eq_lo_taken : 0;
    float dropped = 0.f;
#pragma unroll 16
    for (int k = 0; k < P / 2; ++k) {
        const float v = mine[k];
        const float a = fabsf(v);
        bool take = a > tau;
        if (!take && a == tau && eq_taken < need) {
            take = true;
            ++eq_taken;
        }
        if (take) {
            if (active && pos < s0) {
                supp[i * s0 + pos] = h * (P / 2) + k;
                coef[i * s0 + pos] = v;
            }
            ++pos;
        } else {
            dropped += v * v;
        }
    }
    dropped += other_half(dropped);
    if (active && h == 0) err[i] = dropped;
}

// p = 256 on the bf16 matrix cores (see energy_split_kernel for the arithmetic): the four
// wavefronts of a workgroup take four 32-signal tiles of ONE block and share its rows, staged
// through LDS 32 atoms at a time (48 KiB in the split operand order, double-buffered); each
// wavefront keeps its signals' three bf16 parts (192 registers) and the whole projection
// (8 accumulator tiles, 128 registers) in registers and selects from there.  Dsb is the whole
// dictionary in the split operand order (dict_swizzle_split_kernel).
// Workgroup ids are dealt out so that the workgroups of one XCD (ids equal modulo 8) take a
// contiguous run of tiles, that is, few blocks, whose rows then stay in that XCD's L2.
template <int P, int S>
__global__ __launch_bounds__(256) void select_wide_split_kernel(const float* __restrict__ Y,
                                                                const u32x4* __restrict__ Dsb, int K, int s0,
                                                                const int32_t* __restrict__ offsets,
                                                                const int32_t* __restrict__ perm,
                                                                int32_t* __restrict__ supp,
                                                                float* __restrict__ coef,
                                                                float* __restrict__ err) {
    constexpr int KS16 = P / 16;
    constexpr int MT = P / 32;
    constexpr int STAGE_U = KS16 * 3 * 64;     // 16-byte units of 32 rows
    constexpr int FPT = STAGE_U / 256;
    static_assert(STAGE_U % 256 == 0 && S <= 16, "shape");

    extern __shared__ int lds[];               // unit_start[K+1] | tmp[16] | pad | Qs[2][STAGE_U] | stage[4][..]
    int* unit_start = lds;
    int* tmp = lds + (K + 1);
    const int head = ((K + 1 + 16) + 3) & ~3;
    u32x4(*Qs)[STAGE_U] = reinterpret_cast<u32x4(*)[STAGE_U]>(lds + head);
    int* stage_all = reinterpret_cast<int*>(Qs + 2);

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, n = lane & 31;

    // units of four tiles per block
    wg_exclusive_scan4([&](int j) { return (((offsets[j + 1] - offsets[j] + 31) >> 5) + 3) >> 2; }, K,
                       unit_start, tmp);
    const int per_xcd = gridDim.x >> 3;        // the grid is a multiple of 8 (launcher)
    const int id = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (id >= unit_start[K]) return;           // uniform over the workgroup

    const int j = upper_slot(unit_start, K, id);
    const int pos0 = offsets[j] + ((id - unit_start[j]) * 4 + wave) * 32;
    const int cnt = min(32, offsets[j + 1] - pos0);        // <= 0: this wavefront has no tile (it still
    const bool active = n < cnt;                           // takes part in the staging and the barriers)
    const int64_t i = active ? perm[pos0 + n] : -1;

    u32x4 pre[FPT];
    const u32x4* Qj = Dsb + (int64_t)j * MT * STAGE_U;
    auto fetch = [&](int s) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) pre[r] = Qj[(int64_t)s * STAGE_U + tid + 256 * r];
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int r = 0; r < FPT; ++r) Qs[buf][tid + 256 * r] = pre[r];
    };
    fetch(0);

    // B operand: the three bf16 parts of this lane's dims (ks*16 + h*8 .. +7) of its signal
    u32x4 yq[KS16][3];
#pragma unroll
    for (int ks = 0; ks < KS16; ++ks) {
        f32x4 v0 = {0.f, 0.f, 0.f, 0.f}, v1 = v0;
        if (active) {
            const f32x4* src = reinterpret_cast<const f32x4*>(Y + i * P + ks * 16 + h * 8);
            v0 = src[0];
            v1 = src[1];
        }
        const Bf16x3Pair a = split_bf16x3(v0.x, v0.y), b = split_bf16x3(v0.z, v0.w);
        const Bf16x3Pair c = split_bf16x3(v1.x, v1.y), d = split_bf16x3(v1.z, v1.w);
        yq[ks][0] = u32x4{a.hi, b.hi, c.hi, d.hi};
        yq[ks][1] = u32x4{a.mid, b.mid, c.mid, d.mid};
        yq[ks][2] = u32x4{a.lo, b.lo, c.lo, d.lo};
    }
    stash(0);
    __syncthreads();

    // the six partial products, smallest first: (A part, B part)
    constexpr int TA[6] = {2, 0, 1, 1, 0, 0};
    constexpr int TB[6] = {0, 2, 1, 0, 1, 0};
    const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f,
                         0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16 acc[MT];
#pragma unroll
    for (int s = 0; s < MT; ++s) {
        const int cur = s & 1;
        if (s + 1 < MT) fetch(s + 1);
#pragma unroll
        for (int ks = 0; ks < KS16; ++ks) {
            u32x4 a[3];
#pragma unroll
            for (int pl = 0; pl < 3; ++pl) a[pl] = Qs[cur][(ks * 3 + pl) * 64 + lane];
#pragma unroll
            for (int t = 0; t < 6; ++t)
                acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[TA[t]]),
                                                                 __builtin_bit_cast(bf16x8, yq[ks][TB[t]]),
                                                                 (ks == 0 && t == 0) ? zero : acc[s], 0, 0, 0);
        }
        if (s + 1 < MT) stash(cur ^ 1);
        __syncthreads();
    }

    tile_select<P, S, false>(acc, h, n, active, i, s0, nullptr, stage_all + wave * kSelectStageWords, supp, coef,
                             err);
}

template <int P, int S>
hipError_t launch_wide_ps(const float* Y, int64_t m, const float* D, int K, int s0,
                          const Workspace& ws, int32_t* supp, float* coef, float* err, bool split,
                          hipStream_t st) {
    (void)D;                                   // the kernels read ws.dsb / ws.dsw, the same Q in operand order
    if (split) {
        // a multiple of 8, so that the kernel's dealing of ids over the XCDs covers every unit
        const int64_t max_units = (((m + 127) / 128 + K) + 7) & ~(int64_t)7;
        const int head = ((K + 1 + 16) + 3) & ~3;
        const size_t lds = (size_t)head * sizeof(int) + (size_t)2 * (P / 16) * 3 * 64 * 16 +
                           (size_t)4 * kSelectStageWords * sizeof(int);
        if (hipError_t e =
                ws.raised->ensure(reinterpret_cast<const void*>(&select_wide_split_kernel<P, S>), lds);
            e != hipSuccess)
            return e;
        hipLaunchKernelGGL((select_wide_split_kernel<P, S>), dim3((unsigned)max_units), dim3(256), lds, st, Y,
                           reinterpret_cast<const u32x4*>(ws.dsb), K, s0, ws.offsets, ws.perm, supp, coef, err);
        return hipGetLastError();
    }
    const int64_t max_tiles = (m + 31) / 32 + K;
    dim3 grid((unsigned)((max_tiles + 3) / 4));
    const size_t lds = (K + 1 + 16) * sizeof(int) + 4 * 32 * (P + 1) * sizeof(float);
    if (hipError_t e = ws.raised->ensure(reinterpret_cast<const void*>(&select_wide_kernel<P, S>), lds);
        e != hipSuccess)
        return e;
    hipLaunchKernelGGL((select_wide_kernel<P, S>), grid, dim3(256), lds, st, Y,
                       reinterpret_cast<const f32x4*>(ws.dsw), K, s0, ws.offsets, ws.perm, supp, coef, err);
    return hipGetLastError();
}

template <int P>
hipError_t launch_wide_p(int s0, const float* Y, int64_t m, const float* D, int K,
                         const Workspace& ws, int32_t* supp, float* coef, float* err, bool split,
                         hipStream_t st) {
    if (s0 <= 1) return launch_wide_ps<P, 1>(Y, m, D, K, s0, ws, supp, coef, err, split, st);
    if (s0 <= 2) return launch_wide_ps<P, 2>(Y, m, D, K, s0, ws, supp, coef, err, split, st);
    if (s0 <= 4) return launch_wide_ps<P, 4>(Y, m, D, K, s0, ws, supp, coef, err, split, st);
    if (s0 <= 8) return launch_wide_ps<P, 8>(Y, m, D, K, s0, ws, supp, coef, err, split, st);
    return launch_wide_ps<P, 16>(Y, m, D, K, s0, ws, supp, coef, err, split, st);
}

template <int P, int S>
hipError_t launch_ps(const float* Y, int64_t m, const float* D, int K, int s0, const Workspace& ws,
                     int32_t* supp, float* coef, float* err, hipStream_t st) {
    const int64_t max_tiles = (m + 31) / 32 + K;
    dim3 grid((unsigned)((max_tiles + 3) / 4));
    const size_t lds = ((((K + 1 + 16) + 3) & ~3) + 4 * kSelectStageWords) * sizeof(int) +
                       4 * 32 * (P + 1) * sizeof(float);
    hipLaunchKernelGGL((select_kernel<P, S>), grid, dim3(256), lds, st, Y, D, K, s0, ws.offsets,
                       ws.perm, supp, coef, err);
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

hipError_t launch_select(int p, int K, int s0, const float* Y, int64_t m, const float* D,
                         const Workspace& ws, int32_t* supp, float* coef, float* err, bool ops_valid,
                         bool split, hipStream_t st) {
    if (p == 256 && !ops_valid) {              // the p = 256 kernels read Q in operand order
        hipError_t e = split ? launch_dict_swizzle_split(p, K, D, ws.dsb, 2, st)
                             : launch_dict_swizzle(p, K, D, ws.dsw, st);
        if (e != hipSuccess) return e;
    }
    switch (p) {
        case 16: return launch_p<16>(s0, Y, m, D, K, ws, supp, coef, err, st);
        case 32: return launch_p<32>(s0, Y, m, D, K, ws, supp, coef, err, st);
        case 64: return launch_p<64>(s0, Y, m, D, K, ws, supp, coef, err, st);
        case 256: return launch_wide_p<256>(s0, Y, m, D, K, ws, supp, coef, err, split, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sbo
