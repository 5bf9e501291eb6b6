// Internal declarations shared by the libsbo translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <stdlib.h>
#include <vector>

#include "../../include/sbo.h"

namespace sbo {

constexpr int kWave = 64;

// ---- grouping geometry -----------------------------------------------------
// One wavefront owns one chunk of consecutive signals; a chunk is a multiple of
// 64 signals, sized so that there are at most ~1024 chunks.
struct GroupGeom {
    int chunk;     // signals per chunk (multiple of 512)
    int n_chunks;  // ceil(m / chunk)
};
inline GroupGeom group_geom(int64_t m) {
    int64_t c = (m + 1023) / 1024;
    c = ((c + 511) / 512) * 512;           // whole workgroups of the coding kernels (128, 256 or 512 signals)
    if (c < 512) c = 512;
    GroupGeom g;
    g.chunk = (int)c;
    g.n_chunks = (int)((m + c - 1) / c);
    return g;
}

// ---- accumulation geometry ---------------------------------------------------
// Each block's sorted signal list is cut into pieces of `piece` signals; one
// workgroup reduces one piece into a partial p x p matrix.
constexpr int kNumCU = 256;
inline int accum_piece(int64_t m, int K, int p) {
    // One workgroup per CU for every p (8 wavefronts with 150 KiB of LDS for p <= 64, 512
    // registers per lane for p = 256), and all pieces resident in one round: pieces <= CUs where
    // K allows.
    const int target = K < kNumCU / 2 ? kNumCU - K : kNumCU / 2;
    int64_t c = (m + target - 1) / target;
    c = ((c + 63) / 64) * 64;
    if (c < (p <= 64 ? 64 : 256)) c = p <= 64 ? 64 : 256;
    if (c > 4096) c = 4096;
    return (int)c;
}
// Piece size of the stand-alone accumulation for p <= 64, whose workgroups fill a whole CU:
// as few pieces as keep every CU busy in a single round (pieces <= CUs where K allows), capped
// because the kernel keeps a piece's signal ids in LDS.
constexpr int kTallMaxPiece = 4096;
inline int accum_tall_piece(int64_t m, int K) {
    const int target = K < kNumCU / 2 ? kNumCU - K : kNumCU / 2;
    int64_t c = (m + target - 1) / target;
    c = ((c + 63) / 64) * 64;
    if (c > kTallMaxPiece) c = kTallMaxPiece;
    return (int)(c < 64 ? 64 : c);
}
inline int accum_max_pieces(int64_t m, int K, int p) {
    int piece = accum_piece(m, K, p);
    return (int)((m + piece - 1) / piece) + K;
}

// ---- Jacobi stopping threshold ---------------------------------------------------
// A sweep in which every pair already had a cosine below this is the last one.
constexpr float kPolarDone = 1e-4f;

// ---- kernels that need more dynamic LDS than the default limit ---------------------
// Their limit is raised once per context (a context belongs to one device and its calls do
// not overlap), before the first launch; the context remembers which kernels have been done.
struct LdsRaised {
    std::vector<const void*> fns;
    hipError_t ensure(const void* fn, size_t bytes) {
        for (const void* f : fns)
            if (f == fn) return hipSuccess;
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        if (e == hipSuccess) fns.push_back(fn);
        return e;
    }
};

// ---- device workspace layout ---------------------------------------------------
struct Workspace {
    // grouping
    int32_t* chunk_count;  // [n_chunks_max][K]
    int32_t* chunk_base;   // [n_chunks_max][K]
    int32_t* counts;       // [K]
    int32_t* offsets;      // [K+1]
    int32_t* perm;         // [m_max]
    // coding
    float* energy;         // [m_max] kept energy in the winning block
    float* dsw;            // [ceil(K*p/64)*64][p] dictionary in MFMA operand order
    unsigned* dsh;         // p > 64 only: the same rows as two fp16 parts (the energy kernel's order there)
    unsigned* dsb;         // the same rows in parts: three bf16 (6 bytes per entry) or, for the energy kernel at
                           // p <= 64, two fp16 (4 bytes per entry), in the split operand orders
    float* part_E;         // [kEnergySplitRows][m_max] split coding / resolution pass: best energy per row
    int32_t* part_j;       // same shape: its block
    // accumulation
    float* partial;        // [max_pieces][p][p]
    float* M;              // [K][p][p]
    float* vwork;          // p > 64 only: [K][p][p] the V of the wide Jacobi SVD
    float* jac_a;          // p > 64 only: scratch of the wide Jacobi (polar_wide_scratch_bytes)
    // worst-W selection
    int32_t* sel_hist;     // [4][256] digit histograms of the radix select
    int32_t* sel_state;    // [4][2] (key prefix, entries still to take) after each pass
    int32_t* sel_cnt;      // [ceil(m_max / kSelChunk)][2] entries above / equal to the threshold
    int32_t* sel_base;     // same shape: exclusive sums of sel_cnt over the chunks
    int32_t* sel_ids;      // [m_max] worst-W set inside sbo_learn
    double* sq_out;        // [1] squared-error total inside sbo_learn
    int32_t* sweeps;       // [K] most recent SVD stage: Jacobi sweeps, or minus the Newton-Schulz steps
    int32_t* ns_fallback;  // [K] 1 = Newton-Schulz left the block to the Jacobi kernel
    int32_t* sq_counter;   // [1] workgroups of the fused squared-error sum that have finished (0 between launches)
    bool parts_accum = false;   // p = 256: the accumulation on the bf16 matrix cores (any coding arithmetic but fp32)
    int32_t* flag_ids;     // [m_max] signals whose block the screening pass of the coding kernel left undecided
    int32_t* flag_count;   // [1] how many (0 between calls: the grouping's scan kernel clears it)
    // iterate
    double* sq_partial;    // [kSqBlocks]
    size_t bytes;
    // host side: launch state of the owning context (not device memory)
    LdsRaised* raised;
};
constexpr int kSqBlocks = 256;
constexpr int kEnergySplitBelow = 192;       // coding launches with fewer workgroups split the blocks
constexpr int kEnergySplitRows = 16;         // at most this many workgroup rows
constexpr int kEnergySplitSignals = 49152;   // and only up to this many signals (scratch size)
constexpr int kSelChunk = 2048;              // signals per workgroup in the worst-W compaction

size_t workspace_layout(int p, int K, int s0, int64_t m_max, Workspace* ws, char* base);

}  // namespace sbo

struct sbo_span {
    int stage;
    hipEvent_t beg, end;
};

struct sbo_ctx {
    int p, K, s0;                    // K = blocks in use (<= K_cap, see sbo_set_blocks)
    int K_cap;                       // blocks the workspace was sized for
    int64_t m_max;
    hipStream_t stream;
    char* ws_base;
    sbo::Workspace ws;
    int svd_method;                  // SBO_SVD_AUTO or SBO_SVD_JACOBI (sbo_set_option)
    int coding_arith;                // SBO_ARITH_* (sbo_set_option)
    sbo::LdsRaised raised;
    int timing;
    std::vector<sbo_span> spans;     // event pool; the first n_spans are in use
    size_t n_spans;
};

// ---- kernel launchers (each returns a hipError_t from the launch) ----------------
namespace sbo {

// dsw = D rewritten by launch_dict_swizzle into the energy kernel's operand order.
hipError_t launch_dict_swizzle(int p, int K, const float* D, float* dsw, hipStream_t st);
// dsb = D in the operand order of the split coding kernels; kind 2: three bf16 parts per entry,
// kind 3 (p <= 64): two fp16 parts per entry (device_utils.h).
hipError_t launch_dict_swizzle_split(int p, int K, const float* D, unsigned* dsb, int kind, hipStream_t st);
// chunk_count != nullptr: also add the per-chunk histograms of the chosen blocks into it (the
// first step of launch_group; the array must be zero on entry, launch_group leaves it so).
// part_E / part_j ([kEnergySplitRows][m_max], may be nullptr): scratch for small m (at most
// kEnergySplitSignals), where the blocks are split over several workgroup rows to fill the chip,
// and for the resolution pass of the screening (scr), which is always split that way.
// dsb != nullptr: the projection runs on the bf16 (dsb_kind 2) or fp16 (dsb_kind 3, p <= 64) matrix
// cores from the split dictionary (dsw is then not read); otherwise on the fp32 matrix instruction
// from dsw.
// scr != nullptr (with dsb, p <= 64, enough signals to fill the chip): a screening pass with half
// the matrix work decides the block of every signal whose two best energies are further apart
// than the screening error allows, and the full products are formed only for the rest, listed in
// scr->ids ([m]) / scr->count ([1], zero on entry; launch_group sets it back to zero).  The
// energies written for decided signals are then the screened ones.
struct EnergyScreen {
    int32_t* ids;
    int32_t* count;
};
hipError_t launch_energy(int p, int K, int s0, const float* Y, int64_t m, const float* dsw,
                         const unsigned* dsb, int dsb_kind, int32_t* blk, float* energy, int32_t* chunk_count,
                         float* part_E, int32_t* part_j, LdsRaised* raised, const EnergyScreen* scr,
                         hipStream_t st);

hipError_t launch_group(int K, const int32_t* blk, int64_t m, const Workspace& ws, bool have_hist,
                        hipStream_t st);
// The grouping with its scratch in a static device array (no workspace, no allocation).
constexpr int kGroupStaticMaxK = 128;
constexpr int64_t kGroupStaticMaxM = (int64_t)1 << 20;
hipError_t launch_group_static(int K, const int32_t* blk, int64_t m, int32_t* counts, int32_t* offsets,
                               int32_t* perm, hipStream_t st);

// p = 256 reads Q in operand order: ws.dsb (split: the bf16 matrix cores) or ws.dsw (fp32 matrix
// instruction).  ops_valid: that buffer already holds this D (launch_dict_swizzle[_split]);
// otherwise it is rewritten first.  p <= 64 reads D itself and ignores both flags.
hipError_t launch_select(int p, int K, int s0, const float* Y, int64_t m, const float* D,
                         const Workspace& ws, int32_t* supp, float* coef, float* err, bool ops_valid,
                         bool split, hipStream_t st);

hipError_t launch_accumulate(int p, int K, int s0, const float* Y, int64_t m, const int32_t* supp,
                             const float* coef, const Workspace& ws, float* M, hipStream_t st);

// Fused select + per-piece accumulation (p <= 64); the piece results land in ws.partial
// and launch_accum_reduce sums them into M.
hipError_t launch_select_accum(int p, int K, int s0, const float* Y, int64_t m, const float* D,
                               const Workspace& ws, int32_t* supp, float* coef, float* err,
                               hipStream_t st);
// err, sq_out != nullptr: the same launch also forms *sq_out = sum of err[0..m).
hipError_t launch_accum_reduce(int p, int K, int64_t m, const Workspace& ws, float* M,
                               const float* err, double* sq_out, hipStream_t st);

// The SVD update Q_j = U V^T of every block with counts[j] > 0 (counts == nullptr: all).
// p <= 64: Newton-Schulz on the matrix cores (polar_ns.hip) first, then the Jacobi SVD for the
// blocks it leaves flagged (rank-deficient ones); p = 256: the same two steps spread over the whole
// chip (polar_wide_ns.hip, polar_wide.hip).
// jacobi_only != 0: the Jacobi SVD for every block (SBO_SVD_JACOBI).
// Uses ws.vwork and ws.jac_a (p = 256), ws.sweeps (per block: Jacobi sweeps, or minus the
// Newton-Schulz steps), ws.ns_fallback.
// eig_sv != nullptr switches to eigen mode (always Jacobi): M[j] symmetric positive
// semidefinite, D[j] receives its eigenvectors as atoms by descending eigenvalue and
// eig_sv[j][p] the square roots of the eigenvalues.
// write_ops (p <= 64): the rows of every updated block are also written in the coding kernel's
// operand order: 1 = into ws.dsw (what launch_dict_swizzle would produce from the new D), 2 / 3 =
// into ws.dsb (launch_dict_swizzle_split with kind 2: three bf16 parts / 3: two fp16 parts), 0 = neither.
hipError_t launch_polar(int p, int K, const float* M, const int32_t* counts, float* D,
                        const Workspace& ws, int jacobi_only, float* eig_sv, int write_ops,
                        hipStream_t st);

// Total squared error riding along in a launch (sq_total.h): out == nullptr = none.
struct SqTotalArgs {
    const float* err = nullptr;
    int64_t m = 0;
    double* part = nullptr;     // ws.sq_partial
    int* counter = nullptr;     // ws.sq_counter (zero between launches)
    double* out = nullptr;
    int nb = 0;                 // workgroups (<= kSqBlocks)
};
// Newton-Schulz for p <= 64 with the Jacobi SVD in the same workgroup for a block that does not
// converge.  M == nullptr: P_j = the sum of block j's pieces in `partial` (fused select +
// accumulate, cut from `offsets` with `piece` signals per piece).
hipError_t launch_polar_ns(int p, int K, const float* M, const float* partial, const int32_t* offsets,
                           int piece, const int32_t* counts, float* D, float* dsw, unsigned* dsb, int dsb_kind,
                           int32_t* fallback, int32_t* iters, const SqTotalArgs& sq, LdsRaised* raised,
                           hipStream_t st);
// The SVD update straight from the piece results of launch_select_accum (p <= 64, Newton-Schulz
// path): what launch_accum_reduce + launch_polar do, in one launch.  err / sq_out as for
// launch_accum_reduce.
hipError_t launch_polar_from_pieces(int p, int K, int64_t m, float* D, const Workspace& ws, int write_ops,
                                    const float* err, double* sq_out, hipStream_t st);

// p = 256 variant of launch_polar (polar_wide.hip) and the size of its scratch (working
// copy of P_j, rotation log, sweep counts).
size_t polar_wide_scratch_bytes(int K);
// only != nullptr: blocks with only[j] == 0 are skipped.
hipError_t launch_polar_wide(int K, const float* M, const int32_t* counts, float* D, float* vwork,
                             float* jac_a, float* eig_sv, int32_t* sweeps, const int32_t* only,
                             LdsRaised* raised, hipStream_t st);
// p = 256 Newton-Schulz over the whole chip (polar_wide_ns.hip); scratch as for the Jacobi variant.
size_t polar_wide_ns_scratch_bytes(int K);
hipError_t launch_polar_wide_ns(int K, const float* M, const int32_t* counts, float* D, float* scratch,
                                int32_t* fallback, int32_t* iters, LdsRaised* raised, hipStream_t st);

// ids == nullptr: sum over all m signals; otherwise over the m listed ones.
hipError_t launch_sqerr(const float* err, const int32_t* ids, int64_t m, const Workspace& ws,
                        double* out, hipStream_t st);

// A signal set as one block: ws.perm = ids clamped to [0, m), ws.counts = {n}, ws.offsets = {0, n}.
hipError_t launch_single_block(const int32_t* ids, int64_t n, int64_t m, const Workspace& ws,
                               hipStream_t st);

// n_blocks signal sets of per_block signals each (ids[n_blocks][per_block]) as K = n_blocks blocks:
// ws.perm = the ids clamped to [0, m), ws.counts[j] = per_block, ws.offsets[j] = j * per_block.
hipError_t launch_equal_blocks(const int32_t* ids, int n_blocks, int64_t per_block, int64_t m,
                               const Workspace& ws, hipStream_t st);

// G[j] = sum over the signals of block j (ws.perm / ws.offsets for K blocks, n signals in all)
// of y y^T.
hipError_t launch_gram(int p, int K, const float* Y, int64_t n, const Workspace& ws, float* G,
                       hipStream_t st);

// ids[0..W) = the W signals with the largest err (ties: lower index), ascending.
hipError_t launch_worst(const float* err, int64_t m, int64_t W, const Workspace& ws, int32_t* ids,
                        hipStream_t st);

}  // namespace sbo
