// C-ABI of libsbo: argument checks, workspace, stage sequencing and timing.
// All arithmetic is in the kernels; this file only enqueues them.
#include "sbo_internal.h"

#include <cmath>
#include <new>
#include <string>

namespace sbo {

static size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

static int max_chunks() { return 1025; }

static int max_pieces_bound(int64_t m_max, int K, int p) {
    const int min_piece = p <= 64 ? 64 : 256;  // smallest piece size accum_piece() can return
    return (int)((m_max + min_piece - 1) / min_piece) + K + 1;
}

size_t workspace_layout(int p, int K, int s0, int64_t m_max, Workspace* ws, char* base) {
    (void)s0;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char* ptr = base ? base + off : nullptr;
        off += align_up(bytes);
        return ptr;
    };
    Workspace w;
    w.chunk_count = (int32_t*)take((size_t)max_chunks() * K * 4);
    w.chunk_base = (int32_t*)take((size_t)max_chunks() * K * 4);
    w.counts = (int32_t*)take((size_t)K * 4);
    w.offsets = (int32_t*)take((size_t)(K + 1) * 4);
    w.perm = (int32_t*)take((size_t)m_max * 4);
    w.energy = (float*)take((size_t)m_max * 4);
    w.dsw = (float*)take((size_t)((K * p + 63) / 64) * 64 * p * 4);
    w.dsb = (unsigned*)take((size_t)((K * p + 63) / 64) * 64 * p * 6);
    w.dsh = (unsigned*)take(p > 64 ? (size_t)((K * p + 63) / 64) * 64 * p * 4 : 0);
    const size_t split_m = (size_t)m_max;      // small m: one entry per signal; resolution pass: per list entry
    w.part_E = (float*)take((size_t)kEnergySplitRows * split_m * 4);
    w.part_j = (int32_t*)take((size_t)kEnergySplitRows * split_m * 4);
    w.partial = (float*)take((size_t)max_pieces_bound(m_max, K, p) * p * p * 4);
    w.M = (float*)take((size_t)K * p * p * 4);
    w.vwork = (float*)take(p > 64 ? (size_t)K * p * p * 4 : 0);
    const size_t wide_a = polar_wide_scratch_bytes(K), wide_b = polar_wide_ns_scratch_bytes(K);
    w.jac_a = (float*)take(p > 64 ? (wide_a > wide_b ? wide_a : wide_b) : 0);
    const size_t sel_chunks = (size_t)((m_max + kSelChunk - 1) / kSelChunk);
    w.sel_hist = (int32_t*)take((size_t)4 * 256 * 4);
    w.sel_state = (int32_t*)take((size_t)4 * 2 * 4);
    w.sel_cnt = (int32_t*)take(sel_chunks * 2 * 4);
    w.sel_base = (int32_t*)take(sel_chunks * 2 * 4);
    w.sel_ids = (int32_t*)take((size_t)m_max * 4);
    w.sq_out = (double*)take(8);
    w.sq_counter = (int32_t*)take(4);
    w.flag_ids = (int32_t*)take((size_t)m_max * 4);
    w.flag_count = (int32_t*)take(4);
    w.sweeps = (int32_t*)take((size_t)K * 4);
    w.ns_fallback = (int32_t*)take((size_t)K * 4);
    w.sq_partial = (double*)take((size_t)kSqBlocks * 8);
    w.bytes = off;
    w.raised = nullptr;
    if (ws) *ws = w;
    return off;
}

static bool shape_ok(int p, int K, int s0, int64_t m_max) {
    if (!(p == 16 || p == 32 || p == 64 || p == 256)) return false;
    if (K < 1 || K > 1024) return false;
    if (s0 < 1 || s0 > 16 || s0 > p) return false;
    if (m_max < 1) return false;
    const int64_t lim = ((int64_t)1 << 31) / (p > s0 ? p : s0);
    if (m_max >= lim) return false;
    return true;
}

static thread_local std::string g_hip_text = "no HIP error recorded";

static int hip_fail(hipError_t e) {
    g_hip_text = std::string("HIP error: ") + hipGetErrorString(e);
    return SBO_EHIP;
}

#define SBO_HIP(expr)                                   \
    do {                                                \
        hipError_t e_ = (expr);                         \
        if (e_ != hipSuccess) return sbo::hip_fail(e_); \
    } while (0)

// Records a begin event now and an end event at scope exit when timing is on.
struct StageTimer {
    sbo_ctx* c;
    long idx;                                  // index into c->spans, -1 = not timing
    StageTimer(sbo_ctx* ctx, int stage) : c(ctx), idx(-1) {
        if (!c->timing || (c->timing == 2 && stage != SBO_STAGE_ENERGY)) return;
        if (c->n_spans == c->spans.size()) {
            sbo_span s;
            s.stage = stage;
            if (hipEventCreate(&s.beg) != hipSuccess) return;
            if (hipEventCreate(&s.end) != hipSuccess) {
                (void)hipEventDestroy(s.beg);
                return;
            }
            c->spans.push_back(s);
        }
        idx = (long)c->n_spans++;
        c->spans[idx].stage = stage;
        (void)hipEventRecord(c->spans[idx].beg, c->stream);
    }
    ~StageTimer() {
        if (idx >= 0) (void)hipEventRecord(c->spans[idx].end, c->stream);
    }
};

static int check_call(const sbo_ctx* c, int64_t m) {
    if (!c) return SBO_EINVAL;
    if (m < 1 || m > c->m_max) return SBO_EINVAL;
    return SBO_OK;
}

static int run_group(sbo_ctx* c, const int32_t* blk, int64_t m, bool have_hist = false) {
    StageTimer t(c, SBO_STAGE_GROUP);
    SBO_HIP(launch_group(c->K, blk, m, c->ws, have_hist, c->stream));
    return SBO_OK;
}

// The coding kernel reads the split dictionary (bf16 matrix cores) or the fp32 one.
static bool use_split(const sbo_ctx* c) { return c->coding_arith != SBO_ARITH_F32; }
// Which operand order the coding kernel of this context reads (the write_ops / kind values of
// launch_polar and launch_dict_swizzle_split): 1 fp32, 2 three bf16 parts, 3 two fp16 parts.
static int ops_kind(const sbo_ctx* c) {
    if (c->coding_arith == SBO_ARITH_F32) return 1;
    return c->coding_arith == SBO_ARITH_F16X2 ? 3 : 2;
}
// The buffer the energy kernel reads: at p = 256 the fp16 order has a buffer of its own, because
// the select kernel there reads the three-bf16 order from ws.dsb.
static unsigned* energy_parts(const sbo_ctx* c) {
    return c->p > 64 && ops_kind(c) == 3 ? c->ws.dsh : c->ws.dsb;
}

// D in the operand order(s) the coding kernels of this context read (tiny; outside the stages).
static int run_swizzle(sbo_ctx* c, const float* D) {
    if (use_split(c)) {
        SBO_HIP(launch_dict_swizzle_split(c->p, c->K, D, energy_parts(c), ops_kind(c), c->stream));
        if (energy_parts(c) != c->ws.dsb)       // p = 256: the select kernel's order as well
            SBO_HIP(launch_dict_swizzle_split(c->p, c->K, D, c->ws.dsb, 2, c->stream));
    }
    else SBO_HIP(launch_dict_swizzle(c->p, c->K, D, c->ws.dsw, c->stream));
    return SBO_OK;
}

static int run_energy(sbo_ctx* c, const float* Y, int64_t m, int32_t* blk) {
    StageTimer t(c, SBO_STAGE_ENERGY);     // also leaves the chunk histograms of the grouping
    const EnergyScreen scr{c->ws.flag_ids, c->ws.flag_count};
    SBO_HIP(launch_energy(c->p, c->K, c->s0, Y, m, c->ws.dsw, use_split(c) ? energy_parts(c) : nullptr, ops_kind(c), blk,
                          c->ws.energy, c->ws.chunk_count, c->ws.part_E, c->ws.part_j, &c->raised,
                          c->coding_arith == SBO_ARITH_BF16X3_SCREEN ? &scr : nullptr, c->stream));
    return SBO_OK;
}

static int run_code(sbo_ctx* c, const float* Y, int64_t m, const float* D, int32_t* blk,
                    int32_t* supp, float* coef, float* err) {
    int rc = run_swizzle(c, D);
    if (rc) return rc;
    rc = run_energy(c, Y, m, blk);
    if (rc) return rc;
    rc = run_group(c, blk, m, true);           // the energy kernel left the chunk histograms
    if (rc) return rc;
    {
        StageTimer t(c, SBO_STAGE_SELECT);         // p = 256 reads the operand order run_swizzle wrote
        SBO_HIP(launch_select(c->p, c->K, c->s0, Y, m, D, c->ws, supp, coef, err, true, use_split(c), c->stream));
    }
    return SBO_OK;
}

// Accumulate + SVD for signals already grouped in the workspace.
static int run_update_grouped(sbo_ctx* c, const float* Y, int64_t m, const int32_t* supp,
                              const float* coef, float* D) {
    {
        StageTimer t(c, SBO_STAGE_ACCUM);
        SBO_HIP(launch_accumulate(c->p, c->K, c->s0, Y, m, supp, coef, c->ws, c->ws.M, c->stream));
    }
    {
        StageTimer t(c, SBO_STAGE_SVD);
        SBO_HIP(launch_polar(c->p, c->K, c->ws.M, c->ws.counts, D, c->ws, c->svd_method, nullptr, 0,
                             c->stream));
    }
    return SBO_OK;
}

// The SVD update from the piece results of launch_select_accum (p <= 64); err / sq_out: also
// the squared-error total of the coding pass.  One launch on the default path; with the Jacobi
// SVD for every block the pieces are summed by their own launch first.
static int run_polar_pieces(sbo_ctx* c, int64_t m, float* D, int write_ops, const float* err, double* sq_out,
                            int K = -1) {
    if (K < 0) K = c->K;
    if (c->svd_method == SBO_SVD_JACOBI) {
        {
            StageTimer t(c, SBO_STAGE_ACCUM);
            SBO_HIP(launch_accum_reduce(c->p, K, m, c->ws, c->ws.M, err, sq_out, c->stream));
        }
        StageTimer t(c, SBO_STAGE_SVD);
        SBO_HIP(launch_polar(c->p, K, c->ws.M, c->ws.counts, D, c->ws, 1, nullptr, write_ops, c->stream));
        return SBO_OK;
    }
    StageTimer t(c, SBO_STAGE_SVD);
    SBO_HIP(launch_polar_from_pieces(c->p, K, m, D, c->ws, write_ops, err, sq_out, c->stream));
    return SBO_OK;
}

}  // namespace sbo

using namespace sbo;

extern "C" {

size_t sbo_workspace_bytes(int p, int K, int s0, int64_t m_max) {
    if (!shape_ok(p, K, s0, m_max)) return 0;
    return workspace_layout(p, K, s0, m_max, nullptr, nullptr);
}

int sbo_create(sbo_ctx** out, int p, int K, int s0, int64_t m_max, void* hip_stream) {
    if (!out || !shape_ok(p, K, s0, m_max)) return SBO_EINVAL;
    sbo_ctx* c = new (std::nothrow) sbo_ctx();
    if (!c) return SBO_ENOMEM;
    c->p = p;
    c->K = K;
    c->K_cap = K;
    c->s0 = s0;
    c->m_max = m_max;
    c->stream = (hipStream_t)hip_stream;
    c->svd_method = SBO_SVD_AUTO;
    c->coding_arith = SBO_ARITH_F16X2;
    c->timing = 0;
    c->n_spans = 0;
    const size_t bytes = workspace_layout(p, K, s0, m_max, nullptr, nullptr);
    void* base = nullptr;
    hipError_t e = hipMalloc(&base, bytes);
    if (e != hipSuccess) {
        delete c;
        if (e == hipErrorOutOfMemory) return SBO_ENOMEM;
        return hip_fail(e);
    }
    c->ws_base = (char*)base;
    workspace_layout(p, K, s0, m_max, &c->ws, c->ws_base);
    c->ws.raised = &c->raised;
    c->ws.parts_accum = c->coding_arith != SBO_ARITH_F32;
    // Two pieces of the workspace carry an invariant between calls: the chunk histograms and the
    // finished-workgroup counter are zero whenever no call is in flight.
    e = hipMemsetAsync(c->ws.chunk_count, 0, (size_t)max_chunks() * K * 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws.sq_counter, 0, 4, c->stream);
    if (e == hipSuccess) e = hipMemsetAsync(c->ws.flag_count, 0, 4, c->stream);
    if (e != hipSuccess) {
        (void)hipFree(c->ws_base);
        delete c;
        return hip_fail(e);
    }
    *out = c;
    return SBO_OK;
}

int sbo_destroy(sbo_ctx* c) {
    if (!c) return SBO_EINVAL;
    hipError_t e = hipStreamSynchronize(c->stream);
    for (auto& s : c->spans) {
        (void)hipEventDestroy(s.beg);
        (void)hipEventDestroy(s.end);
    }
    hipError_t e2 = hipFree(c->ws_base);
    delete c;
    if (e != hipSuccess) return hip_fail(e);
    if (e2 != hipSuccess) return hip_fail(e2);
    return SBO_OK;
}

int sbo_code(sbo_ctx* c, const float* Y, int64_t m, const float* D, int32_t* blk, int32_t* supp,
             float* coef, float* err) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !D || !blk || !supp || !coef || !err) return SBO_EINVAL;
    c->n_spans = 0;
    return run_code(c, Y, m, D, blk, supp, coef, err);
}

int sbo_group(sbo_ctx* c, const int32_t* blk, int64_t m, int32_t* counts, int32_t* offsets,
              int32_t* perm) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!blk) return SBO_EINVAL;
    c->n_spans = 0;
    rc = run_group(c, blk, m);
    if (rc) return rc;
    if (counts)
        SBO_HIP(hipMemcpyAsync(counts, c->ws.counts, (size_t)c->K * 4, hipMemcpyDeviceToDevice,
                               c->stream));
    if (offsets)
        SBO_HIP(hipMemcpyAsync(offsets, c->ws.offsets, (size_t)(c->K + 1) * 4,
                               hipMemcpyDeviceToDevice, c->stream));
    if (perm)
        SBO_HIP(hipMemcpyAsync(perm, c->ws.perm, (size_t)m * 4, hipMemcpyDeviceToDevice, c->stream));
    return SBO_OK;
}

int sbo_group_static(const int32_t* blk, int64_t m, int K, int32_t* counts, int32_t* offsets,
                     int32_t* perm, void* hip_stream) {
    if (!blk || !counts || !offsets || !perm) return SBO_EINVAL;
    if (K < 1 || K > SBO_GROUP_STATIC_MAX_K || m < 1 || m > SBO_GROUP_STATIC_MAX_M) {
        g_hip_text = "sbo_group_static: K or m beyond the static scratch (K <= 128, m <= 1048576)";
        return SBO_ELIMIT;
    }
    static_assert(SBO_GROUP_STATIC_MAX_K == kGroupStaticMaxK && SBO_GROUP_STATIC_MAX_M == kGroupStaticMaxM,
                  "header and kernel limits differ");
    SBO_HIP(launch_group_static(K, blk, m, counts, offsets, perm, (hipStream_t)hip_stream));
    return SBO_OK;
}

int sbo_accumulate(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk, const int32_t* supp,
                   const float* coef, float* M) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !blk || !supp || !coef || !M) return SBO_EINVAL;
    c->n_spans = 0;
    rc = run_group(c, blk, m);
    if (rc) return rc;
    StageTimer t(c, SBO_STAGE_ACCUM);
    SBO_HIP(launch_accumulate(c->p, c->K, c->s0, Y, m, supp, coef, c->ws, M, c->stream));
    return SBO_OK;
}

int sbo_polar(sbo_ctx* c, const float* M, const int32_t* counts, float* D) {
    if (!c || !M || !D) return SBO_EINVAL;
    c->n_spans = 0;
    StageTimer t(c, SBO_STAGE_SVD);
    SBO_HIP(launch_polar(c->p, c->K, M, counts, D, c->ws, c->svd_method, nullptr, 0, c->stream));
    return SBO_OK;
}

int sbo_update(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk, const int32_t* supp,
               const float* coef, float* D, int32_t* counts) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !blk || !supp || !coef || !D) return SBO_EINVAL;
    c->n_spans = 0;
    rc = run_group(c, blk, m);
    if (rc) return rc;
    rc = run_update_grouped(c, Y, m, supp, coef, D);
    if (rc) return rc;
    if (counts)
        SBO_HIP(hipMemcpyAsync(counts, c->ws.counts, (size_t)c->K * 4, hipMemcpyDeviceToDevice,
                               c->stream));
    return SBO_OK;
}

int sbo_iterate(sbo_ctx* c, const float* Y, int64_t m, float* D, int n_iter, int32_t* blk,
                int32_t* supp, float* coef, float* err, double* sqerr_per_iter) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !D || !blk || !supp || !coef || !err || n_iter < 1) return SBO_EINVAL;
    c->n_spans = 0;
    const bool fused = c->p <= 64;             // select and accumulate share one pass over Y
    for (int it = 0; it < n_iter; ++it) {
        if (!fused) {
            rc = run_code(c, Y, m, D, blk, supp, coef, err);
            if (rc) return rc;
            if (sqerr_per_iter) SBO_HIP(launch_sqerr(err, nullptr, m, c->ws, sqerr_per_iter + it, c->stream));
            rc = run_update_grouped(c, Y, m, supp, coef, D);   // grouping reused
            if (rc) return rc;
            continue;
        }
        // The dictionary in the coding kernel's operand order: rewritten from D at the start
        // of the call, kept up to date by the SVD kernel afterwards.
        if (it == 0) {
            rc = run_swizzle(c, D);
            if (rc) return rc;
        }
        rc = run_energy(c, Y, m, blk);
        if (rc) return rc;
        rc = run_group(c, blk, m, true);
        if (rc) return rc;
        {
            StageTimer t(c, SBO_STAGE_SELECT);  // includes the per-piece accumulation
            SBO_HIP(launch_select_accum(c->p, c->K, c->s0, Y, m, D, c->ws, supp, coef, err, c->stream));
        }
        rc = run_polar_pieces(c, m, D, ops_kind(c), err, sqerr_per_iter ? sqerr_per_iter + it : nullptr);
        if (rc) return rc;
    }
    return SBO_OK;
}

static int run_train_rounds(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk, float* D, int R,
                            int32_t* supp, float* coef, float* err) {
    int rc = run_group(c, blk, m);             // the assignment, hence the grouping, is fixed
    if (rc) return rc;
    for (int r = 0; r < R; ++r) {
        if (c->p <= 64) {
            {
                StageTimer t(c, SBO_STAGE_SELECT);
                SBO_HIP(launch_select_accum(c->p, c->K, c->s0, Y, m, D, c->ws, supp, coef, err,
                                            c->stream));
            }
            rc = run_polar_pieces(c, m, D, 0, nullptr, nullptr);
            if (rc) return rc;
            continue;
        } else {
            {
                StageTimer t(c, SBO_STAGE_SELECT);
                SBO_HIP(launch_select(c->p, c->K, c->s0, Y, m, D, c->ws, supp, coef, err, false,
                                      use_split(c), c->stream));
            }
            StageTimer t(c, SBO_STAGE_ACCUM);
            SBO_HIP(launch_accumulate(c->p, c->K, c->s0, Y, m, supp, coef, c->ws, c->ws.M, c->stream));
        }
        StageTimer t(c, SBO_STAGE_SVD);
        SBO_HIP(launch_polar(c->p, c->K, c->ws.M, c->ws.counts, D, c->ws, c->svd_method, nullptr, 0,
                             c->stream));
    }
    return SBO_OK;
}

int sbo_train_rounds(sbo_ctx* c, const float* Y, int64_t m, const int32_t* blk, float* D, int R,
                     int32_t* supp, float* coef, float* err) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !blk || !D || !supp || !coef || !err || R < 1) return SBO_EINVAL;
    c->n_spans = 0;
    return run_train_rounds(c, Y, m, blk, D, R, supp, coef, err);
}

int sbo_set_blocks(sbo_ctx* c, int K) {
    if (!c || K < 1 || K > c->K_cap) return SBO_EINVAL;
    c->K = K;
    return SBO_OK;
}

int sbo_sqerr(sbo_ctx* c, const float* err, int64_t m, double* out) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!err || !out) return SBO_EINVAL;
    SBO_HIP(launch_sqerr(err, nullptr, m, c->ws, out, c->stream));
    return SBO_OK;
}

int sbo_worst(sbo_ctx* c, const float* err, int64_t m, int64_t W, int32_t* ids) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!err || !ids || W < 1 || W > m) return SBO_EINVAL;
    SBO_HIP(launch_worst(err, m, W, c->ws, ids, c->stream));
    return SBO_OK;
}

// Gram matrix of the set -> its eigenvectors by descending eigenvalue (ws.perm etc. hold the set).
static int run_init_base(sbo_ctx* c, const float* Y, int64_t n, float* Q, float* sv) {
    SBO_HIP(launch_gram(c->p, 1, Y, n, c->ws, c->ws.M, c->stream));
    SBO_HIP(launch_polar(c->p, 1, c->ws.M, nullptr, Q, c->ws, 0, sv ? sv : c->ws.energy, 0,
                         c->stream));              // energy[m_max >= p] as a sink
    return SBO_OK;
}

int sbo_init_base(sbo_ctx* c, const float* Y, int64_t m, const int32_t* ids, int64_t n, float* Q,
                  float* sv) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !ids || !Q || n < 1 || n > m) return SBO_EINVAL;
    if (c->m_max < c->p) return SBO_EINVAL;    // the workspace doubles as scratch of p floats
    c->n_spans = 0;
    SBO_HIP(launch_single_block(ids, n, m, c->ws, c->stream));
    return run_init_base(c, Y, n, Q, sv);
}

// ws.perm etc. already hold the set (launch_single_block).
static int run_new_base(sbo_ctx* c, const float* Y, int64_t n, int R, int have_q0, float* Q,
                        int32_t* supp, float* coef, float* err, double* sqerr_per_round) {
    if (!have_q0) {
        int rc = run_init_base(c, Y, n, Q, nullptr);
        if (rc) return rc;
    }
    for (int r = 0; r < R; ++r) {
        if (c->p <= 64) {
            SBO_HIP(launch_select_accum(c->p, 1, c->s0, Y, n, Q, c->ws, supp, coef, err, c->stream));
        } else {
            SBO_HIP(launch_select(c->p, 1, c->s0, Y, n, Q, c->ws, supp, coef, err, false, use_split(c), c->stream));
            SBO_HIP(launch_accumulate(c->p, 1, c->s0, Y, n, supp, coef, c->ws, c->ws.M, c->stream));
        }
        if (sqerr_per_round)
            SBO_HIP(launch_sqerr(err, c->ws.perm, n, c->ws, sqerr_per_round + r, c->stream));
        if (c->p <= 64) {
            int rc = run_polar_pieces(c, n, Q, 0, nullptr, nullptr, 1);
            if (rc) return rc;
        } else {
            SBO_HIP(launch_polar(c->p, 1, c->ws.M, c->ws.counts, Q, c->ws, c->svd_method, nullptr, 0,
                                 c->stream));
        }
    }
    return SBO_OK;
}

int sbo_new_base(sbo_ctx* c, const float* Y, int64_t m, const int32_t* ids, int64_t n, int R,
                 int have_q0, float* Q, int32_t* supp, float* coef, float* err,
                 double* sqerr_per_round) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !ids || !Q || !supp || !coef || !err || n < 1 || n > m || R < 0) return SBO_EINVAL;
    if (c->m_max < c->p) return SBO_EINVAL;
    c->n_spans = 0;
    SBO_HIP(launch_single_block(ids, n, m, c->ws, c->stream));
    return run_new_base(c, Y, n, R, have_q0, Q, supp, coef, err, sqerr_per_round);
}

// RMSE of the codes in err (Section 4), read back to the host (synchronises the stream).
static int host_rmse(sbo_ctx* c, const float* err, int64_t m, double* out) {
    SBO_HIP(launch_sqerr(err, nullptr, m, c->ws, c->ws.sq_out, c->stream));
    double sq = 0.0;
    SBO_HIP(hipMemcpyAsync(&sq, c->ws.sq_out, sizeof(double), hipMemcpyDeviceToHost, c->stream));
    SBO_HIP(hipStreamSynchronize(c->stream));
    *out = sqrt(sq / ((double)c->p * (double)m));
    return SBO_OK;
}

int sbo_learn(sbo_ctx* c, const float* Y, int64_t m, float* D, const int32_t* init_ids, int K0,
              int64_t P0, int R, int64_t W, int K_max, double target_rmse, int32_t* blk,
              int32_t* supp, float* coef, float* err, int* K_final, double* rmse_hist, int* n_hist) {
    int rc = check_call(c, m);
    if (rc) return rc;
    if (!Y || !D || !init_ids || !blk || !supp || !coef || !err || !K_final || !rmse_hist || !n_hist)
        return SBO_EINVAL;
    if (K0 < 1 || K0 > K_max || K_max > c->K_cap || P0 < 1 || P0 > m || W < 1 || W > m || R < 1)
        return SBO_EINVAL;
    if (c->m_max < c->p) return SBO_EINVAL;
    c->n_spans = 0;
    const int K_before = c->K;
    const size_t pp = (size_t)c->p * c->p;
    auto fail = [&](int code) {
        c->K = K_before;
        return code;
    };

    // Initialisation: K0 orthobases, each trained on its own signal set; then represent.
    // p <= 64: all K0 at once, the sets as K0 blocks of one grouping (eq. (5) for every block,
    // then R rounds of the fused select + accumulate and the SVD update over K0 blocks; a
    // signal that sits in two sets only has its scratch rows of supp / coef / err written
    // twice, which nothing reads).  Otherwise, and when the sets do not fit the workspace, one
    // after the other.
    const int64_t n_init = (int64_t)K0 * P0;
    if (c->p <= 64 && n_init <= c->m_max && (int64_t)K0 * c->p <= c->m_max) {
        SBO_HIP(launch_equal_blocks(init_ids, K0, P0, m, c->ws, c->stream));
        SBO_HIP(launch_gram(c->p, K0, Y, n_init, c->ws, c->ws.M, c->stream));
        SBO_HIP(launch_polar(c->p, K0, c->ws.M, nullptr, D, c->ws, 0, c->ws.energy, 0, c->stream));
        for (int r = 0; r < R; ++r) {
            SBO_HIP(launch_select_accum(c->p, K0, c->s0, Y, n_init, D, c->ws, supp, coef, err, c->stream));
            rc = run_polar_pieces(c, n_init, D, 0, nullptr, nullptr, K0);
            if (rc) return fail(rc);
        }
    } else {
        for (int j = 0; j < K0; ++j) {
            SBO_HIP(launch_single_block(init_ids + (size_t)j * P0, P0, m, c->ws, c->stream));
            rc = run_new_base(c, Y, P0, R, 0, D + j * pp, supp, coef, err, nullptr);
            if (rc) return fail(rc);
        }
    }
    int K = K0;
    c->K = K;
    rc = run_code(c, Y, m, D, blk, supp, coef, err);
    if (rc) return fail(rc);
    int n = 0;
    rc = host_rmse(c, err, m, &rmse_hist[n]);
    if (rc) return fail(rc);
    ++n;

    // Iterations: grow by one orthobase trained on the worst-W set, represent, train every
    // orthobase over its own signals, check the stopping rule.
    while (K < K_max && rmse_hist[n - 1] > target_rmse) {
        if (hipError_t e = launch_worst(err, m, W, c->ws, c->ws.sel_ids, c->stream); e != hipSuccess)
            return fail(hip_fail(e));
        if (hipError_t e = launch_single_block(c->ws.sel_ids, W, m, c->ws, c->stream); e != hipSuccess)
            return fail(hip_fail(e));
        rc = run_new_base(c, Y, W, R, 0, D + K * pp, supp, coef, err, nullptr);
        if (rc) return fail(rc);
        ++K;
        c->K = K;
        rc = run_code(c, Y, m, D, blk, supp, coef, err);
        if (rc) return fail(rc);
        rc = run_train_rounds(c, Y, m, blk, D, R, supp, coef, err);
        if (rc) return fail(rc);
        rc = host_rmse(c, err, m, &rmse_hist[n]);
        if (rc) return fail(rc);
        ++n;
    }
    *K_final = K;
    *n_hist = n;
    c->K = K_before;
    return SBO_OK;
}

int sbo_svd_sweeps(sbo_ctx* c, int32_t* sweeps) {
    if (!c || !sweeps) return SBO_EINVAL;
    SBO_HIP(hipMemcpyAsync(sweeps, c->ws.sweeps, (size_t)c->K * 4, hipMemcpyDeviceToHost, c->stream));
    SBO_HIP(hipStreamSynchronize(c->stream));
    return SBO_OK;
}

int sbo_set_option(sbo_ctx* c, int option, int value) {
    if (!c) return SBO_EINVAL;
    switch (option) {
        case SBO_OPT_SVD_METHOD:
            if (value != SBO_SVD_AUTO && value != SBO_SVD_JACOBI) return SBO_EINVAL;
            c->svd_method = value;
            return SBO_OK;
        case SBO_OPT_CODING_ARITH:
            if (value != SBO_ARITH_F32 && value != SBO_ARITH_BF16X3 && value != SBO_ARITH_BF16X3_SCREEN &&
                value != SBO_ARITH_F16X2)
                return SBO_EINVAL;
            c->coding_arith = value;
            c->ws.parts_accum = value != SBO_ARITH_F32;
            return SBO_OK;
        default: return SBO_EINVAL;
    }
}

int sbo_set_timing(sbo_ctx* c, int enable) {
    if (!c) return SBO_EINVAL;
    c->timing = enable == 2 ? 2 : (enable ? 1 : 0);
    c->n_spans = 0;
    return SBO_OK;
}

int sbo_stage_ms(sbo_ctx* c, float* ms) {
    if (!c || !ms) return SBO_EINVAL;
    for (int s = 0; s < SBO_N_STAGES; ++s) ms[s] = 0.f;
    SBO_HIP(hipStreamSynchronize(c->stream));
    for (size_t i = 0; i < c->n_spans; ++i) {
        float t = 0.f;
        SBO_HIP(hipEventElapsedTime(&t, c->spans[i].beg, c->spans[i].end));
        ms[c->spans[i].stage] += t;
    }
    return SBO_OK;
}

const char* sbo_strerror(int code) {
    switch (code) {
        case SBO_OK: return "success";
        case SBO_EINVAL: return "invalid argument or unsupported shape";
        case SBO_ENOMEM: return "out of device memory";
        case SBO_ELIMIT: return g_hip_text.c_str();
        case SBO_EHIP: return g_hip_text.c_str();
        default: return "unknown error code";
    }
}

}  // extern "C"
