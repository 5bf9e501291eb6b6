"""Helpers for the GPU parity tests: run the C-ABI entry points on numpy inputs and
compare their outputs with the oracle's under the stated tolerances."""
from __future__ import annotations

import numpy as np

import paper_1412_4944_amd as sbo

BLOCK_GAP = 1e-5     # oracle top-two block energies closer than this * ||y||^2: block not compared
SUPP_GAP = 1e-5      # oracle s0-th / (s0+1)-th magnitudes closer than this * ||y||: support not compared
COEF_TOL = 1e-4      # |coef_gpu - coef_oracle| <= COEF_TOL * ||y||
ERR_TOL = 1e-4       # |err_gpu - err_oracle|   <= ERR_TOL * ||y||^2
Q_TOL = 1e-4         # max-abs on blocks with sigma_min > 1e-3 * sigma_max
ORTHO_TOL = 1e-5     # max |Q^T Q - I| of every block written by the GPU


class Sbo:
    """One libsbo context plus device copies; everything returned is numpy."""

    def __init__(self, p, K, s0, m_max, jacobi_only=False, arith=None):
        import torch
        self.torch = torch
        self.dev = torch.device("cuda:0")
        self.p, self.K, self.s0 = p, K, s0
        self.ctx = sbo.sbo_create(p, K, s0, m_max)
        if jacobi_only:
            self.svd_jacobi(True)
        if arith is not None:
            self.coding_arith(arith)

    def coding_arith(self, name):
        """"f32": fp32 matrix instruction; "bf16x3": three-part bf16 split on the bf16 matrix cores;
        "screen": the same with the block choice screened by the three largest partial products."""
        sbo.sbo_set_option(self.ctx, sbo.SBO_OPT_CODING_ARITH,
                           {"f32": sbo.SBO_ARITH_F32, "bf16x3": sbo.SBO_ARITH_BF16X3,
                            "screen": sbo.SBO_ARITH_BF16X3_SCREEN, "f16x2": sbo.SBO_ARITH_F16X2}[name])

    def svd_jacobi(self, on):
        """Jacobi SVD for every orthobase (on) or the default Newton-Schulz + Jacobi fallback."""
        sbo.sbo_set_option(self.ctx, sbo.SBO_OPT_SVD_METHOD, sbo.SBO_SVD_JACOBI if on else sbo.SBO_SVD_AUTO)

    def close(self):
        if self.ctx is not None:
            sbo.sbo_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *a):
        self.close()

    def dev_f32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev)

    def dev_i32(self, a):
        return self.torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(self.dev)

    def outputs(self, m):
        t = self.torch
        return (t.full((m,), -7, dtype=t.int32, device=self.dev),
                t.full((m, self.s0), -7, dtype=t.int32, device=self.dev),
                t.full((m, self.s0), float("nan"), dtype=t.float32, device=self.dev),
                t.full((m,), float("nan"), dtype=t.float32, device=self.dev))

    def code(self, Y, D):
        Yd, Dd = self.dev_f32(Y), self.dev_f32(D)
        blk, supp, coef, err = self.outputs(Y.shape[0])
        sbo.sbo_code(self.ctx, Yd, Dd, blk, supp, coef, err)
        self.torch.cuda.synchronize()
        return blk.cpu().numpy(), supp.cpu().numpy(), coef.cpu().numpy(), err.cpu().numpy()

    def group(self, blk):
        t = self.torch
        m = len(blk)
        counts = t.full((self.K,), -7, dtype=t.int32, device=self.dev)
        offsets = t.full((self.K + 1,), -7, dtype=t.int32, device=self.dev)
        perm = t.full((m,), -7, dtype=t.int32, device=self.dev)
        sbo.sbo_group(self.ctx, self.dev_i32(blk), counts, offsets, perm)
        t.cuda.synchronize()
        return counts.cpu().numpy(), offsets.cpu().numpy(), perm.cpu().numpy()

    def accumulate(self, Y, blk, supp, coef):
        t = self.torch
        M = t.full((self.K, self.p, self.p), float("nan"), dtype=t.float32, device=self.dev)
        sbo.sbo_accumulate(self.ctx, self.dev_f32(Y), self.dev_i32(blk), self.dev_i32(supp),
                           self.dev_f32(coef), M)
        t.cuda.synchronize()
        return M.cpu().numpy()

    def polar(self, M, D_old, counts=None):
        Dd = self.dev_f32(D_old)
        sbo.sbo_polar(self.ctx, self.dev_f32(M), None if counts is None else self.dev_i32(counts), Dd)
        self.torch.cuda.synchronize()
        return Dd.cpu().numpy()

    def update(self, Y, blk, supp, coef, D):
        t = self.torch
        Dd = self.dev_f32(D)
        counts = t.full((self.K,), -7, dtype=t.int32, device=self.dev)
        sbo.sbo_update(self.ctx, self.dev_f32(Y), self.dev_i32(blk), self.dev_i32(supp),
                       self.dev_f32(coef), Dd, counts)
        t.cuda.synchronize()
        return Dd.cpu().numpy(), counts.cpu().numpy()

    def train_rounds(self, Y, blk, D, R):
        Yd, Dd = self.dev_f32(Y), self.dev_f32(D)
        _b, supp, coef, err = self.outputs(Y.shape[0])
        sbo.sbo_train_rounds(self.ctx, Yd, self.dev_i32(blk), Dd, R, supp, coef, err)
        self.torch.cuda.synchronize()
        return Dd.cpu().numpy(), supp.cpu().numpy(), coef.cpu().numpy(), err.cpu().numpy()

    def sqerr(self, err):
        out = self.torch.zeros((1,), dtype=self.torch.float64, device=self.dev)
        sbo.sbo_sqerr(self.ctx, self.dev_f32(err), out)
        self.torch.cuda.synchronize()
        return float(out.item())

    def worst(self, err, W):
        ids = self.torch.full((W,), -7, dtype=self.torch.int32, device=self.dev)
        sbo.sbo_worst(self.ctx, self.dev_f32(err), W, ids)
        self.torch.cuda.synchronize()
        return ids.cpu().numpy()

    def init_base(self, Y, ids):
        t = self.torch
        Q = t.full((self.p, self.p), float("nan"), dtype=t.float32, device=self.dev)
        sv = t.full((self.p,), float("nan"), dtype=t.float32, device=self.dev)
        sbo.sbo_init_base(self.ctx, self.dev_f32(Y), self.dev_i32(ids), Q, sv)
        t.cuda.synchronize()
        return Q.cpu().numpy(), sv.cpu().numpy()

    def new_base(self, Y, ids, R, Q0=None):
        """Returns Q, the code arrays (rows outside the set keep their fill values) and the
        per-round squared errors."""
        t = self.torch
        m = Y.shape[0]
        Q = self.dev_f32(Q0) if Q0 is not None else t.full((self.p, self.p), float("nan"),
                                                           dtype=t.float32, device=self.dev)
        _b, supp, coef, err = self.outputs(m)
        sq = t.zeros((max(R, 1),), dtype=t.float64, device=self.dev)
        sbo.sbo_new_base(self.ctx, self.dev_f32(Y), self.dev_i32(ids), R, Q0 is not None, Q, supp, coef,
                         err, sq)
        t.cuda.synchronize()
        return Q.cpu().numpy(), supp.cpu().numpy(), coef.cpu().numpy(), err.cpu().numpy(), sq.cpu().numpy()[:R]

    def iterate(self, Y, D, n_iter):
        t = self.torch
        Yd, Dd = self.dev_f32(Y), self.dev_f32(D)
        blk, supp, coef, err = self.outputs(Y.shape[0])
        sq = t.zeros((n_iter,), dtype=t.float64, device=self.dev)
        sbo.sbo_iterate(self.ctx, Yd, Dd, n_iter, blk, supp, coef, err, sq)
        t.cuda.synchronize()
        return (Dd.cpu().numpy(), blk.cpu().numpy(), supp.cpu().numpy(), coef.cpu().numpy(),
                err.cpu().numpy(), sq.cpu().numpy())


def compare_code(Y, D, s0, oracle_out, gpu_out, max_exempt_frac=0.01):
    """Element-by-element comparison of one coding pass.  Returns the fraction of
    signals exempted as near-ties."""
    oblk, osupp, ocoef, oerr, oE = oracle_out
    gblk, gsupp, gcoef, gerr = gpu_out
    Y64 = np.asarray(Y, np.float64)
    D64 = np.asarray(D, np.float64)
    m, p = Y64.shape
    K = D64.shape[0]
    n2 = (Y64 ** 2).sum(1)
    nrm = np.sqrt(n2)
    assert gblk.min() >= 0 and gblk.max() < K
    assert gsupp.min() >= 0 and gsupp.max() < p
    assert (np.diff(gsupp, axis=1) > 0).all(), "support not strictly ascending"
    assert np.isfinite(gcoef).all() and np.isfinite(gerr).all()

    # block index: bit-exact unless the oracle's two best energies nearly tie
    if K > 1:
        top2 = np.sort(oE, axis=1)[:, -2:]
        block_tie = (top2[:, 1] - top2[:, 0]) < BLOCK_GAP * np.maximum(n2, 1e-300)
    else:
        block_tie = np.zeros(m, bool)
    bad_blk = gblk != oblk
    assert not (bad_blk & ~block_tie).any(), \
        f"{(bad_blk & ~block_tie).sum()} block mismatches outside the near-tie exemption"

    same_blk = ~bad_blk
    # support: bit-exact unless the s0-th and (s0+1)-th magnitudes nearly tie
    bad_supp = same_blk & (gsupp != osupp).any(axis=1)
    ids = np.nonzero(bad_supp)[0]
    supp_tie = np.zeros(m, bool)
    if ids.size and s0 < p:
        C = np.einsum("nkd,nd->nk", D64[oblk[ids]], Y64[ids])
        mags = -np.sort(-np.abs(C), axis=1)
        supp_tie[ids] = (mags[:, s0 - 1] - mags[:, s0]) < SUPP_GAP * np.maximum(nrm[ids], 1e-300)
    assert not (bad_supp & ~supp_tie).any(), \
        f"{(bad_supp & ~supp_tie).sum()} support mismatches outside the near-tie exemption"

    ok = same_blk & ~bad_supp
    dcoef = np.abs(gcoef[ok].astype(np.float64) - ocoef[ok])
    assert (dcoef <= COEF_TOL * nrm[ok, None] + 1e-30).all(), f"coef off by {dcoef.max()}"
    derr = np.abs(gerr[ok].astype(np.float64) - oerr[ok])
    assert (derr <= ERR_TOL * n2[ok] + 1e-30).all(), f"err off by {derr.max()}"

    # exempted signals must still be valid s0-term codes: the GPU's own choice, evaluated
    # in fp64, has to be as good as the oracle's up to the tie gap
    ex = np.nonzero(~ok)[0]
    if ex.size:
        atoms = D64[gblk[ex, None], gsupp[ex]]
        x = np.einsum("ntd,nd->nt", atoms, Y64[ex])
        np.testing.assert_allclose(gcoef[ex], x, rtol=0, atol=COEF_TOL * nrm[ex].max())
        res = ((Y64[ex] - np.einsum("nt,ntd->nd", x, atoms)) ** 2).sum(1)
        assert (res <= oerr[ex] + 4 * max(BLOCK_GAP, SUPP_GAP) * n2[ex] + 1e-30).all()
        assert (np.abs(gerr[ex] - res) <= ERR_TOL * n2[ex] + 1e-30).all()
    frac = ex.size / m
    assert frac <= max_exempt_frac, f"exempt fraction {frac}"
    return frac


def compare_assigned_code(Y, D, blk, s0, oracle_out, gpu_out, max_exempt_frac=0.01):
    """Codes computed with the block assignment GIVEN (frozen-assignment rounds, a new orthobase
    on a set): per block, the same gated comparison as compare_code with that block as the only
    candidate (support bit-exact unless the s0-th / (s0+1)-th magnitudes nearly tie, and then a
    valid code whose error is within the gap).  oracle_out / gpu_out = (supp, coef, err) over
    the rows of Y.  Returns the exempt fraction over all signals."""
    so, co, eo = oracle_out
    sg, cg, eg = gpu_out
    blk = np.asarray(blk)
    m = Y.shape[0]
    exempt = 0.0
    for j in np.unique(blk):
        ids = np.nonzero(blk == j)[0]
        z = np.zeros(ids.size, np.int32)
        frac = compare_code(Y[ids], np.asarray(D)[j:j + 1], s0, (z, so[ids], co[ids], eo[ids], None),
                            (z, sg[ids], cg[ids], eg[ids]), max_exempt_frac=1.0)
        exempt += frac * ids.size
    exempt /= m
    assert exempt <= max_exempt_frac, f"exempt fraction {exempt}"
    return exempt


def compare_Q(D_gpu, D_oracle, M_oracle, updated):
    """Q_j within Q_TOL max-abs where M_j is well conditioned; orthonormal always;
    Q^T P symmetric PSD (polar factor property) on every updated block."""
    K, p, _ = D_gpu.shape
    worst = 0.0
    for j in range(K):
        Qg = D_gpu[j].astype(np.float64).T                 # p x p, columns = atoms
        assert np.abs(Qg.T @ Qg - np.eye(p)).max() <= ORTHO_TOL, f"block {j} not orthonormal"
        if not updated[j]:
            continue
        P = M_oracle[j].T
        sv = np.linalg.svd(P, compute_uv=False)
        H = Qg.T @ P
        scale = sv[0]
        assert np.abs(H - H.T).max() <= 2e-4 * scale, f"block {j}: Q^T P not symmetric"
        assert np.linalg.eigvalsh((H + H.T) / 2).min() >= -2e-4 * scale
        if sv[-1] > 1e-3 * sv[0]:
            d = np.abs(Qg - D_oracle[j].T).max()
            worst = max(worst, d)
            assert d <= Q_TOL, f"block {j}: Q off by {d}"
    return worst
