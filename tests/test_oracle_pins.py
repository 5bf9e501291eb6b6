"""Pins for the CPU oracle: each check ties an oracle function to something
other than itself (closed forms, brute force, library routines it does not
call, invariants the paper's constraints imply).  CPU only."""
import itertools
import json
import os

import numpy as np
import pytest
import scipy.linalg

import sbo_synth as synth
from oracle import sbo_oracle as orc

HERE = os.path.dirname(os.path.abspath(__file__))


def _tiny(keep=True, **kw):
    return synth.generate(synth.CONFIGS["tiny"], keep_fp64=keep, **kw)


# ----------------------------------------------------------------- generator
def test_generator_onbs_orthonormal_1e12():
    rng = np.random.default_rng(7)
    for p in (2, 8, 16, 64):
        Q = synth.random_onb(rng, p)
        assert np.abs(Q.T @ Q - np.eye(p)).max() < 1e-12
    D = synth.random_dictionary(rng, 3, 16)
    for j in range(3):
        assert np.abs(D[j] @ D[j].T - np.eye(16)).max() < 1e-12


def test_generator_snr_exact_and_shapes():
    cfg = synth.custom("c", p=16, K=3, m=500, s0=2, snr_db=20.0)
    pr = synth.generate(cfg, keep_fp64=True)
    clean = np.einsum("nt,ntd->nd", pr.coef, pr.D_planted64[pr.blk[:, None], pr.supp])
    noise = pr.Y64 - clean
    snr = 10 * np.log10((clean ** 2).sum() / (noise ** 2).sum())
    assert abs(snr - 20.0) < 1e-9
    assert pr.Y.dtype == np.float32 and pr.Y.shape == (500, 16)
    assert (np.diff(pr.supp, axis=1) > 0).all()


# ------------------------------------------------------------ hand-worked 2-D
def test_hand_worked_2d_example():
    g = json.load(open(os.path.join(HERE, "golden", "hand_2d.json")))
    Q = np.array(g["Q"], float)
    Y = np.array(g["Y"], float)
    blk, supp, coef, err, E = orc.o_code(Y, Q, 1)
    assert blk.tolist() == g["blk"]
    assert supp.tolist() == g["supp"]
    np.testing.assert_allclose(coef, g["coef"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(err, g["err"], rtol=0, atol=1e-14)
    np.testing.assert_allclose(E, g["energy"], rtol=0, atol=1e-14)
    Dn, M = orc.o_update(Y, blk, supp, coef, Q)
    # P (column-major p x p) for block 0 is [[9,0],[3,25]]; atom-major storage is its transpose
    np.testing.assert_allclose(M[0].T, [[9, 0], [3, 25]], atol=1e-14)
    s2 = np.sqrt(2.0)
    np.testing.assert_allclose(M[1].T, [[4 * s2, -3 / s2], [4 * s2, 6 / s2]], atol=1e-14)
    for j, (num, den) in enumerate(g["polar_tan"]):
        h = np.hypot(num, den)
        R = np.array([[den, -num], [num, den]]) / h       # rotation by atan(num/den)
        np.testing.assert_allclose(Dn[j].T, R, atol=1e-14)


# ------------------------------------------------------------------- coding
def test_parseval_and_closed_form_error():
    pr = _tiny()
    D = synth.random_dictionary(np.random.default_rng(3), 4, 16)   # fp64-orthonormal
    Y = pr.Y64 + 0.05 * np.random.default_rng(4).standard_normal(pr.Y64.shape)
    blk, supp, coef, err, E = orc.o_code(Y, D, 3)
    n2 = (Y ** 2).sum(axis=1)
    # Parseval: all p coefficients in any one orthobase carry the full energy
    _, _, cfull, efull, Efull = orc.o_code(Y, D, 16)
    np.testing.assert_allclose(Efull, n2[:, None] * np.ones((1, 4)), rtol=1e-12)
    assert np.abs(efull).max() <= 1e-24 * n2.max() + 1e-26
    # err computed directly equals ||y||^2 - E_kept
    np.testing.assert_allclose(err, n2 - E[np.arange(len(blk)), blk], rtol=0, atol=1e-12 * n2.max())
    # kept energy equals the sum of the reported coefficients squared
    np.testing.assert_allclose((coef ** 2).sum(1), E[np.arange(len(blk)), blk], rtol=1e-12)


@pytest.mark.parametrize("p,s0", [(4, 1), (6, 2), (8, 3), (8, 5)])
def test_top_s0_is_best_s0_term_fit_bruteforce(p, s0):
    rng = np.random.default_rng(100 + p + s0)
    K = 3
    D = synth.random_dictionary(rng, K, p)
    Y = rng.standard_normal((12, p))
    blk, supp, coef, err, E = orc.o_code(Y, D, s0)
    for i in range(Y.shape[0]):
        best = (np.inf, None, None)
        per_block_min = []
        for j in range(K):
            Q = D[j].T
            bj = np.inf
            for S in itertools.combinations(range(p), s0):
                x, *_ = np.linalg.lstsq(Q[:, S], Y[i], rcond=None)
                r = ((Y[i] - Q[:, S] @ x) ** 2).sum()
                bj = min(bj, r)
                if r < best[0] - 1e-13:
                    best = (r, j, S)
            per_block_min.append(bj)
        assert best[1] == blk[i]
        assert list(best[2]) == supp[i].tolist()
        assert abs(best[0] - err[i]) < 1e-12
        np.testing.assert_allclose((Y[i] ** 2).sum() - E[i], per_block_min, atol=1e-12)


def test_tie_breaks_and_zero_signal():
    # two identical blocks -> lowest block index; equal magnitudes -> lowest atom index
    I = np.eye(4)
    D = np.stack([I, I])
    Y = np.array([[1.0, -1.0, 1.0, 1.0], [0, 0, 0, 0], [0.5, 2.0, -2.0, 0.1]])
    blk, supp, coef, err, E = orc.o_code(Y, D, 2)
    assert blk.tolist() == [0, 0, 0]
    assert supp.tolist() == [[0, 1], [0, 1], [1, 2]]
    np.testing.assert_allclose(coef, [[1, -1], [0, 0], [2, -2]])
    np.testing.assert_allclose(err, [2.0, 0.0, 0.26])


def test_planted_recovery_noiseless_fp64():
    pr = _tiny()
    blk, supp, coef, err, E = orc.o_code(pr.Y64, pr.D_planted64, pr.cfg.s0)
    assert (blk == pr.blk).all()
    assert (supp == pr.supp).all()
    np.testing.assert_allclose(coef, pr.coef, rtol=0, atol=1e-12)
    n2 = (pr.Y64 ** 2).sum(1)
    assert (err <= 1e-24 * n2 + 1e-28).all()
    # the same on the fp32-rounded inputs the GPU sees
    blk, supp, coef, err, E = orc.o_code(pr.Y, pr.D_planted, pr.cfg.s0)
    assert (blk == pr.blk).all() and (supp == pr.supp).all()
    assert (err <= 1e-12 * n2).all()


def test_block_argmax_bruteforce():
    rng = np.random.default_rng(11)
    D = synth.random_dictionary(rng, 5, 8)
    Y = rng.standard_normal((40, 8))
    blk, supp, coef, err, E = orc.o_code(Y, D, 3)
    for i in range(40):
        en = []
        for j in range(5):
            c = np.array([D[j, k] @ Y[i] for k in range(8)])
            en.append(np.sort(c ** 2)[-3:].sum())
        assert int(np.argmax(en)) == blk[i]
        np.testing.assert_allclose(en, E[i], rtol=1e-12)


# ----------------------------------------------------------------- grouping
def test_grouping_invariants():
    rng = np.random.default_rng(5)
    K = 7
    blk = rng.integers(0, K, 1000).astype(np.int32)
    blk[blk == 3] = 2                                  # an empty block
    counts, offsets, perm = orc.o_group(blk, K)
    assert counts.sum() == 1000 and counts[3] == 0
    assert sorted(perm.tolist()) == list(range(1000))
    assert (np.diff(blk[perm]) >= 0).all()
    assert offsets[0] == 0 and offsets[-1] == 1000
    for j in range(K):
        seg = perm[offsets[j]:offsets[j + 1]]
        assert (blk[seg] == j).all() and (np.diff(seg) > 0).all()
        assert len(seg) == counts[j]


# ------------------------------------------------------------------- update
def test_accumulate_matches_loop_definition_and_trace_identity():
    pr = _tiny()
    D = pr.D_init.astype(np.float64)
    blk, supp, coef, err, E = orc.o_code(pr.Y, D, pr.cfg.s0)
    M = orc.o_accumulate(pr.Y, blk, supp, coef, pr.cfg.K)
    M2 = np.zeros_like(M)
    for i in range(pr.Y.shape[0]):                     # column k of P gains x_i[k] * y_i
        for t in range(pr.cfg.s0):
            M2[blk[i], supp[i, t]] += coef[i, t] * pr.Y[i].astype(np.float64)
    np.testing.assert_allclose(M, M2, atol=1e-12)
    # sum_j tr(Q_j^T P_j) = total kept energy
    tr = sum(np.trace(D[j] @ M[j].T) for j in range(pr.cfg.K))
    assert abs(tr - E[np.arange(len(blk)), blk].sum()) < 1e-9


def test_polar_factor_against_scipy_and_invariants():
    rng = np.random.default_rng(9)
    for p in (2, 5, 16, 64):
        P = rng.standard_normal((p, p))
        Q = orc.o_polar(P.T).T
        assert np.abs(Q.T @ Q - np.eye(p)).max() < 1e-12
        U = scipy.linalg.polar(P)[0]
        np.testing.assert_allclose(Q, U, atol=1e-10)
        H = Q.T @ P
        assert np.abs(H - H.T).max() < 1e-10
        assert np.linalg.eigvalsh((H + H.T) / 2).min() > -1e-10
        nuc = np.linalg.svd(P, compute_uv=False).sum()
        assert abs(np.trace(H) - nuc) < 1e-9
        for _ in range(5):
            R = synth.random_onb(rng, p)
            assert np.trace(R.T @ P) <= nuc + 1e-9


def test_update_is_procrustes_decrease_and_keeps_empty_block():
    pr = _tiny()
    D = pr.D_init.astype(np.float64)
    blk, supp, coef, err, E = orc.o_code(pr.Y, D, pr.cfg.s0)
    blk = blk.copy()
    moved = blk == 2
    blk[moved] = 1                                     # block 2 has no signals
    Dn, M = orc.o_update(pr.Y, blk, supp, coef, D)
    np.testing.assert_array_equal(Dn[2], D[2])
    Y = pr.Y.astype(np.float64)
    for j in (0, 1, 3):
        ids = np.nonzero(blk == j)[0]
        X = np.zeros((16, ids.size))
        X[supp[ids], np.arange(ids.size)[:, None]] = coef[ids]
        before = np.linalg.norm(Y[ids].T - D[j].T @ X)
        after = np.linalg.norm(Y[ids].T - Dn[j].T @ X)
        assert after <= before + 1e-12
        assert np.abs(Dn[j] @ Dn[j].T - np.eye(16)).max() < 1e-12


def test_fixed_point_at_planted_dictionary():
    pr = _tiny()
    blk, supp, coef, err, E = orc.o_code(pr.Y64, pr.D_planted64, pr.cfg.s0)
    Dn, M = orc.o_update(pr.Y64, blk, supp, coef, pr.D_planted64)
    assert np.abs(Dn - pr.D_planted64).max() < 1e-12
    blk, supp, coef, err, E = orc.o_code(pr.Y, pr.D_planted, pr.cfg.s0)
    Dn, M = orc.o_update(pr.Y, blk, supp, coef, pr.D_planted)
    assert np.abs(Dn - pr.D_planted).max() < 5e-6


# ---------------------------------------------------------------- iteration
@pytest.mark.parametrize("name,m", [("tiny", None), ("patch8", 2048)])
def test_iteration_error_non_increasing(name, m):
    pr = synth.generate(synth.CONFIGS[name], m=m)
    D, last, sq = orc.o_iterate(pr.Y, pr.D_init, pr.cfg.s0, 5, round_f32=False)
    assert (np.diff(sq) <= 1e-9 * sq[0]).all()
    assert sq[-1] < sq[0]
    assert orc.rmse(sq[0], pr.cfg.p, pr.Y.shape[0]) == pytest.approx(
        np.sqrt(sq[0] / pr.Y.size), rel=1e-15)
    for j in range(pr.cfg.K):
        assert np.abs(D[j] @ D[j].T - np.eye(pr.cfg.p)).max() < 1e-12


def test_frozen_assignment_rounds_monotone_and_consistent():
    pr = synth.generate(synth.CONFIGS["patch8"], m=3000)
    D0 = pr.D_init.astype(np.float64)
    blk = orc.o_code(pr.Y, D0, pr.cfg.s0)[0]
    D3, (supp, coef, err), sq = orc.o_train_rounds(pr.Y, blk, D0, pr.cfg.s0, 4, round_f32=False)
    # SELECT is the best s0-term code for the current basis and Q = U V^T the best basis for
    # the current code, so the error cannot increase from one round to the next
    assert (np.diff(sq) <= 1e-9 * sq[0]).all() and sq[-1] < sq[0]
    for j in range(pr.cfg.K):
        assert np.abs(D3[j] @ D3[j].T - np.eye(pr.cfg.p)).max() < 1e-12
    # one round from the coding pass's assignment = coding + update
    b, s_, c_, e_, _ = orc.o_code(pr.Y, D0, pr.cfg.s0)
    D1a, _ = orc.o_update(pr.Y, b, s_, c_, D0)
    D1b, (s2, c2, e2), sq1 = orc.o_train_rounds(pr.Y, b, D0, pr.cfg.s0, 1, round_f32=False)
    np.testing.assert_allclose(D1a, D1b, atol=1e-12)
    assert (s2 == s_).all() and np.allclose(c2, c_) and np.allclose(e2, e_)
    # per-round error recomputed from a dense reconstruction of the last round's code
    Y = pr.Y.astype(np.float64)
    rec = np.einsum("nt,ntd->nd", coef, D3[blk[:, None], supp])   # not the basis the code was made for
    assert ((Y - rec) ** 2).sum() <= sq[-1] + 1e-9                 # the later update only helps


def test_rmse_definition_against_dense_reconstruction():
    pr = _tiny()
    D = pr.D_init.astype(np.float64)
    blk, supp, coef, err, E = orc.o_code(pr.Y, D, pr.cfg.s0)
    K, p = pr.cfg.K, pr.cfg.p
    X = np.zeros((K * p, pr.Y.shape[0]))
    for i in range(pr.Y.shape[0]):
        X[blk[i] * p + supp[i], i] = coef[i]
    Dfull = np.concatenate([D[j].T for j in range(K)], axis=1)      # p x Kp = [Q_1 ... Q_K]
    fro = np.linalg.norm(pr.Y.T.astype(np.float64) - Dfull @ X)
    assert orc.rmse(err.sum(), p, pr.Y.shape[0]) == pytest.approx(fro / np.sqrt(pr.Y.size), rel=1e-12)
    assert (np.count_nonzero(X, axis=0) <= pr.cfg.s0).all()


# ------------------------------------------- worst-W set, base initialisation, new base
def test_worst_set_defining_inequalities_and_ties():
    rng = np.random.default_rng(31)
    err = rng.random(500)
    err[[7, 70, 170, 270]] = 0.5                      # exact ties at a value inside the range
    for W in (0, 1, 17, 250, 500):
        ids = orc.o_worst(err, W)
        assert ids.size == W and (np.diff(ids) > 0).all()
        rest = np.setdiff1d(np.arange(500), ids)
        if W and rest.size:
            assert err[ids].min() >= err[rest].max()
    # ties: with k of the four equal values to take, the k lowest indices are taken
    above = int((err > 0.5).sum())
    for k in (1, 2, 3):
        ids = orc.o_worst(err, above + k)
        tied = [i for i in (7, 70, 170, 270) if i in set(ids.tolist())]
        assert tied == [7, 70, 170, 270][:k]
    # brute force on a tiny case: exhaustive check of "no outsider beats an insider"
    e = np.array([0.1, 0.9, 0.9, 0.3, 0.0, 0.9])
    assert orc.o_worst(e, 2).tolist() == [1, 2]
    assert orc.o_worst(e, 4).tolist() == [1, 2, 3, 5]


def test_init_base_hand_worked_diagonal_and_rank_one():
    # Y_sub = diag(3, 1) padded with a zero signal: U = I (up to sign), sv = (3, 1)
    Y = np.array([[3.0, 0.0], [0.0, 1.0], [0.0, 0.0]])
    Q0, sv = orc.o_init_base(Y, [0, 1, 2])
    assert np.allclose(np.abs(Q0), np.eye(2), atol=1e-14) and np.allclose(sv, [3, 1])
    # order of the rows follows the singular values, not the input order
    Q0, sv = orc.o_init_base(Y, [1, 0])
    assert np.allclose(sv, [3, 1]) and np.allclose(np.abs(Q0), np.eye(2), atol=1e-14)
    # rank one: first atom = +-y/||y||, the rest an orthonormal completion
    y = np.array([[1.0, 2.0, 2.0]])
    Q0, sv = orc.o_init_base(np.repeat(y, 4, axis=0), [0, 1, 2, 3])
    assert np.allclose(np.abs(Q0[0]), y[0] / 3.0, atol=1e-14)
    assert np.allclose(sv, [6.0, 0, 0], atol=1e-12)
    assert np.abs(Q0 @ Q0.T - np.eye(3)).max() < 1e-12


def test_init_base_diagonalises_gram_and_recovers_planted_factor():
    rng = np.random.default_rng(32)
    p, n = 16, 200
    U = synth.random_onb(rng, p)
    s = np.linspace(5.0, 0.5, p)                      # distinct, descending
    W, _ = np.linalg.qr(rng.standard_normal((n, p)))
    Ysub = (U * s) @ W.T                              # p x n with known SVD
    Y = np.vstack([rng.standard_normal((50, p)), Ysub.T])   # the set sits at rows 50..249
    ids = np.arange(50, 250)
    Q0, sv = orc.o_init_base(Y, ids)
    assert np.allclose(sv, s, rtol=1e-12)
    assert np.abs(np.abs(Q0 @ U) - np.eye(p)).max() < 1e-10         # rows = +-columns of U, in order
    # independent route: eigen-decomposition of the Gram matrix (routine the oracle does not call)
    G = Ysub @ Ysub.T
    lam, E = np.linalg.eigh(G)
    assert np.allclose(lam[::-1], sv ** 2, rtol=1e-10)
    assert np.abs(np.abs(Q0 @ E[:, ::-1]) - np.eye(p)).max() < 1e-8
    assert np.abs(Q0 @ G @ Q0.T - np.diag(sv ** 2)).max() < 1e-10 * lam.max()
    # fewer signals than dimensions: still a complete orthobase
    Q0, sv = orc.o_init_base(Y, ids[:5])
    assert np.abs(Q0 @ Q0.T - np.eye(p)).max() < 1e-12 and (sv[5:] == 0).all()


def test_new_base_error_monotone_and_planted_fixed_point():
    pr = synth.generate(synth.custom("nb", p=16, K=1, m=600, s0=3, snr_db=None), keep_fp64=True)
    ids = np.arange(100, 500)
    # eq. (5) start, then rounds: the error of the codes never increases
    Q, sq = orc.o_new_base(pr.Y64, ids, 3, 6, round_f32=False)
    assert np.abs(Q @ Q.T - np.eye(16)).max() < 1e-12
    assert (np.diff(sq) <= 1e-12 * sq[0]).all()
    # started at the planted orthobase of noiseless data, training stays there with zero error
    Q, sq = orc.o_new_base(pr.Y64, ids, 3, 3, Q0=pr.D_planted64[0], round_f32=False)
    assert np.abs(Q - pr.D_planted64[0]).max() < 1e-10 and sq.max() < 1e-20 * (pr.Y64[ids] ** 2).sum()
    # the rounds are Algorithm 1 on the set alone: same as coding + update on the extracted signals
    sub = pr.Y64[ids]
    Q0, _ = orc.o_init_base(pr.Y64, ids)
    blk, supp, coef, err, _ = orc.o_code(sub, Q0[None], 3)
    Q1, _M = orc.o_update(sub, blk, supp, coef, Q0[None])
    Qa, sqa = orc.o_new_base(pr.Y64, ids, 3, 1, round_f32=False)
    assert np.abs(Qa - Q1[0]).max() < 1e-12 and abs(sqa[0] - err.sum()) <= 1e-12 * err.sum()


def test_learn_history_monotone_stops_and_matches_manual_steps():
    pr = synth.generate(synth.custom("lrn", p=16, K=3, m=900, s0=3, snr_db=25.0), keep_fp64=True)
    rng = np.random.default_rng(51)
    sets = [np.sort(rng.choice(900, 120, replace=False)) for _ in range(2)]
    D, blk, hist = orc.o_learn(pr.Y64, 3, sets, R=2, W=150, K_max=5, round_f32=False)
    assert D.shape == (5, 16, 16) and hist.size == 4            # K0 = 2, three growth iterations
    assert (np.diff(hist) <= 1e-12).all(), hist                 # the RMSE history never increases
    for j in range(5):
        assert np.abs(D[j] @ D[j].T - np.eye(16)).max() < 1e-12
    assert blk.min() >= 0 and blk.max() < 5
    # stopping rule: a target already met after the initial representation stops at once,
    # a target met after the first iteration stops there
    D0, _b, h0 = orc.o_learn(pr.Y64, 3, sets, R=2, W=150, K_max=5, target_rmse=hist[0] * 1.01, round_f32=False)
    assert D0.shape[0] == 2 and h0.size == 1 and h0[0] == hist[0]
    D1, _b, h1 = orc.o_learn(pr.Y64, 3, sets, R=2, W=150, K_max=5, target_rmse=(hist[1] + hist[2]) / 2,
                             round_f32=False)
    assert D1.shape[0] == 4 and np.allclose(h1, hist[:3], rtol=0, atol=1e-15)
    # recomposition of the first iteration from the pinned pieces
    Da = np.stack([orc.o_new_base(pr.Y64, ids, 3, 2, round_f32=False)[0] for ids in sets])
    _blk, _s, _c, err, _E = orc.o_code(pr.Y64, Da, 3)
    assert abs(orc.rmse(err.sum(), 16, 900) - hist[0]) < 1e-15
    Qn = orc.o_new_base(pr.Y64, orc.o_worst(err, 150), 3, 2, round_f32=False)[0]
    Db = np.concatenate([Da, Qn[None]])
    blk1 = orc.o_code(pr.Y64, Db, 3)[0]
    _D, (_s, _c, e1), _sq = orc.o_train_rounds(pr.Y64, blk1, Db, 3, 2, round_f32=False)
    assert abs(orc.rmse(e1.sum(), 16, 900) - hist[1]) < 1e-15


def test_hand_worked_2d_worst_set_and_base_initialisation():
    g = json.load(open(os.path.join(HERE, "golden", "hand_2d.json")))
    h = json.load(open(os.path.join(HERE, "golden", "hand_2d_next.json")))
    Y = np.array(g["Y"], float)
    D = np.array(g["Q"], float)
    err = orc.o_code(Y, D, 1)[3]
    assert np.allclose(err, h["err"], atol=1e-14)
    for W, ids in h["worst"].items():
        assert orc.o_worst(err, int(W)).tolist() == ids
    Q0, sv = orc.o_init_base(Y, h["init_set"])
    assert np.allclose(sv, h["singular_values"], rtol=1e-14)
    assert np.allclose(np.abs(Q0), h["Q0_abs_atoms"], atol=1e-14)
    assert abs(Q0[0, 0] / Q0[0, 1] - h["Q0_atom0_over_atom0_ratio"]) < 1e-12     # same sign inside the atom
