"""CPU oracle for one Single Block Orthogonal (SBO) dictionary-learning iteration.

TEST INFRASTRUCTURE ONLY.  Plain, slow, fp64 numpy written from the paper's
definitions; it shares no code with the HIP path, and the product never calls
it.  Every stage of the iteration is exact (no approximation), so each function
is the plain definition written out; library routines used as steps: matmul,
stable argsort, bincount, LAPACK SVD.

Layouts (same as the GPU boundary, cast to fp64 on entry)
  Y : (m, p)     signal-major, row i = y_i
  D : (K, p, p)  atom-major, D[j, k, :] = atom k of Q_j, i.e. D[j] = Q_j^T

Pins (tests/test_oracle_pins.py): Parseval, brute-force best s0-term fit,
closed-form error, brute-force block argmax, planted recovery, hand-worked 2-D
example, grouping invariants, dense Y_j X_j^T identity, scipy polar factor,
nuclear-norm maximality, Procrustes decrease, fixed point, monotone iteration and
monotone frozen-assignment rounds; worst-W set against its defining inequalities;
base initialisation against the eigen-decomposition of the Gram matrix, a rank-one
case, a hand-worked diagonal case and a planted factorisation; new-base training
against monotone error and the planted fixed point; the whole of Algorithm 2 against
its stopping conditions, a monotone RMSE history and a step-by-step recomposition.
No function here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np


def o_code(Y, D, s0, chunk=8192):
    """Single-block sparse coding of every signal (Section 2, eq. (4); Section 3.1).

    For signal y and every block j: c = Q_j^T y; keep the s0 entries of largest
    magnitude (ties: lower atom index first); E_j = sum of the kept c^2; the
    block with the largest E_j wins (ties: lowest j).  Returns
      blk  (m,)    int32   winning block
      supp (m,s0)  int32   kept atom indices inside that block, ascending
      coef (m,s0)  float64 kept coefficients, paired with supp
      err  (m,)    float64 ||y - Q_blk x||^2 evaluated directly
      E    (m,K)   float64 kept energy for every block (for tie gating in tests)
    """
    Y = np.asarray(Y, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64)
    m, p = Y.shape
    K = D.shape[0]
    assert D.shape == (K, p, p) and 1 <= s0 <= p
    blk = np.empty(m, np.int32)
    supp = np.empty((m, s0), np.int32)
    coef = np.empty((m, s0), np.float64)
    err = np.empty(m, np.float64)
    E = np.empty((m, K), np.float64)
    A = D.reshape(K * p, p)                      # row (j*p + k) = atom k of Q_j
    for a in range(0, m, chunk):
        b = min(m, a + chunk)
        y = Y[a:b]
        n = b - a
        C = (y @ A.T).reshape(n, K, p)           # C[i, j, k] = <atom k of Q_j, y_i>
        order = np.argsort(-np.abs(C), axis=2, kind="stable")[:, :, :s0]
        kept = np.take_along_axis(C, order, axis=2)
        En = (kept ** 2).sum(axis=2)
        j = np.argmax(En, axis=1)                # first maximum = lowest block index
        rows = np.arange(n)
        S = np.sort(order[rows, j], axis=1)
        x = C[rows[:, None], j[:, None], S]
        atoms = D[j[:, None], S]                 # (n, s0, p)
        resid = y - np.einsum("nt,ntd->nd", x, atoms)
        blk[a:b] = j
        supp[a:b] = S
        coef[a:b] = x
        err[a:b] = (resid ** 2).sum(axis=1)
        E[a:b] = En
    return blk, supp, coef, err, E


def o_group(blk, K):
    """Bucket the signals by chosen block (Section 3.3, grouping before training):
    counts per block, exclusive offsets, and the stable permutation that lists
    signal ids block by block in original order."""
    blk = np.asarray(blk)
    counts = np.bincount(blk, minlength=K).astype(np.int32)
    offsets = np.zeros(K + 1, np.int64)
    offsets[1:] = np.cumsum(counts)
    perm = np.argsort(blk, kind="stable").astype(np.int32)
    return counts, offsets.astype(np.int32), perm


def o_accumulate(Y, blk, supp, coef, K):
    """P = Y_j X_j^T for every block (Algorithm 1, step 5), atom-major:
    M[j, k, :] = column k of Y_j X_j^T = sum over the block's signals of x_i[k] * y_i."""
    Y = np.asarray(Y, dtype=np.float64)
    m, p = Y.shape
    M = np.zeros((K, p, p), np.float64)
    for j in range(K):
        ids = np.nonzero(np.asarray(blk) == j)[0]
        if ids.size == 0:
            continue
        X = np.zeros((p, ids.size), np.float64)
        X[np.asarray(supp)[ids], np.arange(ids.size)[:, None]] = np.asarray(coef, np.float64)[ids]
        P = Y[ids].T @ X.T                       # (p, p) = Y_j X_j^T
        M[j] = P.T
    return M


def o_polar(M_am):
    """Q = U V^T from the SVD of one p x p matrix P (Algorithm 1, steps 6-7).
    Input and output atom-major (the transpose of P, resp. of Q)."""
    P = np.asarray(M_am, dtype=np.float64).T
    U, _, Vt = np.linalg.svd(P)
    return (U @ Vt).T


def o_update(Y, blk, supp, coef, D):
    """Train every orthobase over its own signals with one round (Algorithm 2,
    step 5 with R = 1): Q_j <- U V^T of SVD(Y_j X_j^T).  A block that no signal
    chose keeps its basis.  Returns the new D (fp64, atom-major) and M."""
    D = np.asarray(D, dtype=np.float64)
    K = D.shape[0]
    M = o_accumulate(Y, blk, supp, coef, K)
    counts = np.bincount(np.asarray(blk), minlength=K)
    Dn = D.copy()
    for j in range(K):
        if counts[j] > 0:
            Dn[j] = o_polar(M[j])
    return Dn, M


def o_train_rounds(Y, blk, D, s0, R, round_f32=True):
    """R rounds of single-orthobase training with the block assignment frozen (Algorithm 1
    run for R rounds on every block over its own signals; Algorithm 2, step 5): per block
    and round, X = SELECT(Q^T Y_j, s0), P = Y_j X^T, Q = U V^T.  Returns the final D, the
    codes of the last round and the total squared error of every round's code."""
    Y = np.asarray(Y, dtype=np.float64)
    D = np.asarray(D, dtype=np.float64).copy()
    blk = np.asarray(blk)
    m, p = Y.shape
    K = D.shape[0]
    supp = np.zeros((m, s0), np.int32)
    coef = np.zeros((m, s0), np.float64)
    err = np.zeros(m, np.float64)
    sq = []
    for _ in range(R):
        for j in range(K):
            ids = np.nonzero(blk == j)[0]
            if ids.size == 0:
                continue
            _b, S, x, e, _E = o_code(Y[ids], D[j:j + 1], s0)   # one block: plain SELECT
            supp[ids], coef[ids], err[ids] = S, x, e
        sq.append(err.sum())
        D, _M = o_update(Y, blk, supp, coef, D)
        if round_f32:
            D = D.astype(np.float32).astype(np.float64)
    return D, (supp, coef, err), np.array(sq)


def o_iterate(Y, D, s0, n_iter, round_f32=True):
    """n_iter x (coding; update).  Returns the final D, the outputs of the last
    coding pass, and the total squared error of every coding pass.  With
    round_f32 the dictionary is rounded to float32 after each update, as the
    GPU boundary stores it."""
    D = np.asarray(D, dtype=np.float64)
    sq = []
    last = None
    for _ in range(n_iter):
        blk, supp, coef, err, _E = o_code(Y, D, s0)
        sq.append(err.sum())
        D, _M = o_update(Y, blk, supp, coef, D)
        if round_f32:
            D = D.astype(np.float32).astype(np.float64)
        last = (blk, supp, coef, err)
    return D, last, np.array(sq)


def o_worst(err, W):
    """The W worst represented signals (Algorithm 2, step 3): the W largest squared
    residuals; among equal residuals the lower signal index is taken first.  Returns the
    chosen signal ids in ascending order."""
    err = np.asarray(err, dtype=np.float64)
    assert 0 <= W <= err.size
    order = np.argsort(-err, kind="stable")      # descending error, ties by index
    return np.sort(order[:W]).astype(np.int32)


def o_init_base(Y, ids):
    """Starting orthobase for a set of signals (eq. (5)): Y_sub = U S V^T, Q_0 = U.
    Returns (Q0, sv): Q0 atom-major (row k = left singular vector k, singular values in
    descending order; the sign of a row is not determined) and the p singular values
    (zeros appended when the set has fewer than p signals)."""
    Y = np.asarray(Y, dtype=np.float64)
    sub = Y[np.asarray(ids, dtype=np.int64)].T       # p x n
    U, sv, _ = np.linalg.svd(sub, full_matrices=True)
    p = sub.shape[0]
    full = np.zeros(p)
    full[:sv.size] = sv
    return U.T.copy(), full


def o_new_base(Y, ids, s0, R, Q0=None, round_f32=True):
    """A new orthobase trained on a set of signals (Algorithm 2, steps 1 and 3): start
    from eq. (5) unless Q0 is given, then R rounds of Algorithm 1 on those signals.
    Returns (Q, sq): Q atom-major and the total squared error of every round's code."""
    Y = np.asarray(Y, dtype=np.float64)
    ids = np.asarray(ids, dtype=np.int64)
    if Q0 is None:
        Q0, _ = o_init_base(Y, ids)
        if round_f32:
            Q0 = Q0.astype(np.float32).astype(np.float64)
    sub = Y[ids]
    D, _codes, sq = o_train_rounds(sub, np.zeros(ids.size, np.int32), Q0[None], s0, R,
                                   round_f32=round_f32)
    return D[0], sq


def o_learn(Y, s0, init_sets, R, W, K_max, target_rmse=0.0, round_f32=True):
    """Algorithm 2 as a whole.  init_sets: K0 index arrays, the randomly chosen signals each
    initial orthobase is trained on (the random draw is the caller's).  Steps: train the K0
    initial orthobases (eq. (5) start + R rounds each); represent every signal; then, while
    fewer than K_max orthobases exist and the RMSE is above target_rmse: train a new
    orthobase on the W worst represented signals and append it; represent every signal;
    train every orthobase over its own signals for R rounds; evaluate the stopping rule.
    The error used by the stopping rule and by the next worst-W set is that of the codes of
    the last training round (taken before that round's update, which can only lower it).
    Returns (D, blk, rmse_history): rmse_history[0] after the initial representation, then
    one entry per iteration."""
    Y = np.asarray(Y, dtype=np.float64)
    m, p = Y.shape
    cast = (lambda a: a.astype(np.float32).astype(np.float64)) if round_f32 else (lambda a: a)
    D = np.stack([cast(o_new_base(Y, ids, s0, R, round_f32=round_f32)[0]) for ids in init_sets])
    blk, _supp, _coef, err, _E = o_code(Y, D, s0)
    hist = [rmse(err.sum(), p, m)]
    while D.shape[0] < K_max and hist[-1] > target_rmse:
        ids = o_worst(err.astype(np.float32) if round_f32 else err, W)
        Qn = cast(o_new_base(Y, ids, s0, R, round_f32=round_f32)[0])
        D = np.concatenate([D, Qn[None]], axis=0)
        blk = o_code(Y, D, s0)[0]
        D, (_supp, _coef, err), _sq = o_train_rounds(Y, blk, D, s0, R, round_f32=round_f32)
        hist.append(rmse(err.sum(), p, m))
    return D, blk, np.array(hist)


def rmse(sqerr_total, p, m):
    """RMSE = ||Y - DX||_F / sqrt(p m) (Section 4)."""
    return float(np.sqrt(sqerr_total / (p * m)))
