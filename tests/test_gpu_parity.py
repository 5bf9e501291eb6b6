"""GPU parity: the HIP path, called through the C-ABI, against the fp64 oracle on the
same seeded inputs.  Tolerances are the ones stated in tests/gpu_util.py."""
import numpy as np
import pytest

import sbo_synth as synth
from oracle import sbo_oracle as orc
from gpu_util import Sbo, compare_assigned_code, compare_code, compare_Q
import paper_1412_4944_amd as sbo

pytestmark = pytest.mark.gpu


def _problem(name, m=None, **kw):
    if name in synth.CONFIGS:
        return synth.generate(synth.CONFIGS[name], m=m)
    return synth.generate(synth.custom(name, m=m, **kw))


CODE_CASES = [
    ("tiny", dict()),
    ("patch8", dict(m=4096 + 77)),                       # several tiles + ragged tail
    ("headline", dict(m=3000)),
    ("p32", dict(p=32, K=6, m=1500, s0=4)),
    ("p32_oddK", dict(p=32, K=5, m=700, s0=16)),
    ("p16_oddK", dict(p=16, K=3, m=333, s0=2)),
    ("p16_full", dict(p=16, K=2, m=200, s0=16)),
    ("p16_s9", dict(p=16, K=4, m=257, s0=9)),
    ("p64_s1", dict(p=64, K=3, m=129, s0=1)),
    ("p64_s16", dict(p=64, K=4, m=640, s0=16)),
    ("p64_s5", dict(p=64, K=7, m=1000, s0=5)),
    ("K1", dict(p=64, K=1, m=100, s0=8)),
    ("m1", dict(p=64, K=4, m=1, s0=3)),
    ("p256", dict(p=256, K=3, m=333, s0=12, snr_db=25.0)),
    ("p256_s8", dict(p=256, K=2, m=150, s0=8, snr_db=25.0)),
    ("p256_s1", dict(p=256, K=2, m=70, s0=1, snr_db=25.0)),
]


ARITH = ["f32", "bf16x3", "screen", "f16x2"]     # the two ways the projection onto all K orthobases is multiplied out


@pytest.mark.parametrize("arith", ARITH)
@pytest.mark.parametrize("name,kw", CODE_CASES, ids=[c[0] for c in CODE_CASES])
def test_code_matches_oracle(name, kw, arith):
    pr = _problem(name, **kw)
    cfg = pr.cfg
    print(f"case {name} {arith}: p={cfg.p} K={cfg.K} m={pr.Y.shape[0]} s0={cfg.s0}", flush=True)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0], arith=arith) as g:
        for D in (pr.D_init, pr.D_planted):
            o = orc.o_code(pr.Y, D, cfg.s0)
            out = g.code(pr.Y, D)
            # s0 = p keeps everything: all blocks tie exactly, so every signal is exempt
            frac = compare_code(pr.Y, D, cfg.s0, o, out,
                                max_exempt_frac=1.0 if cfg.s0 == cfg.p else 0.01)
            print(f"  exempt fraction {frac:.5f}", flush=True)


@pytest.mark.parametrize("p", [16, 64, 256])
@pytest.mark.parametrize("arith", ARITH)
def test_code_ties_zero_signal_and_duplicates(arith, p):
    # identical blocks (block tie -> lowest index), equal magnitudes (atom tie -> lowest
    # index), an all-zero signal; every expected value follows from the tie rules alone
    K, s0 = 4, 3
    rng = np.random.default_rng(3)
    Q = synth.random_onb(rng, p).T.astype(np.float32)
    D = np.stack([np.eye(p, dtype=np.float32), Q, np.eye(p, dtype=np.float32), Q])
    Y = np.zeros((70, p), np.float32)
    Y[0, [2, 5, 7, 9]] = [1.0, -1.0, 1.0, 1.0]          # four equal magnitudes, keep 2,5,7
    Y[1] = 0.0
    Y[2, [0, p - 1]] = [3.0, -3.0]                       # fewer non-zeros than s0
    Y[3:] = rng.standard_normal((67, p)).astype(np.float32)
    Y[40] = Y[39]                                        # duplicate signals
    o = orc.o_code(Y, D, s0)
    with Sbo(p, K, s0, 70, arith=arith) as g:
        blk, supp, coef, err = g.code(Y, D)
    assert blk[0] == 0 and supp[0].tolist() == [2, 5, 7] and coef[0].tolist() == [1.0, -1.0, 1.0]
    assert err[0] == 1.0
    assert blk[1] == 0 and supp[1].tolist() == [0, 1, 2] and (coef[1] == 0).all() and err[1] == 0
    assert blk[2] == 0 and supp[2].tolist() == [0, 1, p - 1] and coef[2].tolist() == [3.0, 0.0, -3.0]
    assert (blk[40], supp[40].tolist(), coef[40].tolist()) == (blk[39], supp[39].tolist(), coef[39].tolist())
    assert (blk < 2).all()                               # blocks 2,3 duplicate 0,1: lowest index wins
    compare_code(Y, D, s0, o, (blk, supp, coef, err), max_exempt_frac=0.05)


@pytest.mark.parametrize("p,K,s0", [(64, 5, 8), (16, 3, 4), (256, 2, 12)])
@pytest.mark.parametrize("arith", ARITH)
def test_code_over_signal_scales_and_dynamic_range(arith, p, K, s0):
    """Coding does not depend on the scale of a signal (the fp16 arithmetic rescales every signal by
    a power of two, the others work on the values as they are): signals scaled by 1e-12 .. 1e12
    (squares stay inside the fp32 range), signals with one dimension 1e4 times the others, and a
    signal of a single non-zero entry."""
    rng = np.random.default_rng(91 + p)
    pr = _problem(f"scales_p{p}", p=p, K=K, m=700, s0=s0, snr_db=25.0)
    Y = pr.Y.copy()
    m = Y.shape[0]
    Y *= (10.0 ** rng.uniform(-12, 12, size=(m, 1))).astype(np.float32)
    Y[5::50, 3] *= 1e4
    Y[7] = 0.0
    Y[7, p - 2] = -2.5e-9
    D = pr.D_planted
    print(f"case {arith}: p={p} K={K} m={m} s0={s0}", flush=True)
    o = orc.o_code(Y, D, s0)
    with Sbo(p, K, s0, m, arith=arith) as g:
        out = g.code(Y, D)
    frac = compare_code(Y, D, s0, o, out, max_exempt_frac=0.01)
    print(f"  exempt fraction {frac:.5f}", flush=True)


@pytest.mark.parametrize("K,m", [(4, 1024), (32, 5000), (128, 70001), (1, 100), (1000, 3000), (7, 1)])
def test_group_matches_oracle(K, m):
    rng = np.random.default_rng(K * 1000 + m)
    w = (np.arange(K) + 1.0) ** -1.1
    blk = rng.choice(K, size=m, p=w / w.sum()).astype(np.int32)
    if K > 3:
        blk[blk == 2] = 1                                # an empty block
    print(f"case K={K} m={m}", flush=True)
    with Sbo(64, K, 4, m) as g:
        counts, offsets, perm = g.group(blk)
    oc, oo, op = orc.o_group(blk, K)
    np.testing.assert_array_equal(counts, oc)
    np.testing.assert_array_equal(offsets, oo)
    np.testing.assert_array_equal(perm, op)


UPDATE_CASES = [
    ("tiny", dict()),
    ("patch8", dict(m=4096 + 77)),
    ("headline", dict(m=20000)),
    ("p32", dict(p=32, K=6, m=3000, s0=4)),
    ("p16_oddK", dict(p=16, K=3, m=999, s0=2)),
    ("p256", dict(p=256, K=2, m=2500, s0=12, snr_db=25.0)),
]


@pytest.mark.parametrize("name,kw", UPDATE_CASES, ids=[c[0] for c in UPDATE_CASES])
def test_update_stages_match_oracle_teacher_forced(name, kw):
    pr = _problem(name, **kw)
    cfg = pr.cfg
    print(f"case {name}: p={cfg.p} K={cfg.K} m={pr.Y.shape[0]} s0={cfg.s0}", flush=True)
    blk, supp, coef, err, E = orc.o_code(pr.Y, pr.D_init, cfg.s0)
    coef32 = coef.astype(np.float32)
    Dn, M = orc.o_update(pr.Y, blk, supp, coef32, pr.D_init)
    counts = np.bincount(blk, minlength=cfg.K)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0]) as g:
        Mg = g.accumulate(pr.Y, blk, supp, coef32)
        Mg2 = g.accumulate(pr.Y, blk, supp, coef32)
        assert np.array_equal(Mg, Mg2), "accumulation not bitwise repeatable"
        for j in range(cfg.K):
            scale = np.abs(M[j]).max() + 1e-30
            assert np.abs(Mg[j] - M[j]).max() <= 2e-5 * scale * max(1.0, np.sqrt(counts[j] / 64.0)), \
                f"M[{j}] off by {np.abs(Mg[j] - M[j]).max() / scale} rel"
        Dp = g.polar(M.astype(np.float32), pr.D_init, counts.astype(np.int32))
        w1 = compare_Q(Dp, Dn, M, counts > 0)
        Dg, cg = g.update(pr.Y, blk, supp, coef32, pr.D_init)
        np.testing.assert_array_equal(cg, counts)
        w2 = compare_Q(Dg, Dn, M, counts > 0)
        Dg2, _ = g.update(pr.Y, blk, supp, coef32, pr.D_init)
        assert np.array_equal(Dg, Dg2), "update not bitwise repeatable"
        print(f"  worst |Q - Q_oracle|: polar {w1:.2e}, update {w2:.2e}", flush=True)


def test_polar_rank_deficient_and_empty_blocks():
    p, K = 64, 5
    rng = np.random.default_rng(17)
    M = rng.standard_normal((K, p, p))
    M[1][:, :] = 0.0
    M[1][:5] = rng.standard_normal((5, p))               # rank 5: most atoms never used
    M[2][7] = 0.0                                        # one unused atom
    M[3] = 0.0                                           # all-zero but counted as non-empty
    u, s, vt = np.linalg.svd(M[4])
    M[4] = (u * np.geomspace(1, 1e-6, p)) @ vt           # ill-conditioned but full rank
    D_old = synth.random_dictionary(rng, K, p).astype(np.float32)
    counts = np.array([10, 10, 10, 10, 10], np.int32)
    counts0 = counts.copy()
    counts0[0] = 0
    with Sbo(p, K, 4, 16) as g:
        Dg = g.polar(M.astype(np.float32), D_old, counts0)
        np.testing.assert_array_equal(Dg[0], D_old[0])   # empty block keeps its basis
        Dg = g.polar(M.astype(np.float32), D_old, None)
    M32 = M.astype(np.float32).astype(np.float64)
    Dn = np.stack([orc.o_polar(M32[j]) for j in range(K)])
    compare_Q(Dg, Dn, M32, np.ones(K, bool))


@pytest.mark.parametrize("name,kw,iters", [("tiny", dict(), 5), ("patch8", dict(m=8192), 6),
                                           ("p32", dict(p=32, K=6, m=3000, s0=4), 4),
                                           ("p256", dict(p=256, K=2, m=2500, s0=12, snr_db=25.0), 3)])
@pytest.mark.parametrize("arith", ARITH)
def test_iterate_free_running(name, kw, iters, arith):
    pr = _problem(name, **kw)
    cfg = pr.cfg
    print(f"case {name} {arith}: p={cfg.p} K={cfg.K} m={pr.Y.shape[0]} s0={cfg.s0}", flush=True)
    Do, last, sq_o = orc.o_iterate(pr.Y, pr.D_init, cfg.s0, iters)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0], arith=arith) as g:
        Dg, blk, supp, coef, err, sq = g.iterate(pr.Y, pr.D_init, iters)
        Dg2, *_rest, sq2 = g.iterate(pr.Y, pr.D_init, iters)
    assert np.array_equal(Dg, Dg2) and np.array_equal(sq, sq2), "iteration not bitwise repeatable"
    print("  oracle sqerr", sq_o, "\n  gpu    sqerr", sq, flush=True)
    assert (np.diff(sq) <= 1e-6 * sq[0]).all(), "error increased"
    np.testing.assert_allclose(sq, sq_o, rtol=1e-3)
    assert abs(sq[-1] - err.astype(np.float64).sum()) <= 1e-6 * sq[-1] + 1e-12
    for j in range(cfg.K):
        Q = Dg[j].astype(np.float64)
        assert np.abs(Q @ Q.T - np.eye(cfg.p)).max() <= 1e-5


@pytest.mark.parametrize("name,kw", [("tiny", dict()), ("patch8", dict(m=5000)), ("p32", dict(p=32, K=6, m=3000, s0=4)),
                                     ("p64_s5", dict(p=64, K=7, m=2100, s0=5)),
                                     ("p256", dict(p=256, K=2, m=1500, s0=12, snr_db=25.0))])
@pytest.mark.parametrize("arith", ARITH)
def test_iterate_one_step_matches_oracle(name, kw, arith):
    """sbo_iterate(1) (which fuses select and accumulate for p <= 64) against the oracle:
    the coding outputs element by element, the updated dictionary teacher-forced."""
    pr = _problem(name, **kw)
    cfg = pr.cfg
    print(f"case {name} {arith}: p={cfg.p} K={cfg.K} m={pr.Y.shape[0]} s0={cfg.s0}", flush=True)
    o = orc.o_code(pr.Y, pr.D_init, cfg.s0)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0], arith=arith) as g:
        Dg, blk, supp, coef, err, sq = g.iterate(pr.Y, pr.D_init, 1)
        frac = compare_code(pr.Y, pr.D_init, cfg.s0, o, (blk, supp, coef, err))
        # the update the GPU made from ITS code, against the oracle's update from the same code
        Dn, M = orc.o_update(pr.Y, blk, supp, coef, pr.D_init)
        w = compare_Q(Dg, Dn, M, np.bincount(blk, minlength=cfg.K) > 0)
        b2, s2, c2, e2 = g.code(pr.Y, pr.D_init)
    assert np.array_equal(blk, b2) and np.array_equal(supp, s2)
    np.testing.assert_allclose(coef, c2, rtol=0, atol=1e-6 * np.abs(c2).max())
    assert abs(sq[0] - err.astype(np.float64).sum()) <= 1e-6 * sq[0] + 1e-12
    print(f"  exempt {frac:.5f}, worst dQ {w:.2e}", flush=True)


@pytest.mark.parametrize("name,kw,R", [("tiny", dict(), 4), ("patch8", dict(m=6000), 3),
                                       ("p256", dict(p=256, K=2, m=1500, s0=12, snr_db=25.0), 2)])
def test_train_rounds_frozen_assignment(name, kw, R):
    """R rounds of 1ONB per block with the assignment frozen.  Every round is compared with
    the oracle teacher-forced (the GPU starts the round from the oracle's dictionary, so a
    near-tie support flip cannot compound); the R-round call is then compared with the
    chain of single-round calls."""
    pr = _problem(name, **kw)
    cfg = pr.cfg
    m = pr.Y.shape[0]
    print(f"case {name}: p={cfg.p} K={cfg.K} m={m} s0={cfg.s0} R={R}", flush=True)
    blk = orc.o_code(pr.Y, pr.D_init, cfg.s0)[0]
    counts = np.bincount(blk, minlength=cfg.K)
    D = pr.D_init.astype(np.float64)
    with Sbo(cfg.p, cfg.K, cfg.s0, m) as g:
        chain = pr.D_init
        for r in range(R):
            D32 = D.astype(np.float32)
            # oracle round from D32: SELECT in the assigned block, then the update
            so, co, eo = orc.o_train_rounds(pr.Y, blk, D32, cfg.s0, 1)[1]
            Dg, sg, cg, eg = g.train_rounds(pr.Y, blk, D32, 1)
            # supports bit-exact except below the near-tie gap, exempt codes valid in fp64
            frac = compare_assigned_code(pr.Y, D32, blk, cfg.s0, (so, co, eo), (sg, cg, eg))
            Dn, M = orc.o_update(pr.Y, blk, sg, cg, D32)       # from the GPU's own code
            w = compare_Q(Dg, Dn, M, counts > 0)
            print(f"  round {r}: exempt fraction {frac:.5f}, worst dQ {w:.2e}, sqerr {eg.astype(np.float64).sum():.6f}",
                  flush=True)
            D = orc.o_train_rounds(pr.Y, blk, D32, cfg.s0, 1)[0]
            chain, s_ch, c_ch, e_ch = g.train_rounds(pr.Y, blk, chain, 1)
        DR, sR, cR, eR = g.train_rounds(pr.Y, blk, pr.D_init, R)
        DR2, *_ = g.train_rounds(pr.Y, blk, pr.D_init, R)
        D1, s1, c1, e1 = g.train_rounds(pr.Y, blk, pr.D_init, 1)
    assert np.array_equal(DR, DR2), "rounds not bitwise repeatable"
    # one call with R rounds = R calls with one round, bit for bit
    assert np.array_equal(DR, chain) and np.array_equal(sR, s_ch)
    assert np.array_equal(cR, c_ch) and np.array_equal(eR, e_ch)
    assert eR.astype(np.float64).sum() <= e1.astype(np.float64).sum() * (1 + 1e-6), "error increased over rounds"
    for j in range(cfg.K):
        Q = DR[j].astype(np.float64)
        assert np.abs(Q @ Q.T - np.eye(cfg.p)).max() <= 1e-5


def test_teacher_forced_iterations_patch8():
    """Each iteration: the GPU codes with the oracle's dictionary (rounded to fp32) and
    updates from the oracle's code, so chaotic block flips do not compound."""
    pr = _problem("patch8", m=4096)
    cfg = pr.cfg
    D = pr.D_init.astype(np.float64)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0]) as g:
        for it in range(4):
            D32 = D.astype(np.float32)
            o = orc.o_code(pr.Y, D32, cfg.s0)
            frac = compare_code(pr.Y, D32, cfg.s0, o, g.code(pr.Y, D32))
            blk, supp, coef, err, E = o
            coef32 = coef.astype(np.float32)
            Dn, M = orc.o_update(pr.Y, blk, supp, coef32, D32)
            Dg, _ = g.update(pr.Y, blk, supp, coef32, D32)
            w = compare_Q(Dg, Dn, M, np.bincount(blk, minlength=cfg.K) > 0)
            print(f"  iter {it}: exempt {frac:.5f}, worst dQ {w:.2e}", flush=True)
            D = Dn


def test_errors_are_reported_not_faulted():
    import paper_1412_4944_amd as sbo
    import torch
    with Sbo(64, 4, 3, 128) as g:
        Y = g.dev_f32(np.zeros((256, 64)))
        D = g.dev_f32(np.zeros((4, 64, 64)))
        blk, supp, coef, err = g.outputs(256)
        with pytest.raises(sbo.SboError) as e:
            sbo.sbo_code(g.ctx, Y, D, blk, supp, coef, err)      # m > m_max
        assert e.value.code == sbo.binding.SBO_EINVAL
        # out-of-range block ids are dropped by grouping, not dereferenced
        b = np.array([0, 1, 99, -5, 3] + [2] * 100, np.int32)
        counts, offsets, perm = g.group(b)
        assert counts.tolist() == [1, 1, 100, 1] and offsets[-1] == 103
        torch.cuda.synchronize()


@pytest.mark.parametrize("arith", ARITH)
def test_largest_K_and_context_reuse(arith):
    """K = 1024 orthobases (the largest the boundary accepts), most of them empty after
    coding; and one context (sized for m_max) used for calls with smaller and changing m."""
    pr = synth.generate(synth.custom("bigK", p=16, K=1024, m=3000, s0=2, snr_db=20.0))
    cfg = pr.cfg
    with Sbo(16, 1024, 2, 4000, arith=arith) as g:        # m_max > every m used below
        for m in (3000, 777, 2500):
            Y = pr.Y[:m]
            o = orc.o_code(Y, pr.D_init, 2)
            out = g.code(Y, pr.D_init)
            compare_code(Y, pr.D_init, 2, o, out)
            blk, supp, coef, _err = out
            Dg, counts = g.update(Y, blk, supp, coef, pr.D_init)
            assert np.array_equal(counts, np.bincount(blk, minlength=1024))
            Dn, M = orc.o_update(Y, blk, supp, coef, pr.D_init)
            compare_Q(Dg, Dn, M, counts > 0)
            assert np.array_equal(Dg[counts == 0], pr.D_init[counts == 0]), "an empty block changed"
        # iterate in the same context, then code again: the fused path must leave the
        # workspace invariants intact for the call after it
        Y = pr.Y[:1500]
        Dg, blk, supp, coef, err, sq = g.iterate(Y, pr.D_init, 2)
        assert sq[1] <= sq[0] * (1 + 1e-6)
        compare_code(Y, Dg, 2, orc.o_code(Y, Dg, 2), g.code(Y, Dg))


@pytest.mark.parametrize("p", [16, 32, 64, 256])
def test_polar_condition_sweep_and_both_paths(p):
    """The SVD update over a range of condition numbers, once with the default path
    (Newton-Schulz, Jacobi for the blocks it flags) and once with the Jacobi SVD alone: each
    against the oracle, and the two against each other.  The last block is a symmetric positive
    definite matrix (polar factor = I) whose dominant eigenvectors are orthogonal to the vector of
    absolute row sums of its Gram matrix: a scale estimated by power iteration from that vector
    alone would be too small by a factor of 3.7 and send the dominant singular values to -1."""
    rng = np.random.default_rng(23 + p)
    conds = [1.0, 3.0, 30.0, 300.0, 900.0, 3e3, 3e4, 1e6, np.inf]
    K = len(conds) + 1
    M = np.empty((K, p, p))
    for j, c in enumerate(conds):
        u = synth.random_onb(rng, p)
        v = synth.random_onb(rng, p)
        s = np.geomspace(1.0, 1.0 / c, p) if np.isfinite(c) else np.r_[np.geomspace(1.0, 0.1, p - 3), 0, 0, 0]
        M[j] = (u * s) @ v.T * (10.0 ** rng.uniform(-3, 3))          # any overall scale
    # sqrt of kron(I, [[1, -0.6], [-0.6, 1]]): eigenvalues sqrt(1.6) on (1, -1)/sqrt2, sqrt(0.4) on (1, 1)/sqrt2
    a, b = (np.sqrt(1.6) + np.sqrt(0.4)) / 2, (np.sqrt(0.4) - np.sqrt(1.6)) / 2
    M[K - 1] = np.kron(np.eye(p // 2), np.array([[a, b], [b, a]]))
    M32 = M.astype(np.float32)
    D_old = synth.random_dictionary(rng, K, p).astype(np.float32)
    Dn = np.stack([orc.o_polar(M32[j].astype(np.float64)) for j in range(K)])
    assert np.abs(Dn[K - 1] - np.eye(p)).max() < 1e-6                # oracle agrees: polar factor = I
    out = {}
    with Sbo(p, K, min(4, p), 256) as g:
        for mode in ("default", "jacobi"):
            g.svd_jacobi(mode == "jacobi")
            out[mode] = g.polar(M32, D_old, None)
            sweeps = sbo.sbo_svd_sweeps(g.ctx, K)
            w = compare_Q(out[mode], Dn, M32.astype(np.float64), np.ones(K, bool))
            print(f"  p={p} {mode}: worst |Q - Q_oracle| {w:.2e}, per block {sweeps}", flush=True)
            if mode == "default":
                assert all(x < 0 for x in sweeps[:4]), "well-conditioned blocks should not need the fallback"
                assert sweeps[len(conds) - 1] > 0, "the rank-deficient block must go to the Jacobi SVD"
                assert sweeps[K - 1] < 0, "the symmetric block is well conditioned: Newton-Schulz"
            else:
                assert all(x > 0 for x in sweeps)
    good = [j for j, c in enumerate(conds) if c <= 900.0] + [K - 1]
    assert np.abs(out["default"][good] - out["jacobi"][good]).max() <= 1e-4


JACOBI_CASES = [("tiny", dict(), 12), ("patch8", dict(m=4096 + 77), 10),
                ("p256", dict(p=256, K=2, m=1300, s0=12, snr_db=25.0), 2)]


@pytest.mark.parametrize("name,kw,iters", JACOBI_CASES, ids=[c[0] for c in JACOBI_CASES])
def test_jacobi_only_inside_iterate_and_rounds(name, kw, iters):
    """SBO_SVD_JACOBI (the one-sided Jacobi SVD for every orthobase) inside sbo_iterate and
    sbo_train_rounds: every iteration teacher-forced against the oracle's update, then a
    free-running sbo_iterate over all iterations against the oracle's error curve."""
    pr = _problem(name, **kw)
    cfg = pr.cfg
    m = pr.Y.shape[0]
    print(f"case {name}: p={cfg.p} K={cfg.K} m={m} s0={cfg.s0} iters={iters}", flush=True)
    D = pr.D_init.astype(np.float64)
    with Sbo(cfg.p, cfg.K, cfg.s0, m, jacobi_only=True) as g:
        for it in range(min(iters, 4)):
            D32 = D.astype(np.float32)
            o = orc.o_code(pr.Y, D32, cfg.s0)
            Dg, blk, supp, coef, err, sq = g.iterate(pr.Y, D32, 1)
            assert all(x >= 0 for x in sbo.sbo_svd_sweeps(g.ctx, cfg.K)), "Newton-Schulz ran"
            frac = compare_code(pr.Y, D32, cfg.s0, o, (blk, supp, coef, err))
            counts = np.bincount(blk, minlength=cfg.K)
            Dn, M = orc.o_update(pr.Y, blk, supp, coef, D32)   # the oracle's update from the GPU's code
            w = compare_Q(Dg, Dn, M, counts > 0)
            # the same update through the frozen-assignment rounds
            Dr, sr, cr, er = g.train_rounds(pr.Y, blk, D32, 1)
            assert np.array_equal(sr, supp)
            w2 = compare_Q(Dr, Dn, M, counts > 0)
            print(f"  iter {it}: exempt {frac:.5f}, worst dQ iterate {w:.2e} rounds {w2:.2e}", flush=True)
            D = orc.o_update(pr.Y, o[0], o[1], o[2], D32)[0]
        Dg, blk, supp, coef, err, sq = g.iterate(pr.Y, pr.D_init, iters)
        Dg2, *_r, sq2 = g.iterate(pr.Y, pr.D_init, iters)
        assert np.array_equal(Dg, Dg2) and np.array_equal(sq, sq2), "not bitwise repeatable"
        # R rounds in one call against the chain of single rounds (frozen assignment)
        b0 = orc.o_code(pr.Y, pr.D_init, cfg.s0)[0]
        DR, *_x = g.train_rounds(pr.Y, b0, pr.D_init, 3)
        chain = pr.D_init
        for _ in range(3):
            chain, *_x = g.train_rounds(pr.Y, b0, chain, 1)
        assert np.array_equal(DR, chain)
    sq_o = orc.o_iterate(pr.Y, pr.D_init, cfg.s0, iters)[2]
    print("  oracle sqerr", sq_o, "\n  gpu    sqerr", sq, flush=True)
    assert (np.diff(sq) <= 1e-6 * sq[0]).all(), "error increased"
    np.testing.assert_allclose(sq, sq_o, rtol=1e-3)
    for j in range(cfg.K):
        Q = Dg[j].astype(np.float64)
        assert np.abs(Q @ Q.T - np.eye(cfg.p)).max() <= 1e-5


@pytest.mark.parametrize("arith", ARITH)
@pytest.mark.parametrize("jacobi_only", [False, True], ids=["auto", "jacobi"])
def test_iterate_with_rank_deficient_blocks(jacobi_only, arith):
    """Skewed assignment with more orthobases than the data supports: the rare orthobases get
    fewer than p signals, so their P_j are rank-deficient.  Inside sbo_iterate these go to the
    Jacobi SVD (flagged by Newton-Schulz in the default mode), which completes the basis and
    also writes the dictionary copy the next coding pass reads.  Checked: the updated
    dictionary (polar-factor properties on every orthobase, values where P_j is well
    conditioned) and the NEXT coding pass, element by element against the oracle."""
    pr = synth.generate(synth.custom("rankdef", p=64, K=24, m=3000, s0=4, snr_db=20.0, zipf_s=1.3))
    cfg = pr.cfg
    D0 = pr.D_planted                  # signals go to their planted orthobase: skewed counts
    o = orc.o_code(pr.Y, D0, cfg.s0)
    with Sbo(cfg.p, cfg.K, cfg.s0, pr.Y.shape[0], jacobi_only=jacobi_only, arith=arith) as g:
        D1, blk, supp, coef, err, sq = g.iterate(pr.Y, D0, 1)
        sweeps = sbo.sbo_svd_sweeps(g.ctx, cfg.K)
        compare_code(pr.Y, D0, cfg.s0, o, (blk, supp, coef, err))
        counts = np.bincount(blk, minlength=cfg.K)
        small = (counts > 0) & (counts < cfg.p)
        print(f"  counts {counts.tolist()}\n  svd work {sweeps}", flush=True)
        assert small.sum() >= 3 and (counts >= 2 * cfg.p).sum() >= 3, "the case needs small and large blocks"
        for j in np.nonzero(small)[0]:
            assert sweeps[j] > 0, f"rank-deficient block {j} did not go to the Jacobi SVD"
        if not jacobi_only:
            assert any(x < 0 for x in sweeps), "Newton-Schulz handled no block"
        Dn, M = orc.o_update(pr.Y, blk, supp, coef, D0)
        w = compare_Q(D1, Dn, M, counts > 0)
        assert np.array_equal(D1[counts == 0], D0[counts == 0])
        # two iterations in one call: the codes it leaves are those of pass 2, i.e. with D1
        D2, b2, s2, c2, e2, sq2 = g.iterate(pr.Y, D0, 2)
        assert sq2[0] == sq[0] and sq2[1] <= sq2[0] * (1 + 1e-6)
        frac = compare_code(pr.Y, D1, cfg.s0, orc.o_code(pr.Y, D1, cfg.s0), (b2, s2, c2, e2))
        print(f"  worst dQ {w:.2e}; next coding pass: exempt {frac:.5f}", flush=True)
        c2n = np.bincount(b2, minlength=cfg.K)
        Dn2, M2 = orc.o_update(pr.Y, b2, s2, c2, D1)
        compare_Q(D2, Dn2, M2, c2n > 0)
