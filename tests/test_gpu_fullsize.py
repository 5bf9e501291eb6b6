"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  Coding is checked on every signal at the headline and
8x8-patch sizes and on a sample of at least a tenth of the signals at the two largest
sizes (the oracle codes each signal independently of the others); grouping, accumulation
and the SVD update are checked in full against the oracle."""
import numpy as np
import pytest

import sbo_synth as synth
from oracle import sbo_oracle as orc
from gpu_util import Sbo, compare_assigned_code, compare_code, compare_Q

pytestmark = pytest.mark.gpu


# The oracle's results do not depend on how the GPU multiplies: computed once per workload and
# shared by the parametrized cases below.
import functools


@functools.lru_cache(maxsize=2)
def _problem_of(name):
    return synth.generate(synth.CONFIGS[name])


@functools.lru_cache(maxsize=4)
def _oracle_code_of(name, n_sample):
    pr = _problem_of(name)
    cfg = pr.cfg
    ids = _sample_ids(pr.Y.shape[0], n_sample, cfg.number)
    return ids, orc.o_code(pr.Y[ids], pr.D_init, cfg.s0)


@functools.lru_cache(maxsize=4)
def _oracle_curve_of(name):
    pr = _problem_of(name)
    return orc.o_iterate(pr.Y, pr.D_init, pr.cfg.s0, pr.cfg.iters)[2]


def _sample_ids(m, n, seed):
    if n >= m:
        return np.arange(m)
    rng = np.random.default_rng(seed)
    edge = np.array([0, 1, 31, 32, 63, 64, 127, 128, 255, 256, m - 257, m - 129, m - 65, m - 33, m - 2, m - 1])
    ids = np.unique(np.concatenate([edge[(edge >= 0) & (edge < m)], rng.choice(m, size=n, replace=False)]))
    return ids


@pytest.mark.parametrize("name,n_sample,arith", [("headline", 262144, "f32"), ("headline", 262144, "bf16x3"),
                                                 ("headline", 262144, "screen"), ("skew", 110000, "screen"),
                                                 ("headline", 262144, "f16x2"), ("skew", 110000, "f16x2"),
                                                 ("skew", 110000, "f32"), ("skew", 110000, "bf16x3"),
                                                 ("patch16", 14000, "f32"), ("patch16", 14000, "bf16x3"),
                                                 ("patch16", 14000, "f16x2")])
def test_full_size_iteration_against_oracle(name, n_sample, arith):
    cfg = synth.CONFIGS[name]
    print(f"case {name} {arith}: p={cfg.p} K={cfg.K} m={cfg.m} s0={cfg.s0}: generating", flush=True)
    pr = _problem_of(name)
    m = pr.Y.shape[0]
    ids, o = _oracle_code_of(name, n_sample)
    with Sbo(cfg.p, cfg.K, cfg.s0, m, arith=arith) as g:
        print("  coding on the GPU", flush=True)
        blk, supp, coef, err = g.code(pr.Y, pr.D_init)
        frac = compare_code(pr.Y[ids], pr.D_init, cfg.s0, o, (blk[ids], supp[ids], coef[ids], err[ids]))
        print(f"  coding parity on {len(ids)} of {m} signals, exempt fraction {frac:.5f}", flush=True)
        # properties that hold at any size
        assert blk.min() >= 0 and blk.max() < cfg.K
        assert (np.diff(supp, axis=1) > 0).all() and supp.min() >= 0 and supp.max() < cfg.p
        n2 = (pr.Y.astype(np.float64) ** 2).sum(1)
        kept = (coef.astype(np.float64) ** 2).sum(1)
        assert (np.abs(n2 - kept - err) <= 1e-4 * n2 + 1e-30).all()      # Parseval in the chosen orthobase
        assert (err >= 0).all()

        print("  grouping", flush=True)
        counts, offsets, perm = g.group(blk)
        oc, oo, op = orc.o_group(blk, cfg.K)
        np.testing.assert_array_equal(counts, oc)
        np.testing.assert_array_equal(offsets, oo)
        np.testing.assert_array_equal(perm, op)

        print("  accumulation and update (oracle on all signals)", flush=True)
        Dn, M = orc.o_update(pr.Y, blk, supp, coef, pr.D_init)
        Mg = g.accumulate(pr.Y, blk, supp, coef)
        for j in range(cfg.K):
            scale = np.abs(M[j]).max() + 1e-30
            tol = 2e-5 * scale * max(1.0, np.sqrt(counts[j] / 64.0))
            assert np.abs(Mg[j] - M[j]).max() <= tol, f"M[{j}]: {np.abs(Mg[j] - M[j]).max() / scale:.2e} rel"
        Dg, cg = g.update(pr.Y, blk, supp, coef, pr.D_init)
        np.testing.assert_array_equal(cg, counts)
        worst = compare_Q(Dg, Dn, M, counts > 0)
        print(f"  worst |Q - Q_oracle| {worst:.2e}", flush=True)

        print("  two free-running iterations", flush=True)
        Dg2, b2, s2, c2, e2, sq = g.iterate(pr.Y, pr.D_init, 2)
        assert abs(sq[0] - err.astype(np.float64).sum()) <= 1e-6 * sq[0]
        assert sq[1] <= sq[0]
        # first update of the free run equals the teacher-forced update just checked
        o2 = orc.o_code(pr.Y[ids], Dg, cfg.s0)
        compare_code(pr.Y[ids], Dg, cfg.s0, o2, (b2[ids], s2[ids], c2[ids], e2[ids]))


@pytest.mark.parametrize("arith", ["f32", "bf16x3", "screen", "f16x2"])
@pytest.mark.parametrize("name", ["patch8", "headline"])
def test_full_size_configured_iterations(name, arith):
    """The configured number of iterations (10) at the stated size, free-running on both sides:
    the squared-error curve never increases and stays within 1e-3 of the oracle's (Section 4
    RMSE); then the last coding pass, element by element, against the oracle coding with the
    dictionary that pass used."""
    cfg = synth.CONFIGS[name]
    pr = _problem_of(name)
    m, iters = pr.Y.shape[0], cfg.iters
    print(f"case {name} {arith}: p={cfg.p} K={cfg.K} m={m} s0={cfg.s0} iterations={iters}", flush=True)
    with Sbo(cfg.p, cfg.K, cfg.s0, m, arith=arith) as g:
        Dg, blk, supp, coef, err, sq = g.iterate(pr.Y, pr.D_init, iters)
        Dprev, *_r = g.iterate(pr.Y, pr.D_init, iters - 1)     # the dictionary the last pass coded with
    print("  oracle", flush=True)
    sq_o = _oracle_curve_of(name)
    print(f"  oracle sqerr {sq_o}\n  gpu    sqerr {sq}", flush=True)
    assert (np.diff(sq) <= 1e-6 * sq[0]).all(), "error increased"
    np.testing.assert_allclose(sq, sq_o, rtol=1e-3)
    assert abs(sq[-1] - err.astype(np.float64).sum()) <= 1e-6 * sq[-1]
    frac = compare_code(pr.Y, Dprev, cfg.s0, orc.o_code(pr.Y, Dprev, cfg.s0), (blk, supp, coef, err))
    print(f"  last coding pass: exempt fraction {frac:.5f}", flush=True)
    for j in range(cfg.K):
        Q = Dg[j].astype(np.float64)
        assert np.abs(Q @ Q.T - np.eye(cfg.p)).max() <= 1e-5


def test_full_size_patch8_rows():
    """The 8x8-patch configuration at its stated size (m = 16384): every row of the iteration
    against the oracle on all signals, teacher-forced over the configured 10 iterations."""
    cfg = synth.CONFIGS["patch8"]
    pr = synth.generate(cfg)
    m = pr.Y.shape[0]
    D = pr.D_init.astype(np.float64)
    with Sbo(cfg.p, cfg.K, cfg.s0, m) as g:
        for it in range(cfg.iters):
            D32 = D.astype(np.float32)
            o = orc.o_code(pr.Y, D32, cfg.s0)
            frac = compare_code(pr.Y, D32, cfg.s0, o, g.code(pr.Y, D32))
            blk, supp, coef, _err, _E = o
            coef32 = coef.astype(np.float32)
            counts, offsets, perm = g.group(blk)
            oc, oo, op = orc.o_group(blk, cfg.K)
            assert np.array_equal(counts, oc) and np.array_equal(offsets, oo) and np.array_equal(perm, op)
            Dn, M = orc.o_update(pr.Y, blk, supp, coef32, D32)
            Mg = g.accumulate(pr.Y, blk, supp, coef32)
            for j in range(cfg.K):
                scale = np.abs(M[j]).max() + 1e-30
                assert np.abs(Mg[j] - M[j]).max() <= 2e-5 * scale * max(1.0, np.sqrt(counts[j] / 64.0))
            Dg, _c = g.update(pr.Y, blk, supp, coef32, D32)
            w = compare_Q(Dg, Dn, M, counts > 0)
            print(f"  iter {it}: exempt {frac:.5f}, worst dQ {w:.2e}", flush=True)
            D = Dn


def test_full_size_next_rows_headline():
    """Worst-W set, base initialisation and a new orthobase at the headline size, in the
    shapes bench.py times (W = 4096, R = 6), plus the worst-W set of a million residuals."""
    from test_gpu_next_rows import _check_init_base
    cfg = synth.CONFIGS["headline"]
    print(f"case headline next rows: p={cfg.p} K={cfg.K} m={cfg.m}: generating", flush=True)
    pr = synth.generate(cfg)
    m, W, R = pr.Y.shape[0], 4096, 6
    with Sbo(cfg.p, cfg.K, cfg.s0, m) as g:
        blk, supp, coef, err = g.code(pr.Y, pr.D_init)
        print("  worst-W set", flush=True)
        ids = g.worst(err, W)
        assert np.array_equal(ids, orc.o_worst(err, W))
        for W2 in (1, 65536, m):
            assert np.array_equal(g.worst(err, W2), orc.o_worst(err, W2))
        print("  base initialisation on the worst set", flush=True)
        Qg, svg = g.init_base(pr.Y, ids)
        checked, worst = _check_init_base(pr.Y, ids, Qg, svg)
        print(f"  {checked}/{cfg.p} atoms compared, worst {worst:.2e}", flush=True)
        print("  new orthobase, R = 6", flush=True)
        Qn, s2, c2, e2, sq = g.new_base(pr.Y, ids, R)
        Q = Qn.astype(np.float64)
        assert np.abs(Q @ Q.T - np.eye(cfg.p)).max() <= 1e-5
        assert (np.diff(sq) <= 1e-6 * sq[0]).all()
        _Qo, sqo = orc.o_new_base(pr.Y, ids, cfg.s0, R)
        assert np.abs(sq - sqo).max() <= 2e-3 * sqo[0], (sq, sqo)
        # every round teacher-forced: from the oracle's orthobase (rounded to fp32), the codes of
        # the set against the oracle's, the update against the oracle's update from the GPU's codes
        sub, zeros = pr.Y[ids], np.zeros(W, np.int32)
        Qr = orc.o_init_base(pr.Y, ids)[0]
        for r in range(R):
            Q32 = Qr.astype(np.float32)
            so, co, eo = orc.o_train_rounds(sub, zeros, Q32[None], cfg.s0, 1)[1]
            Qg, sg, cg, eg, sq1 = g.new_base(pr.Y, ids, 1, Q0=Q32)
            sg, cg, eg = sg[ids], cg[ids], eg[ids]
            frac = compare_assigned_code(sub, Q32[None], zeros, cfg.s0, (so, co, eo), (sg, cg, eg))
            Dn, M = orc.o_update(sub, zeros, sg, cg, Q32[None])
            w = compare_Q(Qg[None], Dn, M, np.array([True]))
            print(f"  round {r}: exempt fraction {frac:.5f}, worst dQ {w:.2e}", flush=True)
            Qr = orc.o_train_rounds(sub, zeros, Q32[None], cfg.s0, 1)[0][0]
    rng = np.random.default_rng(9)
    big = (rng.random(1 << 20) ** 3).astype(np.float32)
    big[rng.integers(0, 1 << 20, 5000)] = big[17]
    with Sbo(16, 2, 2, 1 << 20) as g:
        for W2 in (1000, 300000):
            assert np.array_equal(g.worst(big, W2), orc.o_worst(big, W2))


def test_full_size_learn_patch8():
    """Algorithm 2 as a whole at the 8x8-patch size with the paper's Table 2 parameters
    (K0 = 5, R = 6), free-running against the oracle."""
    import torch
    import paper_1412_4944_amd as sbo
    cfg = synth.CONFIGS["patch8"]
    pr = synth.generate(cfg)
    m, p, s0 = pr.Y.shape[0], cfg.p, cfg.s0
    K0, P0, R, W, K_max = 5, 2048, 6, 1024, 8
    rng = np.random.default_rng(47)
    sets = np.stack([np.sort(rng.choice(m, P0, replace=False)) for _ in range(K0)]).astype(np.int32)
    print("  oracle", flush=True)
    Do, _blk, hist_o = orc.o_learn(pr.Y, s0, list(sets), R, W, K_max)
    print(f"  oracle history {hist_o}", flush=True)
    with Sbo(p, K_max, s0, m) as g:
        t = g.torch
        D = t.zeros((K_max, p, p), dtype=t.float32, device=g.dev)
        blk, supp, coef, err = g.outputs(m)
        Kf, hist = sbo.sbo_learn(g.ctx, g.dev_f32(pr.Y), D, g.dev_i32(sets), R, W, K_max, 0.0, blk, supp,
                                 coef, err)
        t.cuda.synchronize()
        hist = np.array(hist)
        print(f"  gpu history {hist}", flush=True)
        assert Kf == K_max and hist.size == hist_o.size
        assert (np.diff(hist) <= 1e-6 * hist[0]).all()
        assert np.abs(hist - hist_o).max() <= 1e-2 * hist_o[0]
        Dg = D.cpu().numpy().astype(np.float64)
        for j in range(Kf):
            assert np.abs(Dg[j] @ Dg[j].T - np.eye(p)).max() <= 1e-5


@pytest.mark.parametrize("name", ["headline", "skew"])
def test_screened_block_choice_equals_the_full_products(name):
    """SBO_ARITH_BF16X3_SCREEN decides most signals' orthobase from the three largest partial
    products and forms all six only for the undecided ones: every output must be bit-identical to
    SBO_ARITH_BF16X3, which forms all six for every signal (random initial dictionary: the
    energies of the orthobases are close, many signals are undecided; planted dictionary: few)."""
    cfg = synth.CONFIGS[name]
    pr = _problem_of(name)
    m = pr.Y.shape[0]
    print(f"case {name}: p={cfg.p} K={cfg.K} m={m} s0={cfg.s0}", flush=True)
    with Sbo(cfg.p, cfg.K, cfg.s0, m) as g:
        for D in (pr.D_init, pr.D_planted):
            g.coding_arith("bf16x3")
            ref = g.code(pr.Y, D)
            g.coding_arith("screen")
            out = g.code(pr.Y, D)
            out2 = g.code(pr.Y, D)
            for a, b, c in zip(ref, out, out2):
                assert np.array_equal(a, b), "screened coding differs from the full products"
                assert np.array_equal(b, c), "screened coding is not repeatable"
