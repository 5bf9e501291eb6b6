"""GPU parity at the full sizes of the benchmark configurations, in the launch
configuration bench.py times.  Coding is checked on a sample of signals (the oracle
codes each signal independently of the others); grouping, accumulation and the SVD
update are checked in full against the oracle."""
import numpy as np
import pytest

import sbo_synth as synth
from oracle import sbo_oracle as orc
from gpu_util import Sbo, compare_code, compare_Q

pytestmark = pytest.mark.gpu


def _sample_ids(m, n, seed):
    rng = np.random.default_rng(seed)
    edge = np.array([0, 1, 31, 32, 63, 64, 127, 128, 255, 256, m - 257, m - 129, m - 65, m - 33, m - 2, m - 1])
    ids = np.unique(np.concatenate([edge[(edge >= 0) & (edge < m)], rng.choice(m, size=n, replace=False)]))
    return ids


@pytest.mark.parametrize("name,n_sample", [("headline", 6000), ("skew", 3000), ("patch16", 1500)])
def test_full_size_iteration_against_oracle(name, n_sample):
    cfg = synth.CONFIGS[name]
    print(f"case {name}: p={cfg.p} K={cfg.K} m={cfg.m} s0={cfg.s0}: generating", flush=True)
    pr = synth.generate(cfg)
    m = pr.Y.shape[0]
    ids = _sample_ids(m, n_sample, cfg.number)
    with Sbo(cfg.p, cfg.K, cfg.s0, m) as g:
        print("  coding on the GPU", flush=True)
        blk, supp, coef, err = g.code(pr.Y, pr.D_init)
        o = orc.o_code(pr.Y[ids], pr.D_init, cfg.s0)
        frac = compare_code(pr.Y[ids], pr.D_init, cfg.s0, o, (blk[ids], supp[ids], coef[ids], err[ids]))
        print(f"  sampled coding parity on {len(ids)} signals, exempt fraction {frac:.5f}", flush=True)
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
