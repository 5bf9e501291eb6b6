"""sbo_group_static (the grouping for callers that cannot allocate: static device scratch)
against sbo_group, through the C-ABI: bit-exact, on two calls in a row, the second with a
smaller input, and against the oracle's grouping; limits are rejected with SBO_ELIMIT."""
import numpy as np
import pytest

from oracle import sbo_oracle as orc
from gpu_util import Sbo
import paper_1412_4944_amd as sbo

pytestmark = pytest.mark.gpu


def _blk(K, m, seed):
    rng = np.random.default_rng(seed)
    w = (np.arange(K) + 1.0) ** -1.1
    b = rng.choice(K, size=m, p=w / w.sum()).astype(np.int32)
    if K > 3:
        b[b == 2] = 1                                    # an empty block
    return b


def _static(t, dev, blk, K):
    m = len(blk)
    counts = t.full((K,), -7, dtype=t.int32, device=dev)
    offsets = t.full((K + 1,), -7, dtype=t.int32, device=dev)
    perm = t.full((m,), -7, dtype=t.int32, device=dev)
    bd = t.from_numpy(blk).to(dev)
    sbo.sbo_group_static(bd, K, counts, offsets, perm)
    t.cuda.synchronize()
    return counts.cpu().numpy(), offsets.cpu().numpy(), perm.cpu().numpy()


def test_group_static_matches_group_on_two_calls_in_a_row():
    K = 128
    big, small = _blk(K, 1 << 20, 5), _blk(K, 70001, 6)
    with Sbo(64, K, 4, 1 << 20) as g:
        t, dev = g.torch, g.dev
        for blk in (big, small, _blk(K, 1, 7)):          # the second and third calls are smaller
            print(f"case K={K} m={len(blk)}", flush=True)
            got = _static(t, dev, blk, K)
            ref = g.group(blk)
            for a, b in zip(got, ref):
                assert np.array_equal(a, b)
            for a, b in zip(got, orc.o_group(blk, K)):
                assert np.array_equal(a, b)
    # another K right after, without any context alive
    import torch
    dev = torch.device("cuda:0")
    for K2, m2 in ((7, 5000), (32, 262144), (1, 100)):
        blk = _blk(K2, m2, 8 + K2)
        got = _static(torch, dev, blk, K2)
        for a, b in zip(got, orc.o_group(blk, K2)):
            assert np.array_equal(a, b)


def test_group_static_rejects_sizes_beyond_its_scratch():
    import torch
    dev = torch.device("cuda:0")
    ok = torch.zeros(16, dtype=torch.int32, device=dev)
    out = torch.zeros(300, dtype=torch.int32, device=dev)
    with pytest.raises(sbo.SboError) as e:
        sbo.sbo_group_static(ok, 129, out, out, out)      # K beyond the limit
    assert e.value.code == sbo.binding.SBO_ELIMIT and "static scratch" in str(e.value)
    L = sbo.lib()
    import ctypes
    rc = L.sbo_group_static(ctypes.c_void_p(ok.data_ptr()), (1 << 20) + 1, 4, ctypes.c_void_p(out.data_ptr()),
                            ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(out.data_ptr()), None)
    assert rc == sbo.binding.SBO_ELIMIT                   # m beyond the limit: nothing was enqueued
    assert L.sbo_group_static(None, 16, 4, None, None, None, None) == sbo.binding.SBO_EINVAL
    torch.cuda.synchronize()
