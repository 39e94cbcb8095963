"""The entry point that allocates nothing, apex_replay_sample_noalloc, against apex_replay_sample: same memory,
same uniforms, every output compared; two calls in a row, the second smaller, then the size limit."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_sample_equal, dev, host

pytestmark = pytest.mark.gpu
F32 = np.float32
U64 = 1 << 64


def test_sample_noalloc_equals_sample_on_two_calls_in_a_row():
    from paper_1803_00933_amd import apex
    rng = np.random.default_rng(41)
    C, P, ob, ab = 60_000, 70_000, 4112, 8
    g = apex.Replay(C, P, ob, ab)
    o = oracle.Replay(C, P, ob, ab)
    n = 55_000
    obs = rng.integers(0, 256, (n, ob), dtype=np.uint8)
    act = rng.integers(0, 256, (n, ab), dtype=np.uint8)
    ret, gacc = rng.standard_normal(n).astype(F32), rng.random(n).astype(F32)
    prio = (rng.pareto(0.7, n) + 1e-3).astype(F32)
    assert g.add(dev(prio), dev(obs), dev(act), dev(ret), dev(gacc))[0] == 0
    assert o.add(prio, obs, act, ret, gacc)[0] == 0
    before = torch.cuda.memory_allocated()
    calls = ((4, 512), (1, 37))                       # the second call is smaller than the first
    outs = [(g.alloc_sample_outputs(nb, k), g.alloc_sample_outputs(nb, k)) for nb, k in calls]
    rnds = [rng.integers(0, U64, nb * k, dtype=np.uint64) for nb, k in calls]
    d_rnds = [dev(r) for r in rnds]
    torch.cuda.synchronize()
    held = torch.cuda.memory_allocated()
    for (nb, k), (a, b), rnd in zip(calls, outs, d_rnds):          # back to back, nothing in between
        assert g.sample_noalloc(nb, k, 0.4, rnd, a) == apex.OK
    assert torch.cuda.memory_allocated() == held and held > before
    for (nb, k), (a, b), rnd in zip(calls, outs, d_rnds):
        assert g.sample(nb, k, 0.4, rnd, out=b)[0] == apex.OK
    torch.cuda.synchronize()
    for (nb, k), (a, b), rnd in zip(calls, outs, rnds):
        for name in ("key", "slot", "obs", "act", "ret", "gacc"):
            assert torch.equal(a[name], b[name]), name
        assert torch.equal(a["weight"], b["weight"])               # the same kernels on the same masses
        rco, oo = o.sample(nb, k, 0.4, rnd)                        # and both against the oracle
        assert rco == 0
        assert_sample_equal(a, oo)
    # limits and status codes: nothing is enqueued on error
    big = g.alloc_sample_outputs(1, 8, payload=False)
    rnd8 = dev(np.zeros(8, np.uint64))
    lib = apex.lib
    assert lib.apex_replay_sample_noalloc(g.h, 2, apex.NOALLOC_MAX_SAMPLES // 2 + 1, 0.4, rnd8.data_ptr(), None,
                                          big["slot"].data_ptr(), *([None] * 6)) == apex.ERR_TOO_LARGE
    assert g.sample_noalloc(0, 8, 0.4, rnd8, big) == apex.ERR_INVALID_ARG
    assert g.sample_noalloc(1, 8, 1.5, rnd8, big) == apex.ERR_INVALID_ARG
    g2 = apex.Replay(100, 128, 16, 4, min_size_to_sample=10)
    assert g2.sample_noalloc(1, 8, 0.4, rnd8, big) == apex.ERR_NOT_READY
    # the largest size it takes
    nb, k = 16, apex.NOALLOC_MAX_SAMPLES // 16
    a, b = g.alloc_sample_outputs(nb, k, payload=False), g.alloc_sample_outputs(nb, k, payload=False)
    rnd = dev(rng.integers(0, U64, nb * k, dtype=np.uint64))
    assert g.sample_noalloc(nb, k, 1.0, rnd, a) == apex.OK and g.sample(nb, k, 1.0, rnd, out=b)[0] == apex.OK
    torch.cuda.synchronize()
    for name in ("key", "slot", "weight"):
        assert torch.equal(a[name], b[name]), name
