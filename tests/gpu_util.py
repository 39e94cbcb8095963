"""Helpers shared by the GPU parity tests: host<->device marshalling and the comparison bar."""
import numpy as np
import torch

RTOL, ATOL = 1e-5, 1e-6     # fp32 outputs: 1e-5 relative / 1e-6 absolute; integers are compared exactly


def dev(a):
    """numpy -> device tensor (uint64/uint32 travel as the signed type of the same width)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to("cuda:0")


def host(t, dtype=None):
    a = t.detach().cpu().numpy()
    return a.view(dtype) if dtype is not None else a


def assert_close(gpu, ref, what=""):
    gpu, ref = np.asarray(gpu, np.float64), np.asarray(ref, np.float64)
    err = np.abs(gpu - ref)
    bound = ATOL + RTOL * np.abs(ref)
    assert np.all(err <= bound), "%s: worst excess %g at %s" % (what, (err - bound).max(), np.argmax(err - bound))


def assert_sample_equal(gout, oout, payload=True):
    """GPU sample outputs (dict of device tensors) against the oracle's (dict of numpy arrays)."""
    assert np.array_equal(host(gout["slot"], np.uint32), oout["slot"]), "slot"
    assert np.array_equal(host(gout["key"], np.uint64), oout["key"]), "key"
    assert_close(host(gout["weight"]), oout["weight"], "weight")
    if payload and "obs" in oout:
        assert np.array_equal(host(gout["obs"]), oout["obs"]), "obs"
        assert np.array_equal(host(gout["act"]), oout["act"]), "act"
        assert np.array_equal(host(gout["ret"]).view(np.uint32), oout["ret"].view(np.uint32)), "ret"
        assert np.array_equal(host(gout["gacc"]).view(np.uint32), oout["gacc"].view(np.uint32)), "gacc"


def check_gpu_tree(rep, oracle_rep):
    """Every level of the device tree is the sum of its children, leaves and root equal the oracle's."""
    lay = rep.layout
    levels = [host(rep.level_view(l), np.uint64) for l in range(lay.tree_levels)]
    assert np.array_equal(levels[0], oracle_rep.leaves()), "leaves"
    for l in range(1, lay.tree_levels):
        child = levels[l - 1]
        pad = (-len(child)) % lay.tree_fanout
        sums = np.concatenate([child, np.zeros(pad, np.uint64)]).reshape(-1, lay.tree_fanout).sum(1, dtype=np.uint64)
        assert np.array_equal(levels[l], sums), "level %d" % l
    st = rep.stats()
    assert st["root"] == oracle_rep.root == int(levels[-1].sum(dtype=np.uint64))
    assert (st["head"], st["tail"]) == (oracle_rep.head, oracle_rep.tail)
    assert st["n_stale_dropped"] == oracle_rep.n_stale
    assert st["n_clamped"] == oracle_rep.n_clamped
    return st
