"""GPU parity: the replay verbs against the oracle, element by element, on small and ragged shapes."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, assert_sample_equal, check_gpu_tree, dev, host

pytestmark = pytest.mark.gpu
F32 = np.float32
U64 = 1 << 64


def make_pair(C, P, ob, ab, **kw):
    from paper_1803_00933_amd import apex
    return apex.Replay(C, P, ob, ab, **kw), oracle.Replay(C, P, ob, ab, **kw)


def add_both(g, o, rng, cnt, dist=lambda rng, n: rng.lognormal(0, 1, n)):
    from paper_1803_00933_amd import apex
    obs = rng.integers(0, 256, (cnt, o.obs_bytes), dtype=np.uint8)
    act = rng.integers(0, 256, (cnt, o.act_bytes), dtype=np.uint8)
    ret, gacc = rng.standard_normal(cnt).astype(F32), rng.random(cnt).astype(F32)
    prio = dist(rng, cnt).astype(F32)
    rco, fo = o.add(prio, obs, act, ret, gacc)
    rcg, fg = g.add(dev(prio), dev(obs), dev(act), dev(ret), dev(gacc))
    assert rcg == rco
    if rco == 0:
        assert fg == fo
    return rco


def sample_both(g, o, rng, nb, k, beta=0.4, rnd=None):
    rnd = rng.integers(0, U64, nb * k, dtype=np.uint64) if rnd is None else rnd
    rco, oo = o.sample(nb, k, beta, rnd)
    rcg, go = g.sample(nb, k, beta, dev(rnd))
    assert rcg == rco
    if rco == 0:
        torch.cuda.synchronize()
        assert_sample_equal(go, oo)
    return oo


@pytest.mark.parametrize("P,C,ob,ab", [
    (100, 80, 32, 4),            # one tree level, everything in LDS
    (8192, 4096, 32, 4),         # two levels
    (5000, 4000, 12, 8),         # ragged level sizes, dword copy path
    (300_000, 250_000, 7, 3),    # three levels with ragged tails, byte copy path
    (70_000, 65_000, 4112, 32),  # long-row copy path with a partial last chunk
])
def test_random_operation_sequences(P, C, ob, ab):
    rng = np.random.default_rng(P)
    g, o = make_pair(C, P, ob, ab)
    pareto = lambda rng, n: np.where(rng.random(n) < 0.2, 0.0, rng.pareto(1.1, n) + 1.0)
    for it in range(12):
        cnt = int(rng.integers(1, max(2, P // 4)))
        if o.size + cnt > P:
            assert add_both(g, o, rng, cnt) == oracle.ERR_FULL
            cnt = P - o.size
        if cnt:
            assert add_both(g, o, rng, cnt, pareto if it % 2 else (lambda r, n: r.lognormal(0, 2, n))) == 0
        check_gpu_tree(g, o)
        for nb, k in ((1, 32), (3, 50), (1, 1), (2, 257)):
            oo = sample_both(g, o, rng, nb, k, beta=float(rng.uniform(0, 1)))
        # learner feedback: the sampled keys (with their repeats), some stale and some future keys
        keys = np.concatenate([oo["key"], rng.integers(0, max(1, o.head), 5).astype(np.uint64),
                               np.array([o.tail, o.tail + 7, U64 - 1], np.uint64), oo["key"][:40]])
        newp = pareto(rng, len(keys)).astype(F32)
        newp[:3] = [np.nan, np.inf, 1e30]
        assert o.update_priorities(keys, newp) == 0
        assert g.update_priorities(dev(keys), dev(newp)) == 0
        check_gpu_tree(g, o)
        rco, eo = o.evict()
        rcg, eg = g.evict()
        assert (rcg, eg) == (rco, eo)
        check_gpu_tree(g, o)
        sample_both(g, o, rng, 2, 64)


@pytest.mark.parametrize("P,C,ob,ab", [(5000, 4000, 48, 8), (3000, 2500, 4112, 4)])
def test_add_with_payload_written_in_place(P, C, ob, ab):
    """A producer writes observations and actions of the coming keys straight into the ring (row
    (tail + i) mod P of each column) and adds with NULL for those columns: same memory as a copying add."""
    rng = np.random.default_rng(P + ob)
    g, o = make_pair(C, P, ob, ab)
    for it in range(7):     # wraps around the ring
        cnt = int(rng.integers(1, P - o.size + 1)) if o.size < P else 0
        if cnt:
            obs = rng.integers(0, 256, (cnt, ob), dtype=np.uint8)
            act = rng.integers(0, 256, (cnt, ab), dtype=np.uint8)
            ret, gacc = rng.standard_normal(cnt).astype(F32), rng.random(cnt).astype(F32)
            prio = rng.lognormal(0, 1, cnt).astype(F32)
            rows = torch.from_numpy(((o.tail + np.arange(cnt)) % P).astype(np.int64)).cuda()
            g.obs_view().index_copy_(0, rows, dev(obs))
            g.act_view().index_copy_(0, rows, dev(act))
            assert o.add(prio, obs, act, ret, gacc)[0] == 0
            rc, first = g.add(dev(prio), None, None, dev(ret), dev(gacc))
            assert (rc, first) == (0, o.tail - cnt)
        check_gpu_tree(g, o)
        sample_both(g, o, rng, 2, 96)
        assert g.evict() == o.evict()
    sample_both(g, o, rng, 8, 500)      # the payload of most live keys, as the oracle stored it


def test_large_update_batches_with_heavy_duplication():
    # more than one workgroup's worth of pairs: the two-pass path; few distinct keys: many repeats
    rng = np.random.default_rng(10)
    g, o = make_pair(20_000, 20_000, 16, 4)
    add_both(g, o, rng, 20_000)
    for m, distinct in ((1025, 50), (8192, 300), (5000, 20_000), (1024, 3), (64, 1)):
        keys = rng.integers(0, distinct, m).astype(np.uint64)
        newp = rng.lognormal(0, 1, m).astype(F32)
        assert o.update_priorities(keys, newp) == 0
        assert g.update_priorities(dev(keys), dev(newp)) == 0
        check_gpu_tree(g, o)
    sample_both(g, o, rng, 16, 512)


def test_gather_by_slot():
    rng = np.random.default_rng(9)
    for ob, ab in ((28224, 4), (64, 4), (256, 32), (10, 6)):
        g, o = make_pair(900, 1000, ob, ab)
        add_both(g, o, rng, 950)
        oo = sample_both(g, o, rng, 1, 300)
        out = g.alloc_sample_outputs(1, 300)
        slot = dev(oo["slot"])
        assert g.gather(slot, out["obs"], out["act"], out["ret"], out["gacc"]) == 0
        torch.cuda.synchronize()
        for name in ("obs", "act", "ret", "gacc"):
            assert np.array_equal(host(out[name]), oo[name]), name
        assert g.gather(slot[:0]) == 0


def test_extreme_uniforms_and_edges():
    rng = np.random.default_rng(1)
    g, o = make_pair(6000, 6000, 16, 4)
    add_both(g, o, rng, 6000)
    for fill in (0, U64 - 1, 1 << 63):
        sample_both(g, o, rng, 2, 100, rnd=np.full(200, fill, np.uint64))
    sample_both(g, o, rng, 1, 9000)                      # more samples than transitions
    sample_both(g, o, rng, 1, 65536 // 2)
    # all mass on one transition
    g2, o2 = make_pair(5000, 5000, 16, 4, alpha=1.0, eps=0.0)
    add_both(g2, o2, rng, 5000, lambda r, n: np.where(np.arange(n) == 4321, 1e6, 0.0))
    oo = sample_both(g2, o2, rng, 1, 64)
    assert (oo["slot"] == 4321).sum() >= 63


def test_alpha_zero_and_beta_edges():
    rng = np.random.default_rng(2)
    g, o = make_pair(10_000, 10_000, 16, 4, alpha=0.0)
    add_both(g, o, rng, 10_000)
    oo = sample_both(g, o, rng, 4, 128)
    assert np.all(oo["weight"] == 1.0)
    g, o = make_pair(10_000, 10_000, 16, 4)
    add_both(g, o, rng, 10_000)
    for beta in (0.0, 1.0, 0.4):
        sample_both(g, o, rng, 2, 512, beta=beta)


def test_status_codes():
    from paper_1803_00933_amd import apex
    rng = np.random.default_rng(3)
    g, o = make_pair(100, 128, 16, 4, min_size_to_sample=50)
    rnd = dev(np.zeros(8, np.uint64))
    assert g.sample(1, 8, 0.4, rnd)[0] == apex.ERR_NOT_READY == o.sample(1, 8, 0.4, np.zeros(8, np.uint64))[0]
    add_both(g, o, rng, 49)
    assert g.sample(1, 8, 0.4, rnd)[0] == apex.ERR_NOT_READY
    add_both(g, o, rng, 1)
    assert g.sample(1, 8, 0.4, rnd)[0] == apex.OK
    g2, o2 = make_pair(100, 128, 16, 4)
    assert g2.sample(1, 8, 0.4, rnd)[0] == apex.ERR_EMPTY == o2.sample(1, 8, 0.4, np.zeros(8, np.uint64))[0]
    assert g.sample(0, 8, 0.4, rnd)[0] == apex.ERR_INVALID_ARG
    assert g.sample(1, 0, 0.4, rnd)[0] == apex.ERR_INVALID_ARG
    assert g.sample(1, 8, -1.0, rnd)[0] == apex.ERR_INVALID_ARG
    big = dev(np.zeros(8, np.uint64))
    assert apex.lib.apex_replay_sample(g.h, 2, 40000, 0.4, big.data_ptr(), None, big.data_ptr(), *([None] * 6)) \
        == apex.ERR_TOO_LARGE
    assert apex.lib.apex_replay_sample(g.h, 1, 8, 0.4, big.data_ptr(), None, None, *([None] * 6)) == apex.ERR_INVALID_ARG
    assert g.evict() == (0, 0) and g.add(dev(np.zeros(0, F32)))[0] == apex.OK
    assert g.update_priorities(dev(np.zeros(0, np.uint64)), dev(np.zeros(0, F32))) == apex.OK
    torch.cuda.synchronize()
    check_gpu_tree(g, o)


@pytest.mark.parametrize("P,C", [(128, 100), (1 << 20, 1_000_000)])   # the larger shape has a top level of 256 nodes
def test_fused_steps_refuse_an_empty_or_unready_memory(P, C):
    """Learner steps as one launch each obey the same gate as apex_replay_sample: nothing stored -> EMPTY, fewer
    than min_size_to_sample -> NOT_READY, with or without priorities to write back, and nothing is enqueued
    (tree, counters and buffers stay as they were)."""
    from paper_1803_00933_amd import apex
    rng = np.random.default_rng(17)
    k = 8
    rnd, newp = dev(rng.integers(0, U64, (3, k), dtype=np.uint64)), dev(rng.random((3, k)).astype(F32))
    for min_size, fill, want in ((0, 0, apex.ERR_EMPTY), (50, 0, apex.ERR_NOT_READY), (50, 49, apex.ERR_NOT_READY)):
        g, o = make_pair(C, P, 16, 4, min_size_to_sample=min_size)
        if fill:
            assert add_both(g, o, rng, fill) == 0
        pipe = apex.Pipeline(g, 4, 1, k)
        for s_ in pipe.sets:
            s_["slot"].fill_(-7)
        torch.cuda.synchronize()
        before = g.stats()
        assert o.sample(1, k, 0.4, np.zeros(k, np.uint64))[0] == want
        assert pipe.fork() == 0
        assert pipe.steps(3, 0.4, rnd, newp)[0] == want
        assert pipe.steps(3, 0.4, rnd, None)[0] == want
        assert pipe.join() == 0
        torch.cuda.synchronize()
        assert g.stats() == before
        assert all(int((s_["slot"] != -7).sum()) == 0 for s_ in pipe.sets)
        check_gpu_tree(g, o)
        if fill:                                   # one more transition and the same call goes through
            assert add_both(g, o, rng, 1) == 0
            assert pipe.fork() == 0
            rc, first = pipe.steps(3, 0.4, rnd, newp)
            assert rc == apex.OK and pipe.join() == 0
            torch.cuda.synchronize()
            for i in range(3):
                rco, oo = o.sample(1, k, 0.4, host(rnd[i], np.uint64))
                assert rco == 0 and o.update_priorities(oo["key"], host(newp[i])) == 0
                assert_sample_equal(pipe.sets[(first + i) % 4], oo)
            check_gpu_tree(g, o)
        pipe.close()


def test_tiny_workload_full_trace():
    """The small configuration end to end: 200 rounds of {n-step priorities, add 400, sample 32,
    update with fresh |N(0,1)| errors, evict}; every output of every round is compared."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["tiny"]
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, alpha=w.alpha, eps=w.eps, frac_bits=w.frac_bits)
    key0 = 0
    for rnd_i in range(200):
        d = synth.actor_round(w, rnd_i)
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        rc, prio, ret, gacc, fx = apex.nstep_priorities(dev(d["q_online"]), dev(d["q_target"]), dev(d["action"]),
                                                        dev(d["reward"]), dev(d["discount"]), w.n, w.alpha, w.eps,
                                                        w.frac_bits, w.max_slots)
        assert rc == 0
        obs = synth.obs_rows(w.seed, key0, w.add_count, w.obs_bytes)
        rco, fo = o.add(ref[0].reshape(-1), obs, d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
        rcg, fg = g.add(prio.view(-1), dev(obs), dev(d["act"]), ret.view(-1), gacc.view(-1))   # device to device
        assert (rcg, fg) == (rco, fo) == (0, key0)
        key0 += w.add_count
        torch.cuda.synchronize()
        assert np.array_equal(host(fx, np.uint64), ref[3])
        rnd = synth.uniforms(w.seed, rnd_i, 1, w.k).reshape(-1)
        rco, oo = o.sample(1, w.k, w.beta, rnd)
        rcg, go = g.sample(1, w.k, w.beta, dev(rnd))
        assert rcg == rco == 0
        torch.cuda.synchronize()
        assert_sample_equal(go, oo)
        assert np.array_equal(oo["obs"], np.concatenate([synth.obs_rows(w.seed, int(kk), 1, w.obs_bytes)
                                                         for kk in oo["key"]]))
        newp = synth.priorities(w.td_dist, w.seed, rnd_i, w.k)
        assert o.update_priorities(oo["key"], newp) == 0
        assert g.update_priorities(go["key"], dev(newp)) == 0
        assert g.evict() == o.evict()
        if rnd_i % 10 == 9 or rnd_i < 12:
            st = check_gpu_tree(g, o)
            assert st["size"] == min(key0, w.capacity)
    check_gpu_tree(g, o)


def test_split_calls_on_separate_streams():
    """sample_begin / sample_finish and add_payload / add_publish, tree work and copies on different
    streams ordered by events, against the oracle's plain sequence."""
    rng = np.random.default_rng(12)
    C, P, ob, ab, k, cnt = 3000, 4096, 28224, 4, 128, 500
    g, o = make_pair(C, P, ob, ab)
    add_both(g, o, rng, C)
    tree_s, copy_s = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    outs, refs = [], []
    for step in range(8):
        out = g.alloc_sample_outputs(1, k)
        out["mass"] = torch.empty(k, dtype=torch.int64, device="cuda:0")
        rnd = rng.integers(0, U64, k, dtype=np.uint64)
        newp = rng.lognormal(0, 1, k).astype(F32)
        obs = rng.integers(0, 256, (cnt, ob), dtype=np.uint8)
        act = rng.integers(0, 256, (cnt, ab), dtype=np.uint8)
        ret, gacc, prio = (rng.standard_normal(cnt).astype(F32) for _ in range(3))
        d = [dev(x) for x in (rnd, newp, obs, act, ret, gacc, prio)]
        torch.cuda.synchronize()
        # oracle: sample, update, add, evict
        rco, oo = o.sample(1, k, 0.4, rnd)
        o.update_priorities(oo["key"], newp)
        o.add(prio, obs, act, ret, gacc)
        o.evict()
        # device: the payload copy of the add runs beside the learner step
        assert g.add_payload(cnt, d[2], d[3], d[4], d[5], stream=copy_s) == 0
        payload_done = torch.cuda.Event()
        payload_done.record(copy_s)
        assert g.sample_begin(1, k, d[0], out, stream=tree_s) == 0
        drawn = torch.cuda.Event()
        drawn.record(tree_s)
        copy_s.wait_event(drawn)
        assert g.sample_finish(1, k, 0.4, out, stream=copy_s) == 0
        assert g.update_priorities(out["key"], d[1], stream=tree_s) == 0
        tree_s.wait_event(payload_done)
        assert g.add_publish(d[6], stream=tree_s)[0] == 0
        assert g.evict(stream=tree_s)[0] == 0
        gathered = torch.cuda.Event()
        gathered.record(copy_s)
        tree_s.wait_event(gathered)          # the next payload must not overwrite rows still being read
        copy_s.wait_stream(tree_s)           # and needs the advanced tail
        outs.append(out), refs.append(oo)
    torch.cuda.synchronize()
    for out, oo in zip(outs, refs):
        assert_sample_equal(out, oo)
        assert np.array_equal(host(out["mass"], np.uint64), oo["mass"])
    check_gpu_tree(g, o)


def test_captured_launches_replay_correctly():
    """A captured sequence of add / sample / update / evict is replayed several times, with eager work
    and synchronisations in between; every replay is checked against the oracle doing the same."""
    rng = np.random.default_rng(13)
    C, P, ob, ab, k, cnt = 1000, 2048, 64, 4, 64, 100
    g, o = make_pair(C, P, ob, ab)
    add_both(g, o, rng, C)
    rnd = [rng.integers(0, U64, k, dtype=np.uint64) for _ in range(3)]
    newp = [rng.lognormal(0, 1, k).astype(F32) for _ in range(3)]
    obs = rng.integers(0, 256, (cnt, ob), dtype=np.uint8)
    act = rng.integers(0, 256, (cnt, ab), dtype=np.uint8)
    ret, gacc, prio = (rng.standard_normal(cnt).astype(F32) for _ in range(3))
    d_rnd, d_newp = [dev(x) for x in rnd], [dev(x) for x in newp]
    d_obs, d_act, d_ret, d_gacc, d_prio = (dev(x) for x in (obs, act, ret, gacc, prio))
    outs = [g.alloc_sample_outputs(1, k) for _ in range(3)]

    def sequence():
        assert g.add(d_prio, d_obs, d_act, d_ret, d_gacc)[0] == 0
        for i in range(3):
            assert g.sample(1, k, 0.4, d_rnd[i], out=outs[i])[0] == 0
            assert g.update_priorities(outs[i]["key"], d_newp[i]) == 0
        assert g.evict() == (0, cnt)

    def oracle_sequence():
        o.add(prio, obs, act, ret, gacc)
        res = []
        for i in range(3):
            res.append(o.sample(1, k, 0.4, rnd[i])[1])
            o.update_priorities(res[-1]["key"], newp[i])
        assert o.evict() == (0, cnt)
        return res

    s = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s):
        sequence()
    for replay in range(4):
        graph.replay()
        torch.cuda.synchronize()
        res = oracle_sequence()
        for i in range(3):
            assert_sample_equal(outs[i], res[i])
        assert g.resync() == 0
        check_gpu_tree(g, o)
        if replay == 1:                      # eager work between replays, on the same memory
            add_both(g, o, rng, 50)
            sample_both(g, o, rng, 1, 32)
            assert g.evict() == o.evict()
            assert g.resync() == 0


# One batch per step of 16-byte-aligned rows is one launch per step; 8 x 288 samples per step is above the
# size from which the pipeline sends a step's gather to its copy stream.
# (batches per step, k, observation bytes).  Rows of at most 1 KB make a small add round one launch
# (n-step priorities, payload and masses together), issued by add_end.
PIPELINE_STEP_SHAPES = [(1, 96, 4224), (8, 288, 4224), (1, 64, 256), (1, 64, 100), (1, 32, 7), (1, 32, 1001)]


@pytest.mark.parametrize("depth", [3, 2])      # two buffer sets: too few for the one-launch step, two launches instead
@pytest.mark.parametrize("nb,k,ob", PIPELINE_STEP_SHAPES)
def test_pipeline_matches_the_plain_call_order(nb, k, ob, depth):
    """apex_pipeline_*: learner steps (for steps of several batches: with the gathers on the second
    stream) and add rounds whose payload copy runs beside them, against the oracle doing draw, update,
    [add], [evict] one after the other."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=ob, capacity=3000, max_slots=4096, streams=5, chunk=40, k=k)
    rng = np.random.default_rng(14)
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    add_both(g, o, rng, w.capacity)
    n_steps, per_round = 24, 6
    pipe = apex.Pipeline(g, depth, nb, w.k)
    rnd = rng.integers(0, U64, (n_steps, nb * w.k), dtype=np.uint64)
    newp = rng.lognormal(0, 1, (n_steps, nb * w.k)).astype(F32)
    d_rnd, d_newp = dev(rnd), dev(newp)
    S, T = w.streams, w.chunk
    scratch = [torch.empty(S * T, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    rounds = []
    for i in range(n_steps // per_round):
        d = synth.actor_round(w, i)
        d["obs"] = rng.integers(0, 256, (S * T, w.obs_bytes), dtype=np.uint8)
        rounds.append((d, {k2: dev(v) for k2, v in d.items()}))
    torch.cuda.synchronize()
    assert pipe.fork() == 0
    refs, got = [], []
    for s in range(n_steps):
        if s % per_round == 0:
            d, dd = rounds[s // per_round]
            assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                                  dd["obs"], dd["act"], *scratch) == 0
        rc, first = pipe.steps(1, 0.4, d_rnd[s], d_newp[s])
        assert rc == 0 and first == s % depth
        rco, oo = o.sample(nb, w.k, 0.4, rnd[s])
        o.update_priorities(oo["key"], newp[s])
        refs.append(oo)
        if (s + 1) % per_round == 0:
            evict = (s + 1) % (2 * per_round) == 0
            rc, first_key, ev = pipe.add_end(evict)
            ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                          w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
            rco, fo = o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
            assert (rc, first_key) == (rco, fo)
            if evict:
                assert o.evict() == (0, ev)
        # a set must be consumed before `depth` further steps are issued: copy it out now
        assert pipe.join() == 0
        torch.cuda.synchronize()
        got.append({k2: v.clone() for k2, v in pipe.sets[s % depth].items()})
        assert pipe.fork() == 0
    assert pipe.join() == 0
    torch.cuda.synchronize()
    for out, oo in zip(got, refs):
        assert_sample_equal(out, oo)
    check_gpu_tree(g, o)
    # several steps in one call, no synchronisation in between; the last `depth` sets are checked
    rnd2 = rng.integers(0, U64, (7, nb * w.k), dtype=np.uint64)
    newp2 = rng.lognormal(0, 1, (7, nb * w.k)).astype(F32)
    d2 = (dev(rnd2), dev(newp2))
    torch.cuda.synchronize()
    assert pipe.fork() == 0
    rc, first = pipe.steps(7, 0.4, *d2)
    assert rc == 0 and first == n_steps % depth
    assert pipe.join() == 0
    torch.cuda.synchronize()
    refs2 = []
    for s in range(7):
        rco, oo = o.sample(nb, w.k, 0.4, rnd2[s])
        o.update_priorities(oo["key"], newp2[s])
        refs2.append(oo)
    for s in range(7 - depth, 7):
        assert_sample_equal(pipe.sets[(n_steps + s) % depth], refs2[s])
    check_gpu_tree(g, o)
    pipe.close()


@pytest.mark.parametrize("streams", [48, 30])      # a round on the copy stream (5 MB), one on the learner's stream
def test_wide_steps_are_gathered_before_their_slots_are_reused(streams):
    """A ring with no slack: every add round lands in the slots that the eviction before it has just freed, and
    the batches drawn before that eviction hold many of the evicted keys.  Their gathers, which run on the copy
    streams, have to be through before the round's payload is written; nothing here synchronises in between."""
    from paper_1803_00933_amd import apex, synth
    nb, k, ob, depth, T = 4, 512, 4224, 4, 25
    count = streams * T
    C = 2100
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=ob, capacity=C, max_slots=C + count, streams=streams, chunk=T, k=k)
    rng = np.random.default_rng(streams)
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    add_both(g, o, rng, w.capacity)
    pipe = apex.Pipeline(g, depth, nb, w.k)
    cycles = 3 * depth
    rnd = rng.integers(0, U64, (cycles, nb * w.k), dtype=np.uint64)
    newp = rng.lognormal(0, 1, (cycles, nb * w.k)).astype(F32)
    d_rnd, d_newp = dev(rnd), dev(newp)
    scratch = [torch.empty(count, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    rounds = []
    for i in range(cycles):
        d = synth.actor_round(w, i)
        d["obs"] = rng.integers(0, 256, (count, w.obs_bytes), dtype=np.uint8)
        rounds.append((d, {k2: dev(v) for k2, v in d.items()}))
    torch.cuda.synchronize()
    for c0 in range(0, cycles, depth):
        assert pipe.fork() == 0
        refs = []
        for s in range(c0, c0 + depth):
            d, dd = rounds[s]
            assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                                  dd["obs"], dd["act"], *scratch) == 0
            rc, first = pipe.steps(1, 0.4, d_rnd[s], d_newp[s])
            assert rc == 0 and first == s % depth
            rc, first_key, ev = pipe.add_end(True)
            refs.append(o.sample(nb, w.k, 0.4, rnd[s])[1])
            o.update_priorities(refs[-1]["key"], newp[s])
            ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                          w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
            assert (rc, first_key) == o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1),
                                            ref[2].reshape(-1))
            assert o.evict() == (0, ev) and ev == count
        assert pipe.join() == 0
        torch.cuda.synchronize()
        for s in range(c0, c0 + depth):
            assert_sample_equal(pipe.sets[s % depth], refs[s - c0])
        check_gpu_tree(g, o)
    pipe.close()


def test_pipeline_small_and_large_add_rounds():
    """Small add rounds travel on the learner's stream, large ones on the copy stream: rounds of both kinds
    in one pipeline, with learner steps in between, against the oracle."""
    from paper_1803_00933_amd import apex, synth
    small = synth.WORKLOADS["tiny"].scaled(obs_bytes=4224, capacity=9000, max_slots=12288, streams=4, chunk=25, k=64)
    large = small.scaled(streams=40)              # 1000 rows of 4224 B: above the size that stays on one stream
    rng = np.random.default_rng(21)
    g, o = make_pair(small.capacity, small.max_slots, small.obs_bytes, small.act_bytes)
    add_both(g, o, rng, 8000)
    depth = 4
    pipe = apex.Pipeline(g, depth, 1, small.k)
    assert pipe.fork() == 0
    for i, w in enumerate([small, large, large, small, small, large, small]):
        d = synth.actor_round(w, i)
        n_rows = w.streams * w.chunk
        d["obs"] = rng.integers(0, 256, (n_rows, w.obs_bytes), dtype=np.uint8)
        dd = {k2: dev(v) for k2, v in d.items()}
        scratch = [torch.empty(n_rows, dtype=torch.float32, device="cuda:0") for _ in range(3)]
        rnd = rng.integers(0, U64, (3, w.k), dtype=np.uint64)
        newp = rng.lognormal(0, 1, (3, w.k)).astype(F32)
        d_rnd, d_newp = dev(rnd), dev(newp)
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              dd["obs"], dd["act"], *scratch) == 0
        rc, first = pipe.steps(3, 0.4, d_rnd, d_newp)
        assert rc == 0
        rc, first_key, ev = pipe.add_end(True)
        refs = []
        for s in range(3):
            refs.append(o.sample(1, w.k, 0.4, rnd[s])[1])
            o.update_priorities(refs[-1]["key"], newp[s])
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        rco, fo = o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
        assert (rc, first_key) == (rco, fo)
        assert o.evict() == (0, ev)
        assert pipe.join() == 0
        torch.cuda.synchronize()
        for s in range(3):
            assert_sample_equal(pipe.sets[(first + s) % depth], refs[s])
        check_gpu_tree(g, o)
        assert pipe.fork() == 0
    assert pipe.join() == 0
    # the payload of the last rounds is where the oracle has it
    oo = sample_both(g, o, rng, 1, 64)
    pipe.close()


@pytest.mark.parametrize("ob", [256, 100, 7])
def test_small_add_round_rides_in_the_last_step_launch(ob):
    """With a small add round open (rows of at most 1 KB), the last step launch of a steps call is held back
    and issued by add_end with the round inside it; any other call issues it on its own.  Every order of
    calls against the oracle's plain order: steps, then the round, then the eviction."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=ob, capacity=9000, max_slots=12288, streams=6, chunk=25, k=96)
    rng = np.random.default_rng(ob)
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    add_both(g, o, rng, 8000)
    depth = 5
    pipe = apex.Pipeline(g, depth, 1, w.k)
    n_rows = w.streams * w.chunk
    scratch = [torch.empty(n_rows, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    # (steps calls between add_begin and add_end, write-back, join before add_end, misaligned source rows)
    patterns = [([2], True, False, False), ([1, 1], True, False, False), ([1], True, True, False),
                ([], True, False, False), ([3], True, False, True), ([2], False, False, False),
                ([2], True, False, False)]
    assert pipe.fork() == 0
    for i, (calls, wb, join_between, misaligned) in enumerate(patterns):
        d = synth.actor_round(w, i)
        d["obs"] = rng.integers(0, 256, (n_rows, w.obs_bytes), dtype=np.uint8)
        dd = {k2: dev(v) for k2, v in d.items()}
        if misaligned:   # the same bytes at an address that is no multiple of 16 (nor of 4)
            buf = torch.empty(n_rows * ob + 64, dtype=torch.uint8, device="cuda:0")
            view = buf[3:3 + n_rows * ob].view(n_rows, ob)
            view.copy_(dd["obs"])
            dd["obs"] = view
        total = sum(calls)
        rnd = rng.integers(0, U64, (max(total, 1), w.k), dtype=np.uint64)
        newp = rng.lognormal(0, 1, (max(total, 1), w.k)).astype(F32)
        d_rnd, d_newp = dev(rnd), dev(newp)
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              dd["obs"], dd["act"], *scratch) == 0
        firsts, at = [], 0
        for c in calls:
            rc, first = pipe.steps(c, 0.4, d_rnd[at:at + c], d_newp[at:at + c] if wb else None)
            assert rc == 0
            firsts += [(first + j) % depth for j in range(c)]
            at += c
        if join_between:
            assert pipe.join() == 0
            assert pipe.fork() == 0
        rc, first_key, ev = pipe.add_end(True)
        refs = []
        for s_ in range(total):
            refs.append(o.sample(1, w.k, 0.4, rnd[s_])[1])
            if wb:
                o.update_priorities(refs[-1]["key"], newp[s_])
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        rco, fo = o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
        assert (rc, first_key) == (rco, fo)
        assert o.evict() == (0, ev)
        assert pipe.join() == 0
        torch.cuda.synchronize()
        for s_ in range(total):
            assert_sample_equal(pipe.sets[firsts[s_]], refs[s_])
        check_gpu_tree(g, o)
        sample_both(g, o, rng, 2, 200)      # payload of the rounds added so far
        assert pipe.fork() == 0
    assert pipe.join() == 0
    st = g.stats()
    assert (st["size"], st["n_clamped"], st["n_stale_dropped"]) == (o.size, o.n_clamped, o.n_stale)
    pipe.close()


@pytest.mark.parametrize("ob,seed", [(64, 1), (64, 2), (4224, 3), (1040, 4), (100, 5), (256, 6), (28224, 7), (7, 8)])
def test_pipeline_random_call_orders(ob, seed):
    """Random orders of the pipeline's calls (steps of random length with and without write-back, add rounds
    opened and closed around them, evictions, joins, plain calls on the joined stream in between) against the
    oracle applying the same operations in the order of the calls."""
    from paper_1803_00933_amd import apex, synth
    rng = np.random.default_rng(seed)
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=ob, capacity=6000, max_slots=8192, streams=5, chunk=20, k=int(rng.integers(40, 130)))
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    add_both(g, o, rng, 5000)
    depth = int(rng.integers(3, 7))
    pipe = apex.Pipeline(g, depth, 1, w.k)
    n_rows = w.streams * w.chunk
    scratch = [torch.empty(n_rows, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    keep = []               # device inputs stay alive until the next join
    pending = []            # (buffer set, oracle batch) to compare at the next join
    open_round = None
    assert pipe.fork() == 0
    for it in range(120):
        op = rng.choice(["steps", "steps", "steps", "begin", "end", "join", "plain"])
        if op == "steps":
            n = int(rng.integers(1, depth))          # fewer than the sets, so no set is overwritten before the join
            if len(pending) + n > depth:
                op = "join"
            else:
                wb = rng.random() < 0.8
                rnd = rng.integers(0, U64, (n, w.k), dtype=np.uint64)
                newp = rng.lognormal(0, 1.5, (n, w.k)).astype(F32)
                d_rnd, d_newp = dev(rnd), dev(newp)
                keep += [d_rnd, d_newp]
                rc, first = pipe.steps(n, 0.4, d_rnd, d_newp if wb else None)
                assert rc == 0
                for i in range(n):
                    rco, oo = o.sample(1, w.k, 0.4, rnd[i])
                    assert rco == 0
                    if wb:
                        assert o.update_priorities(oo["key"], newp[i]) == 0
                    pending.append(((first + i) % depth, oo))
        if op == "begin" and open_round is None and o.size + n_rows <= w.max_slots:
            d = synth.actor_round(w, it)
            d["obs"] = rng.integers(0, 256, (n_rows, w.obs_bytes), dtype=np.uint8)
            dd = {k2: dev(v) for k2, v in d.items()}
            keep.append(dd)
            assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                                  dd["obs"], dd["act"], *scratch) == 0
            open_round = d
        elif op == "end" and open_round is not None:
            d, open_round = open_round, None
            evict = bool(rng.random() < 0.5)
            rc, first_key, ev = pipe.add_end(evict)
            ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                          w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
            rco, fo = o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
            assert (rc, first_key) == (rco, fo)
            if evict:
                assert o.evict() == (0, ev)
        elif op in ("join", "plain") and open_round is None:
            assert pipe.join() == 0
            torch.cuda.synchronize()
            for set_index, oo in pending:
                assert_sample_equal(pipe.sets[set_index], oo)
            pending, keep = [], []
            check_gpu_tree(g, o)
            if op == "plain":          # calls outside the pipeline change the first tree copy only
                oo = sample_both(g, o, rng, 1, 48)
                pr = rng.lognormal(0, 1, len(oo["key"])).astype(F32)
                assert g.update_priorities(dev(oo["key"]), dev(pr)) == o.update_priorities(oo["key"], pr) == 0
                if rng.random() < 0.3:
                    assert g.evict() == o.evict()
            assert pipe.fork() == 0
    if open_round is not None:
        rc, first_key, ev = pipe.add_end(False)
        d = open_round
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        assert (rc, first_key) == o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
    assert pipe.join() == 0
    torch.cuda.synchronize()
    for set_index, oo in pending:
        assert_sample_equal(pipe.sets[set_index], oo)
    check_gpu_tree(g, o)
    st = g.stats()
    assert (st["size"], st["n_clamped"], st["n_stale_dropped"]) == (o.size, o.n_clamped, o.n_stale)
    pipe.close()


@pytest.mark.parametrize("nb,k,ob", PIPELINE_STEP_SHAPES)
def test_pipeline_graph_replays(nb, k, ob):
    """One cycle (an add round beside six learner steps, then eviction) captured as a HIP graph by the
    pipeline and replayed; every replay is checked against the oracle, with eager work in between."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=ob, capacity=3000, max_slots=4096, streams=5, chunk=40, k=k)
    rng = np.random.default_rng(15)
    g, o = make_pair(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    add_both(g, o, rng, w.capacity)
    depth, n_steps = 3, 6
    pipe = apex.Pipeline(g, depth, nb, w.k)
    rnd = rng.integers(0, U64, (n_steps, nb * w.k), dtype=np.uint64)
    newp = rng.lognormal(0, 1, (n_steps, nb * w.k)).astype(F32)
    d_rnd, d_newp = dev(rnd), dev(newp)
    S, T = w.streams, w.chunk
    scratch = [torch.empty(S * T, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    d = synth.actor_round(w, 0)
    d["obs"] = rng.integers(0, 256, (S * T, w.obs_bytes), dtype=np.uint8)
    dd = {k2: dev(v) for k2, v in d.items()}
    torch.cuda.synchronize()

    def cycle():
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              dd["obs"], dd["act"], *scratch) == 0
        assert pipe.steps(n_steps, 0.4, d_rnd, d_newp)[0] == 0
        rc, _, ev = pipe.add_end(True)
        assert (rc, ev) == (0, S * T)

    def oracle_cycle():
        res = []
        for s in range(n_steps):
            res.append(o.sample(nb, w.k, 0.4, rnd[s])[1])
            o.update_priorities(res[-1]["key"], newp[s])
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        assert o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))[0] == 0
        assert o.evict() == (0, S * T)
        return res

    assert pipe.capture_begin() == 0
    cycle()
    assert pipe.capture_end() == 0
    for replay in range(4):
        assert pipe.fork() == 0
        assert pipe.replay(1) == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        res = oracle_cycle()
        for s in range(n_steps - depth, n_steps):
            assert_sample_equal(pipe.sets[s % depth], res[s])
        assert g.resync() == 0
        check_gpu_tree(g, o)
        if replay == 1:                       # eager calls between replays, on the same memory
            add_both(g, o, rng, 30)
            sample_both(g, o, rng, 1, 32)
            assert g.evict() == o.evict()
    # several replays back to back
    assert pipe.fork() == 0
    assert pipe.replay(3) == 0
    assert pipe.join() == 0
    torch.cuda.synchronize()
    for _ in range(3):
        res = oracle_cycle()
    for s in range(n_steps - depth, n_steps):
        assert_sample_equal(pipe.sets[s % depth], res[s])
    assert g.resync() == 0
    check_gpu_tree(g, o)
    pipe.close()


@pytest.mark.parametrize("P,C,k,ob", [
    (4096, 3000, 96, 4224),          # one tree level
    (40_000, 30_000, 200, 4112),     # two levels, ragged tails, partial last vector chunk
    (400_000, 300_000, 512, 4224),   # three levels
    (5000, 4000, 1024, 32768),       # as many samples as a workgroup has lanes, largest fused row
    (5000, 4000, 1, 4224),           # batches of one
    (60_000, 50_000, 512, 256),      # short rows (feature vectors): a few lanes of each workgroup copy
    (70_000, 60_000, 300, 4224),     # a top level of 1094 nodes: the drawing wave stages it in chunks of four passes
    (280_000, 250_000, 256, 1040),   # a ragged top level of 4375 nodes (three chunks)
    (4608, 4000, 64, 4112),          # one level of the largest size
    (33_000, 30_000, 517, 2064),     # 516 top nodes (two passes of the drawing wave), k no multiple of 8
    (9000, 8000, 1000, 48),          # two passes over the pending pairs, a ragged last one
    (5000, 4000, 100, 4100),         # rows that are no multiple of 16 bytes: 4-byte vectors, several passes per row
    (3000, 2500, 64, 1001),          # odd row size: byte copies
    (3000, 2500, 96, 56448),         # rows longer than one pass of a workgroup (two frame stacks per transition)
    (3000, 2500, 40, 32784),         # just beyond one pass
])
def test_one_launch_per_learner_step(P, C, k, ob):
    """Sequences of learner steps issued as one launch per step (draw of the next batch inside the launch
    that gathers and writes back the current one, two copies of the tree): every batch of every sequence
    against the oracle doing draw, update, draw, update, with other operations between the sequences.
    Priorities are heavy-tailed so that batches draw the same slot several times."""
    from paper_1803_00933_amd import apex
    rng = np.random.default_rng(P + k)
    g, o = make_pair(C, P, ob, 4)
    heavy = lambda rng, n: (rng.pareto(0.4, n) + 1e-3)
    while o.size < C:
        assert add_both(g, o, rng, min(20_000, C - o.size), heavy) == 0
    depth = 9
    pipe = apex.Pipeline(g, depth, 1, k)
    for seq in range(6):
        n = (8, 2, 8, 8, 1, 7)[seq]           # sequences of one and two steps never read the second tree copy
        rnd = rng.integers(0, U64, (n, k), dtype=np.uint64)
        newp = heavy(rng, (n, k)).astype(F32)
        newp[rng.random((n, k)) < 0.1] = 0.0
        with_update = seq != 3
        d_rnd, d_newp = dev(rnd), dev(newp)
        torch.cuda.synchronize()
        assert pipe.fork() == 0
        rc, first = pipe.steps(n, 0.5, d_rnd, d_newp if with_update else None)
        assert rc == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        dup = 0
        for i in range(n):
            rco, oo = o.sample(1, k, 0.5, rnd[i])
            assert rco == 0
            dup += k - len(np.unique(oo["slot"]))
            if with_update:
                assert o.update_priorities(oo["key"], newp[i]) == 0
            assert_sample_equal(pipe.sets[(first + i) % depth], oo)
        assert k < 64 or n < 7 or dup > 0  # the case the test is about occurs
        check_gpu_tree(g, o)
        # other operations between the sequences: they change the first copy of the tree only
        if seq % 2 == 0:
            assert add_both(g, o, rng, min(500, P - o.size), heavy) == 0
            assert g.evict() == o.evict()
        else:
            oo = sample_both(g, o, rng, 1, min(k, 64))
            pr = heavy(rng, len(oo["key"])).astype(F32)
            assert g.update_priorities(dev(oo["key"]), dev(pr)) == o.update_priorities(oo["key"], pr) == 0
    st = g.stats()
    assert (st["n_clamped"], st["n_stale_dropped"]) == (o.n_clamped, o.n_stale)
    pipe.close()


@pytest.mark.parametrize("ob,k,extra", [(28224, 512, 0), (4224, 100, 0), (64, 128, 0), (4224, 700, 600),
                                        (64, 700, 600), (7, 512, 700)])   # short rows, more than 1024 pairs
def test_finish_with_update_riding_along(ob, k, extra):
    """apex_replay_sample_finish_update == finish, then update (in the gather kernel's extra workgroup when
    the batch fits one; with short rows the first pass of a larger update rides in the gather launch; by
    launches of its own otherwise)."""
    rng = np.random.default_rng(16 + k)
    g, o = make_pair(3000, 4096, ob, 4)
    add_both(g, o, rng, 3000)
    for step in range(4):
        rnd = rng.integers(0, U64, k, dtype=np.uint64)
        rco, oo = o.sample(1, k, 0.4, rnd)
        keys = np.concatenate([oo["key"], rng.integers(0, 3000, extra).astype(np.uint64)])   # extra: > 1024 pairs
        newp = rng.lognormal(0, 1, len(keys)).astype(F32)
        o.update_priorities(keys, newp)
        out = g.alloc_sample_outputs(1, k)
        out["mass"] = torch.empty(k, dtype=torch.int64, device="cuda:0")
        assert g.sample_begin(1, k, dev(rnd), out) == 0
        assert g.sample_finish_update(1, k, 0.4, out, dev(keys), dev(newp)) == 0
        torch.cuda.synchronize()
        assert_sample_equal(out, oo)
        check_gpu_tree(g, o)
        # the batch's own priorities written back by the launch that finishes it
        rnd = rng.integers(0, U64, k, dtype=np.uint64)
        rco, oo = o.sample(1, k, 0.4, rnd)
        newp = rng.lognormal(0, 1, k).astype(F32)
        o.update_priorities(oo["key"], newp)
        assert g.sample_begin(1, k, dev(rnd), out) == 0
        assert g.sample_finish_writeback(1, k, 0.4, out, dev(newp)) == 0
        torch.cuda.synchronize()
        assert_sample_equal(out, oo)
        check_gpu_tree(g, o)
        # several batches per call: samples of different batches collide on heavy transitions
        nb = 3
        rnd = rng.integers(0, U64, nb * k, dtype=np.uint64)
        rco, oo = o.sample(nb, k, 0.4, rnd)
        newp = rng.lognormal(0, 1, nb * k).astype(F32)
        o.update_priorities(oo["key"], newp)
        out3 = g.alloc_sample_outputs(nb, k)
        out3["mass"] = torch.empty(nb * k, dtype=torch.int64, device="cuda:0")
        assert g.sample_begin(nb, k, dev(rnd), out3) == 0
        assert g.sample_finish_writeback(nb, k, 0.4, out3, dev(newp)) == 0
        torch.cuda.synchronize()
        assert_sample_equal(out3, oo)
        check_gpu_tree(g, o)


@pytest.mark.parametrize("m,A", [(512, 18), (96, 1), (3000, 4)])
def test_update_from_learner_q_values(m, A):
    """apex_replay_update_from_q: priorities recomputed from the stored (ret, gacc) and fresh Q-values, in the
    one-workgroup path and in the two-pass path, with repeats and stale keys."""
    rng = np.random.default_rng(17 + m)
    g, o = make_pair(5000, 8192, 16, 4)
    add_both(g, o, rng, 5000)
    add_both(g, o, rng, 2000)
    assert g.evict() == o.evict()                      # keys 0..1999 are stale now
    for it in range(3):
        keys = rng.integers(1500, 7300, m).astype(np.uint64)      # some stale, some not yet added, many repeats
        q_taken = rng.standard_normal(m).astype(F32)
        q_on = np.round(rng.standard_normal((m, A)) * 2).astype(F32) / 2       # ties in the argmax
        q_tg = rng.standard_normal((m, A)).astype(F32)
        rco, p_ref = o.update_from_q(keys, q_taken, q_on, q_tg)
        p_out = torch.empty(m, dtype=torch.float32, device="cuda:0")
        rcg = g.update_from_q(dev(keys), dev(q_taken), dev(q_on), dev(q_tg), p_out)
        assert rcg == rco == 0
        torch.cuda.synchronize()
        assert np.array_equal(host(p_out).view(np.uint32), p_ref.view(np.uint32))
        check_gpu_tree(g, o)
    sample_both(g, o, rng, 2, 128)
