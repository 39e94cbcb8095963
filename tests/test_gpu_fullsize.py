"""GPU parity at the full sizes of the five workloads: the HIP library driven through its C ABI
against the oracle on the same seeded inputs.  Indices, keys, tree sums and eviction are compared
bit for bit at every step; weights to 1e-5 relative / 1e-6 absolute; observation bytes against
their definition as a function of the key (the oracle keeps no 59 GB copy).
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, check_gpu_tree, dev, host

pytestmark = pytest.mark.gpu
F32 = np.float32


class Pair:
    """The device memory and the oracle fed with the same calls."""

    def __init__(self, w):
        from paper_1803_00933_amd import apex
        self.w = w
        self.g = apex.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits)
        self.o = oracle.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits,
                               payload_slots=0)
        self.key0 = 0
        self.round = 0

    def add_round_nstep(self):
        """One round of S x T transitions: n-step priorities on both sides, then add."""
        from paper_1803_00933_amd import apex, synth
        w = self.w
        d = synth.actor_round(w, self.round)
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        rc, prio, ret, gacc, fx = apex.nstep_priorities(dev(d["q_online"]), dev(d["q_target"]), dev(d["action"]),
                                                        dev(d["reward"]), dev(d["discount"]), w.n, w.alpha, w.eps,
                                                        w.frac_bits, w.max_slots)
        assert rc == 0
        obs = synth.obs_rows_torch(w.seed, self.key0, w.add_count, w.obs_bytes, "cuda:0")
        rco, fo = self.o.add(ref[0].reshape(-1))
        rcg, fg = self.g.add(prio.view(-1), obs, dev(d["act"]), ret.view(-1), gacc.view(-1))
        assert (rcg, fg) == (rco, fo) == (0, self.key0)
        if self.round % 16 == 0:
            torch.cuda.synchronize()
            assert np.array_equal(host(fx, np.uint64), ref[3])
            assert np.array_equal(host(prio).view(np.uint32), ref[0].view(np.uint32))
        self.key0 += w.add_count
        self.round += 1

    def add_bulk(self, count, dist, tag_step):
        from paper_1803_00933_amd import synth
        w = self.w
        prio = synth.priorities(dist, w.seed, tag_step, count, tag="bulk")
        obs = synth.obs_rows_torch(w.seed, self.key0, count, w.obs_bytes, "cuda:0")
        assert self.o.add(prio)[0] == 0
        assert self.g.add(dev(prio), obs)[0] == 0
        self.key0 += count

    def evict(self):
        a, b = self.g.evict(), self.o.evict()
        assert a == b
        return a[1]

    def check_obs(self, key, obs_out):
        """Gathered rows are the bytes their keys define."""
        from paper_1803_00933_amd import synth
        w = self.w
        key = np.asarray(key)
        for i in np.linspace(0, len(key) - 1, min(len(key), 24)).astype(int):
            exp = synth.obs_rows(w.seed, int(key[i]), 1, w.obs_bytes)[0]
            assert np.array_equal(host(obs_out[i]), exp), (i, int(key[i]))


def learner_steps(p, steps, nb, beta_of, add_every=0, evict_every=0, add_fn=None, check_obs_every=50):
    """steps x {sample nb x k, update the drawn keys with fresh priorities} with no synchronisation in
    between; every output is kept on the device and compared afterwards."""
    from paper_1803_00933_amd import synth
    w, g, o = p.w, p.g, p.o
    n = nb * w.k
    keys = torch.empty((steps, n), dtype=torch.int64, device="cuda:0")
    slots = torch.empty((steps, n), dtype=torch.int32, device="cuda:0")
    wts = torch.empty((steps, n), dtype=torch.float32, device="cuda:0")
    obs_keep = {}
    ref = []
    scratch_obs = torch.empty((n, w.obs_bytes), dtype=torch.uint8, device="cuda:0")
    scratch_small = g.alloc_sample_outputs(nb, w.k)
    for s in range(steps):
        rnd = synth.uniforms(w.seed, s, nb, w.k).reshape(-1)
        newp = synth.priorities(w.td_dist, w.seed, s, n)
        beta = beta_of(s)
        rco, oo = o.sample(nb, w.k, beta, rnd, payload=False)
        assert rco == 0
        assert o.update_priorities(oo["key"], newp) == 0
        keep = s % check_obs_every == 0
        obs_out = torch.empty_like(scratch_obs) if keep else scratch_obs
        if keep:
            obs_keep[s] = obs_out
        out = dict(key=keys[s], slot=slots[s], weight=wts[s], obs=obs_out, act=scratch_small["act"],
                   ret=scratch_small["ret"], gacc=scratch_small["gacc"])
        assert g.sample(nb, w.k, beta, dev(rnd), out=out)[0] == 0
        assert g.update_priorities(keys[s], dev(newp)) == 0
        ref.append(oo)
        if add_every and (s + 1) % add_every == 0:
            add_fn()
        if evict_every and (s + 1) % evict_every == 0:
            p.evict()
    torch.cuda.synchronize()
    hk, hs, hw = host(keys, np.uint64), host(slots, np.uint32), host(wts)
    for s, oo in enumerate(ref):
        assert np.array_equal(hs[s], oo["slot"]), "slot, step %d" % s
        assert np.array_equal(hk[s], oo["key"]), "key, step %d" % s
        assert_close(hw[s], oo["weight"], "weight, step %d" % s)
    for s, obs_out in obs_keep.items():
        p.check_obs(ref[s]["key"], obs_out)
    return ref


def final_checks(p):
    st = check_gpu_tree(p.g, p.o)
    assert st["size"] == p.o.size
    return st


def test_atari_shape_full_size():
    """2,000,000 transitions of 84x84x4 uint8 (59 GB ring), batch 512, add rounds of 360 x 50."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["atari"]
    p = Pair(w)
    while p.key0 < w.capacity:
        p.add_round_nstep()
    assert p.evict() == p.key0 - w.capacity
    st = final_checks(p)
    assert st["size"] == w.capacity
    learner_steps(p, 200, 1, lambda s: w.beta, add_every=25, evict_every=100, add_fn=p.add_round_nstep)
    final_checks(p)

    # the launch configuration the benchmark times: the library's pipeline, eager and as a replayed graph,
    # in windows of 25 learner steps beside one add round
    depth, steps = 32, 25
    pipe = apex.Pipeline(p.g, depth, 1, w.k)
    first_set = [0]
    rnd = np.stack([synth.uniforms(w.seed, 1000 + s, 1, w.k).reshape(-1) for s in range(steps)])
    newp = np.stack([synth.priorities(w.td_dist, w.seed, 1000 + s, w.k) for s in range(steps)])
    d_rnd, d_newp = dev(rnd), dev(newp)
    d = synth.actor_round(w, 9999)
    dd = {k2: dev(v) for k2, v in d.items()}
    obs = synth.obs_rows_torch(w.seed, 0, w.add_count, w.obs_bytes, "cuda:0")
    scratch = [torch.empty(w.add_count, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    ref_n = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                    w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)

    def cycle():
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              obs, dd["act"], *scratch) == 0
        rc, first_set[0] = pipe.steps(steps, w.beta, d_rnd, d_newp)
        assert rc == 0
        assert pipe.add_end(True)[0] == 0

    def oracle_cycle():
        res = []
        for s in range(steps):
            res.append(p.o.sample(1, w.k, w.beta, rnd[s], payload=False)[1])
            p.o.update_priorities(res[-1]["key"], newp[s])
        assert p.o.add(ref_n[0].reshape(-1))[0] == 0
        p.o.evict()
        return res

    def compare(res):
        for s in range(steps):
            o_, g_ = res[s], pipe.sets[(first_set[0] + s) % depth]
            assert np.array_equal(host(g_["slot"], np.uint32), o_["slot"])
            assert np.array_equal(host(g_["key"], np.uint64), o_["key"])
            assert_close(host(g_["weight"]), o_["weight"], "weight")
            idx = torch.from_numpy(o_["slot"][:32].astype(np.int64)).to("cuda:0")
            assert torch.equal(g_["obs"][:32], p.g.obs_view()[idx])
        # the add round's payload (copied on the second stream) sits in the slots of its keys
        first = p.o.tail - w.add_count
        rows = np.linspace(0, w.add_count - 1, 97).astype(np.int64)
        slots_new = torch.from_numpy((first + rows) % w.max_slots).to("cuda:0")
        rows_t = torch.from_numpy(rows).to("cuda:0")
        assert torch.equal(p.g.obs_view()[slots_new], obs[rows_t])
        assert torch.equal(p.g.act_view()[slots_new], dd["act"][rows_t])
        assert np.array_equal(host(p.g.ret_view()[slots_new]).view(np.uint32), ref_n[1].reshape(-1)[rows].view(np.uint32))

    torch.cuda.synchronize()
    for _ in range(6):                    # 150 learner steps and six add rounds, checked window by window
        assert pipe.fork() == 0
        cycle()
        assert pipe.join() == 0
        torch.cuda.synchronize()
        compare(oracle_cycle())
    final_checks(p)
    assert pipe.capture_begin() == 0
    cycle()
    assert pipe.capture_end() == 0
    for _ in range(3):
        assert pipe.fork() == 0
        assert pipe.replay(1) == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        compare(oracle_cycle())
        assert p.g.resync() == 0
        final_checks(p)
    pipe.close()

    # the paper's prefetch depth as one step: 16 batches of 512 per call, gathers on the copy stream
    nb, calls = 16, 3
    pipe = apex.Pipeline(p.g, 2, nb, w.k)
    rnd16 = np.stack([synth.uniforms(w.seed, 3000 + c, nb, w.k).reshape(-1) for c in range(calls)])
    newp16 = np.stack([synth.priorities(w.td_dist, w.seed, 3000 + c, nb * w.k) for c in range(calls)])
    d_rnd16, d_newp16 = dev(rnd16), dev(newp16)
    torch.cuda.synchronize()
    assert pipe.fork() == 0
    assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                          obs, dd["act"], *scratch) == 0
    for c in range(calls):
        rc, first = pipe.steps(1, w.beta, d_rnd16[c:c + 1], d_newp16[c:c + 1])
        assert rc == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        o_ = p.o.sample(nb, w.k, w.beta, rnd16[c], payload=False)[1]
        p.o.update_priorities(o_["key"], newp16[c])
        g_ = pipe.sets[first]
        assert np.array_equal(host(g_["slot"], np.uint32), o_["slot"])
        assert np.array_equal(host(g_["key"], np.uint64), o_["key"])
        assert_close(host(g_["weight"]), o_["weight"], "weight")
        idx = torch.from_numpy(o_["slot"][::257].astype(np.int64)).to("cuda:0")
        assert torch.equal(g_["obs"][::257], p.g.obs_view()[idx])
        assert pipe.fork() == 0
    assert pipe.add_end(True)[0] == 0
    assert pipe.join() == 0
    assert p.o.add(ref_n[0].reshape(-1))[0] == 0
    p.o.evict()
    final_checks(p)
    pipe.close()


def test_priority_skew_full_size():
    """2^21 slots, Pareto(1.1) priorities with a fifth at zero, 16 prefetched batches of 512 per call,
    beta annealed 0.4 -> 1.0, updates carrying the duplicates the skew produces."""
    from paper_1803_00933_amd import synth
    w = synth.WORKLOADS["skew"]
    p = Pair(w)
    p.add_bulk(w.max_slots, "pareto", 0)
    final_checks(p)
    steps = 1200
    ref = learner_steps(p, steps, w.num_batches, lambda s: 0.4 + 0.6 * s / (steps - 1), check_obs_every=400)
    dup = sum(len(r["key"]) - len(np.unique(r["key"])) for r in ref)
    assert dup > steps          # the skew does make samples collide
    final_checks(p)


def test_continuous_control_shape_full_size():
    """1,000,000 transitions, obs fp32[64], action fp32[8], critic values (A = 1), n = 5, 64 streams x 50."""
    from paper_1803_00933_amd import synth
    w = synth.WORKLOADS["control"]
    p = Pair(w)
    p.add_bulk(w.capacity - 10 * w.add_count, "lognormal1", 0)
    for _ in range(12):
        p.add_round_nstep()
    assert p.evict() == 2 * w.add_count
    learner_steps(p, 300, 1, lambda s: w.beta, add_every=1, evict_every=10, add_fn=p.add_round_nstep)
    final_checks(p)

    # the launch configuration the benchmark times for this shape: the pipeline with an add round (one
    # launch) around every learner step, eviction every 10 rounds; eager, then as a replayed graph
    from paper_1803_00933_amd import apex
    depth, steps = 4, 10
    pipe = apex.Pipeline(p.g, depth, 1, w.k)
    rnd = np.stack([synth.uniforms(w.seed, 2000 + s, 1, w.k).reshape(-1) for s in range(steps)])
    newp = np.stack([synth.priorities(w.td_dist, w.seed, 2000 + s, w.k) for s in range(steps)])
    d_rnd, d_newp = dev(rnd), dev(newp)
    rounds = [synth.actor_round(w, 7000 + i) for i in range(steps)]
    d_rounds = [{k2: dev(v) for k2, v in d.items()} for d in rounds]
    refs_n = [oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots) for d in rounds]
    obs = synth.obs_rows_torch(w.seed, 0, w.add_count, w.obs_bytes, "cuda:0")
    scratch = [torch.empty(w.add_count, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    outs = [{k2: torch.empty_like(v) for k2, v in pipe.sets[0].items() if k2 in ("slot", "key", "weight")}
            for _ in range(steps)]

    def cycle(keep):
        for s in range(steps):
            dd = d_rounds[s]
            assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                                  obs, dd["act"], *scratch) == 0
            rc, first = pipe.steps(1, w.beta, d_rnd[s:s + 1], d_newp[s:s + 1])
            assert rc == 0
            assert pipe.add_end(s == steps - 1)[0] == 0
            if keep:                      # a set is overwritten `depth` steps later: copy it out, in stream order
                assert pipe.join() == 0
                for k2 in outs[s]:
                    outs[s][k2].copy_(pipe.sets[first][k2])
                assert pipe.fork() == 0

    def oracle_cycle():
        res = []
        for s in range(steps):
            res.append(p.o.sample(1, w.k, w.beta, rnd[s], payload=False)[1])
            p.o.update_priorities(res[-1]["key"], newp[s])
            assert p.o.add(refs_n[s][0].reshape(-1))[0] == 0
        p.o.evict()
        return res

    torch.cuda.synchronize()
    assert pipe.fork() == 0
    cycle(keep=True)
    assert pipe.join() == 0
    torch.cuda.synchronize()
    for s, o_ in enumerate(oracle_cycle()):
        assert np.array_equal(host(outs[s]["slot"], np.uint32), o_["slot"]), s
        assert np.array_equal(host(outs[s]["key"], np.uint64), o_["key"]), s
        assert_close(host(outs[s]["weight"]), o_["weight"], "weight")
    final_checks(p)
    assert pipe.capture_begin() == 0
    cycle(keep=False)
    assert pipe.capture_end() == 0
    for _ in range(3):
        assert pipe.fork() == 0
        assert pipe.replay(1) == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        res = oracle_cycle()
        for s in range(steps - depth, steps):
            g_ = pipe.sets[(pipe_first_set(steps, depth, s))]
            assert np.array_equal(host(g_["slot"], np.uint32), res[s]["slot"]), s
            assert_close(host(g_["weight"]), res[s]["weight"], "weight")
        assert p.g.resync() == 0
        final_checks(p)
    pipe.close()


def pipe_first_set(steps, depth, s):
    """The set that step s of the captured cycle fills: the pipeline numbers its steps from its creation, and
    the eager cycle before the capture took `steps` of them."""
    return (steps + s) % depth


def test_scale_stress_full_size():
    """2^24 slots (ring 2^24 + 2^20), batch 4096, 1024 streams x 50 per add round, lognormal(0,2)."""
    from paper_1803_00933_amd import synth
    w = synth.WORKLOADS["scale"]
    p = Pair(w)
    left = w.capacity
    step = 0
    while left > 0:                       # bulk prefill in pieces of 2^21
        cnt = min(left, 1 << 21)
        p.add_bulk(cnt, "lognormal2", step)
        left -= cnt
        step += 1
    st = final_checks(p)
    assert st["size"] == w.capacity
    learner_steps(p, 600, 1, lambda s: w.beta, add_every=8, evict_every=100, add_fn=p.add_round_nstep,
                  check_obs_every=150)
    st = final_checks(p)
    assert st["n_clamped"] == p.o.n_clamped


def test_atari_shape_full_size_through_the_observation_codec():
    """The Atari-shaped memory (2,000,000 rows, 60 GB ring) storing frame-like rows through the block codec:
    filled through the encoder, then the launch configurations the benchmark times on it - pipeline windows of
    25 one-batch steps beside an add round, and calls of 16 batches - against the oracle (indices, keys, weights)
    and against the rows' definition as a function of the key (decoded observations)."""
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["atari"]
    stride = int(apex.lib.apex_codec_row_bytes(w.obs_bytes))
    g = apex.Replay(w.capacity, w.max_slots, stride, w.act_bytes, w.alpha, w.eps, w.frac_bits)
    o = oracle.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits, payload_slots=0)
    key0 = 0
    while key0 < w.capacity:
        prio = synth.priorities("lognormal1", w.seed, key0 // w.add_count, w.add_count, tag="bulk")
        rows = synth.frame_rows_torch(w.seed, key0, w.add_count, w.obs_bytes, "cuda:0")
        assert g.add_payload_encoded(rows) == 0
        assert g.add_publish(dev(prio)) == o.add(prio)
        key0 += w.add_count
    assert g.evict() == o.evict()
    check_gpu_tree(g, o)

    def check_rows(keys, obs_out, n_check=24):
        keys = np.asarray(keys)
        for i in np.linspace(0, len(keys) - 1, min(len(keys), n_check)).astype(int):
            exp = synth.frame_rows(w.seed, int(keys[i]), 1, w.obs_bytes)[0]
            assert np.array_equal(host(obs_out[i]), exp), (i, int(keys[i]))

    d = synth.actor_round(w, 4242)
    dd = {k2: dev(v) for k2, v in d.items()}
    scratch = [torch.empty(w.add_count, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    ref_n = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                    w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)

    # windows of 25 one-batch steps, each beside an add round that is encoded on the copy stream
    depth, steps = 32, 25
    pipe = apex.Pipeline(g, depth, 1, w.k)
    assert pipe.set_codec(w.obs_bytes) == 0
    for window in range(3):
        rnd = np.stack([synth.uniforms(w.seed, 5000 + 100 * window + s, 1, w.k).reshape(-1) for s in range(steps)])
        newp = np.stack([synth.priorities(w.td_dist, w.seed, 5000 + 100 * window + s, w.k) for s in range(steps)])
        d_rnd, d_newp = dev(rnd), dev(newp)
        rows = synth.frame_rows_torch(w.seed, key0, w.add_count, w.obs_bytes, "cuda:0")
        assert pipe.fork() == 0
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              rows, dd["act"], *scratch) == 0
        rc, first = pipe.steps(steps, w.beta, d_rnd, d_newp)
        assert rc == 0
        rc, first_key, ev = pipe.add_end(True)
        assert pipe.join() == 0
        res = []
        for s in range(steps):
            res.append(o.sample(1, w.k, w.beta, rnd[s], payload=False)[1])
            o.update_priorities(res[-1]["key"], newp[s])
        assert (rc, first_key) == o.add(ref_n[0].reshape(-1)) == (0, key0)
        assert o.evict() == (0, ev)
        key0 += w.add_count
        torch.cuda.synchronize()
        for s in range(steps):
            o_, g_ = res[s], pipe.sets[(first + s) % depth]
            assert np.array_equal(host(g_["slot"], np.uint32), o_["slot"])
            assert np.array_equal(host(g_["key"], np.uint64), o_["key"])
            assert_close(host(g_["weight"]), o_["weight"], "weight")
            check_rows(o_["key"], g_["obs"], 6)
        check_gpu_tree(g, o)
    # the round added by the last window is sampled from as well: its rows went through the encoder on the copy stream
    pipe.close()

    # calls of 16 batches: fetched through the decoder on the copy stream
    nb = 16
    pipe = apex.Pipeline(g, 2, nb, w.k)
    assert pipe.set_codec(w.obs_bytes) == 0
    for call in range(2):
        rnd = synth.uniforms(w.seed, 7000 + call, nb, w.k).reshape(-1)
        newp = synth.priorities(w.td_dist, w.seed, 7000 + call, nb * w.k)
        d_rnd, d_newp = dev(rnd[None]), dev(newp[None])
        assert pipe.fork() == 0
        rc, first = pipe.steps(1, w.beta, d_rnd, d_newp)
        assert rc == 0 and pipe.join() == 0
        oo = o.sample(nb, w.k, w.beta, rnd, payload=False)[1]
        o.update_priorities(oo["key"], newp)
        torch.cuda.synchronize()
        g_ = pipe.sets[first]
        assert np.array_equal(host(g_["slot"], np.uint32), oo["slot"])
        assert np.array_equal(host(g_["key"], np.uint64), oo["key"])
        assert_close(host(g_["weight"]), oo["weight"], "weight")
        check_rows(oo["key"], g_["obs"], 48)
    check_gpu_tree(g, o)
    pipe.close()
