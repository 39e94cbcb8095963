"""GPU parity at the full sizes of the five workloads and over their full schedules: the HIP library
driven through its C ABI against the oracle on the same seeded inputs.  Indices, keys, tree sums and
eviction are compared bit for bit at every step; weights to 1e-5 relative / 1e-6 absolute; gathered
observation rows, every row of a batch, against their definition as a function of the oracle's key (the
oracle keeps no 59 GB copy; the rows are regenerated on the device from the keys it drew).
APEX_TEST_SCHEDULE=short in the environment cuts the two long schedules (skew: 10,000 steps, scale: 5,000
steps) to a tenth; the default runs them whole.
"""
import os

import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_close, check_gpu_tree, dev, host

pytestmark = pytest.mark.gpu
F32 = np.float32
SHORT = os.environ.get("APEX_TEST_SCHEDULE", "") == "short"


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
        self.rounds_from = None

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

    def content_keys(self, key):
        """The key whose bytes a stored row holds.  Rows added through this class hold the bytes of their own key;
        rounds_from names the first key of a run of add rounds that all carried the rows of keys 0 .. add_count-1
        (the staging buffer that the pipeline tests re-use)."""
        key = np.asarray(key).astype(np.uint64)
        if self.rounds_from is None:
            return key
        late = key >= np.uint64(self.rounds_from)
        return np.where(late, (key - np.uint64(self.rounds_from)) % np.uint64(self.w.add_count), key)

    def check_obs(self, key, obs_out):
        """Every gathered row is the bytes that its key - the oracle's - defines; compared on the device."""
        from paper_1803_00933_amd import synth
        w = self.w
        key = self.content_keys(key)
        assert obs_out.shape[0] == len(key)
        for lo in range(0, len(key), 2048):                  # 2048 frame stacks = 58 MB of expected bytes at a time
            exp = synth.obs_rows_for_keys_torch(w.seed, key[lo:lo + 2048], w.obs_bytes, "cuda:0")
            if not torch.equal(obs_out[lo:lo + 2048], exp):
                bad = (obs_out[lo:lo + 2048] != exp).any(dim=1).nonzero().reshape(-1)
                raise AssertionError("gathered rows differ from their keys' bytes: rows %s of %d"
                                     % ((bad[:8] + lo).tolist(), len(key)))


def learner_steps(p, steps, nb, beta_of, add_every=0, evict_every=0, add_fn=None, check_obs_every=50, chunk=500):
    """steps x {sample nb x k, update the drawn keys with fresh priorities} with no synchronisation inside a
    chunk of steps; every output is kept on the device and compared when the chunk is done (slots, keys, weights
    of every step; every gathered row of every check_obs_every-th step).  Returns the number of samples that drew
    a transition already drawn in the same call."""
    from paper_1803_00933_amd import synth
    w, g, o = p.w, p.g, p.o
    n = nb * w.k
    chunk = min(chunk, steps)
    keys = torch.empty((chunk, n), dtype=torch.int64, device="cuda:0")
    slots = torch.empty((chunk, n), dtype=torch.int32, device="cuda:0")
    wts = torch.empty((chunk, n), dtype=torch.float32, device="cuda:0")
    scratch_obs = torch.empty((n, w.obs_bytes), dtype=torch.uint8, device="cuda:0")
    scratch_small = g.alloc_sample_outputs(nb, w.k)
    dup = 0
    for c0 in range(0, steps, chunk):
        obs_keep, ref = {}, []
        for s in range(c0, min(c0 + chunk, steps)):
            i = s - c0
            rnd = synth.uniforms(w.seed, s, nb, w.k).reshape(-1)
            newp = synth.priorities(w.td_dist, w.seed, s, n)
            beta = beta_of(s)
            rco, oo = o.sample(nb, w.k, beta, rnd, payload=False)
            assert rco == 0
            assert o.update_priorities(oo["key"], newp) == 0
            keep = s % check_obs_every == 0
            obs_out = torch.empty_like(scratch_obs) if keep else scratch_obs
            if keep:
                obs_keep[i] = obs_out
            out = dict(key=keys[i], slot=slots[i], weight=wts[i], obs=obs_out, act=scratch_small["act"],
                       ret=scratch_small["ret"], gacc=scratch_small["gacc"])
            assert g.sample(nb, w.k, beta, dev(rnd), out=out)[0] == 0
            assert g.update_priorities(keys[i], dev(newp)) == 0
            ref.append(oo)
            if add_every and (s + 1) % add_every == 0:
                add_fn()
            if evict_every and (s + 1) % evict_every == 0:
                p.evict()
        torch.cuda.synchronize()
        hk, hs, hw = host(keys, np.uint64), host(slots, np.uint32), host(wts)
        for i, oo in enumerate(ref):
            assert np.array_equal(hs[i], oo["slot"]), "slot, step %d" % (c0 + i)
            assert np.array_equal(hk[i], oo["key"]), "key, step %d" % (c0 + i)
            assert_close(hw[i], oo["weight"], "weight, step %d" % (c0 + i))
            dup += len(oo["key"]) - len(np.unique(oo["key"]))
        for i, obs_out in obs_keep.items():
            p.check_obs(ref[i]["key"], obs_out)
        print("  steps %d..%d of %d checked" % (c0, c0 + len(ref) - 1, steps), flush=True)
    return dup


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
            if s % 6 == 0:                # all 512 rows of every sixth batch of the window
                p.check_obs(o_["key"], g_["obs"])
        # the add round's payload (copied on the second stream) sits in the slots of its keys
        first = p.o.tail - w.add_count
        rows = np.linspace(0, w.add_count - 1, 97).astype(np.int64)
        slots_new = torch.from_numpy((first + rows) % w.max_slots).to("cuda:0")
        rows_t = torch.from_numpy(rows).to("cuda:0")
        assert torch.equal(p.g.obs_view()[slots_new], obs[rows_t])
        assert torch.equal(p.g.act_view()[slots_new], dd["act"][rows_t])
        assert np.array_equal(host(p.g.ret_view()[slots_new]).view(np.uint32), ref_n[1].reshape(-1)[rows].view(np.uint32))

    p.rounds_from = p.key0                # every round from here on carries the rows of keys 0 .. add_count-1
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
        p.check_obs(o_["key"], g_["obs"])   # all 8192 rows of the call
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
    steps = 1000 if SHORT else 10_000
    dup = learner_steps(p, steps, w.num_batches, lambda s: 0.4 + 0.6 * s / (steps - 1), check_obs_every=400)
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
    steps = 500 if SHORT else 5000        # an add round of 51,200 every 8 steps: 625 rounds = 32,000,000 more
    learner_steps(p, steps, 1, lambda s: w.beta, add_every=8, evict_every=100, add_fn=p.add_round_nstep,
                  check_obs_every=150)    # transitions, 1.9 x the capacity on top of the prefill
    st = final_checks(p)
    assert st["n_clamped"] == p.o.n_clamped
    if not SHORT:
        assert st["tail"] == w.capacity + 625 * w.add_count and st["tail"] > 2 * w.max_slots   # the ring wrapped twice
        assert st["head"] == st["tail"] - w.capacity - (steps % 100) // 8 * w.add_count


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

    def check_rows(keys, obs_out):
        """Every decoded row is the frame-like row that its key - the oracle's - defines."""
        keys = np.asarray(keys)
        for lo in range(0, len(keys), 2048):
            exp = synth.frame_rows_for_keys_torch(w.seed, keys[lo:lo + 2048], w.obs_bytes, "cuda:0")
            assert torch.equal(obs_out[lo:lo + 2048], exp), "decoded rows %d.. differ from their keys' bytes" % lo

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
            if s % 6 == 0:
                check_rows(o_["key"], g_["obs"])
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
        check_rows(oo["key"], g_["obs"])
    check_gpu_tree(g, o)
    pipe.close()
