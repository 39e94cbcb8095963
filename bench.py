#!/usr/bin/env python3
"""Throughput of the replay hot path on one MI355X, Atari-shaped workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one learner step of the paper's Atari setting (Section 4.1) served from a memory of
2,000,000 transitions of 84x84x4 uint8 frames: sample a prioritized batch of 512 (stratified
descent, importance weights, gather of the frame stacks) and write 512 new priorities back.
The actors' side runs inside the timed region at the paper's ratio: every 25 steps one round of
360 streams x 50 transitions goes through n-step priorities and add (about 12.5K inserts per
19 learner steps), and every 100 steps the excess above 2M is evicted, oldest first.
All inputs are synthetic, seeded, and resident in HBM before the clock starts.

Prints one JSON line (see the keys at the bottom).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
ADD_EVERY, EVICT_EVERY = 25, 100

# One byte model for every HBM fraction in the output line: what the method itself has to move per sampled
# transition of this workload -- gather read + write 2 * (28,224 + 4 + 8), sample outputs and uniform 24,
# descent reads 8 * 21, update read-modify-writes 16 * 22 + 12 = 57,030 B -- times the batch of 512.
STEP_ALGORITHMIC_BYTES = 512 * 57030

# HBM traffic of one launch of the learner-step kernel as the hardware counters saw it.  A RECORDED figure, not
# measured by this run: two `rocprofv3 --pmc` runs of this script (FETCH_SIZE, then WRITE_SIZE; KiB per
# dispatch, averaged over the kernel's dispatches), each scaled by what the same counter reads for the plain
# 508,032,000-byte payload copy of an add round in the same run (FETCH_SIZE: 248,074.09 KiB for 496,125 KiB
# read, factor 1.9999; WRITE_SIZE: factor 1.0).  Source: profiles/learner_step_atari_hbm_traffic.txt.
RECORDED_STEP_TRAFFIC = {
    "fetch_kib_per_dispatch": 7647.976, "fetch_scale": 496125.0 / 248074.09,
    "write_kib_per_dispatch": 14321.975, "write_scale": 1.0,
    "source": "profiles/learner_step_atari_hbm_traffic.txt (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, recorded; "
              "not re-measured by this run)",
}
RECORDED_STEP_TRAFFIC_BYTES = int((RECORDED_STEP_TRAFFIC["fetch_kib_per_dispatch"] * RECORDED_STEP_TRAFFIC["fetch_scale"]
                                   + RECORDED_STEP_TRAFFIC["write_kib_per_dispatch"]
                                   * RECORDED_STEP_TRAFFIC["write_scale"]) * 1024)


def normalise_steps(steps, warmup):
    """(K, W) that are actually run for the requested --steps / --warmup.

    The timed schedule is periodic in EVICT_EVERY learner steps (four add rounds and one eviction, after which
    the memory is back at its capacity), and the graph-replay variant records exactly one such cycle, so both
    counts are rounded UP to whole cycles: 20 -> 100, 5 -> 100, 2000 -> 2000, 0 warm-up steps stay 0."""
    if steps < 1 or warmup < 0:
        raise ValueError("--steps must be >= 1 and --warmup >= 0")
    up = lambda v: -(-v // EVICT_EVERY) * EVICT_EVERY
    return up(steps), up(warmup)


def host_cpu():
    """(model name, logical cores) of the machine this runs on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model, os.cpu_count()


def dev(a):
    import torch
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).to("cuda:0")


class GpuJob:
    """The device-resident replay memory plus every pre-generated input of the timed loop."""

    def __init__(self, w, steps_total, log):
        import torch
        from paper_1803_00933_amd import apex, synth
        self.torch, self.apex, self.synth, self.w = torch, apex, synth, w
        self.rep = apex.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits)
        self.n_pool = 4
        self.rounds = []
        for i in range(self.n_pool):
            d = synth.actor_round(w, i)
            t = {k: dev(v) for k, v in d.items()}
            S, T = w.streams, w.chunk
            t["out"] = (torch.empty((S, T), dtype=torch.float32, device="cuda:0"),
                        torch.empty((S, T), dtype=torch.float32, device="cuda:0"),
                        torch.empty((S, T), dtype=torch.float32, device="cuda:0"), None)
            self.rounds.append(t)
        self.obs_stage = torch.empty((w.add_count, w.obs_bytes), dtype=torch.uint8, device="cuda:0")
        self.step = 0
        self.key0 = 0
        # prefill to capacity with hashed frame bytes, then trim
        t0 = time.time()
        n_fill = -(-w.capacity // w.add_count)
        for i in range(n_fill):
            self.obs_stage.copy_(synth.obs_rows_torch(w.seed, self.key0, w.add_count, w.obs_bytes, "cuda:0"))
            self.add_round(i)
        rc, e = self.rep.evict()
        assert rc == 0
        torch.cuda.synchronize()
        st = self.rep.stats()
        assert st["size"] == w.capacity, st
        log("prefill: %d rounds, %.1f s, size %d, root %d" % (n_fill, time.time() - t0, st["size"], st["root"]))
        # learner inputs for every step
        n = steps_total
        self.rnd = dev(np.concatenate([synth.uniforms(w.seed, s, 1, w.k) for s in range(n)]))
        self.td = dev(np.stack([synth.priorities(w.td_dist, w.seed, s, w.k) for s in range(n)]))
        self.outs = [self.rep.alloc_sample_outputs(1, w.k) for _ in range(4)]
        # raw argument lists per step: the timed loop only marshals integers into the C ABI
        self.stream = torch.cuda.current_stream().cuda_stream
        self.sample_args, self.update_args = [], []
        for s in range(n):
            o = self.outs[s % len(self.outs)]
            self.sample_args.append((self.rep.h, 1, w.k, w.beta, self.rnd[s].data_ptr(), o["key"].data_ptr(),
                                     o["slot"].data_ptr(), o["weight"].data_ptr(), o["obs"].data_ptr(),
                                     o["act"].data_ptr(), o["ret"].data_ptr(), o["gacc"].data_ptr(), self.stream))
            self.update_args.append((self.rep.h, w.k, o["key"].data_ptr(), self.td[s].data_ptr(), self.stream))

    def add_round(self, i):
        w, apex = self.w, self.apex
        t = self.rounds[i % self.n_pool]
        rc, prio, ret, gacc, _ = apex.nstep_priorities(t["q_online"], t["q_target"], t["action"], t["reward"],
                                                       t["discount"], w.n, w.alpha, w.eps, w.frac_bits, w.max_slots,
                                                       want_fx=False, out=t["out"])
        assert rc == 0
        rc, first = self.rep.add(prio.view(-1), self.obs_stage, t["act"], ret.view(-1), gacc.view(-1))
        assert rc == 0, rc
        self.key0 += w.add_count

    def learner_step(self, s):
        lib = self.apex.lib
        rc = lib.apex_replay_sample(*self.sample_args[s])
        assert rc == 0, rc
        rc = lib.apex_replay_update_priorities(*self.update_args[s])
        assert rc == 0, rc

    def run(self, first, count, with_actors=True):
        """Everything on one stream, one call after the other."""
        for s in range(first, first + count):
            self.learner_step(s)
            if with_actors:
                if (s + 1) % ADD_EVERY == 0:
                    self.add_round(s // ADD_EVERY)
                if (s + 1) % EVICT_EVERY == 0:
                    rc, e = self.rep.evict()
                    assert rc == 0

    # -- the library's prefetch pipeline: learner steps on one stream, add payloads on a second ----
    def setup_pipeline(self):
        self.pipe = self.apex.Pipeline(self.rep, 8, 1, self.w.k)

    def issue_windows(self, first, count, in_place=False):
        """Same order of tree operations as run(): draw s, update s, [publish the add round], [evict].
        in_place: the observations of the add rounds are not copied (a producer is taken to have written
        them into the ring itself; the other columns and the priorities are handled as usual)."""
        w, pipe = self.w, self.pipe
        assert first % ADD_EVERY == 0 and count % ADD_EVERY == 0
        for f in range(first, first + count, ADD_EVERY):
            t = self.rounds[(f // ADD_EVERY) % self.n_pool]
            prio, ret, gacc, _ = t["out"]
            rc = pipe.add_begin(t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n,
                                None if in_place else self.obs_stage, t["act"], prio, ret, gacc)
            assert rc == 0, rc
            rc, _ = pipe.steps(ADD_EVERY, w.beta, self.rnd[f:f + ADD_EVERY], self.td[f:f + ADD_EVERY])
            assert rc == 0, rc
            rc, _, _ = pipe.add_end(evict=(f + ADD_EVERY) % EVICT_EVERY == 0)
            assert rc == 0, rc

    def run_pipelined_learner_only(self, first, count):
        assert self.pipe.fork() == 0
        rc, _ = self.pipe.steps(count, self.w.beta, self.rnd[first:first + count], self.td[first:first + count])
        assert rc == 0, rc
        assert self.pipe.join() == 0

    def prefetch16_us_per_batch(self, batches, with_actors):
        """The paper's prefetch depth as the unit of work: 16 batches of 512 drawn per call from one state of
        the memory, gathered on the copy stream while the priorities are written back on the tree stream.  With the actors' side:
        the same insert rate (one add round per 25 batches) and eviction every 100 batches."""
        torch, w = self.torch, self.w
        nb = 16
        calls = batches // nb
        pipe = self.apex.Pipeline(self.rep, 2, nb, w.k)
        rnd = self.rnd[:calls * nb].reshape(calls, nb * w.k)
        td = self.td[:calls * nb].reshape(calls, nb * w.k)

        def go(n_calls):
            assert pipe.fork() == 0
            for c in range(n_calls):
                done, due = c * nb // ADD_EVERY, (c + 1) * nb // ADD_EVERY
                if with_actors and due > done:
                    t = self.rounds[done % self.n_pool]
                    prio, ret, gacc, _ = t["out"]
                    assert pipe.add_begin(t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n,
                                          self.obs_stage, t["act"], prio, ret, gacc) == 0
                assert pipe.steps(1, w.beta, rnd[c], td[c])[0] == 0
                if with_actors and due > done:
                    evict = (c + 1) * nb // EVICT_EVERY > c * nb // EVICT_EVERY
                    assert pipe.add_end(evict)[0] == 0
            assert pipe.join() == 0
            if with_actors:                      # leave the memory at its capacity
                assert self.rep.evict(stream=torch.cuda.current_stream())[0] == 0
        go(min(calls, 8))
        dt, _ = self.timed(lambda: go(calls))
        pipe.close()
        return dt / (calls * nb) * 1e6

    def run_pipelined(self, first, count, in_place=False):
        assert self.pipe.fork() == 0
        self.issue_windows(first, count, in_place)
        assert self.pipe.join() == 0

    def capture_cycle(self, first):
        """One EVICT_EVERY-step cycle recorded as a HIP graph; replays re-use its uniforms and TD errors."""
        assert self.pipe.capture_begin() == 0
        self.issue_windows(first, EVICT_EVERY)
        assert self.pipe.capture_end() == 0

    def run_replays(self, reps):
        assert self.pipe.fork() == 0
        assert self.pipe.replay(reps) == 0
        assert self.pipe.join() == 0

    def timed(self, fn):
        torch = self.torch
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        return time.perf_counter() - t0, t_host

    def timed_median(self, fn, reps=5):
        """(median wall time, its host-enqueue time, all wall times) over `reps` runs of fn."""
        runs = sorted(self.timed(fn) for _ in range(reps))
        return runs[reps // 2][0], runs[reps // 2][1], [r[0] for r in runs]

    def step_kernel_us(self, first, count):
        """Average time per launch of the dominant kernel as it runs in the timed loop: the learner-step launch
        (gather of the 512 frame stacks of one batch, its importance weights, the write-back of its priorities
        and the draw of the next batch).  `count` launches back to back on the pipeline's stream, every one
        with other rows (nothing is served from the 256 MB memory-side cache); HIP events on the stream that
        the pipeline's stream is forked from and joined to, so the figure contains the gaps between the
        launches and, once per `count` launches, the standalone first draw."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        self.run_pipelined_learner_only(first, count)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / count * 1e3


def op_timings(job):
    """Device time of the other steps of the path on their own, microseconds (HIP events on the launch
    stream; repeated launches are captured once and replayed so that host launch cost stays out)."""
    torch, w, rep, apex = job.torch, job.w, job.rep, job.apex

    def replayed(fn, n=32, replays=4):
        s = torch.cuda.Stream()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            for i in range(n):
                fn(i)
        g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (n * replays) * 1e3

    out = {}
    t = job.rounds[0]
    out["nstep_priorities_18000"] = replayed(lambda i: apex.nstep_priorities(
        t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n, w.alpha, w.eps, w.frac_bits,
        w.max_slots, want_fx=False, out=t["out"]))
    o = job.outs[0]
    o["mass"] = torch.empty(w.k, dtype=torch.int64, device="cuda:0")
    out["descent_512"] = replayed(lambda i: rep.sample_begin(1, w.k, job.rnd[i], o))
    out["update_512"] = replayed(lambda i: rep.update_priorities(o["key"], job.td[i]))

    def plain_step(i):                       # the plain verbs, one learner step: three launches
        oo = job.outs[i % len(job.outs)]
        assert rep.sample(1, w.k, w.beta, job.rnd[i], out=oo)[0] == 0
        assert rep.update_priorities(oo["key"], job.td[i]) == 0

    out["plain_sample_plus_update_512"] = replayed(plain_step)
    # add rounds and the eviction that follows them change the size of the memory: timed once, eagerly
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    torch.cuda.synchronize()
    ev[0].record()
    n_add = EVICT_EVERY // ADD_EVERY
    for i in range(n_add):
        job.add_round(i)
    ev[1].record()
    rc, e = rep.evict()
    ev[2].record()
    torch.cuda.synchronize()
    assert rc == 0 and e == n_add * w.add_count
    out["add_round_18000_incl_nstep"] = ev[0].elapsed_time(ev[1]) / n_add * 1e3
    out["evict_%d" % e] = ev[1].elapsed_time(ev[2]) * 1e3
    # the payload copy of an add round alone (rows into free ring slots; nothing is published)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for i in range(n_add):
        assert rep.add_payload(w.add_count, job.obs_stage) == 0
    ev[1].record()
    torch.cuda.synchronize()
    out["add_payload_18000"] = ev[0].elapsed_time(ev[1]) / n_add * 1e3
    out["add_payload_GBps"] = 2 * w.add_count * w.obs_bytes / (out["add_payload_18000"] * 1e-6) / 1e9
    return out


def control_numbers(log, steps=1000):
    """The continuous-control-shaped workload (Section 4.2, Appendix D): 1,000,000 transitions of fp32[64]
    observations and fp32[8] actions, n = 5, critic values as the only "action" column; every learner step
    is preceded by an add round of 64 streams x 50 transitions, the excess is evicted every 10 rounds."""
    import torch
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["control"]
    rep = apex.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits)
    rounds = [{k: dev(v) for k, v in synth.actor_round(w, i).items()} for i in range(4)]
    obs = synth.obs_rows_torch(w.seed, 0, w.add_count, w.obs_bytes, "cuda:0")
    scratch = [torch.empty(w.add_count, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    pipe = apex.Pipeline(rep, 8, 1, w.k)

    def add_begin(i):
        t = rounds[i % 4]
        assert pipe.add_begin(t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n, obs,
                              t["act"], *scratch) == 0

    assert pipe.fork() == 0
    for i in range(w.capacity // w.add_count + 1):
        add_begin(i)
        assert pipe.add_end(True)[0] == 0
    assert pipe.join() == 0
    torch.cuda.synchronize()
    assert rep.stats()["size"] == w.capacity
    rnd = dev(np.concatenate([synth.uniforms(w.seed, s, 1, w.k) for s in range(steps)]))
    td = dev(np.stack([synth.priorities(w.td_dist, w.seed, s, w.k) for s in range(steps)]))

    def timed(fn):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e6

    def full():
        assert pipe.fork() == 0
        for s in range(steps):
            add_begin(s)
            assert pipe.steps(1, w.beta, rnd[s:s + 1], td[s:s + 1])[0] == 0
            assert pipe.add_end((s + 1) % 10 == 0)[0] == 0
        assert pipe.join() == 0

    def learner_only():
        assert pipe.fork() == 0
        assert pipe.steps(steps, w.beta, rnd, td)[0] == 0
        assert pipe.join() == 0

    full()
    us_eager = min(timed(full) for _ in range(2))
    # ten steps (one eviction cycle) recorded as a HIP graph and replayed: the eager loop above is bound by
    # the three Python calls per step, not by the device
    assert pipe.capture_begin() == 0
    for s in range(10):
        add_begin(s)
        assert pipe.steps(1, w.beta, rnd[s:s + 1], td[s:s + 1])[0] == 0
        assert pipe.add_end(s == 9)[0] == 0
    assert pipe.capture_end() == 0

    def replays():
        assert pipe.fork() == 0
        assert pipe.replay(steps // 10) == 0
        assert pipe.join() == 0

    replays()
    us_graph = min(timed(replays) for _ in range(2))
    assert rep.resync() == 0
    us_full = min(us_eager, us_graph)
    learner_only()
    us_learner = min(timed(learner_only) for _ in range(2))
    assert rep.stats()["size"] <= w.capacity + 10 * w.add_count
    pipe.close()
    log("control shape: %.2f us/step eager, %.2f as graph replays, with an add round of %d before every step; "
        "%.2f us/step learner only" % (us_eager, us_graph, w.add_count, us_learner))
    return {"workload": "control: capacity 1,000,000 (ring 2^20) x fp32[64] obs + fp32[8] action, n=5, batch 512; "
                        "add round of 64x50 before every learner step, FIFO evict every 10 rounds",
            "us_per_step": us_full, "us_per_step_eager": us_eager, "us_per_step_graph_replays": us_graph,
            "sampled_transitions_per_s": w.k / (us_full * 1e-6),
            "adds_per_s": w.add_count / (us_full * 1e-6),
            "learner_only_us_per_step": us_learner,
            "learner_only_sampled_transitions_per_s": w.k / (us_learner * 1e-6)}


def tree_bound_workloads(log, calls=300):
    """The two tree-bound stress shapes (small rows, so the descent and the updates dominate): `skew` draws 16
    batches of 512 per call from 2^21 Pareto-distributed priorities and writes all 8192 back, duplicates
    included; `scale` draws one batch of 4096 from 2^24 transitions.  Learner calls only, through the
    pipeline; microseconds per call."""
    import torch
    from paper_1803_00933_amd import apex, synth
    out = {}
    for name, dist in (("skew", "pareto"), ("scale", "lognormal2")):
        w = synth.WORKLOADS[name]
        rep = apex.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits)
        left, piece = w.capacity, 0
        while left > 0:
            cnt = min(left, 1 << 21)
            prio = dev(synth.priorities(dist, w.seed, piece, cnt, tag="bulk"))
            obs = torch.zeros((cnt, w.obs_bytes), dtype=torch.uint8, device="cuda:0")
            assert rep.add(prio, obs)[0] == 0
            left -= cnt
            piece += 1
        nb, per = w.num_batches, w.num_batches * w.k
        pipe = apex.Pipeline(rep, 4, nb, w.k)
        rnd = dev(np.stack([synth.uniforms(w.seed, c, nb, w.k).reshape(-1) for c in range(calls)]))
        td = dev(np.stack([synth.priorities(dist, w.seed, c, per) for c in range(calls)]))

        def go():
            assert pipe.fork() == 0
            assert pipe.steps(calls, w.beta, rnd, td)[0] == 0
            assert pipe.join() == 0

        go()
        best = 1e30
        for _ in range(2):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            go()
            torch.cuda.synchronize()
            best = min(best, (time.perf_counter() - t0) / calls * 1e6)
        pipe.close()
        out[name] = {"samples_per_call": per, "us_per_call": best, "sampled_transitions_per_s": per / (best * 1e-6)}
        log("%s shape: %d samples per call, %.2f us per call (draw + weights + gather + update)" % (name, per, best))
        del pipe, rep, rnd, td
        torch.cuda.empty_cache()
    return out


def next_row_numbers(log):
    """The two library features beyond the headline path, each timed on its own: learner-side priorities from
    fresh Q-values fused into the write-back (Algorithm 2, ComputePriorities + SetPriority), and the memory with
    prioritized eviction of the continuous-control variant (Appendix D: eviction by sampling with exponent -0.4)."""
    import torch
    from paper_1803_00933_amd import apex, synth
    out = {}
    rng = np.random.default_rng(5)
    # --- priorities from Q-values, 512 pairs with 18 actions, on the Atari-shaped tree (payload rows of 16 bytes)
    w = synth.WORKLOADS["atari"]
    rep = apex.Replay(w.capacity, w.max_slots, 16, w.act_bytes, w.alpha, w.eps, w.frac_bits)
    for piece in range(8):
        cnt = w.capacity // 8
        prio = dev(synth.priorities("lognormal1", w.seed, piece, cnt, tag="bulk"))
        assert rep.add(prio, torch.zeros((cnt, 16), dtype=torch.uint8, device="cuda:0"), None,
                       torch.zeros(cnt, device="cuda:0"), torch.full((cnt,), 0.97, device="cuda:0"))[0] == 0
    o = rep.alloc_sample_outputs(1, w.k)
    assert rep.sample(1, w.k, w.beta, dev(synth.uniforms(w.seed, 0, 1, w.k).reshape(-1)), out=o)[0] == 0
    q_taken = torch.randn(w.k, device="cuda:0")
    q_on, q_tg = torch.randn((w.k, w.num_actions), device="cuda:0"), torch.randn((w.k, w.num_actions), device="cuda:0")
    n = 200
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=stream):          # launches recorded once: host launch cost stays out
        for _ in range(32):
            assert rep.update_from_q(o["key"], q_taken, q_on, q_tg) == 0
    graph.replay()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    torch.cuda.synchronize()
    ev[0].record()
    for _ in range(4):
        graph.replay()
    ev[1].record()
    torch.cuda.synchronize()
    out["update_from_q_512x18_us"] = ev[0].elapsed_time(ev[1]) / (32 * 4) * 1e3
    del graph, rep
    # --- prioritized eviction, control shape: 32,000 of 1,032,000 transitions in 5 rounds
    w = synth.WORKLOADS["control"]
    g = apex.PeReplay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes)
    assert g.add(dev(synth.priorities("lognormal1", 0, 0, w.capacity, tag="bulk"))) == 0
    times = []
    for r in range(3):
        for i in range(10):
            assert g.add(dev(synth.priorities("lognormal1", 0, 1 + i + 10 * r, w.add_count, tag="bulk"))) == 0
        e = 10 * w.add_count
        rnd = dev(rng.integers(0, 1 << 64, (5, e), dtype=np.uint64))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        rc, evicted = g.evict(5, rnd)
        times.append((time.perf_counter() - t0) * 1e6)
        assert rc == 0 and evicted == e, (rc, evicted)
    out["prioritized_evict_32000_of_1032000_us"] = min(times)
    rnds = dev(rng.integers(0, 1 << 64, (n, w.k), dtype=np.uint64))
    td = torch.rand((n, w.k), device="cuda:0")
    so = g.alloc_sample_outputs(1, w.k)
    for rep_i in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n):
            g.sample(1, w.k, 0.4, rnds[i], out=so)
            g.update_priorities(so["key"], td[i])
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / n * 1e6
    out["prioritized_evict_memory_sample_update_us"] = dt
    # the whole control-shaped schedule on this memory, as Appendix D runs it: an add round of 64 x 50 before
    # every learner step, and every 10 rounds the excess of 32,000 evicted by priority in 5 rounds
    rounds_in = [{k2: dev(v) for k2, v in synth.actor_round(w, i).items()} for i in range(4)]
    obs = synth.obs_rows_torch(w.seed, 0, w.add_count, w.obs_bytes, "cuda:0")
    outs = [torch.empty((w.streams, w.chunk), dtype=torch.float32, device="cuda:0") for _ in range(3)] + [None]
    rnd_ev = dev(rng.integers(0, 1 << 64, (5, 10 * w.add_count), dtype=np.uint64))
    steps = 100

    def schedule():
        for s in range(steps):
            t = rounds_in[s % 4]
            rc, prio, ret, gacc, _ = apex.nstep_priorities(t["q_online"], t["q_target"], t["action"], t["reward"],
                                                           t["discount"], w.n, w.alpha, w.eps, w.frac_bits, w.max_slots,
                                                           want_fx=False, out=outs)
            assert rc == 0 and g.add(prio.view(-1), obs, t["act"], ret.view(-1), gacc.view(-1)) == 0
            g.sample(1, w.k, 0.4, rnds[s], out=so)
            g.update_priorities(so["key"], td[s])
            if (s + 1) % 10 == 0:
                rc, evicted = g.evict(5, rnd_ev)
                assert rc == 0 and evicted == 10 * w.add_count, (rc, evicted)

    for rep_i in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        schedule()
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps * 1e6
    out["prioritized_evict_memory_control_schedule_plain_calls_us_per_step"] = dt

    # the same schedule through the calls that keep the host out of the loop: an actor round as one launch, a
    # learner step as two, the eviction enqueued (its count confirmed later from a snapshot)
    # (argument lists made beforehand: the timed loop only marshals integers into the C ABI)
    stream = torch.cuda.current_stream().cuda_stream
    round_args = [(g.h, w.streams, w.chunk, w.n, w.num_actions, t["q_online"].data_ptr(), t["q_target"].data_ptr(),
                   t["action"].data_ptr(), t["reward"].data_ptr(), t["discount"].data_ptr(), obs.data_ptr(),
                   t["act"].data_ptr(), stream) for t in rounds_in]
    step_args = [(g.h, w.k, 0.4, rnds[i].data_ptr(), td[i].data_ptr(), so["key"].data_ptr(), so["slot"].data_ptr(),
                  so["weight"].data_ptr(), so["obs"].data_ptr(), so["act"].data_ptr(), so["ret"].data_ptr(),
                  so["gacc"].data_ptr(), stream) for i in range(n)]
    lib = apex.lib

    def schedule_fused(n_steps):
        for s in range(n_steps):
            assert lib.apex_pe_add_round(*round_args[s % 4]) == 0
            assert lib.apex_pe_sample_update(*step_args[s % n]) == 0
            if (s + 1) % 10 == 0:
                rc, asked = g.evict_enqueue(3, rnd_ev)
                assert rc == 0 and asked == 10 * w.add_count, (rc, asked)

    steps_f = 1000
    best = 1e30
    for rep_i in range(3):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        schedule_fused(steps_f)
        t_host = time.perf_counter() - t0
        torch.cuda.synchronize()
        best = min(best, (time.perf_counter() - t0) / steps_f * 1e6)
    st = g.stats()
    assert st["size"] == w.capacity and st["evicted"] == st["inserted"] - w.capacity, st
    out["prioritized_evict_memory_control_schedule_us_per_step"] = best
    out["prioritized_evict_memory_control_schedule_host_us_per_step"] = t_host / steps_f * 1e6
    g.close()
    out["observation_codec"] = codec_numbers(log)
    log("next rows: %s" % {k: (round(v, 2) if not isinstance(v, dict) else v) for k, v in out.items()})
    return out


def frame_like_rows(n, raw_bytes, flat_share, seed):
    """Stand-in for game screens (no frames of the suite are in the container): every 64-byte block of a row is
    one of 8 background bytes with probability flat_share, uniform random bytes otherwise."""
    import torch
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(seed)
    nb = raw_bytes // 64
    rows = torch.randint(0, 256, (n, nb, 64), dtype=torch.uint8, device="cuda:0", generator=gen)
    flat = torch.rand((n, nb, 1), device="cuda:0", generator=gen) < flat_share
    pal = (torch.randint(0, 8, (n, nb, 1), device="cuda:0", generator=gen) * 31).to(torch.uint8)
    return torch.where(flat, pal, rows).view(n, raw_bytes)


def codec_schedule_us(job, K, log, flat_share=0.8):
    """The headline schedule (one batch of 512 per learner step, an add round of 360 x 50 every 25 steps, FIFO
    eviction every 100) on a memory that stores its observations through the codec, fed with frame-like rows:
    add rounds are encoded on the copy stream, the step launch decodes as it gathers."""
    import torch
    from paper_1803_00933_amd import apex
    w = job.w
    stride = int(apex.lib.apex_codec_row_bytes(w.obs_bytes))
    rep = apex.Replay(w.capacity, w.max_slots, stride, w.act_bytes, w.alpha, w.eps, w.frac_bits)
    pipe = apex.Pipeline(rep, 8, 1, w.k)
    assert pipe.set_codec(w.obs_bytes) == 0
    stage = frame_like_rows(w.add_count, w.obs_bytes, flat_share, seed=5)

    def add_begin(i):
        t = job.rounds[i % job.n_pool]
        prio, ret, gacc, _ = t["out"]
        assert pipe.add_begin(t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n, stage,
                              t["act"], prio, ret, gacc) == 0

    assert pipe.fork() == 0
    n_fill = -(-w.capacity // w.add_count)
    for i in range(n_fill):
        add_begin(i)
        assert pipe.add_end(i == n_fill - 1)[0] == 0
    assert pipe.join() == 0
    torch.cuda.synchronize()
    assert rep.stats()["size"] == w.capacity

    def run(first, count):
        assert pipe.fork() == 0
        for f in range(first, first + count, ADD_EVERY):
            add_begin(f // ADD_EVERY)
            assert pipe.steps(ADD_EVERY, w.beta, job.rnd[f:f + ADD_EVERY], job.td[f:f + ADD_EVERY])[0] == 0
            assert pipe.add_end((f + ADD_EVERY) % EVICT_EVERY == 0)[0] == 0
        assert pipe.join() == 0

    def learner_only(count):
        assert pipe.fork() == 0
        assert pipe.steps(count, w.beta, job.rnd[:count], job.td[:count])[0] == 0
        assert pipe.join() == 0

    run(0, EVICT_EVERY)
    dt, _, _ = job.timed_median(lambda: run(0, K), reps=3)
    assert rep.stats()["size"] == w.capacity
    dt_learner, _, _ = job.timed_median(lambda: learner_only(K), reps=3)
    pipe.close()
    # the paper's prefetch depth as the unit of work: 16 batches per call, fetched through the decoder
    nb = 16
    calls = K // nb
    pipe16 = apex.Pipeline(rep, 2, nb, w.k)
    assert pipe16.set_codec(w.obs_bytes) == 0
    rnd = job.rnd[:calls * nb].reshape(calls, nb * w.k)
    td = job.td[:calls * nb].reshape(calls, nb * w.k)

    def go16(with_actors):
        assert pipe16.fork() == 0
        for c in range(calls):
            done, due = c * nb // ADD_EVERY, (c + 1) * nb // ADD_EVERY
            if with_actors and due > done:
                t = job.rounds[done % job.n_pool]
                prio, ret, gacc, _ = t["out"]
                assert pipe16.add_begin(t["q_online"], t["q_target"], t["action"], t["reward"], t["discount"], w.n,
                                        stage, t["act"], prio, ret, gacc) == 0
            assert pipe16.steps(1, w.beta, rnd[c], td[c])[0] == 0
            if with_actors and due > done:
                assert pipe16.add_end((c + 1) * nb // EVICT_EVERY > c * nb // EVICT_EVERY)[0] == 0
        assert pipe16.join() == 0
        if with_actors:
            assert rep.evict(stream=torch.cuda.current_stream())[0] == 0

    go16(True)
    dt16, _, _ = job.timed_median(lambda: go16(True), reps=3)
    dt16_learner, _, _ = job.timed_median(lambda: go16(False), reps=3)
    pipe16.close()
    rep.close()
    del rep, stage
    torch.cuda.empty_cache()
    res = {"flat_blocks_share": flat_share,
           "per_batch_steps_us_per_step": dt / K * 1e6, "per_batch_steps_learner_only_us_per_step": dt_learner / K * 1e6,
           "16_batches_per_call_us_per_batch": dt16 / (calls * nb) * 1e6,
           "16_batches_per_call_learner_only_us_per_batch": dt16_learner / (calls * nb) * 1e6}
    log("pipeline with the observation codec, frame-like rows (%d %% flat blocks): %s"
        % (int(flat_share * 100), {k2: round(v, 2) for k2, v in res.items()}))
    return res


def codec_numbers(log):
    """The observation codec (Section 4.1: observations are stored compressed) on frame-stack rows: the payload
    of an add round encoded on its way into the ring, batches decoded on their way out, against the plain
    copies of the same rows.  Device time from HIP events; a ring of 2^18 rows (7.5 GB) drawn from at random."""
    import torch
    from paper_1803_00933_amd import apex, synth
    w = synth.WORKLOADS["atari"]
    raw, P = w.obs_bytes, 1 << 18
    stride = int(apex.lib.apex_codec_row_bytes(raw))
    res = {"raw_bytes": raw, "row_stride": stride}
    rng = np.random.default_rng(11)
    slot512 = [dev(rng.integers(0, P - w.add_count, 512).astype(np.int32)) for _ in range(16)]
    slot8k = [dev(rng.integers(0, P - w.add_count, 8192).astype(np.int32)) for _ in range(4)]
    out512 = [torch.empty((512, raw), dtype=torch.uint8, device="cuda:0") for _ in range(4)]
    out8k = torch.empty((8192, raw), dtype=torch.uint8, device="cuda:0")
    prio = torch.ones(w.add_count, device="cuda:0")

    def timed(fn, n):
        fn(0)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(n):
            fn(i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n * 1e3

    for share in (0.8, 0.0):
        rows = frame_like_rows(w.add_count, raw, share, seed=3)
        rep = apex.Replay(P - w.add_count, P, stride, w.act_bytes, w.alpha, w.eps, w.frac_bits)
        for _ in range((P - w.add_count) // w.add_count):           # fill through the encoder
            assert rep.add_payload_encoded(rows) == 0
            assert rep.add_publish(prio)[0] == 0
        torch.cuda.synchronize()
        nb = raw // 64
        blocks = rows.view(w.add_count, nb, 64)
        n_raw = (blocks != blocks[:, :, :1]).any(dim=2).sum(dim=1).to(torch.float64).mean().item()
        used = (stride - 64 * nb - (nb + 15) // 16 * 16) + (nb - n_raw) + 64 * n_raw
        tag = "flat_%d%%" % int(share * 100)
        res[tag] = {
            "bytes_per_row_that_carry_data": used, "ratio": raw / used,
            "add_payload_encoded_18000_us": timed(lambda i: rep.add_payload_encoded(rows), 8),
            "gather_decoded_512_us": timed(lambda i: rep.gather_decoded(slot512[i % 16], out512[i % 4]), 64),
            "gather_decoded_8192_us": timed(lambda i: rep.gather_decoded(slot8k[i % 4], out8k), 8),
        }
        if share == 0.0:       # the plain copies of rows of the same stride, for comparison
            enc_rows = rep.obs_view()[:w.add_count].clone()
            out512s = [torch.empty((512, stride), dtype=torch.uint8, device="cuda:0") for _ in range(4)]
            out8ks = torch.empty((8192, stride), dtype=torch.uint8, device="cuda:0")
            res["plain_copies"] = {
                "add_payload_18000_us": timed(lambda i: rep.add_payload(w.add_count, obs=enc_rows), 8),
                "gather_512_us": timed(lambda i: rep.gather(slot512[i % 16], obs=out512s[i % 4]), 64),
                "gather_8192_us": timed(lambda i: rep.gather(slot8k[i % 4], obs=out8ks), 8),
            }
            del enc_rows, out512s, out8ks
        rep.close()
        del rep, rows
        torch.cuda.empty_cache()
    log("observation codec: %s" % res)
    return res


def profile_loop(job, n, log):
    """--profile-loop: only the launches that the rocprofv3 passes under profiles/ look at, each kind n times
    with other rows or uniforms every time, so that per-kernel averages of counters mean something:
    (a) learner steps as one launch each (learner_step_kernel: gather + weights + write-back + next draw),
    (b) plain gathers of 512 frame stacks (copy_rows_long_kernel, no side jobs),
    (c) draws of 512 samples (sample_descent_kernel),
    (d) gathers of 16 batches = 8192 frame stacks with their weights (copy_rows_long_kernel with weights)."""
    torch, w, rep = job.torch, job.w, job.rep
    job.setup_pipeline()
    job.run_pipelined_learner_only(0, n)
    torch.cuda.synchronize()
    st = rep.stats()
    gen = torch.Generator(device="cuda:0")
    gen.manual_seed(1)
    head_slot = st["head"] % w.max_slots
    slots = ((torch.randint(0, st["size"], (n, w.k), device="cuda:0", generator=gen) + head_slot) % w.max_slots).to(torch.int32)
    outs = [torch.empty((w.k, w.obs_bytes), dtype=torch.uint8, device="cuda:0") for _ in range(4)]
    for i in range(n):
        assert rep.gather(slots[i], obs=outs[i % 4]) == 0
    torch.cuda.synchronize()
    o = job.outs[0]
    o["mass"] = torch.empty(w.k, dtype=torch.int64, device="cuda:0")
    for i in range(n):
        assert rep.sample_begin(1, w.k, job.rnd[i], o) == 0
    torch.cuda.synchronize()
    nb = 16
    o16 = rep.alloc_sample_outputs(nb, w.k)
    o16["mass"] = torch.empty(nb * w.k, dtype=torch.int64, device="cuda:0")
    for c in range(max(1, n // nb)):
        assert rep.sample_begin(nb, w.k, job.rnd[c * nb:(c + 1) * nb], o16) == 0
        assert rep.sample_finish(nb, w.k, w.beta, o16) == 0
    torch.cuda.synchronize()
    log("profile loop: %d fused steps, %d gathers of %d rows, %d draws, %d gathers of %d rows"
        % (n, n, w.k, n, max(1, n // nb), nb * w.k))


def cpu_baseline(w, budget_steps, budget_seconds, log):
    """The oracle, untouched, on one host core: same schedule, bounded sample -- whole cycles of EVICT_EVERY
    steps until budget_seconds have passed, at most budget_steps."""
    import oracle
    from paper_1803_00933_amd import synth
    payload_slots = 1 << 15                      # frame rows aliased modulo 32768 slots (0.9 GB): timing only
    o = oracle.Replay(w.capacity, w.max_slots, w.obs_bytes, w.act_bytes, w.alpha, w.eps, w.frac_bits,
                      payload_slots=payload_slots)
    rng = np.random.default_rng(0)
    n_fill = -(-w.capacity // w.add_count)
    for i in range(n_fill):
        o.add(synth.priorities("lognormal1", w.seed, i, w.add_count, tag="bulk"))
    o.evict()
    obs = rng.integers(0, 256, (w.add_count, w.obs_bytes), dtype=np.uint8)
    rounds = [synth.actor_round(w, i) for i in range(2)]
    rnd = [synth.uniforms(w.seed, s, 1, w.k).reshape(-1) for s in range(budget_steps)]
    td = [synth.priorities(w.td_dist, w.seed, s, w.k) for s in range(budget_steps)]
    def step(s):
        rc, out = o.sample(1, w.k, w.beta, rnd[s % len(rnd)])
        o.update_priorities(out["key"], td[s % len(td)])
        if (s + 1) % ADD_EVERY == 0:
            d = rounds[(s // ADD_EVERY) % 2]
            prio, ret, gacc, _ = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"],
                                                         d["discount"], w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
            o.add(prio.reshape(-1), obs, d["act"], ret.reshape(-1), gacc.reshape(-1))
        if (s + 1) % EVICT_EVERY == 0:
            o.evict()

    for s in range(EVICT_EVERY):                 # one untimed cycle: first touch of the payload pages
        step(s)
    t0 = time.perf_counter()
    done = 0
    for s in range(budget_steps):
        if s % EVICT_EVERY == 0 and s and time.perf_counter() - t0 >= budget_seconds:
            break
        done = s + 1
        step(EVICT_EVERY + s)
    dt = time.perf_counter() - t0
    budget_steps = done
    model, nproc = host_cpu()
    log("cpu oracle: %d steps in %.2f s on one core of %d (%s)" % (budget_steps, dt, nproc, model))
    return {"value": w.k * budget_steps / dt, "unit": "transitions/s", "cores": 1, "kind": "oracle",
            "cpu_model": model, "host_logical_cores": nproc,
            "sample": "%d learner steps of the same schedule (batch %d, add round every %d steps, evict every %d) "
                      "after one untimed cycle, single thread; tree and keys at full size, frame rows aliased modulo %d slots to fit host "
                      "memory" % (budget_steps, w.k, ADD_EVERY, EVICT_EVERY, payload_slots),
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000,
                    help="learner steps to time; rounded up to whole cycles of %d (the schedule's period)" % EVICT_EVERY)
    ap.add_argument("--warmup", type=int, default=200, help="untimed steps before them; rounded up the same way")
    ap.add_argument("--cpu-steps", type=int, default=8000,
                    help="most learner steps timed on the CPU oracle (0 = skip) ...")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="... which stops at the first whole cycle after this many seconds")
    ap.add_argument("--extras", choices=("on", "off"), default="on",
                    help="the other workload shapes and library features beside the headline (control, skew, scale, "
                         "learner-side priorities, prioritized eviction, observation codec): about ten seconds more")
    ap.add_argument("--no-control", action="store_true", help="same as --extras off")
    ap.add_argument("--profile-loop", type=int, default=0, metavar="N",
                    help="after the prefill run only N launches of each kernel that the counter passes under "
                         "profiles/ look at, print no result line (for use under rocprofv3)")
    ap.add_argument("--quiet", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU (the replay memory lives in one MI355X's HBM); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)
    try:
        K, W = normalise_steps(args.steps, args.warmup)       # before anything is allocated
    except ValueError as e:
        print("bench.py: %s" % e, file=sys.stderr)
        sys.exit(2)
    extras = not args.no_control and args.extras == "on"

    def log(msg):
        if not args.quiet:
            print("[bench] " + msg, file=sys.stderr, flush=True)

    t_start = time.time()
    import torch
    from paper_1803_00933_amd import synth
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    w = synth.WORKLOADS["atari"]
    if (K, W) != (args.steps, args.warmup):
        log("--steps %d --warmup %d run as %d timed steps after %d of warm-up (whole cycles of %d)"
            % (args.steps, args.warmup, K, W, EVICT_EVERY))
    torch.cuda.set_stream(torch.cuda.Stream())      # plain calls go to an ordinary stream, not the null stream
    K_roof = max(K, 1000)                           # launches behind the roofline figure (learner-only loop)
    if args.profile_loop > 0:
        profile_loop(GpuJob(w, args.profile_loop, log), args.profile_loop, log)
        return
    job = GpuJob(w, max(W + 2 * K, W + K_roof), log)

    job.setup_pipeline()
    job.run(0, W)
    # (1) every call on one stream, in order
    dt_serial, host_serial = job.timed(lambda: job.run(W, K, with_actors=True))
    log("one stream: %.2f us/step (host enqueue %.2f us/step)" % (dt_serial / K * 1e6, host_serial / K * 1e6))
    dt_learner, _ = job.timed(lambda: job.run(W + K, K, with_actors=False))
    log("one stream, learner steps only: %.2f us/step" % (dt_learner / K * 1e6))
    # (2) the library's pipeline (one launch per learner step; add payloads on a second stream)
    job.run_pipelined(0, EVICT_EVERY)               # one untimed cycle in this launch mode
    dt_pipe, host_pipe, reps_pipe = job.timed_median(lambda: job.run_pipelined(W, K))
    log("pipeline, two streams: %.2f us/step, median of %d runs (%s; host enqueue %.2f us/step)"
        % (dt_pipe / K * 1e6, len(reps_pipe), " ".join("%.2f" % (t / K * 1e6) for t in reps_pipe), host_pipe / K * 1e6))
    # (learner steps alone are cheap: always at least 1,000 of them, so that the start of a run does not weigh)
    dt_pipe_learner, _, _ = job.timed_median(lambda: job.run_pipelined_learner_only(W, K_roof))
    dt_pipe_learner *= K / K_roof
    log("pipeline, learner steps only: %.2f us/step (median of 5 runs of %d steps)" % (dt_pipe_learner / K * 1e6, K_roof))
    dt_in_place, _, _ = job.timed_median(lambda: job.run_pipelined(W, K, in_place=True))
    log("pipeline, observations of the add rounds written in place by their producer (no copy): %.2f us/step"
        % (dt_in_place / K * 1e6))
    us_codec = codec_schedule_us(job, K, log) if extras else None
    K16 = max(K, 400) // 16 * 16
    us16 = job.prefetch16_us_per_batch(K16, with_actors=False)
    us16_full = job.prefetch16_us_per_batch(K16, with_actors=True)
    log("pipeline, 16 batches of 512 per call: %.2f us per batch learner only, %.2f with adds and eviction"
        % (us16, us16_full))
    mode, dt = "apex_pipeline: two streams, eager launches", dt_pipe
    # (3) one cycle of the same pipeline captured as a HIP graph and replayed
    job.capture_cycle(W)
    job.run_replays(max(1, W // EVICT_EVERY))
    dt_graph, host_graph, reps_graph = job.timed_median(lambda: job.run_replays(K // EVICT_EVERY))
    assert job.rep.resync() == 0
    log("pipeline, graph replays: %.2f us/step (host %.2f us/step)" % (dt_graph / K * 1e6, host_graph / K * 1e6))
    if dt_graph < dt:
        mode, dt = "apex_pipeline: two streams, one HIP graph per %d-step cycle" % EVICT_EVERY, dt_graph
    if dt_serial < dt:
        mode, dt = "plain calls on one stream, eager launches", dt_serial
    st = job.rep.stats()
    assert st["size"] == w.capacity, st
    log("state after run: %s" % st)

    step_us = job.step_kernel_us(W, K_roof)
    achieved = STEP_ALGORITHMIC_BYTES / (step_us * 1e-6) / 1e9
    log("learner-step kernel: %.2f us/launch over %d launches, %.0f GB/s of algorithmic bytes"
        % (step_us, K_roof, achieved))

    ops = op_timings(job)
    log("other steps alone, us: %s" % {k: round(v, 2) for k, v in ops.items()})
    del job
    torch.cuda.empty_cache()
    control = control_numbers(log) if extras else None
    tree_bound = tree_bound_workloads(log) if extras else None
    next_rows = next_row_numbers(log) if extras else None
    cpu = cpu_baseline(w, args.cpu_steps, args.cpu_seconds, log) if args.cpu_steps > 0 else None

    def frac(us):
        return STEP_ALGORITHMIC_BYTES / (us * 1e-6) / 1e9 / HBM_PEAK_GBS

    line = {
        "metric": "sampled transitions/s (sample+IS+gather+update) at 2M slots, batch 512",
        "value": w.k * K / dt,
        "unit": "transitions/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "steps_requested": args.steps, "warmup_requested": args.warmup,
        "ms_per_step": dt / K * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u64",
        "data": "synthetic",
        "config": {"workload": "atari: capacity 2,000,000 (ring 2^21) x uint8[84*84*4], 18 actions, n=3, alpha 0.6, "
                               "beta 0.4, batch 512; add round of 360x50 every 25 steps, FIFO evict every 100",
                   "capacity": w.capacity, "max_slots": w.max_slots, "obs_bytes": w.obs_bytes, "batch": w.k,
                   "add_round": w.add_count, "add_every": ADD_EVERY, "evict_every": EVICT_EVERY,
                   "launch_mode": mode,
                   "steps_note": "steps and warmup are what was run: the requested counts rounded up to whole "
                                 "cycles of %d steps, the period of the schedule" % EVICT_EVERY},
        "priority_updates_per_s": w.k * K / dt,
        "adds_per_s": w.add_count * (K // ADD_EVERY) / dt,
        "nstep_priorities_per_s": w.add_count / (ops["nstep_priorities_18000"] * 1e-6),
        "ops_us": ops,
        "observation_codec_schedule": us_codec,
        "repetitions": {"n": 5, "value_is": "median",
                        "pipeline_us_per_step": [t / K * 1e6 for t in reps_pipe],
                        "pipeline_graph_us_per_step": [t / K * 1e6 for t in reps_graph]},
        "variants_us_per_step": {"one_stream": dt_serial / K * 1e6, "one_stream_learner_only": dt_learner / K * 1e6,
                                 "pipeline": dt_pipe / K * 1e6, "pipeline_learner_only": dt_pipe_learner / K * 1e6,
                                 "pipeline_graph": dt_graph / K * 1e6,
                                 "pipeline_add_payload_in_place": dt_in_place / K * 1e6,
                                 "pipeline_16_batches_per_call_learner_only": us16,
                                 "pipeline_16_batches_per_call": us16_full},
        "hbm_frac_of_step": {"bytes_per_step": STEP_ALGORITHMIC_BYTES,
                             "pipeline_learner_only": frac(dt_pipe_learner / K * 1e6),
                             "pipeline_16_batches_per_call_learner_only": frac(us16)},
        "roofline": {"bound": "hbm", "kernel": "learner_step_kernel<u32x4,512,4,1,0> (gather of one batch of frame "
                                               "stacks + IS weights + priority write-back + draw of the next "
                                               "batch; distinct rows every launch)",
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": RECORDED_STEP_TRAFFIC_BYTES, "traffic_source": RECORDED_STEP_TRAFFIC["source"],
                     "bytes_per_launch": STEP_ALGORITHMIC_BYTES, "bytes_model": "512 x 57,030 B per sampled transition",
                     "us_per_launch": step_us, "launches_timed": K_roof,
                     "timing": "HIP events around back-to-back launches of the learner-only loop: launch to "
                               "launch, gaps included"},
        "roofline_add_payload": {"bound": "hbm", "kernel": "copy_rows_dense_kernel<u32x4,2> (18,000 frame stacks "
                                                           "of an add round into the ring)",
                                 "achieved": ops["add_payload_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                                 "frac": ops["add_payload_GBps"] / HBM_PEAK_GBS,
                                 "bytes_per_launch": 2 * w.add_count * w.obs_bytes,
                                 "us_per_launch": ops["add_payload_18000"]},
        "control_workload": control,
        "tree_bound_workloads": tree_bound,
        "next_rows": next_rows,
        "extras_run": extras,
        "cpu_baseline": cpu,
        "wall_seconds": time.time() - t_start,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
