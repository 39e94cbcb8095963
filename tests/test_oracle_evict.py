"""Pins for the oracle's memory with prioritized eviction (Appendix "Continuous Control: Additional Details":
eviction by proportional prioritized sampling with exponent alpha_evict): hand-worked rounds, eviction
frequencies, brute force in Python integers, structural invariants."""
import bisect
import math

import numpy as np
import pytest

import oracle

F32 = np.float32
U64 = 1 << 64


def check(r):
    """Both trees sum up; occupied slots, free ring and size agree."""
    leaves = {}
    for which in (False, True):
        nodes = r.nodes(which)
        half = len(nodes) // 2
        assert np.array_equal(nodes[1:half], nodes[2:2 * half:2] + nodes[3:2 * half:2])
        leaves[which] = r.leaves(which)
        assert int(nodes[1]) == sum(int(v) for v in leaves[which])
    live = set(np.nonzero(leaves[False])[0].tolist())
    assert live == set(np.nonzero(leaves[True])[0].tolist())
    ring, P = r.free_ring(), r.max_slots
    free = [int(ring[i % P]) for i in range(r.free_head, r.free_tail)]
    assert len(set(free)) == len(free) and not (set(free) & live) and len(free) + len(live) == P
    assert r.size == len(live) == r.inserted - r.evicted
    return leaves, free


def test_hand_worked_eviction_rounds():
    # alpha_evict = -1, eps = 0, priorities 1 2 4 8: eviction masses 8 4 2 1 (units of 2^21), total 15
    r = oracle.PrioritizedEvictionReplay(2, 4, 4, 4, alpha=1.0, alpha_evict=-1.0, eps=0.0)
    rc, keys = r.add(np.array([1, 2, 4, 8], F32))
    assert rc == 0 and keys.tolist() == [(1 << 32) | s for s in range(4)]
    assert r.leaves(True).tolist() == [8 << 21, 4 << 21, 2 << 21, 1 << 21]
    assert r.leaves(False).tolist() == [1 << 24, 2 << 24, 4 << 24, 8 << 24]
    # e = 2.  round 0: two strata of width 7.5; uniforms 0 -> points 0 and 7.5, both inside slot 0 = [0, 8): one
    # eviction.  round 1: one stratum over the rest (4 2 1); uniform 0 -> point 0 -> slot 1.
    rc, e = r.evict(2, np.zeros(4, np.uint64))
    assert (rc, e) == (0, 2) and r.size == 2
    assert r.leaves(True).tolist() == [0, 0, 2 << 21, 1 << 21]
    leaves, free = check(r)
    assert free == [0, 1]                                        # freed in this order, re-used in this order
    rc, keys = r.add(np.array([16, 32], F32))
    assert keys.tolist() == [(2 << 32) | 0, (2 << 32) | 1]       # second tenants of slots 0 and 1
    # the first tenants' keys are stale now; the new ones work
    r.update_priorities(np.array([(1 << 32) | 0, (2 << 32) | 1], np.uint64), np.array([1, 1], F32))
    assert r.n_stale == 1 and r.leaves(False)[1] == 1 << 24 and r.leaves(False)[0] == 16 << 24
    # with one round only, the repeat in round 0 leaves the eviction one short
    r2 = oracle.PrioritizedEvictionReplay(2, 4, 4, 4, alpha=1.0, alpha_evict=-1.0, eps=0.0)
    r2.add(np.array([1, 2, 4, 8], F32))
    assert r2.evict(1, np.zeros(2, np.uint64)) == (0, 1) and r2.size == 3
    # top of the strata: points just below 7.5 and 15 -> slots 0 and 3
    r3 = oracle.PrioritizedEvictionReplay(2, 4, 4, 4, alpha=1.0, alpha_evict=-1.0, eps=0.0)
    r3.add(np.array([1, 2, 4, 8], F32))
    assert r3.evict(1, np.full(2, U64 - 1, np.uint64)) == (0, 2)
    assert r3.leaves(True).tolist() == [0, 4 << 21, 2 << 21, 0]


def test_single_evictions_follow_p_to_the_alpha_evict():
    alpha_e, P, G = -0.4, 12, 2048
    rng = np.random.default_rng(0)
    prio = rng.lognormal(0, 1, P).astype(F32)
    counts = np.zeros(P)
    for g in range(G):
        r = oracle.PrioritizedEvictionReplay(P - 1, P, 4, 4, alpha_evict=alpha_e, eps=0.0)
        r.add(prio)
        u = np.array([(g << 53) + (1 << 52)], np.uint64)          # mid-points of a regular grid
        assert r.evict(1, u) == (0, 1)
        counts[int(np.nonzero(r.leaves() == 0)[0][0])] += 1
    share = prio.astype(np.float64) ** float(F32(alpha_e))
    share /= share.sum()
    assert np.all(np.abs(counts - share * G) <= 1.0 + 1e-5 * G)
    assert counts[np.argmin(prio)] == counts.max()               # the smallest TD error goes most often


@pytest.mark.parametrize("P,C,rounds", [(64, 40, 6), (1000, 900, 4), (4096, 3000, 8)])
def test_eviction_equals_brute_force(P, C, rounds):
    rng = np.random.default_rng(P)
    r = oracle.PrioritizedEvictionReplay(C, P, 4, 4)
    assert r.add(rng.lognormal(0, 2, P).astype(F32))[0] == 0
    e = P - C
    rnd = rng.integers(0, U64, (rounds, e), dtype=np.uint64)
    mass = [int(v) for v in r.leaves(True)]
    order = []
    remaining = e
    for rd in range(rounds):
        if not remaining:
            break
        cum, run = [], 0
        for m in mass:
            run += m
            cum.append(run)
        w = run // remaining
        cand = [bisect.bisect_right(cum, j * w + (int(rnd[rd, j]) * w >> 64)) for j in range(remaining)]
        acc = [c for j, c in enumerate(cand) if j == 0 or c != cand[j - 1]]
        for c in acc:
            mass[c] = 0
        order += acc
        remaining -= len(acc)
    rc, got = r.evict(rounds, rnd)
    assert (rc, got) == (0, len(order)) and got > 0.9 * e
    leaves, free = check(r)
    assert free == order
    assert [int(v) for v in leaves[True]] == mass


def test_random_sequences_keep_the_structure_sound():
    rng = np.random.default_rng(5)
    P, C = 512, 400
    r = oracle.PrioritizedEvictionReplay(C, P, 8, 4)
    store = {}
    for it in range(30):
        cnt = int(rng.integers(1, P - r.size + 1))
        obs = rng.integers(0, 256, (cnt, 8), dtype=np.uint8)
        rc, keys = r.add(rng.lognormal(0, 1, cnt).astype(F32), obs, np.zeros((cnt, 4), np.uint8),
                         np.zeros(cnt, F32), np.zeros(cnt, F32))
        assert rc == 0 and len(set(keys.tolist())) == cnt
        for k_, o_ in zip(keys, obs):
            assert int(k_) not in store                            # keys are never re-issued
            store[int(k_)] = o_
        assert r.add(np.ones(P, F32))[0] == oracle.ERR_FULL
        check(r)
        rc, out = r.sample(2, 32, 0.4, rng.integers(0, U64, 64, dtype=np.uint64))
        for k_, o_ in zip(out["key"], out["obs"]):
            assert np.array_equal(store[int(k_)], o_)
        assert r.update_priorities(out["key"], rng.lognormal(0, 1, 64).astype(F32)) == 0
        before = r.size
        rc, e = r.evict(10, rng.integers(0, U64, (10, max(1, before - C)), dtype=np.uint64))
        assert e == max(0, before - C) and r.size == min(before, C)
        leaves, free = check(r)
        dead = [k_ for k_ in store if leaves[False][k_ & 0xffffffff] == 0 or r.gen()[k_ & 0xffffffff] != k_ >> 32]
        stale0 = r.n_stale
        r.update_priorities(np.array(dead[:50], np.uint64), np.ones(len(dead[:50]), F32))
        assert r.n_stale == stale0 + len(dead[:50])                # evicted keys are not valid any more


def test_sampling_matches_the_fifo_memory_while_nothing_was_evicted():
    rng = np.random.default_rng(6)
    P = 300
    prio = rng.lognormal(0, 1, P).astype(F32)
    a, b = oracle.PrioritizedEvictionReplay(P, P, 4, 4, payload=False), oracle.Replay(P, P, 4, 4, payload_slots=0)
    a.add(prio), b.add(prio)
    rnd = rng.integers(0, U64, 3 * 50, dtype=np.uint64)
    oa, ob = a.sample(3, 50, 0.4, rnd)[1], b.sample(3, 50, 0.4, rnd)[1]
    assert np.array_equal(oa["slot"], ob["slot"]) and np.array_equal(oa["weight"], ob["weight"])
    assert np.array_equal(oa["key"], (np.uint64(1) << np.uint64(32)) | ob["key"])
    # eviction masses are the quantiser at the eviction exponent
    for s in range(0, P, 37):
        x = float(F32(prio[s]) + F32(1e-6))
        exact = math.pow(x, float(F32(-0.4)))
        assert abs(int(a.leaves(True)[s]) / 2 ** 24 - exact) <= 1e-5 * exact + 2 ** -24
