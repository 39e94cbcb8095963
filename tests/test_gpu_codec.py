"""GPU parity of the observation codec (Section 4.1: observations stored compressed, decompressed when batches
are fetched): rows encoded on their way into the ring against the oracle's encoding, byte for byte where the
format defines the bytes; batches decoded on their way out against the raw rows the oracle stored."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import assert_sample_equal, check_gpu_tree, dev, host
from test_oracle_codec import frame_like

F32 = np.float32
U64 = 1 << 64


def defined_parts_equal(enc_gpu, enc_ref, raw_bytes):
    nb = raw_bytes // 64
    M = (8 * ((nb + 63) // 64) + 15) // 16 * 16
    V = (nb + 15) // 16 * 16
    assert np.array_equal(enc_gpu[:, :M], enc_ref[:, :M]), "mask"
    kept = np.unpackbits(enc_ref[:, :M], axis=1, bitorder="little")[:, :nb].astype(bool)
    assert np.array_equal(enc_gpu[:, M:M + nb][~kept], enc_ref[:, M:M + nb][~kept]), "bytes of the flat blocks"
    img_gpu = enc_gpu[:, M + V:M + V + raw_bytes].reshape(-1, nb, 64)
    img_ref = enc_ref[:, M + V:M + V + raw_bytes].reshape(-1, nb, 64)
    assert np.array_equal(img_gpu[kept], img_ref[kept]), "blocks kept as they are"


@pytest.mark.gpu
@pytest.mark.parametrize("raw_bytes,extra", [(64, 0), (256, 16), (4160, 0), (28224, 0), (36864, 64), (135168, 0)])
@pytest.mark.parametrize("flat_share", [0.0, 0.5, 0.95, 1.0])
def test_rows_through_the_codec(raw_bytes, extra, flat_share):
    from paper_1803_00933_amd import apex
    rng = np.random.default_rng(raw_bytes + int(100 * flat_share))
    stride = oracle.codec_row_bytes(raw_bytes)
    assert apex.lib.apex_codec_row_bytes(raw_bytes) == stride
    P, Cap = 700, 500
    g = apex.Replay(Cap, P, stride + extra, 4)
    o = oracle.Replay(Cap, P, raw_bytes, 4)
    for rnd_round in range(5):                       # wraps around the ring
        cnt = int(rng.integers(1, P - o.size + 1))
        raw = frame_like(rng, cnt, raw_bytes, flat_share)
        act = rng.integers(0, 256, (cnt, 4), dtype=np.uint8)
        ret, gacc = rng.standard_normal(cnt).astype(F32), rng.random(cnt).astype(F32)
        prio = rng.lognormal(0, 1, cnt).astype(F32)
        first_slot = o.tail % P
        assert g.add_payload_encoded(dev(raw), dev(act), dev(ret), dev(gacc)) == 0
        rc, first = g.add_publish(dev(prio))
        assert (rc, first) == o.add(prio, raw, act, ret, gacc)
        torch.cuda.synchronize()
        rows = (first_slot + np.arange(cnt)) % P
        enc_gpu = host(g.obs_view())[rows][:, :stride]
        enc_ref, _ = oracle.codec_encode(raw)
        defined_parts_equal(enc_gpu, enc_ref, raw_bytes)
        check_gpu_tree(g, o)
        # a batch: drawn as usual, fetched through the decoder
        k = 96
        rnd = rng.integers(0, U64, 2 * k, dtype=np.uint64)
        rco, oo = o.sample(2, k, 0.4, rnd)
        rcg, go = g.sample(2, k, 0.4, dev(rnd), payload=False)
        assert rcg == rco == 0
        dec = torch.empty((2 * k, raw_bytes), dtype=torch.uint8, device="cuda:0")
        small = dict(act=torch.empty((2 * k, 4), dtype=torch.uint8, device="cuda:0"),
                     ret=torch.empty(2 * k, dtype=torch.float32, device="cuda:0"),
                     gacc=torch.empty(2 * k, dtype=torch.float32, device="cuda:0"))
        assert g.gather_decoded(go["slot"], dec, **small) == 0
        torch.cuda.synchronize()
        go.update(obs=dec, **small)
        assert_sample_equal(go, oo)
        assert g.evict() == o.evict()


@pytest.mark.gpu
@pytest.mark.parametrize("raw_bytes,flat_share,nb,k,depth", [
    (4160, 0.7, 1, 80, 4), (28224, 0.8, 1, 80, 4), (28224, 0.0, 1, 80, 4), (256, 0.5, 1, 80, 4), (32768, 0.9, 1, 80, 4),
    (4160, 0.7, 4, 512, 2),          # steps of several batches: fetched through the decoder on the copy stream
])
def test_pipeline_with_the_codec(raw_bytes, flat_share, nb, k, depth):
    """The pipeline's fast path with observations stored encoded: add rounds encoded on the copy stream (or on
    the learner's stream when small), learner steps that decode while they gather, against the oracle that
    stores the raw rows."""
    from paper_1803_00933_amd import apex, synth
    rng = np.random.default_rng(raw_bytes + 7)
    stride = oracle.codec_row_bytes(raw_bytes)
    small = synth.WORKLOADS["tiny"].scaled(obs_bytes=stride, capacity=2500, max_slots=4096, streams=4, chunk=25, k=k)
    large = small.scaled(streams=48)
    g = apex.Replay(small.capacity, small.max_slots, stride, small.act_bytes)
    o = oracle.Replay(small.capacity, small.max_slots, raw_bytes, small.act_bytes)
    cnt = 2000
    raw = frame_like(rng, cnt, raw_bytes, flat_share)
    act = rng.integers(0, 256, (cnt, small.act_bytes), dtype=np.uint8)
    ret, gacc = rng.standard_normal(cnt).astype(F32), rng.random(cnt).astype(F32)
    prio = rng.lognormal(0, 1, cnt).astype(F32)
    assert g.add_payload_encoded(dev(raw), dev(act), dev(ret), dev(gacc)) == 0
    assert g.add_publish(dev(prio)) == o.add(prio, raw, act, ret, gacc)
    pipe = apex.Pipeline(g, depth, nb, small.k)
    assert pipe.set_codec(raw_bytes) == 0
    n_steps = min(3, depth - 1)
    assert pipe.fork() == 0
    for i, w in enumerate([small, large, small, large, large]):
        d = synth.actor_round(w, i)
        n_rows = w.streams * w.chunk
        d["obs"] = frame_like(rng, n_rows, raw_bytes, flat_share)
        dd = {k2: dev(v) for k2, v in d.items()}
        scratch = [torch.empty(n_rows, dtype=torch.float32, device="cuda:0") for _ in range(3)]
        rnd = rng.integers(0, U64, (n_steps, nb * w.k), dtype=np.uint64)
        newp = rng.lognormal(0, 1, (n_steps, nb * w.k)).astype(F32)
        d_rnd, d_newp = dev(rnd), dev(newp)
        assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                              dd["obs"], dd["act"], *scratch) == 0
        rc, first = pipe.steps(n_steps, 0.4, d_rnd, d_newp)
        assert rc == 0
        rc, first_key, ev = pipe.add_end(True)
        refs = []
        for s_ in range(n_steps):
            refs.append(o.sample(nb, w.k, 0.4, rnd[s_])[1])
            o.update_priorities(refs[-1]["key"], newp[s_])
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        assert (rc, first_key) == o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))
        assert o.evict() == (0, ev)
        assert pipe.join() == 0
        torch.cuda.synchronize()
        for s_ in range(n_steps):
            assert_sample_equal(pipe.sets[(first + s_) % depth], refs[s_])
        check_gpu_tree(g, o)
        assert pipe.fork() == 0
    assert pipe.join() == 0
    # back to plain rows: the sets receive the encoded rows as they are stored
    assert pipe.set_codec(0) == 0
    assert pipe.set_codec(100) == apex.ERR_INVALID_ARG
    assert pipe.set_codec(raw_bytes + 64) == apex.ERR_TOO_LARGE
    pipe.close()


@pytest.mark.gpu
@pytest.mark.parametrize("raw_bytes,nb,k,depth", [(4160, 1, 80, 3), (28224, 1, 64, 3), (4160, 4, 512, 2)])
def test_pipeline_graph_replays_with_the_codec(raw_bytes, nb, k, depth):
    """One cycle with the codec on (an add round encoded on the copy stream beside learner steps that decode
    while they gather, then eviction) recorded as a HIP graph and replayed; every replay against the oracle,
    with eager calls on the same memory in between."""
    from paper_1803_00933_amd import apex, synth
    rng = np.random.default_rng(raw_bytes + nb)
    stride = oracle.codec_row_bytes(raw_bytes)
    w = synth.WORKLOADS["tiny"].scaled(obs_bytes=stride, capacity=2500, max_slots=4096, streams=6, chunk=30, k=k)
    g = apex.Replay(w.capacity, w.max_slots, stride, w.act_bytes)
    o = oracle.Replay(w.capacity, w.max_slots, raw_bytes, w.act_bytes)

    def eager_add(cnt):
        raw = frame_like(rng, cnt, raw_bytes, 0.7)
        act = rng.integers(0, 256, (cnt, w.act_bytes), dtype=np.uint8)
        ret, gacc = rng.standard_normal(cnt).astype(F32), rng.random(cnt).astype(F32)
        prio = rng.lognormal(0, 1, cnt).astype(F32)
        assert g.add_payload_encoded(dev(raw), dev(act), dev(ret), dev(gacc)) == 0
        assert g.add_publish(dev(prio)) == o.add(prio, raw, act, ret, gacc)

    eager_add(w.capacity)
    pipe = apex.Pipeline(g, depth, nb, w.k)
    assert pipe.set_codec(raw_bytes) == 0
    n_steps = depth - 1 if nb > 1 else 5
    rnd = rng.integers(0, U64, (n_steps, nb * w.k), dtype=np.uint64)
    newp = rng.lognormal(0, 1, (n_steps, nb * w.k)).astype(F32)
    d_rnd, d_newp = dev(rnd), dev(newp)
    n_rows = w.streams * w.chunk
    scratch = [torch.empty(n_rows, dtype=torch.float32, device="cuda:0") for _ in range(3)]
    d = synth.actor_round(w, 0)
    d["obs"] = frame_like(rng, n_rows, raw_bytes, 0.7)
    dd = {k2: dev(v) for k2, v in d.items()}
    torch.cuda.synchronize()

    def oracle_cycle():
        res = []
        for s in range(n_steps):
            res.append(o.sample(nb, w.k, 0.4, rnd[s])[1])
            o.update_priorities(res[-1]["key"], newp[s])
        ref = oracle.nstep_priorities(d["q_online"], d["q_target"], d["action"], d["reward"], d["discount"],
                                      w.n, w.alpha, w.eps, w.frac_bits, w.max_slots)
        assert o.add(ref[0].reshape(-1), d["obs"], d["act"], ref[1].reshape(-1), ref[2].reshape(-1))[0] == 0
        assert o.evict() == (0, n_rows)
        return res

    assert pipe.capture_begin() == 0
    assert pipe.add_begin(dd["q_online"], dd["q_target"], dd["action"], dd["reward"], dd["discount"], w.n,
                          dd["obs"], dd["act"], *scratch) == 0
    assert pipe.steps(n_steps, 0.4, d_rnd, d_newp)[0] == 0
    rc, _, ev = pipe.add_end(True)
    assert (rc, ev) == (0, n_rows)
    assert pipe.capture_end() == 0
    first_kept = max(0, n_steps - depth)
    for replay in range(3):
        assert pipe.fork() == 0
        assert pipe.replay(1) == 0
        assert pipe.join() == 0
        torch.cuda.synchronize()
        res = oracle_cycle()
        for s in range(first_kept, n_steps):
            assert_sample_equal(pipe.sets[s % depth], res[s])
        assert g.resync() == 0
        check_gpu_tree(g, o)
        if replay == 0:                       # eager calls between replays, on the same memory
            eager_add(30)
            assert g.evict() == o.evict()
    pipe.close()


@pytest.mark.gpu
def test_codec_status_codes():
    from paper_1803_00933_amd import apex
    g = apex.Replay(100, 128, 288, 4)                      # rows for 256 raw bytes
    raw = torch.zeros((4, 256), dtype=torch.uint8, device="cuda:0")
    slot = torch.zeros(4, dtype=torch.int32, device="cuda:0")
    assert g.add_payload_encoded(raw) == 0
    assert g.add_payload_encoded(torch.zeros((4, 320), dtype=torch.uint8, device="cuda:0")) == apex.ERR_TOO_LARGE
    assert g.add_payload_encoded(torch.zeros((4, 100), dtype=torch.uint8, device="cuda:0")) == apex.ERR_INVALID_ARG
    buf = torch.zeros(4 * 256 + 16, dtype=torch.uint8, device="cuda:0")
    assert g.add_payload_encoded(buf[4:4 + 1024].view(4, 256)) == apex.ERR_INVALID_ARG     # misaligned rows
    assert g.gather_decoded(slot, torch.zeros((4, 320), dtype=torch.uint8, device="cuda:0")) == apex.ERR_TOO_LARGE
    assert g.gather_decoded(slot, torch.zeros((4, 96), dtype=torch.uint8, device="cuda:0")) == apex.ERR_INVALID_ARG
    assert g.add_payload_encoded(torch.zeros((200, 256), dtype=torch.uint8, device="cuda:0")) == apex.ERR_FULL
    torch.cuda.synchronize()


@pytest.mark.parametrize("raw_bytes", [0, 1, 64, 100, 128, 256, 4096, 4160, 28224, 262144, 262208, 1 << 20])
def test_row_bytes_matches_the_oracle(raw_bytes):
    """Host-only: the stride the library reports is the oracle's."""
    from paper_1803_00933_amd import apex
    assert apex.lib.apex_codec_row_bytes(raw_bytes) == oracle.codec_row_bytes(raw_bytes)
