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
    n_raw = enc_ref[:, :4].copy().view("<u4")[:, 0].astype(np.int64)
    assert np.array_equal(enc_gpu[:, :16 + M], enc_ref[:, :16 + M]), "header or mask"
    for i in range(len(enc_ref)):
        nf = nb - n_raw[i]
        assert np.array_equal(enc_gpu[i, 16 + M:16 + M + nf], enc_ref[i, 16 + M:16 + M + nf]), "flat values of row %d" % i
        a, b = 16 + M + V, 16 + M + V + 64 * n_raw[i]
        assert np.array_equal(enc_gpu[i, a:b], enc_ref[i, a:b]), "kept blocks of row %d" % i


@pytest.mark.gpu
@pytest.mark.parametrize("raw_bytes,extra", [(64, 0), (256, 16), (4160, 0), (28224, 0), (36864, 64)])
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
def test_codec_status_codes():
    from paper_1803_00933_amd import apex
    g = apex.Replay(100, 128, 304, 4)                      # rows for 256 raw bytes
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
    """Host-only: the stride the library reports is the oracle's (the library also refuses rows beyond 256 KB)."""
    from paper_1803_00933_amd import apex
    want = oracle.codec_row_bytes(raw_bytes) if raw_bytes <= 262144 else 0
    assert apex.lib.apex_codec_row_bytes(raw_bytes) == want
