"""Thin ctypes binding of ``libapex_replay.so`` (declared in ``include/apex_replay.h``).

Argument marshalling only: every step of the replay path runs in the library's HIP kernels.
PyTorch supplies device memory (``tensor.data_ptr()``) and the current stream, nothing else.
There is no fallback: if the library has not been built, importing this module raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# (APEX_REPLAY_LIB names another build of the same library, e.g. the one with sanitized host code)
LIB_PATH = os.environ.get("APEX_REPLAY_LIB") or os.path.join(_HERE, "libapex_replay.so")

OK, ERR_INVALID_ARG, ERR_FULL, ERR_NOT_READY, ERR_EMPTY, ERR_HIP, ERR_TOO_LARGE = 0, -1, -2, -3, -4, -5, -6
STATUS_NAMES = {0: "APEX_OK", -1: "APEX_ERR_INVALID_ARG", -2: "APEX_ERR_FULL", -3: "APEX_ERR_NOT_READY",
                -4: "APEX_ERR_EMPTY", -5: "APEX_ERR_HIP", -6: "APEX_ERR_TOO_LARGE"}
MAX_SAMPLES_PER_CALL = 65536
MAX_BATCHES_PER_CALL = 1024
NOALLOC_MAX_SAMPLES = 16384
TREE_MAX_LEVELS = 8

EXPORTS = ["apex_replay_workspace_bytes", "apex_replay_create", "apex_replay_destroy", "apex_replay_layout",
           "apex_nstep_priorities", "apex_replay_add", "apex_replay_add_payload", "apex_replay_add_publish",
           "apex_replay_sample", "apex_replay_sample_noalloc", "apex_replay_sample_begin", "apex_replay_sample_finish",
           "apex_replay_sample_finish_update", "apex_replay_sample_finish_writeback", "apex_replay_gather",
           "apex_replay_update_priorities", "apex_replay_update_from_q", "apex_replay_evict", "apex_replay_resync", "apex_replay_stats",
           "apex_last_hip_error", "apex_pipeline_create", "apex_pipeline_destroy", "apex_pipeline_fork",
           "apex_pipeline_join", "apex_pipeline_steps", "apex_pipeline_add_begin", "apex_pipeline_add_end",
           "apex_pipeline_capture_begin", "apex_pipeline_capture_end", "apex_pipeline_replay",
           "apex_pe_workspace_bytes", "apex_pe_create", "apex_pe_destroy", "apex_pe_layout", "apex_pe_add",
           "apex_pe_sample", "apex_pe_update_priorities", "apex_pe_evict", "apex_pe_stats",
           "apex_pe_evict_enqueue", "apex_pe_add_round", "apex_pe_sample_update",
           "apex_codec_row_bytes", "apex_replay_add_payload_encoded", "apex_replay_gather_decoded",
           "apex_pipeline_set_codec"]


class Config(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("max_slots", C.c_uint64), ("obs_bytes", C.c_uint32),
                ("act_bytes", C.c_uint32), ("alpha", C.c_float), ("eps", C.c_float), ("frac_bits", C.c_uint32),
                ("reserved", C.c_uint32), ("min_size_to_sample", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("size", "head", "tail", "root", "n_stale_dropped", "n_clamped")]


class Layout(C.Structure):
    _fields_ = [("obs_offset", C.c_uint64), ("act_offset", C.c_uint64), ("ret_offset", C.c_uint64),
                ("gacc_offset", C.c_uint64), ("tree_levels", C.c_uint32), ("tree_fanout", C.c_uint32),
                ("level_offset", C.c_uint64 * TREE_MAX_LEVELS), ("level_size", C.c_uint64 * TREE_MAX_LEVELS)]


class BatchBuffers(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("key", "slot", "mass", "weight", "obs", "act", "ret", "gacc")]


class PeConfig(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("max_slots", C.c_uint64), ("obs_bytes", C.c_uint32),
                ("act_bytes", C.c_uint32), ("alpha", C.c_float), ("alpha_evict", C.c_float), ("eps", C.c_float),
                ("frac_bits", C.c_uint32)]


class PeStats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in ("size", "inserted", "evicted", "root", "root_evict", "free_head",
                                          "free_tail", "n_stale_dropped", "n_clamped")]


class PeLayout(C.Structure):
    _fields_ = [("obs_offset", C.c_uint64), ("act_offset", C.c_uint64), ("ret_offset", C.c_uint64),
                ("gacc_offset", C.c_uint64), ("tree_levels", C.c_uint32), ("tree_fanout", C.c_uint32),
                ("level_offset", C.c_uint64 * TREE_MAX_LEVELS), ("level_size", C.c_uint64 * TREE_MAX_LEVELS),
                ("evict_tree_offset", C.c_uint64), ("gen_offset", C.c_uint64), ("free_ring_offset", C.c_uint64)]


PE_MAX_EVICT_PER_CALL = 1 << 20

if not os.path.exists(LIB_PATH):
    raise ImportError("%s is missing: build it first (python paper_1803_00933_amd/build.py or "
                      "__graft_entry__.build()); there is no fallback path" % LIB_PATH)

lib = C.CDLL(LIB_PATH)
_vp, _u32, _u64, _f32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_float
lib.apex_replay_workspace_bytes.argtypes = [C.POINTER(Config)] + [C.POINTER(C.c_size_t)] * 3
lib.apex_replay_create.argtypes = [C.POINTER(Config), _vp, _vp, _vp, C.POINTER(_vp)]
lib.apex_replay_destroy.argtypes = [_vp]
lib.apex_replay_layout.argtypes = [_vp, C.POINTER(Layout)]
lib.apex_nstep_priorities.argtypes = [_u32, _u32, _u32, _u32, _vp, _vp, _vp, _vp, _vp, _f32, _f32, _u32, _u64,
                                      _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_add.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp, C.POINTER(_u64), _vp]
lib.apex_replay_sample.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_sample_noalloc.argtypes = lib.apex_replay_sample.argtypes
lib.apex_replay_add_payload.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_add_publish.argtypes = [_vp, _u64, _vp, C.POINTER(_u64), _vp]
lib.apex_replay_sample_begin.argtypes = [_vp, _u32, _u32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_sample_finish.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_sample_finish_update.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _u64, _vp, _vp, _vp]
lib.apex_replay_sample_finish_writeback.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_resync.argtypes = [_vp, _vp]
lib.apex_replay_gather.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_update_priorities.argtypes = [_vp, _u64, _vp, _vp, _vp]
lib.apex_codec_row_bytes.restype = C.c_size_t
lib.apex_codec_row_bytes.argtypes = [_u32]
lib.apex_replay_add_payload_encoded.argtypes = [_vp, _u64, _vp, _u32, _vp, _vp, _vp, _vp]
lib.apex_replay_gather_decoded.argtypes = [_vp, _u64, _vp, _u32, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_update_from_q.argtypes = [_vp, _u64, _vp, _u32, _vp, _vp, _vp, _vp, _vp]
lib.apex_replay_evict.argtypes = [_vp, C.POINTER(_u64), _vp]
lib.apex_replay_stats.argtypes = [_vp, C.POINTER(Stats), _vp]
lib.apex_last_hip_error.argtypes = []
lib.apex_pipeline_create.argtypes = [_vp, _u32, C.POINTER(BatchBuffers), _u32, _u32, C.POINTER(_vp)]
lib.apex_pipeline_destroy.argtypes = [_vp]
lib.apex_pipeline_fork.argtypes = [_vp, _vp]
lib.apex_pipeline_join.argtypes = [_vp, _vp]
lib.apex_pipeline_steps.argtypes = [_vp, _u32, _f32, _vp, _vp, C.POINTER(_u32)]
lib.apex_pipeline_set_codec.argtypes = [_vp, _u32]
lib.apex_pipeline_add_begin.argtypes = [_vp, _u32, _u32, _u32, _u32] + [_vp] * 10
lib.apex_pipeline_add_end.argtypes = [_vp, C.c_int, C.POINTER(_u64), C.POINTER(_u64)]
lib.apex_pipeline_capture_begin.argtypes = [_vp]
lib.apex_pipeline_capture_end.argtypes = [_vp]
lib.apex_pipeline_replay.argtypes = [_vp, _u32]
lib.apex_pe_workspace_bytes.argtypes = [C.POINTER(PeConfig)] + [C.POINTER(C.c_size_t)] * 3
lib.apex_pe_create.argtypes = [C.POINTER(PeConfig), _vp, _vp, _vp, C.POINTER(_vp)]
lib.apex_pe_destroy.argtypes = [_vp]
lib.apex_pe_layout.argtypes = [_vp, C.POINTER(PeLayout)]
lib.apex_pe_add.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_pe_sample.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
lib.apex_pe_update_priorities.argtypes = [_vp, _u64, _vp, _vp, _vp]
lib.apex_pe_evict.argtypes = [_vp, _u32, _vp, C.POINTER(_u64), _vp]
lib.apex_pe_stats.argtypes = [_vp, C.POINTER(PeStats), _vp]
lib.apex_pe_evict_enqueue.argtypes = [_vp, _u32, _vp, C.POINTER(_u64), _vp]
lib.apex_pe_add_round.argtypes = [_vp, _u32, _u32, _u32, _u32] + [_vp] * 8
lib.apex_pe_sample_update.argtypes = [_vp, _u32, _f32] + [_vp] * 10
for _name in EXPORTS:
    getattr(lib, _name).restype = C.c_int


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device, contiguous tensors only"
    return t.data_ptr()


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def workspace_bytes(cfg: Config):
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    rc = lib.apex_replay_workspace_bytes(C.byref(cfg), C.byref(a), C.byref(b), C.byref(c))
    return rc, a.value, b.value, c.value


def nstep_priorities(q_online, q_target, action, reward, discount, n, alpha, eps, frac_bits, max_slots=0,
                     want_fx=True, out=None, stream=None):
    """Device tensors: q_* [S,T+n,A] fp32, action int32 / reward / discount fp32 [S,T+n].
    Returns (rc, prio, ret, gacc, prio_fx) with outputs of shape [S,T]."""
    S, L, A = q_online.shape
    T = L - n
    dev = q_online.device
    if out is None:
        prio = torch.empty((S, T), dtype=torch.float32, device=dev)
        ret = torch.empty_like(prio)
        gacc = torch.empty_like(prio)
        fx = torch.empty((S, T), dtype=torch.int64, device=dev) if want_fx else None
    else:
        prio, ret, gacc, fx = out
    rc = lib.apex_nstep_priorities(S, T, n, A, _ptr(q_online), _ptr(q_target), _ptr(action), _ptr(reward),
                                   _ptr(discount), alpha, eps, frac_bits, max_slots, _ptr(prio), _ptr(ret),
                                   _ptr(gacc), _ptr(fx), _stream(stream))
    return rc, prio, ret, gacc, fx


class Replay:
    """Owns the three device regions (as torch tensors) and the library handle."""

    def __init__(self, capacity, max_slots, obs_bytes, act_bytes, alpha=0.6, eps=1e-6, frac_bits=24,
                 min_size_to_sample=0, device="cuda:0"):
        self.cfg = Config(capacity, max_slots, obs_bytes, act_bytes, alpha, eps, frac_bits, 0, min_size_to_sample)
        rc, sb, tb, cb = workspace_bytes(self.cfg)
        if rc != OK:
            raise ValueError("configuration rejected: %s" % STATUS_NAMES.get(rc, rc))
        self.device = torch.device(device)
        self.storage = torch.empty(sb, dtype=torch.uint8, device=self.device)
        self.tree = torch.empty(tb // 8, dtype=torch.int64, device=self.device)
        self.scratch = torch.empty(cb, dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize(self.device)
        h = _vp(None)
        rc = lib.apex_replay_create(C.byref(self.cfg), self.storage.data_ptr(), self.tree.data_ptr(),
                                    self.scratch.data_ptr(), C.byref(h))
        if rc != OK:
            raise RuntimeError("apex_replay_create: %s (hip %d)" % (STATUS_NAMES.get(rc, rc), lib.apex_last_hip_error()))
        self.h = h
        self.capacity, self.max_slots, self.obs_bytes, self.act_bytes = capacity, max_slots, obs_bytes, act_bytes
        lay = Layout()
        lib.apex_replay_layout(self.h, C.byref(lay))
        self.layout = lay

    def close(self):
        if getattr(self, "h", None) and lib is not None:     # (lib is None while the interpreter shuts down)
            lib.apex_replay_destroy(self.h)
            self.h = None

    __del__ = close

    # -- views of the caller-owned regions (for tests) ------------------------------------------
    def obs_view(self):
        o = self.layout.obs_offset
        return self.storage[o:o + self.max_slots * self.obs_bytes].view(self.max_slots, self.obs_bytes)

    def act_view(self):
        o = self.layout.act_offset
        return self.storage[o:o + self.max_slots * self.act_bytes].view(self.max_slots, self.act_bytes)

    def ret_view(self):
        o = self.layout.ret_offset
        return self.storage[o:o + self.max_slots * 4].view(torch.float32)

    def gacc_view(self):
        o = self.layout.gacc_offset
        return self.storage[o:o + self.max_slots * 4].view(torch.float32)

    def level_view(self, l):
        o, n = self.layout.level_offset[l], self.layout.level_size[l]
        return self.tree[o:o + n]

    # -- the replay verbs -----------------------------------------------------------------------
    def add(self, prio, obs=None, act=None, ret=None, gacc=None, stream=None):
        first = _u64(0)
        rc = lib.apex_replay_add(self.h, prio.shape[0], _ptr(obs), _ptr(act), _ptr(ret), _ptr(gacc), _ptr(prio),
                                 C.byref(first), _stream(stream))
        return rc, int(first.value)

    def alloc_sample_outputs(self, num_batches, k, payload=True):
        n, dev = num_batches * k, self.device
        out = dict(key=torch.empty(n, dtype=torch.int64, device=dev),
                   slot=torch.empty(n, dtype=torch.int32, device=dev),
                   weight=torch.empty(n, dtype=torch.float32, device=dev))
        if payload:
            out.update(obs=torch.empty((n, self.obs_bytes), dtype=torch.uint8, device=dev),
                       act=torch.empty((n, self.act_bytes), dtype=torch.uint8, device=dev),
                       ret=torch.empty(n, dtype=torch.float32, device=dev),
                       gacc=torch.empty(n, dtype=torch.float32, device=dev))
        return out

    def sample(self, num_batches, k, beta, rnd, out=None, payload=True, stream=None):
        if out is None:
            out = self.alloc_sample_outputs(num_batches, k, payload)
        rc = lib.apex_replay_sample(self.h, num_batches, k, beta, _ptr(rnd), _ptr(out.get("key")), _ptr(out["slot"]),
                                    _ptr(out.get("weight")), _ptr(out.get("obs")), _ptr(out.get("act")),
                                    _ptr(out.get("ret")), _ptr(out.get("gacc")), _stream(stream))
        return rc, out

    def sample_noalloc(self, num_batches, k, beta, rnd, out, stream=None):
        """apex_replay_sample_noalloc into caller-made outputs (see alloc_sample_outputs)."""
        return lib.apex_replay_sample_noalloc(self.h, num_batches, k, beta, _ptr(rnd), _ptr(out.get("key")),
                                              _ptr(out["slot"]), _ptr(out.get("weight")), _ptr(out.get("obs")),
                                              _ptr(out.get("act")), _ptr(out.get("ret")), _ptr(out.get("gacc")),
                                              _stream(stream))

    def add_payload(self, count, obs=None, act=None, ret=None, gacc=None, stream=None):
        return lib.apex_replay_add_payload(self.h, count, _ptr(obs), _ptr(act), _ptr(ret), _ptr(gacc), _stream(stream))

    def add_publish(self, prio, stream=None):
        first = _u64(0)
        rc = lib.apex_replay_add_publish(self.h, prio.shape[0], _ptr(prio), C.byref(first), _stream(stream))
        return rc, int(first.value)

    def sample_begin(self, num_batches, k, rnd, out, stream=None):
        """out needs 'slot' and 'mass' (int64 [nb*k]); 'key', 'act', 'ret', 'gacc' are optional."""
        return lib.apex_replay_sample_begin(self.h, num_batches, k, _ptr(rnd), _ptr(out.get("key")), _ptr(out["slot"]),
                                            _ptr(out["mass"]), _ptr(out.get("act")), _ptr(out.get("ret")),
                                            _ptr(out.get("gacc")), _stream(stream))

    def sample_finish(self, num_batches, k, beta, out, stream=None):
        return lib.apex_replay_sample_finish(self.h, num_batches, k, beta, _ptr(out["slot"]), _ptr(out.get("mass")),
                                             _ptr(out.get("weight")), _ptr(out.get("obs")), _stream(stream))

    def sample_finish_update(self, num_batches, k, beta, out, key, prio, stream=None):
        return lib.apex_replay_sample_finish_update(self.h, num_batches, k, beta, _ptr(out["slot"]),
                                                    _ptr(out.get("mass")), _ptr(out.get("weight")),
                                                    _ptr(out.get("obs")), key.shape[0], _ptr(key), _ptr(prio),
                                                    _stream(stream))

    def sample_finish_writeback(self, num_batches, k, beta, out, prio, stream=None):
        return lib.apex_replay_sample_finish_writeback(self.h, num_batches, k, beta, _ptr(out["key"]), _ptr(out["slot"]),
                                                       _ptr(out["mass"]), _ptr(out.get("weight")), _ptr(out.get("obs")),
                                                       _ptr(prio), _stream(stream))

    def resync(self, stream=None):
        return lib.apex_replay_resync(self.h, _stream(stream))

    def gather(self, slot, obs=None, act=None, ret=None, gacc=None, stream=None):
        return lib.apex_replay_gather(self.h, slot.shape[0], _ptr(slot), _ptr(obs), _ptr(act), _ptr(ret), _ptr(gacc),
                                      _stream(stream))

    def update_priorities(self, key, prio, stream=None):
        return lib.apex_replay_update_priorities(self.h, key.shape[0], _ptr(key), _ptr(prio), _stream(stream))

    def add_payload_encoded(self, raw_obs, act=None, ret=None, gacc=None, stream=None):
        """raw_obs: uint8 [count, raw_bytes], stored through the observation codec."""
        return lib.apex_replay_add_payload_encoded(self.h, raw_obs.shape[0], _ptr(raw_obs), raw_obs.shape[1], _ptr(act),
                                                   _ptr(ret), _ptr(gacc), _stream(stream))

    def gather_decoded(self, slot, obs, act=None, ret=None, gacc=None, stream=None):
        """obs: uint8 [count, raw_bytes] receives the decoded observations of the slots."""
        return lib.apex_replay_gather_decoded(self.h, slot.shape[0], _ptr(slot), obs.shape[1], _ptr(obs), _ptr(act),
                                              _ptr(ret), _ptr(gacc), _stream(stream))

    def update_from_q(self, key, q_taken, q_online_next, q_target_next, prio_out=None, stream=None):
        return lib.apex_replay_update_from_q(self.h, key.shape[0], _ptr(key), q_online_next.shape[1], _ptr(q_taken),
                                             _ptr(q_online_next), _ptr(q_target_next), _ptr(prio_out),
                                             _stream(stream))

    def evict(self, stream=None):
        e = _u64(0)
        rc = lib.apex_replay_evict(self.h, C.byref(e), _stream(stream))
        return rc, int(e.value)

    def stats(self, stream=None):
        st = Stats()
        rc = lib.apex_replay_stats(self.h, C.byref(st), _stream(stream))
        if rc != OK:
            raise RuntimeError("apex_replay_stats: %s" % STATUS_NAMES.get(rc, rc))
        return {n: int(getattr(st, n)) for n, _ in Stats._fields_}


class Pipeline:
    """Binding of apex_pipeline_*: the verbs on two internal streams.  Owns `depth` output sets."""

    def __init__(self, rep: Replay, depth, num_batches, k):
        self.rep, self.depth, self.nb, self.k = rep, depth, num_batches, k
        self.sets = []
        arr = (BatchBuffers * depth)()
        for i in range(depth):
            o = rep.alloc_sample_outputs(num_batches, k)
            o["mass"] = torch.empty(num_batches * k, dtype=torch.int64, device=rep.device)
            self.sets.append(o)
            for name, _ in BatchBuffers._fields_:
                setattr(arr[i], name, o[name].data_ptr())
        h = _vp(None)
        rc = lib.apex_pipeline_create(rep.h, depth, arr, num_batches, k, C.byref(h))
        if rc != OK:
            raise RuntimeError("apex_pipeline_create: %s" % STATUS_NAMES.get(rc, rc))
        self.h = h

    def close(self):
        if getattr(self, "h", None) and lib is not None:
            lib.apex_pipeline_destroy(self.h)
            self.h = None

    __del__ = close

    def fork(self, after=None):
        return lib.apex_pipeline_fork(self.h, _stream(after))

    def join(self, stream=None):
        return lib.apex_pipeline_join(self.h, _stream(stream))

    def set_codec(self, raw_bytes):
        """Observations through the block codec: the sets' 'obs' become [nb*k, raw_bytes] views of their buffers."""
        rc = lib.apex_pipeline_set_codec(self.h, raw_bytes)
        if rc == OK:
            for o in self.sets:
                base = o.setdefault("obs_buffer", o["obs"])
                n = self.nb * self.k
                o["obs"] = base.view(-1)[:n * raw_bytes].view(n, raw_bytes) if raw_bytes else base
        return rc

    def steps(self, n, beta, rnd, new_prio=None):
        first = _u32(0)
        rc = lib.apex_pipeline_steps(self.h, n, beta, _ptr(rnd), _ptr(new_prio), C.byref(first))
        return rc, int(first.value)

    def add_begin(self, q_online, q_target, action, reward, discount, n, obs, act, prio, ret, gacc):
        S, L, A = q_online.shape
        return lib.apex_pipeline_add_begin(self.h, S, L - n, n, A, _ptr(q_online), _ptr(q_target), _ptr(action),
                                           _ptr(reward), _ptr(discount), _ptr(obs), _ptr(act), _ptr(prio), _ptr(ret),
                                           _ptr(gacc))

    def capture_begin(self):
        return lib.apex_pipeline_capture_begin(self.h)

    def capture_end(self):
        return lib.apex_pipeline_capture_end(self.h)

    def replay(self, times=1):
        return lib.apex_pipeline_replay(self.h, times)

    def add_end(self, evict=False):
        first, ev = _u64(0), _u64(0)
        rc = lib.apex_pipeline_add_end(self.h, int(evict), C.byref(first), C.byref(ev))
        return rc, int(first.value), int(ev.value)


class PeReplay:
    """Binding of apex_pe_*: the memory with prioritized eviction.  Owns its three device regions."""

    def __init__(self, capacity, max_slots, obs_bytes, act_bytes, alpha=0.6, alpha_evict=-0.4, eps=1e-6, frac_bits=24,
                 device="cuda:0"):
        self.cfg = PeConfig(capacity, max_slots, obs_bytes, act_bytes, alpha, alpha_evict, eps, frac_bits)
        a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
        rc = lib.apex_pe_workspace_bytes(C.byref(self.cfg), C.byref(a), C.byref(b), C.byref(c))
        if rc != OK:
            raise ValueError("configuration rejected: %s" % STATUS_NAMES.get(rc, rc))
        self.device = torch.device(device)
        self.storage = torch.empty(a.value, dtype=torch.uint8, device=self.device)
        self.tree = torch.empty(b.value // 8, dtype=torch.int64, device=self.device)
        self.scratch = torch.empty(c.value, dtype=torch.uint8, device=self.device)
        torch.cuda.synchronize(self.device)
        h = _vp(None)
        rc = lib.apex_pe_create(C.byref(self.cfg), self.storage.data_ptr(), self.tree.data_ptr(),
                                self.scratch.data_ptr(), C.byref(h))
        if rc != OK:
            raise RuntimeError("apex_pe_create: %s" % STATUS_NAMES.get(rc, rc))
        self.h = h
        self.capacity, self.max_slots, self.obs_bytes, self.act_bytes = capacity, max_slots, obs_bytes, act_bytes
        self.layout = PeLayout()
        lib.apex_pe_layout(self.h, C.byref(self.layout))

    def close(self):
        if getattr(self, "h", None) and lib is not None:
            lib.apex_pe_destroy(self.h)
            self.h = None

    __del__ = close

    def level_view(self, l, evict_tree=False):
        o = self.layout.level_offset[l] + (self.layout.evict_tree_offset if evict_tree else 0)
        return self.tree[o:o + self.layout.level_size[l]]

    def gen_view(self):
        o = self.layout.gen_offset
        return self.scratch[o:o + 4 * self.max_slots].view(torch.int32)

    def free_ring_view(self):
        o = self.layout.free_ring_offset
        return self.scratch[o:o + 4 * self.max_slots].view(torch.int32)

    def obs_view(self):
        o = self.layout.obs_offset
        return self.storage[o:o + self.max_slots * self.obs_bytes].view(self.max_slots, self.obs_bytes)

    def add(self, prio, obs=None, act=None, ret=None, gacc=None, stream=None):
        return lib.apex_pe_add(self.h, prio.shape[0], _ptr(obs), _ptr(act), _ptr(ret), _ptr(gacc), _ptr(prio),
                               _stream(stream))

    def alloc_sample_outputs(self, num_batches, k):
        n, dev = num_batches * k, self.device
        return dict(key=torch.empty(n, dtype=torch.int64, device=dev), slot=torch.empty(n, dtype=torch.int32, device=dev),
                    weight=torch.empty(n, dtype=torch.float32, device=dev),
                    obs=torch.empty((n, self.obs_bytes), dtype=torch.uint8, device=dev),
                    act=torch.empty((n, self.act_bytes), dtype=torch.uint8, device=dev),
                    ret=torch.empty(n, dtype=torch.float32, device=dev),
                    gacc=torch.empty(n, dtype=torch.float32, device=dev))

    def sample(self, num_batches, k, beta, rnd, out=None, stream=None):
        if out is None:
            out = self.alloc_sample_outputs(num_batches, k)
        rc = lib.apex_pe_sample(self.h, num_batches, k, beta, _ptr(rnd), _ptr(out.get("key")), _ptr(out["slot"]),
                                _ptr(out.get("weight")), _ptr(out.get("obs")), _ptr(out.get("act")),
                                _ptr(out.get("ret")), _ptr(out.get("gacc")), _stream(stream))
        return rc, out

    def update_priorities(self, key, prio, stream=None):
        return lib.apex_pe_update_priorities(self.h, key.shape[0], _ptr(key), _ptr(prio), _stream(stream))

    def evict(self, rounds, rnd, stream=None):
        e = _u64(0)
        rc = lib.apex_pe_evict(self.h, rounds, _ptr(rnd), C.byref(e), _stream(stream))
        return rc, int(e.value)

    def evict_enqueue(self, rounds, rnd, stream=None):
        """apex_pe_evict_enqueue: returns (rc, number of evictions asked for) without waiting for the eviction."""
        e = _u64(0)
        rc = lib.apex_pe_evict_enqueue(self.h, rounds, _ptr(rnd), C.byref(e), _stream(stream))
        return rc, int(e.value)

    def add_round(self, q_online, q_target, action, reward, discount, n, obs, act=None, stream=None):
        S, L, A = q_online.shape
        return lib.apex_pe_add_round(self.h, S, L - n, n, A, _ptr(q_online), _ptr(q_target), _ptr(action), _ptr(reward),
                                     _ptr(discount), _ptr(obs), _ptr(act), _stream(stream))

    def sample_update(self, k, beta, rnd, new_prio, out, stream=None):
        return lib.apex_pe_sample_update(self.h, k, beta, _ptr(rnd), _ptr(new_prio), _ptr(out["key"]), _ptr(out["slot"]),
                                         _ptr(out.get("weight")), _ptr(out.get("obs")), _ptr(out.get("act")),
                                         _ptr(out.get("ret")), _ptr(out.get("gacc")), _stream(stream))

    def stats(self, stream=None):
        st = PeStats()
        rc = lib.apex_pe_stats(self.h, C.byref(st), _stream(stream))
        if rc != OK:
            raise RuntimeError("apex_pe_stats: %s" % STATUS_NAMES.get(rc, rc))
        return {n: int(getattr(st, n)) for n, _ in PeStats._fields_}
