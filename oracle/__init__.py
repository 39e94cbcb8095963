"""CPU oracle of the Ape-X replay-memory hot path -- TEST INFRASTRUCTURE ONLY.

ctypes front end of ``apex_oracle.c``.  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import this package; the product package never
does.  Nothing here touches a GPU.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "apex_oracle.c")
_SO = os.path.join(_HERE, "libapex_oracle.so")

OK, ERR_INVALID_ARG, ERR_FULL, ERR_NOT_READY, ERR_EMPTY = 0, -1, -2, -3, -4


_SO_SAN = os.path.join(_HERE, "libapex_oracle_san.so")
SANITIZE_ENV = "APEX_ORACLE_SANITIZE"      # "1": load the build with AddressSanitizer + UndefinedBehaviorSanitizer


def build(force=False, sanitize=False):
    """Compile the oracle with the host C compiler (no HIP, no GPU).  sanitize: the same source with
    -fsanitize=address,undefined (the process that loads it needs the AddressSanitizer runtime preloaded;
    tests/test_host_sanitizers.py does that in a child process)."""
    so = _SO_SAN if sanitize else _SO
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(_SRC):
        tmp = so + ".tmp.%d" % os.getpid()
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=undefined"] if sanitize else ["-O2"]
        subprocess.check_call(["gcc"] + opt + ["-std=c11", "-ffp-contract=off", "-mfma", "-Wall", "-Wextra",
                                               "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, so)
    return so


_lib = None
_u64, _u32, _f32, _i32, _vp = C.c_uint64, C.c_uint32, C.c_float, C.c_int32, C.c_void_p


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build(sanitize=os.environ.get(SANITIZE_ENV, "") == "1"))
        L.oracle_pow_spec.restype = _f32
        L.oracle_pow_spec.argtypes = [_f32, _f32]
        L.oracle_quantise.restype = _u64
        L.oracle_quantise.argtypes = [_f32, _f32, _f32, _u32, _u64, C.POINTER(C.c_int)]
        L.oracle_qmax.restype = _u64
        L.oracle_qmax.argtypes = [_u64]
        L.oracle_nstep_priorities.restype = None
        L.oracle_nstep_priorities.argtypes = [_u32, _u32, _u32, _u32, _vp, _vp, _vp, _vp, _vp,
                                              _f32, _f32, _u32, _u64, _vp, _vp, _vp, _vp]
        L.oracle_replay_create.restype = _vp
        L.oracle_replay_create.argtypes = [_u64, _u64, _u32, _u32, _f32, _f32, _u32, _u64, _u64]
        L.oracle_replay_destroy.restype = None
        L.oracle_replay_destroy.argtypes = [_vp]
        L.oracle_replay_add.restype = C.c_int
        L.oracle_replay_add.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp, C.POINTER(_u64)]
        L.oracle_replay_sample.restype = C.c_int
        L.oracle_replay_sample.argtypes = [_vp, _u32, _u32, _f32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]
        L.oracle_replay_sample_linear.restype = C.c_int
        L.oracle_replay_sample_linear.argtypes = [_vp, _u32, _vp, _vp]
        L.oracle_replay_update_priorities.restype = C.c_int
        L.oracle_replay_update_priorities.argtypes = [_vp, _u64, _vp, _vp]
        L.oracle_replay_update_from_q.restype = C.c_int
        L.oracle_replay_update_from_q.argtypes = [_vp, _u64, _vp, _u32, _vp, _vp, _vp, _vp]
        L.oracle_replay_evict.restype = C.c_int
        L.oracle_replay_evict.argtypes = [_vp, C.POINTER(_u64)]
        for name in ("head", "tail", "root", "n_stale", "n_clamped", "tree_leaves"):
            f = getattr(L, "oracle_replay_" + name)
            f.restype, f.argtypes = _u64, [_vp]
        L.oracle_replay_nodes.restype = C.POINTER(_u64)
        L.oracle_replay_nodes.argtypes = [_vp]
        L.oracle_replay_leaves.restype = None
        L.oracle_replay_leaves.argtypes = [_vp, _u64, _u64, _vp]
        L.oracle_codec_row_bytes.restype = _u64
        L.oracle_codec_row_bytes.argtypes = [_u32]
        L.oracle_codec_encode_row.restype = C.c_int
        L.oracle_codec_encode_row.argtypes = [_vp, _u32, _vp, C.POINTER(_u64)]
        L.oracle_codec_decode_row.restype = C.c_int
        L.oracle_codec_decode_row.argtypes = [_vp, _u32, _vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(_vp)


def _arr(a, dtype):
    if a is None:
        return None
    return np.ascontiguousarray(a, dtype=dtype)


def pow_spec(x, alpha):
    return float(lib().oracle_pow_spec(float(x), float(alpha)))


def qmax(max_slots):
    return int(lib().oracle_qmax(int(max_slots)))


def quantise(p, alpha, eps, frac_bits, qmax_):
    c = C.c_int(0)
    q = lib().oracle_quantise(float(p), float(alpha), float(eps), int(frac_bits), int(qmax_), C.byref(c))
    return int(q), bool(c.value)


def nstep_priorities(q_online, q_target, action, reward, discount, n, alpha, eps, frac_bits, max_slots=0):
    """q_*: [S,T+n,A] fp32; action/reward/discount: [S,T+n].  Returns prio, ret, gacc, prio_fx of shape [S,T]."""
    q_online = _arr(q_online, np.float32)
    q_target = _arr(q_target, np.float32)
    action = _arr(action, np.int32)
    reward = _arr(reward, np.float32)
    discount = _arr(discount, np.float32)
    S, L, A = q_online.shape
    T = L - n
    prio = np.empty((S, T), np.float32)
    ret = np.empty((S, T), np.float32)
    gacc = np.empty((S, T), np.float32)
    fx = np.empty((S, T), np.uint64)
    lib().oracle_nstep_priorities(S, T, n, A, _p(q_online), _p(q_target), _p(action), _p(reward), _p(discount),
                                  alpha, eps, frac_bits, max_slots, _p(prio), _p(ret), _p(gacc), _p(fx))
    return prio, ret, gacc, fx


def codec_row_bytes(raw_bytes):
    """Stride of an encoded observation row (0: raw_bytes is no positive multiple of 64)."""
    return int(lib().oracle_codec_row_bytes(int(raw_bytes)))


def codec_encode(rows):
    """rows: uint8 [n, raw_bytes] -> (encoded uint8 [n, codec_row_bytes], bytes that carry data [n])."""
    rows = _arr(rows, np.uint8)
    n, raw_bytes = rows.shape
    cap = codec_row_bytes(raw_bytes)
    if not cap:
        raise ValueError("raw_bytes must be a positive multiple of 64")
    enc = np.empty((n, cap), np.uint8)
    used = np.empty(n, np.uint64)
    u = _u64(0)
    for i in range(n):
        rc = lib().oracle_codec_encode_row(_p(rows[i]), raw_bytes, _p(enc[i]), C.byref(u))
        assert rc == OK
        used[i] = u.value
    return enc, used


def codec_decode(enc, raw_bytes):
    """enc: uint8 [n, >= codec_row_bytes(raw_bytes)] -> uint8 [n, raw_bytes]."""
    enc = _arr(enc, np.uint8)
    out = np.empty((enc.shape[0], raw_bytes), np.uint8)
    for i in range(enc.shape[0]):
        assert lib().oracle_codec_decode_row(_p(enc[i]), raw_bytes, _p(out[i])) == OK
    return out


class Replay:
    """Plain array sum-tree + ring; mirrors the six replay verbs."""

    def __init__(self, capacity, max_slots, obs_bytes, act_bytes, alpha=0.6, eps=1e-6, frac_bits=24,
                 min_size_to_sample=0, payload_slots=None):
        if payload_slots is None:
            payload_slots = max_slots
        self.h = lib().oracle_replay_create(capacity, max_slots, obs_bytes, act_bytes, alpha, eps, frac_bits,
                                            min_size_to_sample, payload_slots)
        if not self.h:
            raise ValueError("oracle_replay_create rejected the configuration")
        self.capacity, self.max_slots = capacity, max_slots
        self.obs_bytes, self.act_bytes = obs_bytes, act_bytes
        self.has_payload = payload_slots > 0

    def close(self):
        if self.h:
            lib().oracle_replay_destroy(self.h)
            self.h = None

    __del__ = close

    head = property(lambda s: int(lib().oracle_replay_head(s.h)))
    tail = property(lambda s: int(lib().oracle_replay_tail(s.h)))
    size = property(lambda s: s.tail - s.head)
    root = property(lambda s: int(lib().oracle_replay_root(s.h)))
    n_stale = property(lambda s: int(lib().oracle_replay_n_stale(s.h)))
    n_clamped = property(lambda s: int(lib().oracle_replay_n_clamped(s.h)))

    def leaves(self, first=0, count=None):
        count = self.max_slots - first if count is None else count
        out = np.empty(count, np.uint64)
        lib().oracle_replay_leaves(self.h, first, count, _p(out))
        return out

    def nodes(self):
        n = 2 * int(lib().oracle_replay_tree_leaves(self.h))
        return np.ctypeslib.as_array(lib().oracle_replay_nodes(self.h), shape=(n,)).copy()

    def add(self, prio, obs=None, act=None, ret=None, gacc=None):
        prio = _arr(prio, np.float32)
        count = prio.shape[0]
        obs, act = _arr(obs, np.uint8), _arr(act, np.uint8)
        ret, gacc = _arr(ret, np.float32), _arr(gacc, np.float32)
        first = _u64(0)
        rc = lib().oracle_replay_add(self.h, count, _p(obs), _p(act), _p(ret), _p(gacc), _p(prio), C.byref(first))
        return rc, int(first.value)

    def sample(self, num_batches, k, beta, rnd, payload=True):
        rnd = _arr(rnd, np.uint64)
        assert rnd.size == num_batches * k
        n = num_batches * k
        out = dict(key=np.zeros(n, np.uint64), slot=np.zeros(n, np.uint32), weight=np.zeros(n, np.float32),
                   mass=np.zeros(n, np.uint64))
        if payload and self.has_payload:
            out.update(obs=np.zeros((n, self.obs_bytes), np.uint8), act=np.zeros((n, self.act_bytes), np.uint8),
                       ret=np.zeros(n, np.float32), gacc=np.zeros(n, np.float32))
        rc = lib().oracle_replay_sample(self.h, num_batches, k, beta, _p(rnd), _p(out["key"]), _p(out["slot"]),
                                        _p(out["weight"]), _p(out["mass"]), _p(out.get("obs")), _p(out.get("act")),
                                        _p(out.get("ret")), _p(out.get("gacc")))
        return rc, out

    def sample_linear(self, k, rnd):
        rnd = _arr(rnd, np.uint64)
        slot = np.zeros(k, np.uint32)
        rc = lib().oracle_replay_sample_linear(self.h, k, _p(rnd), _p(slot))
        return rc, slot

    def update_priorities(self, key, prio):
        key, prio = _arr(key, np.uint64), _arr(prio, np.float32)
        return lib().oracle_replay_update_priorities(self.h, key.shape[0], _p(key), _p(prio))

    def update_from_q(self, key, q_taken, q_online_next, q_target_next):
        key = _arr(key, np.uint64)
        q_taken, qo, qt = _arr(q_taken, np.float32), _arr(q_online_next, np.float32), _arr(q_target_next, np.float32)
        prio = np.zeros(key.shape[0], np.float32)
        rc = lib().oracle_replay_update_from_q(self.h, key.shape[0], _p(key), qo.shape[1], _p(q_taken), _p(qo), _p(qt),
                                               _p(prio))
        return rc, prio

    def evict(self):
        e = _u64(0)
        rc = lib().oracle_replay_evict(self.h, C.byref(e))
        return rc, int(e.value)


class PrioritizedEvictionReplay:
    """Replay memory whose eviction is proportional prioritized sampling with its own exponent."""

    def __init__(self, capacity, max_slots, obs_bytes, act_bytes, alpha=0.6, alpha_evict=-0.4, eps=1e-6, frac_bits=24,
                 payload=True):
        L = lib()
        if not hasattr(L, "_pe_ready"):
            L.oracle_pe_create.restype = _vp
            L.oracle_pe_create.argtypes = [_u64, _u64, _u32, _u32, _f32, _f32, _f32, _u32, C.c_int]
            L.oracle_pe_destroy.restype = None
            L.oracle_pe_destroy.argtypes = [_vp]
            L.oracle_pe_add.restype = C.c_int
            L.oracle_pe_add.argtypes = [_vp, _u64, _vp, _vp, _vp, _vp, _vp, _vp]
            L.oracle_pe_sample.restype = C.c_int
            L.oracle_pe_sample.argtypes = [_vp, _u32, _u32, _f32] + [_vp] * 9
            L.oracle_pe_update_priorities.restype = C.c_int
            L.oracle_pe_update_priorities.argtypes = [_vp, _u64, _vp, _vp]
            L.oracle_pe_evict.restype = C.c_int
            L.oracle_pe_evict.argtypes = [_vp, _u32, _vp, C.POINTER(_u64)]
            for name in ("size", "root", "root_evict", "inserted", "evicted", "free_head", "free_tail", "n_stale",
                         "n_clamped", "tree_leaves"):
                f = getattr(L, "oracle_pe_" + name)
                f.restype, f.argtypes = _u64, [_vp]
            L.oracle_pe_leaves.restype = None
            L.oracle_pe_leaves.argtypes = [_vp, C.c_int, _vp]
            L.oracle_pe_nodes.restype = None
            L.oracle_pe_nodes.argtypes = [_vp, C.c_int, _vp]
            L.oracle_pe_gen.restype = None
            L.oracle_pe_gen.argtypes = [_vp, _vp]
            L.oracle_pe_free_ring.restype = None
            L.oracle_pe_free_ring.argtypes = [_vp, _vp]
            L._pe_ready = True
        self.h = L.oracle_pe_create(capacity, max_slots, obs_bytes, act_bytes, alpha, alpha_evict, eps, frac_bits,
                                    int(payload))
        if not self.h:
            raise ValueError("oracle_pe_create rejected the configuration")
        self.capacity, self.max_slots, self.obs_bytes, self.act_bytes = capacity, max_slots, obs_bytes, act_bytes
        self.has_payload = payload

    def close(self):
        if self.h:
            lib().oracle_pe_destroy(self.h)
            self.h = None

    __del__ = close

    def _get(self, name):
        return int(getattr(lib(), "oracle_pe_" + name)(self.h))

    size = property(lambda s: s._get("size"))
    root = property(lambda s: s._get("root"))
    root_evict = property(lambda s: s._get("root_evict"))
    inserted = property(lambda s: s._get("inserted"))
    evicted = property(lambda s: s._get("evicted"))
    free_head = property(lambda s: s._get("free_head"))
    free_tail = property(lambda s: s._get("free_tail"))
    n_stale = property(lambda s: s._get("n_stale"))
    n_clamped = property(lambda s: s._get("n_clamped"))

    def leaves(self, evict_tree=False):
        out = np.empty(self.max_slots, np.uint64)
        lib().oracle_pe_leaves(self.h, int(evict_tree), _p(out))
        return out

    def nodes(self, evict_tree=False):
        out = np.empty(2 * self._get("tree_leaves"), np.uint64)
        lib().oracle_pe_nodes(self.h, int(evict_tree), _p(out))
        return out

    def gen(self):
        out = np.empty(self.max_slots, np.uint32)
        lib().oracle_pe_gen(self.h, _p(out))
        return out

    def free_ring(self):
        out = np.empty(self.max_slots, np.uint32)
        lib().oracle_pe_free_ring(self.h, _p(out))
        return out

    def add(self, prio, obs=None, act=None, ret=None, gacc=None):
        prio = _arr(prio, np.float32)
        obs, act = _arr(obs, np.uint8), _arr(act, np.uint8)
        ret, gacc = _arr(ret, np.float32), _arr(gacc, np.float32)
        keys = np.zeros(prio.shape[0], np.uint64)
        rc = lib().oracle_pe_add(self.h, prio.shape[0], _p(obs), _p(act), _p(ret), _p(gacc), _p(prio), _p(keys))
        return rc, keys

    def sample(self, num_batches, k, beta, rnd, payload=True):
        rnd = _arr(rnd, np.uint64)
        n = num_batches * k
        out = dict(key=np.zeros(n, np.uint64), slot=np.zeros(n, np.uint32), weight=np.zeros(n, np.float32),
                   mass=np.zeros(n, np.uint64))
        if payload and self.has_payload:
            out.update(obs=np.zeros((n, self.obs_bytes), np.uint8), act=np.zeros((n, self.act_bytes), np.uint8),
                       ret=np.zeros(n, np.float32), gacc=np.zeros(n, np.float32))
        rc = lib().oracle_pe_sample(self.h, num_batches, k, beta, _p(rnd), _p(out["key"]), _p(out["slot"]),
                                    _p(out["weight"]), _p(out["mass"]), _p(out.get("obs")), _p(out.get("act")),
                                    _p(out.get("ret")), _p(out.get("gacc")))
        return rc, out

    def update_priorities(self, key, prio):
        key, prio = _arr(key, np.uint64), _arr(prio, np.float32)
        return lib().oracle_pe_update_priorities(self.h, key.shape[0], _p(key), _p(prio))

    def evict(self, rounds, rnd):
        rnd = _arr(rnd, np.uint64)
        e = _u64(0)
        rc = lib().oracle_pe_evict(self.h, rounds, _p(rnd), C.byref(e))
        return rc, int(e.value)
