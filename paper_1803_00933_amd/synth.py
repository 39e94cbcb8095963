"""Seeded synthetic inputs shaped like the paper's workloads.

This module only *draws inputs* (Q-values, rewards, terminations, uniforms, TD errors,
observation bytes).  It holds none of the replay method's arithmetic, so that both the
HIP library and the independent CPU oracle can be fed from it.

Every draw is a pure function of (seed, purpose tag, counter): ``numpy`` Philox streams
keyed by those integers, so any round of any schedule can be regenerated on its own.
Observation bytes are a pure function of (seed, key) through a 64-bit integer mixer, so a
59 GB store can be checked row by row without keeping a second copy.
"""
from dataclasses import dataclass, replace

import numpy as np

# ----------------------------------------------------------------------------------
# workload shapes
# ----------------------------------------------------------------------------------


@dataclass(frozen=True)
class Workload:
    name: str
    capacity: int           # soft limit on stored transitions
    max_slots: int          # physical ring size P
    obs_bytes: int          # opaque observation payload per transition
    act_bytes: int          # 4 = int32 action, 32 = fp32[8] action
    num_actions: int        # A (1 = critic values, continuous control)
    n: int                  # n-step
    gamma: float
    alpha: float
    beta: float
    eps: float
    frac_bits: int
    streams: int            # S actor streams per add round
    chunk: int              # T transitions per stream per round
    k: int                  # batch size
    num_batches: int        # batches per sample call
    td_dist: str            # distribution of the learner's new |TD| errors
    seed: int = 0

    @property
    def add_count(self):
        return self.streams * self.chunk

    def scaled(self, **kw):
        return replace(self, **kw)


WORKLOADS = {
    # capacity 4096, obs fp32[8], 4 actions, 8 streams x 50, batch 32
    "tiny": Workload("tiny", 4096, 8192, 32, 4, 4, 3, 0.99, 0.6, 0.4, 1e-6, 24, 8, 50, 32, 1, "absnormal"),
    # 2M transitions of 84x84x4 uint8, 18 actions, 360 streams x 50, batch 512
    "atari": Workload("atari", 2_000_000, 1 << 21, 84 * 84 * 4, 4, 18, 3, 0.99, 0.6, 0.4, 1e-6, 24,
                      360, 50, 512, 1, "lognormal1"),
    # 2^21 slots of 64 B, Pareto priorities, 16 prefetched batches of 512
    "skew": Workload("skew", 1 << 21, 1 << 21, 64, 4, 18, 3, 0.99, 0.6, 0.4, 1e-6, 24,
                     360, 50, 512, 16, "pareto"),
    # 1M transitions, obs fp32[64], action fp32[8], critic values, n=5, 64 streams x 50
    "control": Workload("control", 1_000_000, 1 << 20, 256, 32, 1, 5, 0.99, 0.6, 0.4, 1e-6, 24,
                        64, 50, 512, 1, "lognormal1"),
    # 2^24 slots of 128 B, 1024 streams x 50, batch 4096
    "scale": Workload("scale", 1 << 24, (1 << 24) + (1 << 20), 128, 4, 18, 3, 0.99, 0.6, 0.4, 1e-6, 24,
                      1024, 50, 4096, 1, "lognormal2"),
}

_TAGS = {"chunk": 1, "rnd": 2, "td": 3, "bulk": 4}


def _rng(seed, tag, counter):
    return np.random.Generator(np.random.Philox(key=[(int(seed) << 8) | _TAGS[tag], int(counter)]))


# ----------------------------------------------------------------------------------
# actor side: one round of S streams x (T+n) rows
# ----------------------------------------------------------------------------------

def actor_round(w: Workload, rnd_index: int, p_done: float = 0.05, with_payload: bool = True):
    """Inputs of one add round.  Q-values and rewards N(0,1); each step ends its episode with
    probability ``p_done`` (discount 0, else gamma); actions uniform."""
    g = _rng(w.seed, "chunk", rnd_index)
    S, L, A = w.streams, w.chunk + w.n, w.num_actions
    out = {
        "q_online": g.standard_normal((S, L, A), dtype=np.float32),
        "q_target": g.standard_normal((S, L, A), dtype=np.float32),
        "action": g.integers(0, A, (S, L), dtype=np.int32),
        "reward": g.standard_normal((S, L), dtype=np.float32),
    }
    done = g.random((S, L)) < p_done
    out["discount"] = np.where(done, np.float32(0.0), np.float32(w.gamma)).astype(np.float32)
    if with_payload:
        if w.act_bytes == 4:
            out["act"] = np.ascontiguousarray(out["action"][:, :w.chunk]).reshape(-1, 1).view(np.uint8)
        else:
            a = g.uniform(-1.0, 1.0, (S * w.chunk, w.act_bytes // 4)).astype(np.float32)
            out["act"] = a.view(np.uint8)
    return out


# ----------------------------------------------------------------------------------
# learner side
# ----------------------------------------------------------------------------------

def uniforms(seed: int, step: int, num_batches: int, k: int):
    """uint64 uniforms for one sample call, shape [num_batches, k]."""
    return _rng(seed, "rnd", step).integers(0, 1 << 64, (num_batches, k), dtype=np.uint64)


def priorities(dist: str, seed: int, step: int, m: int, tag: str = "td"):
    """m non-negative fp32 priorities (stand-ins for |TD errors|)."""
    g = _rng(seed, tag, step)
    if dist == "absnormal":
        p = np.abs(g.standard_normal(m))
    elif dist == "lognormal1":
        p = g.lognormal(0.0, 1.0, m)
    elif dist == "lognormal2":
        p = g.lognormal(0.0, 2.0, m)
    elif dist == "pareto":                      # Pareto(shape 1.1), a fifth forced to zero
        p = g.pareto(1.1, m) + 1.0
        p[g.random(m) < 0.2] = 0.0
    elif dist == "ones":
        p = np.ones(m)
    else:
        raise ValueError(dist)
    return p.astype(np.float32)


# ----------------------------------------------------------------------------------
# observation bytes as a function of the key
# ----------------------------------------------------------------------------------

_K1, _K2 = 0x9E3779B97F4A7C15, 0xD1B54A32D192ED03
_M1, _M2 = 0xBF58476D1CE4E5B9, 0x94D049BB133111EB


def obs_rows(seed: int, first_key: int, count: int, obs_bytes: int):
    """uint8 [count, obs_bytes]: row i holds the bytes of key first_key+i (numpy, host)."""
    words = (obs_bytes + 7) // 8
    with np.errstate(over="ignore"):
        key = (np.arange(count, dtype=np.uint64) + np.uint64(first_key))[:, None]
        j = np.arange(words, dtype=np.uint64)[None, :]
        z = key * np.uint64(_K1) + j * np.uint64(_K2) + np.uint64(seed)
        z ^= z >> np.uint64(30)
        z *= np.uint64(_M1)
        z ^= z >> np.uint64(27)
        z *= np.uint64(_M2)
        z ^= z >> np.uint64(31)
    return np.ascontiguousarray(z.view(np.uint8).reshape(count, words * 8)[:, :obs_bytes])


def frame_rows(seed: int, first_key: int, count: int, obs_bytes: int, flat_per_256: int = 205):
    """Frame-like rows as a function of the key (a stand-in for game screens): the bytes of :func:`obs_rows`,
    except that a 64-byte block whose first byte is below flat_per_256 (about 80 % of them) is flat, filled with
    one of 8 background values chosen by its second byte.  obs_bytes must be a multiple of 64."""
    assert obs_bytes % 64 == 0
    rows = obs_rows(seed, first_key, count, obs_bytes).reshape(count, obs_bytes // 64, 64)
    flat = rows[:, :, 0] < flat_per_256
    value = (rows[:, :, 1] & 7) * 31
    return np.where(flat[:, :, None], value[:, :, None], rows).astype(np.uint8).reshape(count, obs_bytes)


def frame_rows_torch(seed: int, first_key: int, count: int, obs_bytes: int, device, flat_per_256: int = 205):
    """Same bytes as :func:`frame_rows`, produced on ``device``."""
    import torch
    assert obs_bytes % 64 == 0
    rows = obs_rows_torch(seed, first_key, count, obs_bytes, device).reshape(count, obs_bytes // 64, 64)
    flat = rows[:, :, 0] < flat_per_256
    value = (rows[:, :, 1] & 7) * 31
    return torch.where(flat[:, :, None], value[:, :, None], rows).reshape(count, obs_bytes).contiguous()


def _s64(v):
    return v - (1 << 64) if v >= (1 << 63) else v


def obs_rows_torch(seed: int, first_key: int, count: int, obs_bytes: int, device):
    """Same bytes as :func:`obs_rows`, produced on ``device`` with integer tensor ops
    (obs_bytes must be a multiple of 8)."""
    import torch
    key = torch.arange(first_key, first_key + count, dtype=torch.int64, device=device)
    return obs_rows_for_keys_torch(seed, key, obs_bytes, device)


def obs_rows_for_keys_torch(seed: int, keys, obs_bytes: int, device):
    """uint8 [len(keys), obs_bytes] on ``device``: row i holds the bytes of key keys[i] (any order, repeats allowed;
    a numpy uint64 / int64 array or an int64 tensor).  The bytes of :func:`obs_rows` for the same keys."""
    import torch
    assert obs_bytes % 8 == 0
    words = obs_bytes // 8
    if not torch.is_tensor(keys):
        keys = torch.from_numpy(np.ascontiguousarray(np.asarray(keys).astype(np.uint64)).view(np.int64))
    key = keys.to(device=device, dtype=torch.int64).reshape(-1)[:, None]
    count = key.shape[0]
    j = torch.arange(words, dtype=torch.int64, device=device)[None, :]
    z = key * _s64(_K1) + j * _s64(_K2) + _s64(seed)

    def lsr(v, s):
        return (v >> s) & ((1 << (64 - s)) - 1)

    z = z ^ lsr(z, 30)
    z = z * _s64(_M1)
    z = z ^ lsr(z, 27)
    z = z * _s64(_M2)
    z = z ^ lsr(z, 31)
    return z.view(torch.uint8).reshape(count, obs_bytes)


def frame_rows_for_keys_torch(seed: int, keys, obs_bytes: int, device, flat_per_256: int = 205):
    """The bytes of :func:`frame_rows` for the keys given, produced on ``device``."""
    import torch
    assert obs_bytes % 64 == 0
    rows = obs_rows_for_keys_torch(seed, keys, obs_bytes, device)
    count = rows.shape[0]
    rows = rows.reshape(count, obs_bytes // 64, 64)
    flat = rows[:, :, 0] < flat_per_256
    value = (rows[:, :, 1] & 7) * 31
    return torch.where(flat[:, :, None], value[:, :, None], rows).reshape(count, obs_bytes).contiguous()
