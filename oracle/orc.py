"""ctypes access to the CPU oracle (oracle/tj_oracle.c).

Test infrastructure only: imported by tests, the smoke check and the
benchmark's CPU-baseline leg.  Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from .build_oracle import LIB, build_oracle

_lib = None

PARAMS, TARGET, GRADS, ADAM_M, ADAM_V = 0, 1, 2, 3, 4
LAST_Q_S, LAST_Q_NEXT_ONLINE, LAST_Q_NEXT_TARGET, LAST_Y, LAST_DELTA = 0, 1, 2, 3, 4

_vp, _u64, _i64, _u32, _i32, _dbl = C.c_void_p, C.c_uint64, C.c_int64, C.c_uint32, C.c_int, C.c_double


def lib():
    global _lib
    if _lib is None:
        path = os.environ.get("ORC_LIB", LIB)   # e.g. the sanitizer build (see build_oracle.py)
        if path == LIB and not os.path.exists(LIB):
            build_oracle()
        L = C.CDLL(path)
        L.orc_rng64.restype = _u64
        L.orc_rng64.argtypes = [_u64, _u64]
        L.orc_mulhi64.restype = _u64
        L.orc_mulhi64.argtypes = [_u64, _u64]
        L.orc_sample.restype = _i32
        L.orc_sample.argtypes = [_vp, _u64, _i64, _i64, _u64, _u32, _vp, _vp]
        L.orc_actor_act.restype = None
        L.orc_actor_act.argtypes = [_vp, _vp, _u32, C.c_double, _u64, _vp, _vp, _vp]
        L.orc_sample_excluding.restype = _i32
        L.orc_sample_excluding.argtypes = [_vp, _u64, _u64, _u64, _u64, _i64, _i64, _u64, _u32, _vp, _vp]
        L.orc_buffer_create.restype = _vp
        L.orc_buffer_create.argtypes = [_u64, _u32, _u32]
        L.orc_buffer_destroy.argtypes = [_vp]
        L.orc_buffer_insert.restype = _i32
        L.orc_buffer_insert.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _vp, _vp]
        L.orc_buffer_count.restype = _u64
        L.orc_buffer_count.argtypes = [_vp]
        L.orc_buffer_head.restype = _u64
        L.orc_buffer_head.argtypes = [_vp]
        L.orc_buffer_versions.restype = _vp
        L.orc_buffer_versions.argtypes = [_vp]
        L.orc_buffer_sample.restype = _i32
        L.orc_buffer_sample.argtypes = [_vp, _u32, _i64, _i64, _u64, _vp, _vp]
        L.orc_buffer_gather.argtypes = [_vp, _vp, _u32, _vp, _vp, _vp, _vp, _vp]
        L.orc_learner_create.restype = _vp
        L.orc_learner_create.argtypes = [_vp, _i32, _i32, _i32, _i32, _i32, _dbl, _dbl, _dbl, _dbl,
                                         _dbl, _dbl, _i64, _i32]
        L.orc_learner_destroy.argtypes = [_vp]
        L.orc_learner_num_params.restype = _u64
        L.orc_learner_num_params.argtypes = [_vp]
        L.orc_learner_num_actions.restype = _i32
        L.orc_learner_num_actions.argtypes = [_vp]
        L.orc_learner_get_t.restype = _i64
        L.orc_learner_get_t.argtypes = [_vp]
        L.orc_learner_set_t.argtypes = [_vp, _i64]
        L.orc_learner_set_state.restype = _i32
        L.orc_learner_set_state.argtypes = [_vp, _i32, _vp]
        L.orc_learner_get_state.restype = _i32
        L.orc_learner_get_state.argtypes = [_vp, _i32, _vp]
        L.orc_learner_forward.argtypes = [_vp, _i32, _vp, _u32, _vp]
        L.orc_learner_min_abs_preactivation.restype = _dbl
        L.orc_learner_min_abs_preactivation.argtypes = [_vp, _vp, _u32, _vp]
        L.orc_learner_step.restype = _dbl
        L.orc_learner_step.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _vp, _vp]
        L.orc_learner_last.restype = _i32
        L.orc_learner_last.argtypes = [_vp, _i32, _vp]
        L.orc_learner_last_astar.restype = _i32
        L.orc_learner_last_astar.argtypes = [_vp, _vp]
        L.orc_num_threads.restype = _i32
        L.orc_gae.restype = None
        L.orc_gae.argtypes = [_u32, _u32, _vp, _vp, _vp, _dbl, _dbl, _vp, _vp]
        L.orc_ppo_loss.restype = None
        L.orc_ppo_loss.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _vp, _dbl, _dbl, _dbl, _vp]
        L.orc_ppo_step.restype = None
        L.orc_ppo_step.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _vp, _dbl, _dbl, _dbl, _vp]
        L.orc_ppo_act.restype = None
        L.orc_ppo_act.argtypes = [_vp, _vp, _u32, _u64, _vp, _vp, _vp, _vp]
        _lib = L
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def _c(a, dtype):
    return np.ascontiguousarray(a, dtype=dtype)


def rng64(seed: int, j: int) -> int:
    return lib().orc_rng64(seed & (2**64 - 1), j)


def mulhi64(a: int, b: int) -> int:
    return lib().orc_mulhi64(a, b)


def num_threads() -> int:
    return lib().orc_num_threads()


def sample(version, count, cur, max_st, seed, batch):
    """(status, idx[batch] uint32, K) from a version array."""
    version = _c(version, np.int32)
    idx = np.empty(batch, dtype=np.uint32)
    K = C.c_uint64(0)
    st = lib().orc_sample(_p(version), count, cur, max_st, seed, batch, _p(idx), C.byref(K))
    return st, idx, K.value


def sample_excluding(version, count, capacity, ex_begin, ex_len, cur, max_st, seed, batch):
    """As sample(), with the slots (ex_begin + t) mod capacity, t < ex_len, not eligible."""
    version = _c(version, np.int32)
    idx = np.empty(batch, dtype=np.uint32)
    K = C.c_uint64(0)
    st = lib().orc_sample_excluding(_p(version), count, capacity, ex_begin, ex_len, cur, max_st, seed, batch,
                                    _p(idx), C.byref(K))
    return st, idx, K.value


def balance_plan(tr_learner, tr_actor, batch, serial_batch, serial_buffer, capacity):
    """(status, dict) of the production / consumption balance (Eq. 2-3)."""
    out = np.zeros(7, np.float64)
    f = lib().orc_balance_plan
    f.restype = _i32
    f.argtypes = [C.c_double, C.c_double, _u64, _u64, _u64, _u64, _vp]
    st = f(tr_learner, tr_actor, batch, serial_batch, serial_buffer, capacity, _p(out))
    keys = ("max_staleness", "rows_per_version", "window", "ratio", "target_ratio", "throughput", "cut")
    return st, dict(zip(keys, out))


def gae(reward, value, done, gamma: float, lam: float):
    """Advantages and returns of rollouts stored environment-major: reward, done [n_env][T],
    value [n_env][T + 1] (the last column bootstraps).  Returns (adv, ret), float64 [n_env][T]."""
    reward, value, done = _c(reward, np.float32), _c(value, np.float32), _c(done, np.uint8)
    n_env, T = reward.shape
    assert value.shape == (n_env, T + 1) and done.shape == (n_env, T)
    adv, ret = np.empty((n_env, T), np.float64), np.empty((n_env, T), np.float64)
    lib().orc_gae(n_env, T, _p(reward), _p(value), _p(done), gamma, lam, _p(adv), _p(ret))
    return adv, ret


class Buffer:
    def __init__(self, capacity: int, obs_elems: int, obs_dtype: str):
        self.capacity, self.obs_elems = capacity, obs_elems
        self.np_dtype = np.float32 if obs_dtype == "f32" else np.uint8
        self.h = lib().orc_buffer_create(capacity, obs_elems, 0 if obs_dtype == "f32" else 1)

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_buffer_destroy(self.h)
            self.h = None

    def insert(self, obs, next_obs, action, reward, done, version) -> int:
        n = len(action)
        obs, next_obs = _c(obs, self.np_dtype), _c(next_obs, self.np_dtype)
        action, reward = _c(action, np.int32), _c(reward, np.float32)
        done, version = _c(done, np.uint8), _c(version, np.int32)
        return lib().orc_buffer_insert(self.h, n, _p(obs), _p(next_obs), _p(action), _p(reward),
                                       _p(done), _p(version))

    @property
    def count(self) -> int:
        return lib().orc_buffer_count(self.h)

    @property
    def head(self) -> int:
        return lib().orc_buffer_head(self.h)

    def versions(self) -> np.ndarray:
        ptr = lib().orc_buffer_versions(self.h)
        arr = np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_int32)), shape=(self.capacity,))
        return arr.copy()

    def sample(self, batch, cur, max_st, seed):
        idx = np.empty(batch, dtype=np.uint32)
        K = C.c_uint64(0)
        st = lib().orc_buffer_sample(self.h, batch, cur, max_st, seed, _p(idx), C.byref(K))
        return st, idx, K.value

    def gather(self, idx):
        idx = _c(idx, np.uint32)
        b = len(idx)
        out = {
            "obs": np.empty((b, self.obs_elems), self.np_dtype),
            "next_obs": np.empty((b, self.obs_elems), self.np_dtype),
            "action": np.empty(b, np.int32),
            "reward": np.empty(b, np.float32),
            "done": np.empty(b, np.uint8),
        }
        lib().orc_buffer_gather(self.h, _p(idx), b, _p(out["obs"]), _p(out["next_obs"]),
                                _p(out["action"]), _p(out["reward"]), _p(out["done"]))
        return out


class FrameBuffer:
    """One u8 frame per slot; observation stacks of `stack` frames are rebuilt when sampling."""

    def __init__(self, capacity: int, frame_elems: int, stack: int):
        L = lib()
        L.orc_frame_buffer_create.restype = _vp
        L.orc_frame_buffer_create.argtypes = [_u64, _u32, _u32]
        L.orc_frame_buffer_destroy.argtypes = [_vp]
        L.orc_frame_buffer_insert.restype = _i32
        L.orc_frame_buffer_insert.argtypes = [_vp, _u32, _vp, _vp, _vp, _vp, _vp]
        L.orc_frame_buffer_sample.restype = _i32
        L.orc_frame_buffer_sample.argtypes = [_vp, _u32, _i64, _i64, _u64, _vp, _vp]
        L.orc_frame_buffer_gather.argtypes = [_vp, _vp, _u32, _vp, _vp, _vp, _vp, _vp]
        for f in ("count", "head"):
            getattr(L, "orc_frame_buffer_" + f).restype = _u64
            getattr(L, "orc_frame_buffer_" + f).argtypes = [_vp]
        for f in ("ages", "versions"):
            getattr(L, "orc_frame_buffer_" + f).restype = _vp
            getattr(L, "orc_frame_buffer_" + f).argtypes = [_vp]
        self.capacity, self.frame_elems, self.stack = capacity, frame_elems, stack
        self.h = L.orc_frame_buffer_create(capacity, frame_elems, stack)

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_frame_buffer_destroy(self.h)
            self.h = None

    def insert(self, frame, action, reward, done, version) -> int:
        frame = _c(frame, np.uint8)
        action, reward = _c(action, np.int32), _c(reward, np.float32)
        done, version = _c(done, np.uint8), _c(version, np.int32)
        return lib().orc_frame_buffer_insert(self.h, len(action), _p(frame), _p(action), _p(reward), _p(done),
                                             _p(version))

    @property
    def count(self) -> int:
        return lib().orc_frame_buffer_count(self.h)

    @property
    def head(self) -> int:
        return lib().orc_frame_buffer_head(self.h)

    def ages(self) -> np.ndarray:
        ptr = lib().orc_frame_buffer_ages(self.h)
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_uint8)), shape=(self.capacity,)).copy()

    def versions(self) -> np.ndarray:
        ptr = lib().orc_frame_buffer_versions(self.h)
        return np.ctypeslib.as_array(C.cast(ptr, C.POINTER(C.c_int32)), shape=(self.capacity,)).copy()

    def sample(self, batch, cur, max_st, seed):
        idx = np.empty(batch, dtype=np.uint32)
        K = C.c_uint64(0)
        st = lib().orc_frame_buffer_sample(self.h, batch, cur, max_st, seed, _p(idx), C.byref(K))
        return st, idx, K.value

    def gather(self, idx):
        idx = _c(idx, np.uint32)
        b, row = len(idx), self.stack * self.frame_elems
        out = {"obs": np.empty((b, row), np.uint8), "next_obs": np.empty((b, row), np.uint8),
               "action": np.empty(b, np.int32), "reward": np.empty(b, np.float32), "done": np.empty(b, np.uint8)}
        lib().orc_frame_buffer_gather(self.h, _p(idx), b, _p(out["obs"]), _p(out["next_obs"]), _p(out["action"]),
                                      _p(out["reward"]), _p(out["done"]))
        return out


class Learner:
    """layers: rows (kind, out, kernel, stride); in_chw: (C, H, W) of one observation."""

    def __init__(self, layers, in_chw, obs_dtype="f32", gamma=0.99, kappa=1.0, lr=1e-3, beta1=0.9,
                 beta2=0.999, eps=1e-8, target_interval=100, emulate_bf16=False):
        spec = _c(np.array(layers, dtype=np.int32).reshape(-1, 4), np.int32)
        self.np_dtype = np.float32 if obs_dtype == "f32" else np.uint8
        self.h = lib().orc_learner_create(_p(spec), len(spec), in_chw[0], in_chw[1], in_chw[2],
                                          0 if obs_dtype == "f32" else 1, gamma, kappa, lr, beta1,
                                          beta2, eps, target_interval, 1 if emulate_bf16 else 0)
        self.n_params = lib().orc_learner_num_params(self.h)
        self.n_actions = lib().orc_learner_num_actions(self.h)
        self.last_batch = 0

    def __del__(self):
        if getattr(self, "h", None):
            lib().orc_learner_destroy(self.h)
            self.h = None

    def set_state(self, which: int, values) -> None:
        v = _c(values, np.float64)
        assert v.size == self.n_params
        assert lib().orc_learner_set_state(self.h, which, _p(v)) == 0

    def get_state(self, which: int) -> np.ndarray:
        out = np.empty(self.n_params, np.float64)
        assert lib().orc_learner_get_state(self.h, which, _p(out)) == 0
        return out

    @property
    def t(self) -> int:
        return lib().orc_learner_get_t(self.h)

    @t.setter
    def t(self, value: int) -> None:
        lib().orc_learner_set_t(self.h, value)

    def forward(self, which: int, obs) -> np.ndarray:
        obs = _c(obs, self.np_dtype)
        b = obs.shape[0]
        q = np.empty((b, self.n_actions), np.float64)
        lib().orc_learner_forward(self.h, which, _p(obs), b, _p(q))
        return q

    def act(self, obs, epsilon: float, seed: int):
        """Epsilon-greedy actions under the online network: (action, q, greedy)."""
        obs = _c(obs, self.np_dtype)
        n = obs.shape[0]
        action, greedy = np.empty(n, np.int32), np.empty(n, np.int32)
        q = np.empty((n, self.n_actions), np.float64)
        lib().orc_actor_act(self.h, _p(obs), n, C.c_double(epsilon), seed, _p(action), _p(q), _p(greedy))
        return action, q, greedy

    def min_abs_preactivation(self, obs) -> np.ndarray:
        """Per sample: the smallest |pre-activation| over the hidden units (online net)."""
        obs = _c(obs, self.np_dtype)
        out = np.empty(obs.shape[0], np.float64)
        lib().orc_learner_min_abs_preactivation(self.h, _p(obs), obs.shape[0], _p(out))
        return out

    def step(self, obs, next_obs, action, reward, done, astar_override=None) -> float:
        obs, next_obs = _c(obs, self.np_dtype), _c(next_obs, self.np_dtype)
        action, reward, done = _c(action, np.int32), _c(reward, np.float32), _c(done, np.uint8)
        b = len(action)
        self.last_batch = b
        ov = None if astar_override is None else _c(astar_override, np.int32)
        return lib().orc_learner_step(self.h, b, _p(obs), _p(next_obs), _p(action), _p(reward),
                                      _p(done), None if ov is None else _p(ov))

    def last(self, which: int) -> np.ndarray:
        b = self.last_batch
        shape = (b, self.n_actions) if which <= 2 else (b,)
        out = np.empty(shape, np.float64)
        assert lib().orc_learner_last(self.h, which, _p(out)) == 0
        return out

    def last_astar(self) -> np.ndarray:
        out = np.empty(self.last_batch, np.int32)
        lib().orc_learner_last_astar(self.h, _p(out))
        return out

    def _ppo_args(self, obs, action, old_logp, adv, ret):
        obs = _c(obs, self.np_dtype)
        action, old_logp = _c(action, np.int32), _c(old_logp, np.float32)
        adv, ret = _c(adv, np.float32), _c(ret, np.float32)
        b = len(action)
        assert obs.shape[0] == b and len(old_logp) == b and len(adv) == b and len(ret) == b
        assert action.min() >= 0 and action.max() < self.n_actions - 1
        return b, obs, action, old_logp, adv, ret

    def ppo_loss(self, obs, action, old_logp, adv, ret, clip=0.2, c_v=0.5, c_e=0.01) -> np.ndarray:
        """Actor-critic objective (the head's last output is the value): [L_pi, L_v, H, loss]."""
        b, obs, action, old_logp, adv, ret = self._ppo_args(obs, action, old_logp, adv, ret)
        out = np.empty(4, np.float64)
        lib().orc_ppo_loss(self.h, b, _p(obs), _p(action), _p(old_logp), _p(adv), _p(ret), clip, c_v, c_e,
                           _p(out))
        return out

    def ppo_step(self, obs, action, old_logp, adv, ret, clip=0.2, c_v=0.5, c_e=0.01) -> np.ndarray:
        """One update on the whole batch; returns [L_pi, L_v, H, loss] before the update."""
        b, obs, action, old_logp, adv, ret = self._ppo_args(obs, action, old_logp, adv, ret)
        out = np.empty(4, np.float64)
        lib().orc_ppo_step(self.h, b, _p(obs), _p(action), _p(old_logp), _p(adv), _p(ret), clip, c_v, c_e,
                           _p(out))
        return out

    def ppo_act(self, obs, seed: int):
        """Sampled actions under the stochastic policy: (action, logp, value, margin), where margin is
        the distance of the uniform draw from the nearest cumulative probability."""
        obs = _c(obs, self.np_dtype)
        n = obs.shape[0]
        action = np.empty(n, np.int32)
        logp, value, margin = np.empty(n), np.empty(n), np.empty(n)
        lib().orc_ppo_act(self.h, _p(obs), n, seed, _p(action), _p(logp), _p(value), _p(margin))
        return action, logp, value, margin
