"""Thin ctypes binding of libtianji_hip.so (see include/tianji.h).

Argument marshalling only: torch supplies device memory and streams, every step
of the path runs in the library's HIP kernels.  There is no CPU fallback: if the
library is missing or no GPU is present the calls raise.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtianji_hip.so")

TJ_OK = 0
TJ_ERR_INVALID_ARG, TJ_ERR_SHAPE, TJ_ERR_ARENA_TOO_SMALL = -1, -2, -3
TJ_ERR_NO_ELIGIBLE, TJ_ERR_CAPACITY, TJ_ERR_DEVICE, TJ_ERR_SCRATCH_LIMIT = -4, -5, -6, -7
TJ_OBS_F32, TJ_OBS_U8 = 0, 1
TJ_PRECISION_FP32, TJ_PRECISION_BF16 = 0, 1
TJ_LAYER_LINEAR, TJ_LAYER_CONV2D = 0, 1
TJ_MAX_LAYERS = 8
(TJ_STATE_PARAMS, TJ_STATE_TARGET, TJ_STATE_GRADS, TJ_STATE_ADAM_M, TJ_STATE_ADAM_V, TJ_STATE_QVALS,
 TJ_STATE_ASTAR, TJ_STATE_WEIGHTS_COMPUTE, TJ_STATE_WEIGHTS_COMPUTE_T, TJ_STATE_WEIGHTS_COMPUTE_TARGET) = range(10)

EXPORTS = [
    "tj_buffer_arena_bytes", "tj_buffer_create", "tj_buffer_destroy", "tj_buffer_insert", "tj_buffer_insert_concurrent", "tj_sample", "tj_sample_noalloc", "tj_buffer_reads_done", "tj_actor_act", "tj_balance_plan", "tj_frame_buffer_arena_bytes", "tj_frame_buffer_create",
    "tj_frame_buffer_destroy", "tj_frame_buffer_insert", "tj_frame_sample", "tj_frame_buffer_status",
    "tj_frame_buffer_field_ptr", "tj_frame_buffer_set_phase_events",
    "tj_buffer_status", "tj_buffer_field_ptr", "tj_learner_num_params", "tj_learner_arena_bytes",
    "tj_learner_create", "tj_learner_destroy", "tj_learner_step", "tj_learner_get_state",
    "tj_learner_set_state", "tj_learner_get_step", "tj_learner_set_step", "tj_strerror",
    "tj_buffer_set_phase_events", "tj_learner_set_phase_events",
    "tj_gae", "tj_ppo_num_params", "tj_ppo_arena_bytes", "tj_ppo_create", "tj_ppo_step", "tj_ppo_evaluate", "tj_ppo_act",
]


class tj_buffer_desc(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("obs_elems", C.c_uint32), ("obs_dtype", C.c_uint32)]


class tj_minibatch(C.Structure):
    _fields_ = [("obs", C.c_void_p), ("next_obs", C.c_void_p), ("action", C.c_void_p),
                ("reward", C.c_void_p), ("done", C.c_void_p), ("idx", C.c_void_p), ("batch", C.c_uint32),
                ("row_index", C.c_void_p), ("n_rows", C.c_uint64), ("plane_index", C.c_void_p)]


class tj_buffer_info(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("head", C.c_uint64), ("count", C.c_uint64),
                ("last_n_eligible", C.c_uint64), ("sticky_error", C.c_int32),
                ("last_excluded_begin", C.c_uint64), ("last_excluded_len", C.c_uint64)]


class tj_balance_in(C.Structure):
    _fields_ = [("tr_learner", C.c_double), ("tr_actor", C.c_double), ("batch", C.c_uint64),
                ("serial_batch", C.c_uint64), ("serial_buffer", C.c_uint64), ("capacity", C.c_uint64)]


class tj_balance_out(C.Structure):
    _fields_ = [("max_staleness", C.c_int64), ("rows_per_version", C.c_double), ("window", C.c_double),
                ("ratio", C.c_double), ("target_ratio", C.c_double), ("throughput", C.c_double),
                ("bottleneck", C.c_int32), ("window_exceeds_capacity", C.c_int32)]


def balance_plan(tr_learner, tr_actor, batch, serial_batch, serial_buffer, capacity):
    """(status, tj_balance_out): the staleness gate that keeps the consumed share of the pool at
    the serial ratio (host arithmetic in the library)."""
    i = tj_balance_in(tr_learner, tr_actor, batch, serial_batch, serial_buffer, capacity)
    o = tj_balance_out()
    f = lib().tj_balance_plan
    f.restype = C.c_int
    f.argtypes = [C.c_void_p, C.c_void_p]
    return f(C.byref(i), C.byref(o)), o


class tj_layer(C.Structure):
    _fields_ = [("kind", C.c_uint32), ("out", C.c_uint32), ("kernel", C.c_uint32), ("stride", C.c_uint32)]


class tj_learner_desc(C.Structure):
    _fields_ = [("n_layers", C.c_uint32), ("layers", tj_layer * TJ_MAX_LAYERS), ("in_c", C.c_uint32),
                ("in_h", C.c_uint32), ("in_w", C.c_uint32), ("obs_dtype", C.c_uint32),
                ("precision", C.c_uint32), ("max_batch", C.c_uint32), ("gamma", C.c_float),
                ("huber_delta", C.c_float), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
                ("eps", C.c_float), ("target_interval", C.c_uint32)]


class tj_ppo_desc(C.Structure):
    _fields_ = [("obs_dim", C.c_uint32), ("n_hidden", C.c_uint32), ("hidden", C.c_uint32 * (TJ_MAX_LAYERS - 1)),
                ("n_actions", C.c_uint32), ("precision", C.c_uint32), ("max_batch", C.c_uint32),
                ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("clip", C.c_float), ("c_v", C.c_float), ("c_e", C.c_float)]


class tj_ppo_batch(C.Structure):
    _fields_ = [("batch", C.c_uint32), ("obs", C.c_void_p), ("action", C.c_void_p), ("old_logp", C.c_void_p),
                ("adv", C.c_void_p), ("ret", C.c_void_p)]


class tj_step_stats(C.Structure):
    _fields_ = [("loss", C.c_float), ("step", C.c_uint32)]


_lib = None


def lib():
    """The loaded library.  torch is imported first so that both share one HIP runtime."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  (loads libamdhip64 before our library binds to it)

        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, u32, u64, i64, sz, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int64, C.c_size_t, C.c_int
        L.tj_buffer_arena_bytes.restype = sz
        L.tj_buffer_arena_bytes.argtypes = [C.POINTER(tj_buffer_desc)]
        L.tj_buffer_create.restype = i32
        L.tj_buffer_create.argtypes = [C.POINTER(tj_buffer_desc), vp, sz, vp, C.POINTER(vp)]
        L.tj_buffer_destroy.restype = i32
        L.tj_buffer_destroy.argtypes = [vp]
        L.tj_buffer_insert.restype = i32
        L.tj_buffer_insert.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp, vp]
        L.tj_actor_act.restype = i32
        L.tj_actor_act.argtypes = [vp, u32, vp, C.c_float, u64, vp, vp, vp, vp]
        L.tj_buffer_insert_concurrent.restype = i32
        L.tj_buffer_insert_concurrent.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp, vp]
        L.tj_sample.restype = i32
        L.tj_sample.argtypes = [vp, u32, i64, i64, u64, C.POINTER(tj_minibatch), vp]
        L.tj_sample_noalloc.restype = i32
        L.tj_sample_noalloc.argtypes = [vp, u32, i64, i64, u64, C.POINTER(tj_minibatch), vp]
        L.tj_buffer_status.restype = i32
        L.tj_buffer_status.argtypes = [vp, C.POINTER(tj_buffer_info), vp]
        L.tj_buffer_reads_done.restype = i32
        L.tj_buffer_reads_done.argtypes = [vp, vp]
        L.tj_buffer_field_ptr.restype = vp
        L.tj_buffer_field_ptr.argtypes = [vp, i32]
        L.tj_learner_num_params.restype = sz
        L.tj_learner_num_params.argtypes = [C.POINTER(tj_learner_desc)]
        L.tj_learner_arena_bytes.restype = sz
        L.tj_learner_arena_bytes.argtypes = [C.POINTER(tj_learner_desc)]
        L.tj_learner_create.restype = i32
        L.tj_learner_create.argtypes = [C.POINTER(tj_learner_desc), vp, sz, vp, vp, vp, C.POINTER(vp)]
        L.tj_learner_destroy.restype = i32
        L.tj_learner_destroy.argtypes = [vp]
        L.tj_learner_step.restype = i32
        L.tj_learner_step.argtypes = [vp, C.POINTER(tj_minibatch), vp, vp]
        L.tj_learner_get_state.restype = i32
        L.tj_learner_get_state.argtypes = [vp, i32, vp, sz, vp]
        L.tj_learner_set_state.restype = i32
        L.tj_learner_set_state.argtypes = [vp, i32, vp, sz, vp]
        L.tj_learner_get_step.restype = i32
        L.tj_learner_get_step.argtypes = [vp, C.POINTER(u64)]
        L.tj_learner_set_step.restype = i32
        L.tj_learner_set_step.argtypes = [vp, u64]
        L.tj_buffer_set_phase_events.restype = i32
        L.tj_buffer_set_phase_events.argtypes = [vp, C.POINTER(vp), u32]
        L.tj_frame_buffer_set_phase_events.restype = i32
        L.tj_frame_buffer_set_phase_events.argtypes = [vp, C.POINTER(vp), u32]
        L.tj_learner_set_phase_events.restype = i32
        L.tj_learner_set_phase_events.argtypes = [vp, C.POINTER(vp), u32]
        L.tj_strerror.restype = C.c_char_p
        L.tj_strerror.argtypes = [i32]
        L.tj_gae.restype = i32
        L.tj_gae.argtypes = [u32, u32, vp, vp, vp, C.c_float, C.c_float, vp, vp, vp]
        L.tj_ppo_num_params.restype = sz
        L.tj_ppo_num_params.argtypes = [C.POINTER(tj_ppo_desc)]
        L.tj_ppo_arena_bytes.restype = sz
        L.tj_ppo_arena_bytes.argtypes = [C.POINTER(tj_ppo_desc)]
        L.tj_ppo_create.restype = i32
        L.tj_ppo_create.argtypes = [C.POINTER(tj_ppo_desc), vp, sz, vp, vp, C.POINTER(vp)]
        L.tj_ppo_step.restype = i32
        L.tj_ppo_step.argtypes = [vp, C.POINTER(tj_ppo_batch), vp, vp]
        L.tj_ppo_evaluate.restype = i32
        L.tj_ppo_evaluate.argtypes = [vp, u32, vp, vp, vp, vp]
        L.tj_ppo_act.restype = i32
        L.tj_ppo_act.argtypes = [vp, u32, vp, u64, vp, vp, vp, vp]
        _lib = L
    return _lib


def tj_strerror(status: int) -> str:
    return lib().tj_strerror(status).decode()


class TjError(RuntimeError):
    def __init__(self, status: int, where: str):
        super().__init__(f"{where}: {tj_strerror(status)} ({status})")
        self.status = status


def _check(status: int, where: str) -> None:
    if status != TJ_OK:
        raise TjError(status, where)


def _stream_ptr(stream=None) -> int:
    import torch

    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def _require_gpu():
    import torch

    if not torch.cuda.is_available():
        raise RuntimeError("no GPU: the HIP path has no CPU fallback")


class Minibatch:
    """Caller-owned device tensors for one minibatch.

    Dense (default): obs / next_obs hold copies of the sampled rows.  With `ring` (a Buffer or a
    FrameBuffer) the minibatch is indirect: no observation tensors exist; `c` is what the sampler
    fills (indices and scalar fields; for a FrameBuffer also the slot of every frame of the two
    stacks) and `c_step` what tj_learner_step reads (the ring's own arrays + those indices)."""

    def __init__(self, batch: int, obs_elems: int, obs_dtype: str, device="cuda:0", ring=None):
        import torch

        tdt = torch.float32 if obs_dtype == "f32" else torch.uint8
        self.batch = batch
        self.ring = ring
        self.action = torch.empty(batch, dtype=torch.int32, device=device)
        self.reward = torch.empty(batch, dtype=torch.float32, device=device)
        self.done = torch.empty(batch, dtype=torch.uint8, device=device)
        self.idx = torch.empty(batch, dtype=torch.int32, device=device)   # bits are uint32
        if ring is None:
            self.obs = torch.empty((batch, obs_elems), dtype=tdt, device=device)
            self.next_obs = torch.empty((batch, obs_elems), dtype=tdt, device=device)
            self.c = tj_minibatch(self.obs.data_ptr(), self.next_obs.data_ptr(), self.action.data_ptr(),
                                  self.reward.data_ptr(), self.done.data_ptr(), self.idx.data_ptr(), batch, None, 0)
            self.c_step = self.c
        elif hasattr(ring, "stack"):     # frame ring: indirect by planes
            assert ring.obs_elems == obs_elems and obs_dtype == "u8"
            self.obs = self.next_obs = None
            self.planes = torch.empty((batch, 2 * ring.stack), dtype=torch.int32, device=device)
            frames = lib().tj_frame_buffer_field_ptr(ring.h, 0)
            self.c = tj_minibatch(None, None, self.action.data_ptr(), self.reward.data_ptr(),
                                  self.done.data_ptr(), self.idx.data_ptr(), batch, None, 0, self.planes.data_ptr())
            self.c_step = tj_minibatch(frames, frames, self.action.data_ptr(), self.reward.data_ptr(),
                                       self.done.data_ptr(), self.idx.data_ptr(), batch, None, ring.capacity,
                                       self.planes.data_ptr())
        else:
            assert ring.obs_elems == obs_elems and ring.obs_dtype == obs_dtype
            self.obs = self.next_obs = None
            self.c = tj_minibatch(None, None, self.action.data_ptr(), self.reward.data_ptr(),
                                  self.done.data_ptr(), self.idx.data_ptr(), batch, None, 0)
            self.c_step = tj_minibatch(lib().tj_buffer_field_ptr(ring.h, 0), lib().tj_buffer_field_ptr(ring.h, 1),
                                       self.action.data_ptr(), self.reward.data_ptr(), self.done.data_ptr(),
                                       self.idx.data_ptr(), batch, self.idx.data_ptr(), ring.capacity)

    def load(self, obs, next_obs, action, reward, done) -> None:
        """Fill from host arrays (tests feed the learner without a ring)."""
        import torch

        if self.ring is not None:
            raise ValueError("an indirect minibatch has no observation tensors to load")

        self.obs.copy_(torch.from_numpy(np.ascontiguousarray(obs)).reshape(self.obs.shape))
        self.next_obs.copy_(torch.from_numpy(np.ascontiguousarray(next_obs)).reshape(self.obs.shape))
        self.action.copy_(torch.from_numpy(np.ascontiguousarray(action, np.int32)))
        self.reward.copy_(torch.from_numpy(np.ascontiguousarray(reward, np.float32)))
        self.done.copy_(torch.from_numpy(np.ascontiguousarray(done, np.uint8)))

    def host(self):
        keys = ("action", "reward", "done") if self.ring is not None else ("obs", "next_obs", "action", "reward", "done")
        out = {k: getattr(self, k).cpu().numpy() for k in keys}
        out["idx"] = self.idx.cpu().numpy().view(np.uint32)
        if getattr(self, "planes", None) is not None:
            out["planes"] = self.planes.cpu().numpy().view(np.uint32)
        return out


class tj_frame_buffer_desc(C.Structure):
    _fields_ = [("capacity", C.c_uint64), ("frame_elems", C.c_uint32), ("stack", C.c_uint32)]


class FrameBuffer:
    """tj_frame_buffer_* (one u8 frame per slot) over a torch-allocated arena."""

    def __init__(self, capacity: int, frame_elems: int, stack: int, device="cuda:0", stream=None):
        import torch

        _require_gpu()
        L = lib()
        vp, u32, u64, i64, i32 = C.c_void_p, C.c_uint32, C.c_uint64, C.c_int64, C.c_int
        L.tj_frame_buffer_arena_bytes.restype = C.c_size_t
        L.tj_frame_buffer_arena_bytes.argtypes = [vp]
        L.tj_frame_buffer_create.restype = i32
        L.tj_frame_buffer_create.argtypes = [vp, vp, C.c_size_t, vp, vp]
        L.tj_frame_buffer_destroy.argtypes = [vp]
        L.tj_frame_buffer_insert.restype = i32
        L.tj_frame_buffer_insert.argtypes = [vp, u32, vp, vp, vp, vp, vp, vp]
        L.tj_frame_sample.restype = i32
        L.tj_frame_sample.argtypes = [vp, u32, i64, i64, u64, vp, vp]
        L.tj_frame_buffer_status.restype = i32
        L.tj_frame_buffer_status.argtypes = [vp, vp, vp]
        L.tj_frame_buffer_field_ptr.restype = vp
        L.tj_frame_buffer_field_ptr.argtypes = [vp, i32]
        self.capacity, self.frame_elems, self.stack, self.device = capacity, frame_elems, stack, device
        self.obs_elems, self.obs_dtype = frame_elems * stack, "u8"
        self.desc = tj_frame_buffer_desc(capacity, frame_elems, stack)
        nbytes = L.tj_frame_buffer_arena_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise TjError(TJ_ERR_INVALID_ARG, "tj_frame_buffer_arena_bytes")
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        self.arena_ptr = (self.arena.data_ptr() + 255) // 256 * 256
        self.arena_bytes = nbytes
        h = C.c_void_p()
        _check(L.tj_frame_buffer_create(C.byref(self.desc), self.arena_ptr, nbytes, _stream_ptr(stream), C.byref(h)),
               "tj_frame_buffer_create")
        self.h = h

    def __del__(self):
        if getattr(self, "h", None):
            lib().tj_frame_buffer_destroy(self.h)
            self.h = None

    def insert(self, frame, action, reward, done, version, stream=None) -> int:
        """Device tensors; returns the status (TJ_ERR_CAPACITY for too many rows)."""
        self._keep = (frame, action, reward, done, version)
        return lib().tj_frame_buffer_insert(self.h, int(action.shape[0]), frame.data_ptr(), action.data_ptr(),
                                            reward.data_ptr(), done.data_ptr(), version.data_ptr(),
                                            _stream_ptr(stream))

    def insert_host(self, frame, action, reward, done, version) -> int:
        import torch

        dev = [torch.from_numpy(np.ascontiguousarray(v)).to(self.device) for v in (frame, action, reward, done, version)]
        st = self.insert(*dev)
        torch.cuda.current_stream().synchronize()
        return st

    def sample(self, mb: Minibatch, current_version: int, max_staleness: int, seed: int, stream=None) -> int:
        return lib().tj_frame_sample(self.h, mb.batch, current_version, max_staleness, seed & (2**64 - 1),
                                     C.byref(mb.c), _stream_ptr(stream))

    def status(self, stream=None):
        info = tj_buffer_info()
        st = lib().tj_frame_buffer_status(self.h, C.byref(info), _stream_ptr(stream))
        return st, info

    def ages(self) -> np.ndarray:
        import torch

        ptr = lib().tj_frame_buffer_field_ptr(self.h, 1)
        off = ptr - self.arena.data_ptr()
        return self.arena[off:off + self.capacity].cpu().numpy()


class Buffer:
    """tj_buffer_* over a torch-allocated arena."""

    def __init__(self, capacity: int, obs_elems: int, obs_dtype: str, device="cuda:0", stream=None):
        import torch

        _require_gpu()
        self.obs_dtype, self.obs_elems, self.capacity, self.device = obs_dtype, obs_elems, capacity, device
        self.desc = tj_buffer_desc(capacity, obs_elems, TJ_OBS_F32 if obs_dtype == "f32" else TJ_OBS_U8)
        nbytes = lib().tj_buffer_arena_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise TjError(TJ_ERR_INVALID_ARG, "tj_buffer_arena_bytes")
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        self.arena_ptr = (self.arena.data_ptr() + 255) // 256 * 256
        self.arena_bytes = nbytes
        h = C.c_void_p()
        _check(lib().tj_buffer_create(C.byref(self.desc), self.arena_ptr, nbytes, _stream_ptr(stream),
                                      C.byref(h)), "tj_buffer_create")
        self.h = h

    def __del__(self):
        if getattr(self, "h", None):
            lib().tj_buffer_destroy(self.h)
            self.h = None

    def insert(self, obs, next_obs, action, reward, done, version, stream=None) -> None:
        """All arguments are device tensors (torch), n = len(action)."""
        n = int(action.shape[0])
        self._keep = (obs, next_obs, action, reward, done, version)   # alive until the next call
        _check(lib().tj_buffer_insert(self.h, n, obs.data_ptr(), next_obs.data_ptr(), action.data_ptr(),
                                      reward.data_ptr(), done.data_ptr(), version.data_ptr(),
                                      _stream_ptr(stream)), "tj_buffer_insert")

    def insert_concurrent(self, obs, next_obs, action, reward, done, version, stream) -> None:
        """Insert on `stream` (a torch stream other than the sampling stream); the source tensors are
        kept alive by the caller until that stream has run the copy."""
        n = int(action.shape[0])
        _check(lib().tj_buffer_insert_concurrent(self.h, n, obs.data_ptr(), next_obs.data_ptr(),
                                                 action.data_ptr(), reward.data_ptr(), done.data_ptr(),
                                                 version.data_ptr(), _stream_ptr(stream)),
               "tj_buffer_insert_concurrent")

    def insert_host(self, rows: dict, stream=None) -> None:
        import torch

        dev = {k: torch.from_numpy(np.ascontiguousarray(v)).to(self.device) for k, v in rows.items()}
        self.insert(dev["obs"], dev["next_obs"], dev["action"], dev["reward"], dev["done"], dev["version"],
                    stream)
        torch.cuda.current_stream().synchronize()

    def sample(self, mb: Minibatch, current_version: int, max_staleness: int, seed: int, stream=None) -> int:
        return lib().tj_sample(self.h, mb.batch, current_version, max_staleness, seed & (2**64 - 1),
                               C.byref(mb.c), _stream_ptr(stream))

    def sample_noalloc(self, mb: Minibatch, current_version: int, max_staleness: int, seed: int, stream=None) -> int:
        return lib().tj_sample_noalloc(self.h, mb.batch, current_version, max_staleness, seed & (2**64 - 1),
                                       C.byref(mb.c), _stream_ptr(stream))

    def status(self, stream=None):
        info = tj_buffer_info()
        st = lib().tj_buffer_status(self.h, C.byref(info), _stream_ptr(stream))
        return st, info

    def reads_done(self, stream=None) -> None:
        """After a Learner.step on an indirect minibatch, where concurrent inserts are in use."""
        _check(lib().tj_buffer_reads_done(self.h, _stream_ptr(stream)), "tj_buffer_reads_done")

    def field(self, name: str):
        """A torch view of one ring field (tests only)."""
        import torch

        fid = ["obs", "next_obs", "action", "reward", "done", "version"].index(name)
        ptr = lib().tj_buffer_field_ptr(self.h, fid)
        off = ptr - self.arena.data_ptr()
        n = self.capacity
        if fid < 2:
            eb = 4 if self.obs_dtype == "f32" else 1
            raw = self.arena[off:off + n * self.obs_elems * eb]
            dt = torch.float32 if self.obs_dtype == "f32" else torch.uint8
            return raw.view(dt).reshape(n, self.obs_elems)
        dt, eb = {2: (torch.int32, 4), 3: (torch.float32, 4), 4: (torch.uint8, 1), 5: (torch.int32, 4)}[fid]
        return self.arena[off:off + n * eb].view(dt)


def make_learner_desc(layers, in_chw, obs_dtype: str, precision: str, max_batch: int, gamma: float,
                      kappa: float, lr: float, beta1: float, beta2: float, eps: float,
                      target_interval: int) -> tj_learner_desc:
    d = tj_learner_desc()
    d.n_layers = len(layers)
    for i, (kind, out, k, s) in enumerate(layers):
        d.layers[i] = tj_layer(kind, out, k, s)
    d.in_c, d.in_h, d.in_w = in_chw
    d.obs_dtype = TJ_OBS_F32 if obs_dtype == "f32" else TJ_OBS_U8
    d.precision = TJ_PRECISION_FP32 if precision == "fp32" else TJ_PRECISION_BF16
    d.max_batch = max_batch
    d.gamma, d.huber_delta, d.lr, d.beta1, d.beta2, d.eps = gamma, kappa, lr, beta1, beta2, eps
    d.target_interval = target_interval
    return d


class Learner:
    """tj_learner_* over a torch-allocated arena."""

    def __init__(self, desc: tj_learner_desc, init_online: np.ndarray, init_target: np.ndarray,
                 device="cuda:0", stream=None):
        import torch

        _require_gpu()
        self.desc = desc
        self.n_params = lib().tj_learner_num_params(C.byref(desc))
        nbytes = lib().tj_learner_arena_bytes(C.byref(desc))
        if nbytes == 0 or self.n_params == 0:
            raise TjError(TJ_ERR_SHAPE, "tj_learner_arena_bytes")
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        self.arena_ptr = (self.arena.data_ptr() + 255) // 256 * 256
        on = np.ascontiguousarray(init_online, np.float32)
        tg = np.ascontiguousarray(init_target, np.float32)
        assert on.size == self.n_params and tg.size == self.n_params
        h = C.c_void_p()
        _check(lib().tj_learner_create(C.byref(desc), self.arena_ptr, nbytes, on.ctypes.data, tg.ctypes.data,
                                       _stream_ptr(stream), C.byref(h)), "tj_learner_create")
        self.h = h
        self.stats = torch.zeros(2, dtype=torch.int32, device=device)   # tj_step_stats {f32, u32}
        self.n_actions = desc.layers[desc.n_layers - 1].out
        self.last_batch = 0

    def __del__(self):
        if getattr(self, "h", None):
            lib().tj_learner_destroy(self.h)
            self.h = None

    def step(self, mb: Minibatch, stream=None) -> int:
        self.last_batch = mb.batch
        return lib().tj_learner_step(self.h, C.byref(mb.c_step), self.stats.data_ptr(), _stream_ptr(stream))

    def act(self, obs, epsilon: float, seed: int, want_q: bool = False, stream=None):
        """Epsilon-greedy actions for a device tensor of observations [n, obs elements]:
        (action int32[n], version int32[n], q float32[n, A] or None), all device tensors."""
        import torch

        n = int(obs.shape[0])
        action = torch.empty(n, dtype=torch.int32, device=obs.device)
        version = torch.empty(n, dtype=torch.int32, device=obs.device)
        q = torch.empty((n, self.n_actions), dtype=torch.float32, device=obs.device) if want_q else None
        _check(lib().tj_actor_act(self.h, n, obs.data_ptr(), epsilon, seed & (2**64 - 1), action.data_ptr(),
                                  version.data_ptr(), q.data_ptr() if want_q else None, _stream_ptr(stream)),
               "tj_actor_act")
        return action, version, q

    def read_stats(self):
        raw = self.stats.cpu().numpy()
        return float(raw.view(np.float32)[0]), int(raw.view(np.uint32)[1])

    def get_state(self, which: int, stream=None) -> np.ndarray:
        if which == TJ_STATE_QVALS:
            n = 3 * self.last_batch * self.n_actions
        elif which == TJ_STATE_ASTAR:
            n = self.last_batch
        else:
            n = self.n_params
        out = np.empty(n, np.float32)
        _check(lib().tj_learner_get_state(self.h, which, out.ctypes.data, n, _stream_ptr(stream)),
               "tj_learner_get_state")
        return out

    def set_state(self, which: int, values, stream=None) -> None:
        v = np.ascontiguousarray(values, np.float32)
        _check(lib().tj_learner_set_state(self.h, which, v.ctypes.data, v.size, _stream_ptr(stream)),
               "tj_learner_set_state")

    @property
    def t(self) -> int:
        t = C.c_uint64(0)
        _check(lib().tj_learner_get_step(self.h, C.byref(t)), "tj_learner_get_step")
        return t.value

    @t.setter
    def t(self, value: int) -> None:
        _check(lib().tj_learner_set_step(self.h, value), "tj_learner_set_step")


def gae(reward, value, done, gamma: float, lam: float, stream=None):
    """tj_gae on device tensors: reward f32 [n_env, T], value f32 [n_env, T + 1], done u8 [n_env, T];
    returns (adv, ret) f32 [n_env, T]."""
    import torch

    n_env, T = int(reward.shape[0]), int(reward.shape[1])
    assert tuple(value.shape) == (n_env, T + 1) and tuple(done.shape) == (n_env, T)
    assert reward.dtype == torch.float32 and value.dtype == torch.float32 and done.dtype == torch.uint8
    assert reward.is_contiguous() and value.is_contiguous() and done.is_contiguous()
    adv, ret = torch.empty_like(reward), torch.empty_like(reward)
    _check(lib().tj_gae(n_env, T, reward.data_ptr(), value.data_ptr(), done.data_ptr(), gamma, lam,
                        adv.data_ptr(), ret.data_ptr(), _stream_ptr(stream)), "tj_gae")
    return adv, ret


class PpoLearner:
    """tj_ppo_* over a torch-allocated arena (state access through tj_learner_*)."""

    def __init__(self, obs_dim: int, hidden, n_actions: int, precision: str, max_batch: int, init: np.ndarray,
                 lr=1e-4, beta1=0.9, beta2=0.999, eps=1e-5, clip=0.2, c_v=0.5, c_e=0.01, device="cuda:0",
                 stream=None):
        import torch

        _require_gpu()
        d = tj_ppo_desc()
        d.obs_dim, d.n_hidden, d.n_actions = obs_dim, len(hidden), n_actions
        for i, h in enumerate(hidden):
            d.hidden[i] = h
        d.precision = TJ_PRECISION_BF16 if precision == "bf16" else TJ_PRECISION_FP32
        d.max_batch = max_batch
        d.lr, d.beta1, d.beta2, d.eps, d.clip, d.c_v, d.c_e = lr, beta1, beta2, eps, clip, c_v, c_e
        self.desc = d
        self.obs_dim, self.hidden, self.n_actions = obs_dim, tuple(hidden), n_actions
        self.n_params = lib().tj_ppo_num_params(C.byref(d))
        nbytes = lib().tj_ppo_arena_bytes(C.byref(d))
        if nbytes == 0 or self.n_params == 0:
            raise TjError(TJ_ERR_SHAPE, "tj_ppo_arena_bytes")
        self.arena = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        self.arena_ptr = (self.arena.data_ptr() + 255) // 256 * 256
        th = np.ascontiguousarray(init, np.float32)
        assert th.size == self.n_params
        h = C.c_void_p()
        _check(lib().tj_ppo_create(C.byref(d), self.arena_ptr, nbytes, th.ctypes.data, _stream_ptr(stream),
                                   C.byref(h)), "tj_ppo_create")
        self.h = h
        self.stats = torch.zeros(5, dtype=torch.int32, device=device)   # tj_ppo_stats {4 x f32, u32}

    def __del__(self):
        if getattr(self, "h", None):
            lib().tj_learner_destroy(self.h)
            self.h = None

    def step(self, obs, action, old_logp, adv, ret, stream=None) -> int:
        """One update on device tensors: obs f32 [B, obs_dim], action i32 [B], old_logp / adv / ret f32 [B]."""
        b = tj_ppo_batch(int(action.shape[0]), obs.data_ptr(), action.data_ptr(), old_logp.data_ptr(),
                         adv.data_ptr(), ret.data_ptr())
        return lib().tj_ppo_step(self.h, C.byref(b), self.stats.data_ptr(), _stream_ptr(stream))

    def evaluate(self, obs, stream=None):
        """(logits f32 [n, A], value f32 [n]) of device observations under the current weights."""
        import torch

        n = int(obs.shape[0])
        logits = torch.empty((n, self.n_actions), dtype=torch.float32, device=obs.device)
        value = torch.empty(n, dtype=torch.float32, device=obs.device)
        _check(lib().tj_ppo_evaluate(self.h, n, obs.data_ptr(), logits.data_ptr(), value.data_ptr(),
                                     _stream_ptr(stream)), "tj_ppo_evaluate")
        return logits, value

    def act(self, obs, seed: int, stream=None):
        """Sampled (action i32 [n], logp f32 [n], value f32 [n]) for device observations."""
        import torch

        n = int(obs.shape[0])
        action = torch.empty(n, dtype=torch.int32, device=obs.device)
        logp = torch.empty(n, dtype=torch.float32, device=obs.device)
        value = torch.empty(n, dtype=torch.float32, device=obs.device)
        _check(lib().tj_ppo_act(self.h, n, obs.data_ptr(), seed & (2**64 - 1), action.data_ptr(), logp.data_ptr(),
                                value.data_ptr(), _stream_ptr(stream)), "tj_ppo_act")
        return action, logp, value

    def read_stats(self):
        """(loss_pi, loss_v, entropy, loss, t) of the last step."""
        raw = self.stats.cpu().numpy()
        f = raw.view(np.float32)
        return float(f[0]), float(f[1]), float(f[2]), float(f[3]), int(raw.view(np.uint32)[4])

    def get_state(self, which: int, stream=None) -> np.ndarray:
        out = np.empty(self.n_params, np.float32)
        _check(lib().tj_learner_get_state(self.h, which, out.ctypes.data, out.size, _stream_ptr(stream)),
               "tj_learner_get_state")
        return out

    def set_state(self, which: int, values, stream=None) -> None:
        v = np.ascontiguousarray(values, np.float32)
        _check(lib().tj_learner_set_state(self.h, which, v.ctypes.data, v.size, _stream_ptr(stream)),
               "tj_learner_set_state")


def learner_for_workload(wl, init_online, init_target, device="cuda:0", max_batch: Optional[int] = None):
    desc = make_learner_desc(wl.layers, wl.in_chw, wl.obs_dtype, wl.precision, max_batch or wl.batch,
                             wl.gamma, wl.kappa, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.target_interval)
    return Learner(desc, init_online, init_target, device=device)


class HipEvents:
    """n timing-enabled hipEvent_t created through the HIP runtime that torch loaded."""

    def __init__(self, n: int):
        import torch  # noqa: F401

        self.rt = C.CDLL("libamdhip64.so.7")
        self.rt.hipEventCreate.argtypes = [C.POINTER(C.c_void_p)]
        self.rt.hipEventElapsedTime.argtypes = [C.POINTER(C.c_float), C.c_void_p, C.c_void_p]
        self.rt.hipEventDestroy.argtypes = [C.c_void_p]
        self.ev = (C.c_void_p * n)()
        for i in range(n):
            e = C.c_void_p()
            if self.rt.hipEventCreate(C.byref(e)) != 0:
                raise RuntimeError("hipEventCreate failed")
            self.ev[i] = e

    def elapsed_ms(self, i: int, j: int) -> float:
        ms = C.c_float(0)
        if self.rt.hipEventElapsedTime(C.byref(ms), self.ev[i], self.ev[j]) != 0:
            raise RuntimeError("hipEventElapsedTime failed")
        return ms.value

    def __del__(self):
        for e in getattr(self, "ev", []):
            if e:
                self.rt.hipEventDestroy(e)
