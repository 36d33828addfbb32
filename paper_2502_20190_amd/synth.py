"""Seeded synthetic inputs shaped like the paper's replay contents.

The paper trains on Gym CartPole and Atari observations (Section 4.1); those
environments are not available here, so every replay row is synthetic: the
shapes, dtypes and value distributions of the workloads, drawn from seeded
generators.  This module serves the HIP path, the CPU oracle and the benchmark
alike and holds none of the method's arithmetic: it only produces inputs
(transitions, version tags, initial weights, optimizer states).

Every chunk of rows is a pure function of (seed, chunk index, row count,
backend): numpy's Philox on the host, torch's device generator on the GPU.  The
two backends give different values; a test uses one backend for both sides.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

MASTER_SEED = 20190


@dataclass(frozen=True)
class Workload:
    """One synthetic workload: ring, sampling gate, network and optimizer."""

    name: str
    capacity: int
    obs_shape: Tuple[int, ...]          # (D,) for vectors, (C, H, W) for pixels
    obs_dtype: str                      # "f32" or "u8"
    n_actions: int
    done_p: float
    version_max: int                    # tags lie in 0..version_max
    version_dist: str                   # "uniform" or "geometric"
    current_version: int
    max_staleness: int
    layers: Tuple[Tuple[int, int, int, int], ...]  # (kind, out, kernel, stride)
    precision: str                      # "fp32" or "bf16"
    batch: int
    steps: int
    lr: float
    gamma: float = 0.99
    kappa: float = 1.0
    beta1: float = 0.9
    beta2: float = 0.999
    eps: float = 1e-8                   # Appendix E, Table 2
    target_interval: int = 100          # Appendix E, Table 2 (64 for pixels)
    geometric_p: float = 0.1
    staleness_sweep: Tuple[int, ...] = field(default_factory=tuple)

    @property
    def obs_elems(self) -> int:
        return int(np.prod(self.obs_shape))

    @property
    def in_chw(self) -> Tuple[int, int, int]:
        if len(self.obs_shape) == 3:
            return tuple(self.obs_shape)  # type: ignore[return-value]
        return (self.obs_elems, 1, 1)

    @property
    def np_obs_dtype(self):
        return np.float32 if self.obs_dtype == "f32" else np.uint8

    @property
    def record_bytes(self) -> int:
        """Bytes of one stored transition that the gather moves (tag excluded)."""
        return 2 * self.obs_elems * (4 if self.obs_dtype == "f32" else 1) + 4 + 4 + 1


LIN, CONV = 0, 1


def _mlp(*outs):
    return tuple((LIN, o, 0, 0) for o in outs)


_NATURE = ((CONV, 32, 8, 4), (CONV, 64, 4, 2), (CONV, 64, 3, 1), (LIN, 512, 0, 0), (LIN, 18, 0, 0))

WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1-tiny", 10_000, (4,), "f32", 2, 0.05, 99, "uniform", 99, 10,
                   _mlp(64, 64, 2), "fp32", 32, 10, 1e-3),
    "c2": Workload("c2-vector-medium", 1_000_000, (128,), "f32", 18, 0.01, 999, "uniform", 999, 32,
                   _mlp(256, 256, 18), "fp32", 512, 1000, 5e-4),
    "c3": Workload("c3-vector-high-throughput", 4_000_000, (256,), "f32", 32, 0.01, 999, "uniform",
                   999, 8, _mlp(1024, 1024, 1024, 32), "bf16", 8192, 1000, 5e-4),
    "c4": Workload("c4-pixel", 1_000_000, (4, 84, 84), "u8", 18, 0.01, 999, "uniform", 999, 32,
                   _NATURE, "bf16", 256, 500, 2.5e-5, target_interval=64),
    "c5": Workload("c5-pixel-large-batch", 2_000_000, (4, 84, 84), "u8", 18, 0.01, 999, "geometric",
                   999, 16, _NATURE, "bf16", 2048, 200, 2.5e-5, target_interval=64,
                   staleness_sweep=(1, 4, 16, 64)),
}


def layer_shapes(layers, in_chw):
    """[(kind, w_shape, fan_in, fan_out, out_chw)] for a layer chain."""
    c, h, w = in_chw
    out = []
    for kind, oc, k, s in layers:
        if kind == CONV:
            oh, ow = (h - k) // s + 1, (w - k) // s + 1
            out.append((kind, (oc, c, k, k), c * k * k, oc * k * k, (oc, oh, ow)))
            c, h, w = oc, oh, ow
        else:
            fin = c * h * w
            out.append((kind, (oc, fin), fin, oc, (oc, 1, 1)))
            c, h, w = oc, 1, 1
    return out


def num_params(layers, in_chw) -> int:
    return sum(int(np.prod(ws)) + ws[0] for _, ws, _, _, _ in layer_shapes(layers, in_chw))


def xavier_init(layers, in_chw, seed: int) -> np.ndarray:
    """Xavier-uniform weights, zero biases, in the flat parameter order:
    layer by layer, weight [out, in] (conv [Cout, Cin, kh, kw]) then bias."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x7761]))
    parts: List[np.ndarray] = []
    for _, ws, fin, fout, _ in layer_shapes(layers, in_chw):
        a = math.sqrt(6.0 / (fin + fout))
        parts.append(rng.uniform(-a, a, size=int(np.prod(ws))).astype(np.float32))
        parts.append(np.zeros(ws[0], dtype=np.float32))
    return np.concatenate(parts)


def midtraining_state(n_params: int, seed: int, grad_scale: float = 1e-3):
    """A plausible optimizer state for starting a comparison away from step 0:
    first moment ~ N(0, scale), second moment ~ scale^2 * chi^2-like, positive."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 0x6D76]))
    m = (grad_scale * rng.standard_normal(n_params)).astype(np.float32)
    v = ((grad_scale ** 2) * (0.1 + rng.random(n_params))).astype(np.float32)
    return m, v


def _versions_np(wl: Workload, rng, n: int) -> np.ndarray:
    if wl.version_dist == "uniform":
        return rng.integers(0, wl.version_max + 1, size=n, dtype=np.int32)
    # geometric on {0,1,2,...}, P(G=g) = p (1-p)^g, counted back from the newest tag
    g = rng.geometric(wl.geometric_p, size=n) - 1
    return np.maximum(0, wl.version_max - g).astype(np.int32)


def make_chunk(wl: Workload, seed: int, chunk: int, n: int) -> Dict[str, np.ndarray]:
    """Host rows of chunk `chunk`: obs, next_obs, action, reward, done, version."""
    rng = np.random.Generator(np.random.Philox(key=[seed, chunk]))
    d = wl.obs_elems
    if wl.obs_dtype == "f32":
        obs = rng.standard_normal((n, d), dtype=np.float32)
        nxt = rng.standard_normal((n, d), dtype=np.float32)
    else:
        obs = rng.integers(0, 256, size=(n, d), dtype=np.uint8)
        nxt = rng.integers(0, 256, size=(n, d), dtype=np.uint8)
    return {
        "obs": obs,
        "next_obs": nxt,
        "action": rng.integers(0, wl.n_actions, size=n, dtype=np.int32),
        "reward": rng.uniform(-1.0, 1.0, size=n).astype(np.float32),
        "done": (rng.random(n) < wl.done_p).astype(np.uint8),
        "version": _versions_np(wl, rng, n),
    }


def make_chunk_device(wl: Workload, seed: int, chunk: int, n: int, device="cuda:0"):
    """Device rows of chunk `chunk` as torch tensors (same fields as make_chunk).
    Used where the ring is too large to stage through host memory."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + chunk) & 0x7FFFFFFFFFFFFFFF)
    d = wl.obs_elems
    if wl.obs_dtype == "f32":
        obs = torch.randn((n, d), generator=g, device=device, dtype=torch.float32)
        nxt = torch.randn((n, d), generator=g, device=device, dtype=torch.float32)
    else:
        obs = torch.randint(0, 256, (n, d), generator=g, device=device, dtype=torch.uint8)
        nxt = torch.randint(0, 256, (n, d), generator=g, device=device, dtype=torch.uint8)
    action = torch.randint(0, wl.n_actions, (n,), generator=g, device=device, dtype=torch.int32)
    reward = torch.rand((n,), generator=g, device=device, dtype=torch.float32) * 2.0 - 1.0
    done = (torch.rand((n,), generator=g, device=device) < wl.done_p).to(torch.uint8)
    if wl.version_dist == "uniform":
        version = torch.randint(0, wl.version_max + 1, (n,), generator=g, device=device,
                                dtype=torch.int32)
    else:
        u = torch.rand((n,), generator=g, device=device, dtype=torch.float64)
        geo = torch.floor(torch.log1p(-u) / math.log1p(-wl.geometric_p))
        version = torch.clamp(wl.version_max - geo, min=0).to(torch.int32)
    return {"obs": obs, "next_obs": nxt, "action": action, "reward": reward, "done": done,
            "version": version}


def make_frame_stream_device(wl: Workload, seed: int, chunk: int, n: int, t0: int, device="cuda:0"):
    """Rows t0 .. t0+n of one environment stream for the frame ring (one u8 frame per row): frames
    uniform, actions / rewards / done as make_chunk_device, and version tags that rise with time so
    that a ring of wl.capacity rows spans the tags 0 .. wl.version_max."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + 7_000_000 + chunk) & 0x7FFFFFFFFFFFFFFF)
    fe = wl.obs_shape[1] * wl.obs_shape[2]
    frame = torch.randint(0, 256, (n, fe), generator=g, device=device, dtype=torch.uint8)
    action = torch.randint(0, wl.n_actions, (n,), generator=g, device=device, dtype=torch.int32)
    reward = torch.rand((n,), generator=g, device=device, dtype=torch.float32) * 2.0 - 1.0
    done = (torch.rand((n,), generator=g, device=device) < wl.done_p).to(torch.uint8)
    per_version = max(1, wl.capacity // (wl.version_max + 1))
    t = torch.arange(t0, t0 + n, device=device, dtype=torch.int64)
    version = torch.clamp(t // per_version, max=wl.version_max).to(torch.int32)
    return {"frame": frame, "action": action, "reward": reward, "done": done, "version": version}


def small_variant(wl: Workload, capacity: int, batch: Optional[int] = None) -> Workload:
    """The same workload on a smaller ring (and batch), for cases the oracle
    finishes in seconds."""
    from dataclasses import replace

    return replace(wl, capacity=capacity, batch=batch or wl.batch)


# ---------------------------------------------------------------- on-policy rollouts
#
# The PPO column of the paper's hyperparameter table: rollouts of 512 steps, the learner's batch
# is the whole buffer (n_env * 512 fresh transitions), hidden width 256.  Inputs only: the
# estimator and the objective live in the library and, separately, in the oracle.

PPO_WORKLOADS = {
    # name: (obs_dim, hidden widths, actions, n_env, rollout, precision)
    "p1": ("p1-ppo-classic-control", 4, (256, 256), 2, 8, 512, "fp32"),
    "p2": ("p2-ppo-vector-large-batch", 256, (1024, 1024, 1024), 31, 64, 512, "bf16"),
}


# Appendix E, Table 2, PPO column (Adam's betas are the usual defaults; the table gives eps and lr)
PPO_HYPER = {"gamma": 0.99, "lam": 0.95, "lr": 1e-4, "beta1": 0.9, "beta2": 0.999, "eps": 1e-5}


def ppo_layers(hidden, n_actions):
    """Actor-critic MLP: shared trunk, head of n_actions logits + 1 state value."""
    return _mlp(*hidden, n_actions + 1)


def make_rollouts(obs_dim: int, n_actions: int, n_env: int, T: int, seed: int, done_p: float = 0.01):
    """Seeded stand-in for what n_env actors send after T steps each (environment-major):
    observations, actions, rewards, episode ends, and what the behaviour policy recorded when it
    acted (state values incl. the bootstrap column, log-probability of the action taken; the
    latter scattered around the uniform policy's so that probability ratios land on both sides
    of the clipping interval)."""
    rng = np.random.default_rng([MASTER_SEED, 77, seed])
    n = n_env * T
    return {
        "obs": rng.standard_normal((n, obs_dim)).astype(np.float32),
        "action": rng.integers(0, n_actions, n).astype(np.int32),
        "reward": rng.uniform(-1.0, 1.0, (n_env, T)).astype(np.float32),
        "done": (rng.random((n_env, T)) < done_p).astype(np.uint8),
        "value": rng.standard_normal((n_env, T + 1)).astype(np.float32),
        "old_logp": (-np.log(n_actions) + 0.25 * rng.standard_normal(n)).astype(np.float32),
    }
