"""GPU parity on randomly drawn network shapes and batch sizes (seeded, so every run sees the same
cases): MLP and convolutional Q-learners and on-policy learners, both precisions, widths and
batches that are multiples of nothing, one-row batches, single-layer networks.  The tile and
kernel choices inside the library depend on the shapes; this walks through many of them.

fp32 cases compare Q-values, loss and gradients only: Adam's first step divides by |g| + eps, so
a weight whose gradient is of the order of eps (1e-8) turns an error of 1e-9 in that gradient
into a visible fraction of the learning rate."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2502_20190_amd import synth
from paper_2502_20190_amd.synth import CONV, LIN

import test_gpu_learner as T
import test_gpu_ppo as P

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def test_random_mlp_shapes(tj, orc):
    rng = np.random.default_rng(1)
    for case in range(60):
        prec = "bf16" if rng.random() < 0.6 else "fp32"
        nl = int(rng.integers(1, 5))
        widths = [int(rng.choice([8, 24, 64, 100, 128, 136, 192, 256, 320, 512, 600, 1024])) for _ in range(nl - 1)]
        A = int(rng.choice([1, 2, 6, 18, 32, 33, 40]))
        D = int(rng.choice([3, 16, 64, 100, 256, 300]))
        B = int(rng.choice([1, 7, 64, 129, 500, 1024, 2048, 3000]))
        ppo = rng.random() < 0.35
        print(f"case {case}: {'on-policy' if ppo else 'q-learning'} {prec} D={D} widths={widths} A={A} B={B}", flush=True)
        if ppo:
            A = max(A, 2)
            g, o = P._pair(tj, orc, D, tuple(widths), A, prec, B, seed=case, lr=1e-3)
            steps = 1 if B < 8 else 8
            rows = P._batch(orc, o, D, A, (B + steps - 1) // steps, steps, 1000 + case, prec, n=B)
            P._step_both(tj, orc, g, o, rows, P.TOL[prec])
        else:
            layers = tuple((LIN, w, 0, 0) for w in widths) + ((LIN, A, 0, 0),)
            wl = replace(synth.WORKLOADS["c2"], obs_shape=(D,), n_actions=A, batch=B, layers=layers,
                         precision=prec, lr=1e-3)
            g, o = T._pair(tj, orc, wl, seed=case)
            rows = T._batch_clear_of_kinks(o, wl, 500 + case, B) if prec == "fp32" else T._batch(wl, 500 + case, B)
            T._step_both(tj, orc, g, o, wl, rows, T.TOL[prec], check_state=(prec == "bf16"))


def test_random_conv_shapes(tj, orc):
    rng = np.random.default_rng(2)
    case = 0
    while case < 40:
        prec = "bf16" if rng.random() < 0.7 else "fp32"
        C = int(rng.choice([1, 2, 4]))
        H = int(rng.choice([20, 28, 36, 44, 52]))
        W = H if rng.random() < 0.7 else H + 2 * int(rng.integers(1, 4))
        layers, h, w, c, ok = [], H, W, C, True
        for li in range(int(rng.integers(1, 4))):
            O, k, s = int(rng.choice([8, 16, 32, 64])), int(rng.choice([3, 4, 8])), int(rng.choice([1, 2, 4]))
            if li == 0 and rng.random() < 0.5:
                O, k, s = 32, 8, 4
            if h < k or w < k:
                ok = False
                break
            layers.append((CONV, O, k, s))
            h, w, c = (h - k) // s + 1, (w - k) // s + 1, O
        if not ok or c * h * w > 6000:
            continue
        A = int(rng.choice([2, 6, 18]))
        layers += [(LIN, int(rng.choice([24, 64, 128])), 0, 0), (LIN, A, 0, 0)]
        B = int(rng.choice([1, 5, 16, 33, 150]))
        obs_dtype = "u8" if rng.random() < 0.8 else "f32"
        print(f"case {case}: {prec} {obs_dtype} in=({C},{H},{W}) layers={[l[1:] for l in layers]} B={B}", flush=True)
        case += 1
        wl = T._conv_workload(prec, obs_dtype=obs_dtype, batch=B, in_chw=(C, H, W), layers=tuple(layers), n_actions=A)
        g, o = T._pair(tj, orc, wl, seed=case)
        rows = T._batch_clear_of_kinks(o, wl, 700 + case, B) if prec == "fp32" else T._batch(wl, 700 + case, B)
        T._step_both(tj, orc, g, o, wl, rows, T.TOL[prec], check_state=(prec == "bf16"))
