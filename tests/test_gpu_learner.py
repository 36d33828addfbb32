"""GPU parity: the learner step (forward x3, TD target, Huber, backward, Adam,
target update) against the CPU oracle, through the C ABI.

Tolerances (relative, per tensor: max|a-b| / max|b|, and for scalars
|a-b| / |b|): 1e-4 for fp32 compute, 2e-2 for bf16 GEMM operands with fp32
accumulation.  The oracle's inputs and states come from the seeded generators
or from the oracle's own earlier steps, never from the GPU."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2502_20190_amd import synth
from paper_2502_20190_amd.synth import LIN
from parity_util import rel_l2, rel_max, rel_scalar, top2_gap

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def _batch(wl, seed, n=None):
    rows = synth.make_chunk(wl, seed, 0, n or wl.batch)
    rows.pop("version")
    return rows


def _batch_clear_of_kinks(o, wl, seed, n=None, margin=5e-6):
    """fp32 comparisons at 1e-4 need inputs away from the ReLU kinks, where the
    gradient jumps by O(1/B) in single rows when a pre-activation changes sign
    under fp32 rounding noise (~1e-6 for these widths).  Samples whose smallest
    hidden |pre-activation| under the ORACLE's current weights is inside the
    margin (a fraction of a percent of them) are re-drawn from another seed."""
    rows = _batch(wl, seed, n)
    for it in range(20):
        bad = o.min_abs_preactivation(rows["obs"]) <= margin
        if not bad.any():
            return rows
        repl = _batch(wl, seed + 7919 * (it + 1), n)
        for f in rows:
            rows[f][bad] = repl[f][bad]
    raise AssertionError("no kink-free batch found")


def _pair(tj, orc, wl, seed=0, max_batch=None, perturb_bias=True, hidden_bias=None):
    theta = synth.xavier_init(wl.layers, wl.in_chw, seed)
    target = synth.xavier_init(wl.layers, wl.in_chw, seed + 1)
    rng = np.random.default_rng(seed + 50)
    if perturb_bias:     # non-zero biases, so that a bias mix-up shows
        theta = (theta + 0.02 * rng.standard_normal(theta.size)).astype(np.float32)
        target = (target + 0.02 * rng.standard_normal(theta.size)).astype(np.float32)
    if hidden_bias is not None:
        # hidden biases of +-hidden_bias (several sigma of the pre-activations): units are mostly
        # on or mostly off, crossings still occur, but few pre-activations sit within fp32 noise of 0
        off = 0
        shapes = synth.layer_shapes(wl.layers, wl.in_chw)
        for i, (_, ws, _, _, _) in enumerate(shapes):
            off += int(np.prod(ws))
            if i < len(shapes) - 1:
                sign = rng.integers(0, 2, ws[0]) * 2 - 1
                theta[off:off + ws[0]] = (hidden_bias * sign).astype(np.float32)
            off += ws[0]
    g = tj.learner_for_workload(wl, theta, target, max_batch=max_batch)
    o = orc.Learner(wl.layers, wl.in_chw, obs_dtype=wl.obs_dtype, gamma=wl.gamma, kappa=wl.kappa, lr=wl.lr,
                    beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, target_interval=wl.target_interval,
                    emulate_bf16=(wl.precision == "bf16"))
    o.set_state(orc.PARAMS, theta.astype(np.float64))
    o.set_state(orc.TARGET, target.astype(np.float64))
    return g, o


def _load_oracle_state_into_gpu(tj, orc, g, o):
    """Teacher forcing, in the allowed direction: the GPU learner takes the ORACLE's state
    (the oracle never receives anything from the GPU).  With bf16 operands, free-running
    trajectories drift apart after a few Adam steps (an update of +-lr on every weight whose
    tiny gradient changes sign), so multi-step bf16 comparisons restart each step from the
    oracle's state and compare one step at a time."""
    g.set_state(tj.TJ_STATE_PARAMS, o.get_state(orc.PARAMS))
    g.set_state(tj.TJ_STATE_TARGET, o.get_state(orc.TARGET))
    g.set_state(tj.TJ_STATE_ADAM_M, o.get_state(orc.ADAM_M))
    g.set_state(tj.TJ_STATE_ADAM_V, o.get_state(orc.ADAM_V))
    g.t = o.t


def _step_both(tj, orc, g, o, wl, rows, tol, check_state=True, sync=False):
    """One step on both sides; compares loss, Q-values, greedy actions, gradients
    and (optionally) the updated state.  Returns the worst relative error seen."""
    if sync:
        _load_oracle_state_into_gpu(tj, orc, g, o)
    b = len(rows["action"])
    mb = tj.Minibatch(b, wl.obs_elems, wl.obs_dtype)
    mb.load(**rows)
    theta_before = o.get_state(orc.PARAMS)
    assert g.step(mb) == tj.TJ_OK
    oloss = o.step(**rows)
    gloss, gt = g.read_stats()
    assert gt == o.t == g.t
    worst = {}
    # Q-values of the three passes
    q = g.get_state(tj.TJ_STATE_QVALS).reshape(3, b, -1)
    for i, which in enumerate((orc.LAST_Q_S, orc.LAST_Q_NEXT_ONLINE, orc.LAST_Q_NEXT_TARGET)):
        worst[f"q{i}"] = rel_max(q[i], o.last(which))
    # greedy actions: equal except where the oracle's own top-2 gap is inside the float noise
    ga, oa = g.get_state(tj.TJ_STATE_ASTAR).astype(np.int32), o.last_astar()
    qn = o.last(orc.LAST_Q_NEXT_ONLINE)
    margin = (1e-5 if wl.precision == "fp32" else 2e-3) * np.abs(qn).max()
    mism = ga != oa
    assert (top2_gap(qn)[mism] < margin).all(), "greedy action differs outside the near-tie margin"
    assert mism.mean() <= 0.01
    worst["loss"] = rel_scalar(gloss, oloss)
    worst["grad"] = rel_max(g.get_state(tj.TJ_STATE_GRADS), o.get_state(orc.GRADS))
    if check_state:
        # updated weights: compare the update itself too (the weights alone hide it)
        gth, oth = g.get_state(tj.TJ_STATE_PARAMS), o.get_state(orc.PARAMS)
        worst["theta"] = rel_max(gth, oth)
        worst["m"] = rel_max(g.get_state(tj.TJ_STATE_ADAM_M), o.get_state(orc.ADAM_M))
        worst["v"] = rel_max(g.get_state(tj.TJ_STATE_ADAM_V), o.get_state(orc.ADAM_V))
        worst["target"] = rel_max(g.get_state(tj.TJ_STATE_TARGET), o.get_state(orc.TARGET))
    bad = {k: v for k, v in worst.items() if not v < tol}
    assert not bad, f"beyond {tol}: {bad} (all: {worst})"
    return worst, (g.get_state(tj.TJ_STATE_PARAMS).astype(np.float64) - theta_before,
                   o.get_state(orc.PARAMS) - theta_before)


def test_c1_ten_free_running_steps(tj, orc):
    """Config 1 (4-64-64-2 fp32, batch 32, lr 1e-3): all ten steps free-running on
    both sides stay inside the fp32 tolerance."""
    wl = synth.WORKLOADS["c1"]
    g, o = _pair(tj, orc, wl, seed=1, perturb_bias=False)
    for step in range(wl.steps):
        worst, _ = _step_both(tj, orc, g, o, wl, _batch_clear_of_kinks(o, wl, 100 + step), TOL["fp32"])
    assert g.t == 10


def test_c2_first_steps_and_update_direction(tj, orc):
    """Config 2 (128-256-256-18 fp32, batch 512): three free-running steps; at step
    one Adam's update is -lr*sign(g) wherever |g| >> eps, which pins the sign."""
    wl = synth.WORKLOADS["c2"]
    g, o = _pair(tj, orc, wl, seed=2)
    for step in range(3):
        worst, (gd, od) = _step_both(tj, orc, g, o, wl, _batch_clear_of_kinks(o, wl, 200 + step),
                                     TOL["fp32"])
        if step == 0:
            big = np.abs(o.get_state(orc.GRADS)) > 1e-5
            np.testing.assert_allclose(gd[big], -wl.lr * np.sign(o.get_state(orc.GRADS)[big]), rtol=2e-3)


def test_midtraining_state_from_the_oracle_side(tj, orc):
    """Both sides start from the same synthetic mid-training optimizer state
    (moments, t = 500), loaded through set_state."""
    wl = replace(synth.WORKLOADS["c2"], batch=256, target_interval=501)
    g, o = _pair(tj, orc, wl, seed=3)
    m, v = synth.midtraining_state(g.n_params, 9)
    g.set_state(tj.TJ_STATE_ADAM_M, m); g.set_state(tj.TJ_STATE_ADAM_V, v); g.t = 500
    o.set_state(orc.ADAM_M, m.astype(np.float64)); o.set_state(orc.ADAM_V, v.astype(np.float64)); o.t = 500
    _step_both(tj, orc, g, o, wl, _batch_clear_of_kinks(o, wl, 31), TOL["fp32"])
    assert g.t == 501
    np.testing.assert_array_equal(g.get_state(tj.TJ_STATE_TARGET), g.get_state(tj.TJ_STATE_PARAMS))


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_ragged_shapes_and_batch_changes(tj, orc, precision):
    """Layer widths and batches that are not multiples of any tile or vector
    size; the batch shrinks and grows between steps; the target syncs at t=2."""
    wl = replace(synth.WORKLOADS["c2"], obs_shape=(20,), n_actions=5, precision=precision,
                 layers=((LIN, 100, 0, 0), (LIN, 36, 0, 0), (LIN, 5, 0, 0)), batch=300,
                 target_interval=2, lr=1e-3)
    g, o = _pair(tj, orc, wl, seed=4, max_batch=300)
    for step, b in enumerate((77, 300, 24, 131, 1)):
        rows = _batch_clear_of_kinks(o, wl, 40 + step, b) if precision == "fp32" else _batch(wl, 40 + step, b)
        _step_both(tj, orc, g, o, wl, rows, TOL[precision])


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_multi_tile_mlp(tj, orc, precision):
    """Several 128 x 128 tiles in every GEMM, a split batch contraction (batch
    2304 > 2 x 1024) with a ragged last slice."""
    wl = replace(synth.WORKLOADS["c2"], obs_shape=(136,), n_actions=18, precision=precision,
                 layers=((LIN, 264, 0, 0), (LIN, 392, 0, 0), (LIN, 18, 0, 0)), batch=2304 + 40)
    g, o = _pair(tj, orc, wl, seed=5)
    for step in range(2):
        rows = _batch_clear_of_kinks(o, wl, 60 + step) if precision == "fp32" else _batch(wl, 60 + step)
        _step_both(tj, orc, g, o, wl, rows, TOL[precision])


def test_bf16_against_the_exact_oracle(tj, orc):
    """bf16 operands against the fp64 oracle without rounding emulation: Q-values
    and loss inside 2e-2, gradients inside 2e-2 in the L2 norm (single ReLU-mask
    flips are jumps of size 1/B in single entries)."""
    wl = replace(synth.WORKLOADS["c3"], obs_shape=(64,), n_actions=8, batch=1024,
                 layers=((LIN, 256, 0, 0), (LIN, 256, 0, 0), (LIN, 8, 0, 0)))
    g, _ = _pair(tj, orc, wl, seed=6)
    theta = g.get_state(tj.TJ_STATE_PARAMS).astype(np.float64)
    target = g.get_state(tj.TJ_STATE_TARGET).astype(np.float64)
    exact = orc.Learner(wl.layers, wl.in_chw, gamma=wl.gamma, kappa=wl.kappa, lr=wl.lr,
                        target_interval=wl.target_interval, emulate_bf16=False)
    exact.set_state(orc.PARAMS, theta); exact.set_state(orc.TARGET, target)
    rows = _batch(wl, 70)
    mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype)
    mb.load(**rows)
    assert g.step(mb) == tj.TJ_OK
    oloss = exact.step(**rows)
    gloss, _ = g.read_stats()
    q = g.get_state(tj.TJ_STATE_QVALS).reshape(3, wl.batch, -1)
    assert rel_max(q[0], exact.last(orc.LAST_Q_S)) < 2e-2
    assert rel_max(q[2], exact.last(orc.LAST_Q_NEXT_TARGET)) < 2e-2
    assert rel_scalar(gloss, oloss) < 2e-2
    assert rel_l2(g.get_state(tj.TJ_STATE_GRADS), exact.get_state(orc.GRADS)) < 2e-2


def test_c3_full_size_step(tj, orc):
    """Config 3 at full size (256-1024-1024-1024-32 bf16, batch 8192), the launch
    configuration the benchmark times, against the bf16-rounding oracle."""
    wl = synth.WORKLOADS["c3"]
    g, o = _pair(tj, orc, wl, seed=7)
    worst, _ = _step_both(tj, orc, g, o, wl, _batch(wl, 80), TOL["bf16"])
    print("c3 full-size worst relative errors:", worst)


def test_learner_argument_errors(tj, orc):
    import ctypes

    wl = synth.WORKLOADS["c1"]
    g, _ = _pair(tj, orc, wl, seed=8)
    mb = tj.Minibatch(64, wl.obs_elems, wl.obs_dtype)          # larger than max_batch = 32
    assert g.step(mb) == tj.TJ_ERR_SHAPE
    L = tj.lib()
    out = np.empty(3, np.float32)
    assert L.tj_learner_get_state(g.h, tj.TJ_STATE_PARAMS, out.ctypes.data, 3, None) == tj.TJ_ERR_INVALID_ARG
    assert L.tj_learner_set_state(g.h, tj.TJ_STATE_GRADS, out.ctypes.data, g.n_params, None) == tj.TJ_ERR_INVALID_ARG
    conv = tj.make_learner_desc([(1, 8, 3, 1), (0, 4, 0, 0)], (1, 8, 8), "u8", "bf16", 8, 0.99, 1.0, 1e-3,
                                0.9, 0.999, 1e-8, 10)
    assert L.tj_learner_num_params(ctypes.byref(conv)) == 8 * 9 + 8 + 4 * 8 * 36 + 4
    assert L.tj_learner_arena_bytes(ctypes.byref(conv)) > 0
    # channels-last rows must be whole 16-byte vectors: 6 output channels are refused
    bad = tj.make_learner_desc([(1, 6, 3, 1), (0, 4, 0, 0)], (1, 8, 8), "u8", "bf16", 8, 0.99, 1.0, 1e-3,
                               0.9, 0.999, 1e-8, 10)
    assert L.tj_learner_arena_bytes(ctypes.byref(bad)) == 0


# ---------------------------------------------------------------- convolutional Q-networks

def _conv_workload(precision, obs_dtype="u8", batch=24, in_chw=(2, 14, 14), layers=None, n_actions=4):
    from paper_2502_20190_amd.synth import CONV

    layers = layers or ((CONV, 8, 4, 2), (CONV, 16, 3, 1), (LIN, 32, 0, 0), (LIN, n_actions, 0, 0))
    return replace(synth.WORKLOADS["c4"], obs_shape=in_chw, obs_dtype=obs_dtype, n_actions=n_actions,
                   layers=layers, precision=precision, batch=batch, lr=1e-3, target_interval=2)


@pytest.mark.parametrize("precision,obs_dtype", [("fp32", "u8"), ("bf16", "u8"), ("fp32", "f32")])
def test_small_conv_net(tj, orc, precision, obs_dtype):
    """Two convolutions (4x4/2, 3x3/1) and two linear layers on 2x14x14 frames: patch matrices,
    channels-last permutations of the weights, col2im input gradients, target sync at t = 2."""
    wl = _conv_workload(precision, obs_dtype)
    g, o = _pair(tj, orc, wl, seed=11)
    for step, b in enumerate((24, 24, 7)):
        rows = _batch_clear_of_kinks(o, wl, 300 + step, b) if precision == "fp32" else _batch(wl, 300 + step, b)
        _step_both(tj, orc, g, o, wl, rows, TOL[precision], sync=(precision == "bf16" and step > 0))


def test_conv_stride_and_kernel_variants(tj, orc):
    """8x8/4 on 4 channels (the first Nature-DQN layer's geometry at small size) followed by 4x4/2."""
    from paper_2502_20190_amd.synth import CONV

    wl = _conv_workload("bf16", batch=10, in_chw=(4, 36, 36),
                        layers=((CONV, 16, 8, 4), (CONV, 16, 4, 2), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6)
    g, o = _pair(tj, orc, wl, seed=12)
    for step in range(2):
        _step_both(tj, orc, g, o, wl, _batch(wl, 320 + step), TOL["bf16"], sync=step > 0)


def test_gathered_conv_operands_with_ragged_batches(tj, orc):
    """Layers that take the patch-matrix-free path (bf16, 32 / 64 output channels, patch length a multiple
    of 64): 8x8/4 -> 32 channels, 4x4/2 -> 64 channels.  Patch counts that are not multiples of the
    32-row stages (21 * 64, 21 * 9, 5 * 9) and a shrinking batch exercise the zero pad rows."""
    from paper_2502_20190_amd.synth import CONV

    wl = _conv_workload("bf16", batch=21, in_chw=(4, 36, 36),
                        layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6)
    g, o = _pair(tj, orc, wl, seed=14)
    for step, b in enumerate((21, 21, 5)):
        _step_both(tj, orc, g, o, wl, _batch(wl, 360 + step, b), TOL["bf16"], sync=step > 0)


@pytest.mark.parametrize("hw,batch", [(36, 300), (100, 140)])
def test_first_conv_kernel_loops_over_images(tj, orc, hw, batch):
    """More images (2 x batch) than the fused first-convolution kernel has blocks (one per CU), so
    every block walks several images: register prefetch of the next frame stack, hand-over between
    the image buffers.  36 x 36 frames fit two image buffers in LDS, 100 x 100 frames only one (the
    variant with two barriers per image)."""
    from paper_2502_20190_amd.synth import CONV

    wl = _conv_workload("bf16", batch=batch, in_chw=(4, hw, hw),
                        layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6)
    g, o = _pair(tj, orc, wl, seed=15)
    _step_both(tj, orc, g, o, wl, _batch(wl, 380), TOL["bf16"])


def test_c5_full_batch_step(tj, orc):
    """Config 5's learner step at full size (Nature-DQN network, batch 2048, bf16), the launch
    configuration the benchmark times for the pixel workloads, against the bf16-rounding oracle."""
    wl = synth.WORKLOADS["c5"]
    g, o = _pair(tj, orc, wl, seed=16)
    worst, _ = _step_both(tj, orc, g, o, wl, _batch(wl, 390), TOL["bf16"])
    print("c5 full-batch worst relative errors:", worst)


@pytest.mark.parametrize("kind", ["mlp-bf16", "mlp-fp32", "conv-bf16"])
def test_steps_are_reproducible_bit_for_bit(tj, kind):
    """Every reduction on the path has a fixed order (no atomics on floating point): two learners
    built from the same state and fed the same minibatches end in identical parameters and
    optimizer moments."""
    from paper_2502_20190_amd.synth import CONV

    if kind == "conv-bf16":
        wl = _conv_workload("bf16", batch=48, in_chw=(4, 36, 36),
                            layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 64, 0, 0), (LIN, 6, 0, 0)), n_actions=6)
    else:
        wl = replace(synth.WORKLOADS["c3"], obs_shape=(96,), n_actions=12, batch=2048, lr=1e-3,
                     precision=kind.split("-")[1],
                     layers=((LIN, 320, 0, 0), (LIN, 256, 0, 0), (LIN, 12, 0, 0)))
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    target = synth.xavier_init(wl.layers, wl.in_chw, 4)
    finals = []
    for run in range(2):
        g = tj.learner_for_workload(wl, theta, target)
        mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype)
        for step in range(4):
            mb.load(**_batch(wl, 900 + step))
            assert g.step(mb) == tj.TJ_OK
        finals.append([g.get_state(w) for w in (tj.TJ_STATE_PARAMS, tj.TJ_STATE_ADAM_M, tj.TJ_STATE_ADAM_V,
                                                 tj.TJ_STATE_GRADS)] + [g.read_stats()])
    for a, b in zip(finals[0][:4], finals[1][:4]):
        assert np.array_equal(a, b)
    assert finals[0][4] == finals[1][4]
    assert not np.array_equal(finals[0][0], theta)


def test_c4_nature_dqn_shape_small_batch(tj, orc):
    """Config 4's network (4x84x84 u8 frames, conv 8x8/4x32, 4x4/2x64, 3x3/1x64, FC 3136-512-18, bf16)
    at batch 16, against the bf16-rounding oracle."""
    wl = replace(synth.WORKLOADS["c4"], batch=16)
    g, o = _pair(tj, orc, wl, seed=13)
    worst, _ = _step_both(tj, orc, g, o, wl, _batch(wl, 340), TOL["bf16"])
    print("c4 network, batch 16, worst relative errors:", worst)


# ---------------------------------------------------------------- policy inference (Algorithm 1, step 1)

def _check_act(tj, orc, g, o, wl, obs, eps, seed, tol):
    import torch

    dev = torch.from_numpy(np.ascontiguousarray(obs)).cuda()
    ga, gv, gq = g.act(dev, eps, seed, want_q=True)
    torch.cuda.synchronize()
    ga, gv, gq = ga.cpu().numpy(), gv.cpu().numpy(), gq.cpu().numpy()
    oa, oq, ogreedy = o.act(obs, eps, seed)
    assert (gv == g.t).all()
    assert rel_max(gq, oq) < tol
    # explore decisions and uniform actions are integer functions of the generator: identical;
    # greedy actions may differ only where the oracle's own top-2 gap is inside the float noise
    margin = (1e-5 if wl.precision == "fp32" else 2e-3) * np.abs(oq).max()
    mism = ga != oa
    assert (top2_gap(oq)[mism] < margin).all() and mism.mean() <= 0.01
    thr = int(eps * 2 ** 24)
    explore = np.array([(orc.rng64(seed, 2 * j) >> 40) < thr for j in range(len(oa))])
    np.testing.assert_array_equal(ga[explore], oa[explore])
    assert not (mism & explore).any()
    return explore.mean()


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_epsilon_greedy_inference_mlp(tj, orc, precision):
    wl = replace(synth.small_variant(synth.WORKLOADS["c2"], capacity=4096, batch=300), precision=precision)
    g, o = _pair(tj, orc, wl, seed=15)
    obs = _batch(wl, 400, 517)["obs"]                       # more rows than the batch (n <= 2 * max_batch)
    for eps, seed in ((0.0, 1), (0.05, 2), (1.0, 3)):
        rate = _check_act(tj, orc, g, o, wl, obs, eps, seed, TOL[precision])
        assert abs(rate - eps) < 0.05
    # after a learner step the stamp is the new version and the actions follow the new weights
    _step_both(tj, orc, g, o, wl, _batch(wl, 401), TOL[precision])
    _check_act(tj, orc, g, o, wl, obs[:64], 0.1, 4, TOL[precision])
    import torch

    assert g.t == 1
    dev = torch.from_numpy(obs).cuda()
    L = tj.lib()
    a = torch.empty(len(obs), dtype=torch.int32, device="cuda")
    assert L.tj_actor_act(g.h, 2 * wl.batch + 1, dev.data_ptr(), 0.1, 0, a.data_ptr(), a.data_ptr(), None,
                          None) == tj.TJ_ERR_SHAPE
    assert L.tj_actor_act(g.h, 8, dev.data_ptr(), 1.5, 0, a.data_ptr(), a.data_ptr(), None,
                          None) == tj.TJ_ERR_INVALID_ARG


def test_epsilon_greedy_inference_conv(tj, orc):
    """Pixel network (the gathered-operand layers and a linear tail), u8 frames."""
    from paper_2502_20190_amd.synth import CONV

    wl = _conv_workload("bf16", batch=12, in_chw=(4, 36, 36),
                        layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6)
    g, o = _pair(tj, orc, wl, seed=16)
    obs = _batch(wl, 410, 19)["obs"]
    for eps, seed in ((0.0, 5), (0.3, 6)):
        _check_act(tj, orc, g, o, wl, obs, eps, seed, TOL["bf16"])
