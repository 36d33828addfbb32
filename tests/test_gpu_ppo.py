"""GPU parity of the on-policy workload (advantage estimation, clipped actor-critic update)
against the CPU oracle, through the C ABI.

Tolerances (relative, per tensor: max|a-b| / max|b|): 1e-5 for the fp32 advantage scan, 1e-4 for
fp32 updates, 2e-2 for bf16 GEMM operands with fp32 accumulation.  Inputs come from the seeded
generators; the oracle never receives anything from the GPU."""
import ctypes as C

import numpy as np
import pytest

from paper_2502_20190_amd import synth
from parity_util import rel_max, rel_scalar

pytestmark = pytest.mark.gpu
TOL = {"fp32": 1e-4, "bf16": 2e-2}


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def _dev(a):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ---------------------------------------------------------------- advantage estimation

@pytest.mark.parametrize("n_env,T,done_p", [(8, 512, 0.01), (3, 17, 0.3), (5, 513, 0.02), (64, 512, 0.01),
                                            (1, 1, 0.0), (2, 1030, 0.005), (7, 8, 0.5), (6, 511, 0.0),
                                            (4, 64, 1.0)])
def test_gae_matches_oracle(tj, orc, n_env, T, done_p):
    import torch

    ro = synth.make_rollouts(4, 2, n_env, T, seed=n_env * 1000 + T, done_p=done_p)
    adv, ret = tj.gae(_dev(ro["reward"]), _dev(ro["value"]), _dev(ro["done"]), 0.99, 0.95)
    torch.cuda.synchronize()
    oadv, oret = orc.gae(ro["reward"], ro["value"], ro["done"], float(np.float32(0.99)), float(np.float32(0.95)))
    assert rel_max(adv.cpu().numpy(), oadv) < 1e-5
    assert rel_max(ret.cpu().numpy(), oret) < 1e-5


def test_gae_full_size_and_degenerate_calls(tj, orc):
    """The benchmark's rollout shape (64 environments x 512 steps), other discount settings, and
    the calls that do nothing or are refused."""
    import torch

    ro = synth.make_rollouts(4, 2, 64, 512, seed=5)
    r, v, d = _dev(ro["reward"]), _dev(ro["value"]), _dev(ro["done"])
    for gamma, lam in ((1.0, 1.0), (0.9, 0.0), (0.0, 0.5)):
        adv, ret = tj.gae(r, v, d, gamma, lam)
        oadv, oret = orc.gae(ro["reward"], ro["value"], ro["done"], gamma, lam)
        assert rel_max(adv.cpu().numpy(), oadv) < 1e-5 and rel_max(ret.cpu().numpy(), oret) < 1e-5
    L = tj.lib()
    out = torch.zeros(4, device="cuda")
    assert L.tj_gae(0, 512, r.data_ptr(), v.data_ptr(), d.data_ptr(), 0.99, 0.95, out.data_ptr(), out.data_ptr(),
                    None) == tj.TJ_OK
    assert L.tj_gae(4, 0, r.data_ptr(), v.data_ptr(), d.data_ptr(), 0.99, 0.95, out.data_ptr(), out.data_ptr(),
                    None) == tj.TJ_OK
    assert L.tj_gae(4, 8, None, v.data_ptr(), d.data_ptr(), 0.99, 0.95, out.data_ptr(), out.data_ptr(),
                    None) == tj.TJ_ERR_INVALID_ARG
    assert L.tj_gae(4, 8, r.data_ptr(), v.data_ptr(), d.data_ptr(), 1.5, 0.95, out.data_ptr(), out.data_ptr(),
                    None) == tj.TJ_ERR_INVALID_ARG
    torch.cuda.synchronize()
    assert not out.any()


# ---------------------------------------------------------------- clipped update

HYPER = {k: synth.PPO_HYPER[k] for k in ("lr", "beta1", "beta2", "eps")}   # the PPO column of the hyperparameter table
COEF = dict(clip=0.2, c_v=0.5, c_e=0.01)


def _pair(tj, orc, obs_dim, hidden, A, precision, max_batch, seed=0, lr=None):
    layers = synth.ppo_layers(hidden, A)
    theta = synth.xavier_init(layers, (obs_dim, 1, 1), seed)
    theta = (theta + 0.02 * np.random.default_rng(seed + 50).standard_normal(theta.size)).astype(np.float32)
    hyper = dict(HYPER)
    if lr is not None:
        hyper["lr"] = lr
    g = tj.PpoLearner(obs_dim, hidden, A, precision, max_batch, theta, **hyper, **COEF)
    o = orc.Learner(layers, (obs_dim, 1, 1), emulate_bf16=(precision == "bf16"), **hyper)
    o.set_state(orc.PARAMS, theta.astype(np.float64))
    return g, o


def _batch(orc, o, obs_dim, A, n_env, T, seed, precision, n=None):
    """Rollouts -> flat batch with oracle-side advantages.  For fp32 comparisons at 1e-4, rows
    within float noise of a ReLU kink or of the clipping boundary (where the gradient jumps by
    O(1/B) in single rows) are re-drawn from another seed; the selection uses the oracle's own
    forward pass."""
    def draw(s):
        ro = synth.make_rollouts(obs_dim, A, n_env, T, seed=s)
        adv, ret = orc.gae(ro["reward"], ro["value"], ro["done"], 0.99, 0.95)
        return dict(obs=ro["obs"], action=ro["action"], old_logp=ro["old_logp"],
                    adv=adv.ravel().astype(np.float32), ret=ret.ravel().astype(np.float32))

    rows = draw(seed)
    if n is not None:
        rows = {k: v[:n] for k, v in rows.items()}
    if precision == "bf16":
        return rows
    for it in range(20):
        z = o.forward(0, rows["obs"])[:, :A]
        logp = z[np.arange(len(z)), rows["action"]] - np.log(np.exp(z - z.max(1, keepdims=True)).sum(1)) - z.max(1)
        rho = np.exp(logp - rows["old_logp"])
        bad = (o.min_abs_preactivation(rows["obs"]) <= 5e-6) | (np.abs(rho - 0.8) < 1e-4) | (np.abs(rho - 1.2) < 1e-4)
        if not bad.any():
            return rows
        repl = draw(seed + 7919 * (it + 1))
        for f in rows:
            rows[f][bad] = repl[f][: len(bad)][bad]
    raise AssertionError("no batch clear of the kinks found")


def _sync(tj, orc, g, o):
    """The GPU learner takes the oracle's state (never the other way round)."""
    g.set_state(tj.TJ_STATE_PARAMS, o.get_state(orc.PARAMS))
    g.set_state(tj.TJ_STATE_ADAM_M, o.get_state(orc.ADAM_M))
    g.set_state(tj.TJ_STATE_ADAM_V, o.get_state(orc.ADAM_V))
    assert tj.lib().tj_learner_set_step(g.h, o.t) == tj.TJ_OK


def _bf16_image(x):
    import torch

    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def _check_compute_copies(tj, g, precision):
    """The weight copies the contraction kernels read are the compute-type image of the master
    weights (identical in fp32, round-to-nearest-even in bf16), straight and transposed."""
    layers = synth.ppo_layers(g.hidden, g.n_actions)
    w = np.zeros(g.n_params, bool)
    off = 0
    for _, ws, _, _, _ in synth.layer_shapes(layers, (g.obs_dim, 1, 1)):
        n = int(np.prod(ws))
        w[off:off + n] = True
        off += n + ws[0]
    theta = g.get_state(tj.TJ_STATE_PARAMS)
    want = _bf16_image(theta) if precision == "bf16" else theta
    for which in (tj.TJ_STATE_WEIGHTS_COMPUTE, tj.TJ_STATE_WEIGHTS_COMPUTE_T):
        copy = g.get_state(which)
        assert np.array_equal(copy[w], want[w]) and np.array_equal(copy[~w], theta[~w])


def _step_both(tj, orc, g, o, rows, tol, sync=False, precision=None):
    if sync:
        _sync(tj, orc, g, o)
    dev = {k: _dev(v) for k, v in rows.items()}
    theta_before_g = g.get_state(tj.TJ_STATE_PARAMS).astype(np.float64)
    theta_before_o = o.get_state(orc.PARAMS)
    assert g.step(dev["obs"], dev["action"], dev["old_logp"], dev["adv"], dev["ret"]) == tj.TJ_OK
    ostats = o.ppo_step(rows["obs"], rows["action"], rows["old_logp"], rows["adv"], rows["ret"], **COEF)
    gs = g.read_stats()
    assert gs[4] == o.t
    worst = {name: rel_scalar(gs[i], ostats[i]) for i, name in enumerate(("loss_pi", "loss_v", "entropy", "loss"))}
    # the policy term averages signed numbers and may sit near zero: measure it against the
    # scale of its summands
    scale = float(np.abs(rows["adv"]).mean())
    worst["loss_pi"] = abs(gs[0] - ostats[0]) / max(abs(ostats[0]), scale)
    worst["loss"] = abs(gs[3] - ostats[3]) / max(abs(ostats[3]), scale)
    og = o.get_state(orc.GRADS)
    worst["grad"] = rel_max(g.get_state(tj.TJ_STATE_GRADS), og)
    worst["theta"] = rel_max(g.get_state(tj.TJ_STATE_PARAMS), o.get_state(orc.PARAMS))
    worst["m"] = rel_max(g.get_state(tj.TJ_STATE_ADAM_M), o.get_state(orc.ADAM_M))
    worst["v"] = rel_max(g.get_state(tj.TJ_STATE_ADAM_V), o.get_state(orc.ADAM_V))
    # the update itself (the weights alone hide it: one step moves a weight by about lr), on the
    # entries whose gradient is at least a tenth of the largest: there the gradient's relative error
    # is at most tol / 0.1, which Adam's normalised step passes on with a factor <= 1
    big = np.abs(og) >= 0.1 * np.abs(og).max()
    dth_g = g.get_state(tj.TJ_STATE_PARAMS).astype(np.float64) - theta_before_g
    dth_o = o.get_state(orc.PARAMS) - theta_before_o
    worst["update/3"] = float(np.abs(dth_g[big] - dth_o[big]).max() / np.abs(dth_o[big]).max()) / 3
    bad = {k: v for k, v in worst.items() if not v < tol}
    assert not bad, f"beyond {tol}: {bad} (all: {worst})"
    if precision is not None:
        _check_compute_copies(tj, g, precision)
    return worst


def test_p1_classic_control_free_running(tj, orc):
    """The small on-policy configuration (4 observations, 256-256 trunk, 2 actions, 8 rollouts
    of 512 steps = batch 4096, fp32): five successive updates on the same batch, as the epochs
    of one PPO iteration; the ratio drifts from the behaviour policy's, clipping sets in."""
    _, D, hidden, A, n_env, T, prec = synth.PPO_WORKLOADS["p1"]
    g, o = _pair(tj, orc, D, hidden, A, prec, n_env * T, seed=1, lr=1e-3)
    rows = _batch(orc, o, D, A, n_env, T, 10, prec)
    theta0 = o.get_state(orc.PARAMS)
    for it in range(5):
        worst = _step_both(tj, orc, g, o, rows, TOL[prec], sync=it > 0, precision=prec)
    # the update itself, not just the weights
    du_g = g.get_state(tj.TJ_STATE_PARAMS).astype(np.float64) - theta0
    du_o = o.get_state(orc.PARAMS) - theta0
    assert rel_max(du_g, du_o) < 1e-3
    print("p1 worst relative errors at the fifth step:", worst)


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_ragged_shapes_and_batch_changes(tj, orc, precision):
    """Widths and batches that are multiples of nothing, a batch that shrinks and grows again
    (pad columns of the transposed activations must read as zero), 63 actions (the most the
    head kernel accepts)."""
    for (D, hidden, A) in ((19, (70, 33), 5), (130, (200,), 63), (7, (), 3), (6, (40,), 1)):
        g, o = _pair(tj, orc, D, hidden, A, precision, 700, seed=3, lr=1e-3)
        for i, n in enumerate((700, 100, 257)):
            rows = _batch(orc, o, D, A, 2, 350, 20 + i, precision, n=n)
            _step_both(tj, orc, g, o, rows, TOL[precision], sync=True, precision=precision)


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_multi_tile_trunk(tj, orc, precision):
    D, hidden, A = 96, (384, 320), 17
    g, o = _pair(tj, orc, D, hidden, A, precision, 1536, seed=4, lr=1e-3)
    rows = _batch(orc, o, D, A, 3, 512, 30, precision)
    _step_both(tj, orc, g, o, rows, TOL[precision], precision=precision)
    _step_both(tj, orc, g, o, rows, TOL[precision], precision=precision)   # free-running: reads the emitted copies


def test_p2_full_size_step(tj, orc):
    """The large on-policy configuration at full size (256 observations, 1024-1024-1024 trunk,
    31 actions + value, 64 rollouts of 512 steps = batch 32768, bf16), the launch configuration
    the benchmark times, against the bf16-rounding oracle."""
    _, D, hidden, A, n_env, T, prec = synth.PPO_WORKLOADS["p2"]
    g, o = _pair(tj, orc, D, hidden, A, prec, n_env * T, seed=7)
    rows = _batch(orc, o, D, A, n_env, T, 40, prec)
    print("p2 full-size worst relative errors:", _step_both(tj, orc, g, o, rows, TOL[prec], precision=prec))


def test_p2_full_size_step_against_the_exact_oracle(tj, orc):
    """The same update against the plain fp64 oracle (no rounding emulation): the three terms of the
    objective and the gradient vector inside 2e-2 (max norm); in the L2 norm the gradient may be at
    most a quarter further from the exact one than the oracle's own bf16-rounding mode is (a ReLU-mask
    flip or a ratio that crosses the clipping boundary under rounding is a jump of size 1/B in single
    rows)."""
    _, D, hidden, A, n_env, T, prec = synth.PPO_WORKLOADS["p2"]
    layers = synth.ppo_layers(hidden, A)
    theta = synth.xavier_init(layers, (D, 1, 1), 7)
    theta = (theta + 0.02 * np.random.default_rng(57).standard_normal(theta.size)).astype(np.float32)
    g = tj.PpoLearner(D, hidden, A, prec, n_env * T, theta, **HYPER, **COEF)
    exact = orc.Learner(layers, (D, 1, 1), emulate_bf16=False, **HYPER)
    rounding = orc.Learner(layers, (D, 1, 1), emulate_bf16=True, **HYPER)
    exact.set_state(orc.PARAMS, theta.astype(np.float64))
    rounding.set_state(orc.PARAMS, theta.astype(np.float64))
    rows = _batch(orc, exact, D, A, n_env, T, 40, prec)
    dev = {k: _dev(v) for k, v in rows.items()}
    assert g.step(dev["obs"], dev["action"], dev["old_logp"], dev["adv"], dev["ret"]) == tj.TJ_OK
    ostats = exact.ppo_step(rows["obs"], rows["action"], rows["old_logp"], rows["adv"], rows["ret"], **COEF)
    rounding.ppo_step(rows["obs"], rows["action"], rows["old_logp"], rows["adv"], rows["ret"], **COEF)
    gs = g.read_stats()
    scale = float(np.abs(rows["adv"]).mean())
    worst = {"loss_pi": abs(gs[0] - ostats[0]) / max(abs(ostats[0]), scale), "loss_v": rel_scalar(gs[1], ostats[1]),
             "entropy": rel_scalar(gs[2], ostats[2])}
    ga, og = g.get_state(tj.TJ_STATE_GRADS).astype(np.float64), exact.get_state(orc.GRADS)
    worst["grad"] = rel_max(ga, og)
    l2_gpu = float(np.linalg.norm(ga - og) / np.linalg.norm(og))
    l2_rounding = float(np.linalg.norm(rounding.get_state(orc.GRADS) - og) / np.linalg.norm(og))
    print("p2 against the exact oracle:", worst, "gradient L2 error", l2_gpu, "of the rounding oracle", l2_rounding)
    bad = {k: v for k, v in worst.items() if not v < 2e-2}
    assert not bad, f"beyond 2e-2: {bad} (all: {worst})"
    assert l2_gpu < max(2e-2, 1.25 * l2_rounding)


def test_p1_fp32_on_the_plain_seeded_batch(tj, orc):
    """fp32 parity on the seeded rollouts as drawn (no row is re-drawn).  The oracle lists the rows
    within float noise of a ReLU kink or of the clipping boundary: they must be rare, and only they
    may carry a differing derivative.  The objective's terms are continuous there (1e-4); gradients are
    compared in the L2 norm with those rows' 1/B shares added to the tolerance."""
    _, D, hidden, A, n_env, T, prec = synth.PPO_WORKLOADS["p1"]
    g, o = _pair(tj, orc, D, hidden, A, prec, n_env * T, seed=11, lr=1e-3)
    rows = _batch(orc, o, D, A, n_env, T, 77, "bf16")            # "bf16": the rows as drawn
    z = o.forward(0, rows["obs"])[:, :A]
    lse = np.log(np.exp(z - z.max(1, keepdims=True)).sum(1)) + z.max(1)
    rho = np.exp(z[np.arange(len(z)), rows["action"]] - lse - rows["old_logp"])
    # 512 hidden units per row: float noise of a pre-activation of size 1 summed over 256 terms is 1e-6
    near = (o.min_abs_preactivation(rows["obs"]) <= 2e-6) | (np.abs(rho - 0.8) < 1e-5) | (np.abs(rho - 1.2) < 1e-5)
    B = len(rho)
    assert near.sum() <= 0.01 * B
    dev = {k: _dev(v) for k, v in rows.items()}
    assert g.step(dev["obs"], dev["action"], dev["old_logp"], dev["adv"], dev["ret"]) == tj.TJ_OK
    ostats = o.ppo_step(rows["obs"], rows["action"], rows["old_logp"], rows["adv"], rows["ret"], **COEF)
    gs = g.read_stats()
    scale = float(np.abs(rows["adv"]).mean())
    assert abs(gs[0] - ostats[0]) / max(abs(ostats[0]), scale) < TOL["fp32"]
    assert rel_scalar(gs[1], ostats[1]) < TOL["fp32"] and rel_scalar(gs[2], ostats[2]) < TOL["fp32"]
    ga, og = g.get_state(tj.TJ_STATE_GRADS).astype(np.float64), o.get_state(orc.GRADS)
    err = float(np.linalg.norm(ga - og) / np.linalg.norm(og))
    print(f"p1: {int(near.sum())} rows near a kink or the clipping boundary, gradient relative L2 error {err:.2e}")
    assert err < TOL["fp32"] + near.sum() / B


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_evaluate_matches_oracle_forward(tj, orc, precision):
    import torch

    D, hidden, A = 24, (128, 64), 6
    g, o = _pair(tj, orc, D, hidden, A, precision, 512, seed=8)
    obs = synth.make_rollouts(D, A, 1, 300, seed=2)["obs"]
    logits, value = g.evaluate(_dev(obs))
    torch.cuda.synchronize()
    z = o.forward(0, obs)
    assert rel_max(logits.cpu().numpy(), z[:, :A]) < TOL[precision]
    assert rel_max(value.cpu().numpy(), z[:, A]) < TOL[precision]


def test_argument_errors(tj, orc):
    import torch

    g, o = _pair(tj, orc, 8, (32,), 4, "fp32", 64, seed=9)
    rows = _batch(orc, o, 8, 4, 1, 128, 3, "fp32")
    dev = {k: _dev(v) for k, v in rows.items()}
    # more rows than max_batch
    assert g.step(dev["obs"], dev["action"], dev["old_logp"], dev["adv"], dev["ret"]) == tj.TJ_ERR_SHAPE
    L = tj.lib()
    b = tj.tj_ppo_batch(64, dev["obs"].data_ptr(), None, dev["old_logp"].data_ptr(), dev["adv"].data_ptr(),
                        dev["ret"].data_ptr())
    assert L.tj_ppo_step(g.h, C.byref(b), None, None) == tj.TJ_ERR_INVALID_ARG
    # a Q-learning step or epsilon-greedy inference on an on-policy handle is refused
    mb = tj.Minibatch(16, 8, "f32")
    assert L.tj_learner_step(g.h, C.byref(mb.c), None, None) == tj.TJ_ERR_INVALID_ARG
    # and the other way round
    wl = synth.WORKLOADS["c1"]
    q = tj.learner_for_workload(wl, synth.xavier_init(wl.layers, wl.in_chw, 1), synth.xavier_init(wl.layers, wl.in_chw, 2))
    b.action = dev["action"].data_ptr()
    assert L.tj_ppo_step(q.h, C.byref(b), None, None) == tj.TJ_ERR_INVALID_ARG
    # descriptors the library refuses
    d = tj.tj_ppo_desc()
    d.obs_dim, d.n_hidden, d.n_actions, d.max_batch = 8, 1, 64, 32
    d.hidden[0] = 16
    d.clip, d.c_v, d.c_e = 0.2, 0.5, 0.01
    assert L.tj_ppo_arena_bytes(C.byref(d)) == 0           # 64 actions: one too many
    d.n_actions, d.clip = 4, 0.0
    assert L.tj_ppo_arena_bytes(C.byref(d)) == 0           # no clipping range
    torch.cuda.synchronize()
    assert g.read_stats()[4] == 0                           # nothing ran


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_updates_are_reproducible_bit_for_bit(tj, orc, precision):
    """Fixed reduction orders: two learners from the same state, the same batch, identical results;
    the advantage scan as well."""
    import torch

    D, hidden, A, n_env, steps = 48, (192, 160), 9, 6, 512
    ro = synth.make_rollouts(D, A, n_env, steps, seed=12)
    dev = {k: _dev(v) for k, v in ro.items()}
    outs = []
    for run in range(2):
        g, _ = _pair(tj, orc, D, hidden, A, precision, n_env * steps, seed=21, lr=1e-3)
        adv, ret = tj.gae(dev["reward"], dev["value"], dev["done"], 0.99, 0.95)
        for it in range(3):
            assert g.step(dev["obs"], dev["action"], dev["old_logp"], adv.view(-1), ret.view(-1)) == tj.TJ_OK
        torch.cuda.synchronize()
        outs.append((adv.cpu().numpy(), ret.cpu().numpy(), g.get_state(tj.TJ_STATE_PARAMS),
                     g.get_state(tj.TJ_STATE_ADAM_V), g.read_stats()))
    for a, b in zip(outs[0][:4], outs[1][:4]):
        assert np.array_equal(a, b)
    assert outs[0][4] == outs[1][4] and outs[0][4][4] == 3


@pytest.mark.parametrize("precision", ["fp32", "bf16"])
def test_acting_under_the_policy(tj, orc, precision):
    """Sampled actions equal the oracle's except where the uniform draw sits within float rounding
    of a cumulative probability (there a neighbouring action is the other valid answer);
    log-probabilities and values within tolerance on the rows that agree."""
    import torch

    D, hidden, A, n = 24, (128, 64), 7, 3000
    g, o = _pair(tj, orc, D, hidden, A, precision, 3072, seed=31)
    obs = synth.make_rollouts(D, A, 1, n, seed=6)["obs"]
    for seed in (1, 2**63 + 5):
        action, logp, value = g.act(_dev(obs), seed)
        torch.cuda.synchronize()
        oa, ologp, ovalue, margin = o.ppo_act(obs, seed)
        ga = action.cpu().numpy()
        mism = ga != oa
        tol_u = 1e-5 if precision == "fp32" else 2e-2
        assert (margin[mism] < tol_u).all() and (np.abs(ga[mism] - oa[mism]) <= 1).all()
        assert mism.mean() < (0.001 if precision == "fp32" else 0.05)
        same = ~mism
        assert np.abs(logp.cpu().numpy()[same] - ologp[same]).max() < TOL[precision] * max(1.0, np.abs(ologp).max())
        assert rel_max(value.cpu().numpy(), ovalue) < TOL[precision]
        assert ga.min() >= 0 and ga.max() < A
    # the draws depend on the seed and on nothing else
    a1, _, _ = g.act(_dev(obs), 9)
    a2, _, _ = g.act(_dev(obs), 9)
    a3, _, _ = g.act(_dev(obs), 10)
    assert torch.equal(a1, a2) and not torch.equal(a1, a3)
    # more observations than the learner was sized for
    big = torch.zeros((3073, D), device="cuda")
    out = torch.zeros(3073, dtype=torch.int32, device="cuda")
    f = torch.zeros(3073, device="cuda")
    assert tj.lib().tj_ppo_act(g.h, 3073, big.data_ptr(), 1, out.data_ptr(), f.data_ptr(), None, None) == tj.TJ_ERR_SHAPE
