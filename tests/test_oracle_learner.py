"""Pins for the oracle's learner step (CPU only): closed forms, Algorithm 1 of
the paper as a special case, finite differences, and library routines (numpy
matmul, torch conv2d / autograd / Adam in fp64) on whole steps."""
import numpy as np
import pytest
import torch

from paper_2502_20190_amd import synth
from paper_2502_20190_amd.synth import CONV, LIN


def _rand_batch(rng, b, in_chw, n_actions, obs_dtype="f32", done_p=0.3):
    d = int(np.prod(in_chw))
    if obs_dtype == "f32":
        obs = rng.standard_normal((b, d)).astype(np.float32)
        nxt = rng.standard_normal((b, d)).astype(np.float32)
    else:
        obs = rng.integers(0, 256, (b, d)).astype(np.uint8)
        nxt = rng.integers(0, 256, (b, d)).astype(np.uint8)
    return dict(obs=obs, next_obs=nxt, action=rng.integers(0, n_actions, b).astype(np.int32),
                reward=rng.uniform(-1, 1, b).astype(np.float32),
                done=(rng.random(b) < done_p).astype(np.uint8))


def _make(orc, layers, in_chw, seed=0, obs_dtype="f32", **kw):
    l = orc.Learner(layers, in_chw, obs_dtype=obs_dtype, **kw)
    theta = synth.xavier_init(layers, in_chw, seed).astype(np.float64)
    target = synth.xavier_init(layers, in_chw, seed + 1).astype(np.float64)
    rng = np.random.default_rng(seed + 100)          # non-zero biases exercise the bias path
    for arr in (theta, target):
        arr += 0.05 * rng.standard_normal(arr.size)
    l.set_state(orc.PARAMS, theta)
    l.set_state(orc.TARGET, target)
    return l, theta, target


def _huber(d, kappa):
    ad = np.abs(d)
    return np.where(ad <= kappa, 0.5 * d * d, kappa * (ad - 0.5 * kappa))


# ---------------------------------------------------------------- TD target

def test_td_target_hand_computed(orc):
    """One linear layer Q = W s + b with hand-picked numbers.  Row 0: online and
    target disagree on the best next action, so the double-DQN target uses the
    target's value at the ONLINE argmax (2.0), not the target's maximum (7.0).
    Row 1: terminal, y = r.  Row 2: tie in the online values, lowest index wins."""
    layers = [(LIN, 3, 0, 0)]
    l = orc.Learner(layers, (3, 1, 1), gamma=0.5, kappa=1.0, lr=0.0)
    W_on = np.eye(3).ravel().tolist() + [0.0, 0.0, 0.0]
    W_tg = np.array([[0, 0, 2.0], [7.0, 0, 0], [0, 1.0, 0]]).ravel().tolist() + [0.0, 0.0, 0.0]
    l.set_state(orc.PARAMS, W_on)
    l.set_state(orc.TARGET, W_tg)
    obs = np.array([[0.25, 0, 0], [0, 0.5, 0], [0, 0, 3.0]], np.float32)
    nxt = np.array([[1.0, 0, 3.0], [9, 9, 9], [4.0, 4.0, 1.0]], np.float32)
    action = np.array([0, 1, 2], np.int32)
    reward = np.array([0.5, -0.25, 1.0], np.float32)
    done = np.array([0, 1, 0], np.uint8)
    loss = l.step(obs, nxt, action, reward, done)
    assert l.last_astar().tolist() == [2, 0, 0]
    # row 0: Q_on(s') = s' = [1, 0, 3] -> a* = 2; Q_tg(s') = [2*3, 7*1, 1*0] = [6, 7, 0], so the
    # target's value at a* is 0: y0 = 0.5 + 0.5*0 = 0.5; delta0 = 0.25 - 0.5 = -0.25
    # row 1: y1 = r = -0.25; delta1 = 0.5 + 0.25 = 0.75
    # row 2: a* = 0; Q_tg(s')[0] = 2*1 = 2; y2 = 1 + 0.5*2 = 2; delta2 = 3 - 2 = 1 (at the kink)
    np.testing.assert_allclose(l.last(orc.LAST_Y), [0.5, -0.25, 2.0], atol=1e-15)
    np.testing.assert_allclose(l.last(orc.LAST_DELTA), [-0.25, 0.75, 1.0], atol=1e-15)
    expect = (0.5 * 0.25 ** 2 + 0.5 * 0.75 ** 2 + 0.5) / 3
    assert loss == pytest.approx(expect, abs=1e-15)
    # and the target's own maximum would have given something else for row 0
    q_tg = l.last(orc.LAST_Q_NEXT_TARGET)
    assert q_tg[0].max() == 7.0 and q_tg[0, 2] == 0.0


def test_algorithm1_special_case(orc):
    """One action, target = online, no terminals, |delta| < 1: the oracle's error
    is minus the paper's TD error delta = r + gamma V(s') - V(s), its loss
    gradient is -(1/B) sum_j delta_j grad V(s_j) (Algorithm 1, policy update), so
    a gradient-descent step on it is the paper's theta += alpha delta grad V."""
    layers = [(LIN, 8, 0, 0), (LIN, 1, 0, 0)]
    in_chw = (4, 1, 1)
    l, theta, _ = _make(orc, layers, in_chw, seed=3, gamma=0.9, lr=0.0)
    l.set_state(orc.TARGET, theta)
    rng = np.random.default_rng(0)
    b = 5
    mb = _rand_batch(rng, b, in_chw, 1, done_p=0.0)
    mb["reward"] *= 0.1
    mb["obs"] *= np.float32(0.3); mb["next_obs"] *= np.float32(0.3)
    v_s = l.forward(0, mb["obs"])[:, 0]
    v_n = l.forward(0, mb["next_obs"])[:, 0]
    delta_paper = mb["reward"] + 0.9 * v_n - v_s
    assert np.abs(delta_paper).max() < 1.0
    # grad V(s_j) by central differences on the forward pass
    h = 1e-6
    gradV = np.zeros((b, theta.size))
    for p in range(theta.size):
        tp = theta.copy(); tp[p] += h; l.set_state(orc.PARAMS, tp)
        up = l.forward(0, mb["obs"])[:, 0]
        tp[p] -= 2 * h; l.set_state(orc.PARAMS, tp)
        dn = l.forward(0, mb["obs"])[:, 0]
        gradV[:, p] = (up - dn) / (2 * h)
    l.set_state(orc.PARAMS, theta)
    l.step(**mb)
    np.testing.assert_allclose(l.last(orc.LAST_DELTA), -delta_paper, atol=1e-14)
    expect = -(delta_paper[:, None] * gradV).sum(0) / b
    np.testing.assert_allclose(l.get_state(orc.GRADS), expect, atol=1e-8)


# ---------------------------------------------------------------- Huber

def test_huber_regions_and_continuity(orc):
    layers = [(LIN, 1, 0, 0)]
    for kappa in (1.0, 0.5):
        l = orc.Learner(layers, (1, 1, 1), gamma=0.0, kappa=kappa, lr=0.0)
        l.set_state(orc.PARAMS, [1.0, 0.0])       # Q(s) = s
        l.set_state(orc.TARGET, [0.0, 0.0])
        s = np.array([[0.3], [-0.2], [5.0], [-7.0], [kappa], [np.nextafter(np.float32(kappa), 9)]],
                     np.float32)
        b = len(s)
        z = np.zeros(b, np.float32)
        loss = l.step(s, s, z.astype(np.int32), z, z.astype(np.uint8))
        d = s[:, 0].astype(np.float64)           # y = 0
        assert loss == pytest.approx(_huber(d, kappa).mean(), rel=1e-15)
        # dL/dw = sum_j clip(d_j) * s_j / B ; dL/db = sum_j clip(d_j) / B
        g = l.get_state(orc.GRADS)
        clip = np.clip(d, -kappa, kappa)
        assert g[0] == pytest.approx((clip * d).sum() / b, rel=1e-14)
        assert g[1] == pytest.approx(clip.sum() / b, rel=1e-14)
    # value continuity at the kink
    assert _huber(np.array([1.0]), 1.0)[0] == 0.5


# ---------------------------------------------------------------- forward vs library routines

def test_linear_layer_is_a_matrix_product(orc):
    rng = np.random.default_rng(5)
    layers = [(LIN, 7, 0, 0)]
    l = orc.Learner(layers, (11, 1, 1))
    W, b = rng.standard_normal((7, 11)), rng.standard_normal(7)
    l.set_state(orc.PARAMS, np.concatenate([W.ravel(), b]))
    x = rng.standard_normal((9, 11)).astype(np.float32)
    np.testing.assert_allclose(l.forward(0, x), x.astype(np.float64) @ W.T + b, rtol=1e-13, atol=1e-13)


def test_mlp_forward_against_numpy(orc):
    layers = [(LIN, 16, 0, 0), (LIN, 8, 0, 0), (LIN, 3, 0, 0)]
    l, theta, target = _make(orc, layers, (6, 1, 1), seed=2)
    x = np.random.default_rng(1).standard_normal((5, 6)).astype(np.float32)
    for which, par in ((0, theta), (1, target)):
        h, off = x.astype(np.float64), 0
        for i, (_, o, _, _) in enumerate(layers):
            fin = h.shape[1]
            W = par[off:off + o * fin].reshape(o, fin); off += o * fin
            b = par[off:off + o]; off += o
            h = h @ W.T + b
            if i < len(layers) - 1:
                h = np.maximum(h, 0)
        np.testing.assert_allclose(l.forward(which, x), h, rtol=1e-12, atol=1e-12)


def test_epsilon_greedy_policy_inference(orc):
    """Algorithm 1, step 1.  Pins: epsilon = 0 is the plain argmax of the forward pass (numpy); the
    decision and the uniform action are literal integer functions of the published generator;
    epsilon = 1 explores always and uniformly (chi-square); the explore rate matches epsilon;
    actions of a shorter batch are a prefix; the online network (not the target) is used."""
    layers = [(LIN, 16, 0, 0), (LIN, 5, 0, 0)]
    l, theta, target = _make(orc, layers, (6, 1, 1), seed=3)
    rng = np.random.default_rng(9)
    x = rng.standard_normal((4000, 6)).astype(np.float32)
    q_on, q_tg = l.forward(0, x), l.forward(1, x)
    a0, q0, g0 = l.act(x, 0.0, 77)
    np.testing.assert_array_equal(a0, q_on.argmax(axis=1))
    np.testing.assert_array_equal(g0, a0)
    np.testing.assert_allclose(q0, q_on, rtol=0, atol=0)
    assert (q_on.argmax(axis=1) != q_tg.argmax(axis=1)).any()        # would notice the wrong network
    for eps in (0.05, 0.5, 1.0):
        a, _, g = l.act(x, eps, 123)
        thr = int(eps * 2 ** 24)
        explore = np.array([(orc.rng64(123, 2 * j) >> 40) < thr for j in range(len(x))])
        uniform = np.array([(orc.rng64(123, 2 * j + 1) * 5) >> 64 for j in range(len(x))])
        np.testing.assert_array_equal(a, np.where(explore, uniform, g))
        np.testing.assert_array_equal(g, g0)
        assert abs(explore.mean() - eps) < 4 * np.sqrt(eps * (1 - eps) / len(x)) + 1e-12
        np.testing.assert_array_equal(l.act(x[:57], eps, 123)[0], a[:57])
    a1 = l.act(x, 1.0, 5)[0]
    counts = np.bincount(a1, minlength=5)
    chi2 = ((counts - len(x) / 5) ** 2 / (len(x) / 5)).sum()
    assert chi2 < 18.47                                               # 4 degrees of freedom, p = 0.001
    # a tie goes to the lowest index
    tie = orc.Learner([(LIN, 3, 0, 0)], (2, 1, 1))
    tie.set_state(orc.PARAMS, np.array([1, 0, 1, 0, 0, 0, 0.5, 0.5, 0.2], np.float64))
    assert tie.act(np.array([[1.0, 3.0]], np.float32), 0.0, 0)[0][0] == 0


def test_conv_1x1_is_a_per_pixel_linear_layer(orc):
    rng = np.random.default_rng(8)
    layers = [(CONV, 5, 1, 1), (LIN, 5 * 3 * 4, 0, 0)]
    l = orc.Learner(layers, (2, 3, 4))
    W, b = rng.standard_normal((5, 2)), rng.standard_normal(5)
    eye = np.eye(60)
    l.set_state(orc.PARAMS, np.concatenate([W.ravel(), b, eye.ravel(), np.zeros(60)]))
    x = rng.standard_normal((3, 2, 3, 4)).astype(np.float32)
    got = l.forward(0, x.reshape(3, -1)).reshape(3, 5, 3, 4)
    want = np.maximum(np.einsum("oc,bchw->bohw", W, x.astype(np.float64)) + b[None, :, None, None], 0)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("k,s", [(3, 1), (4, 2), (8, 4)])
def test_conv_forward_against_torch_conv2d(orc, k, s):
    rng = np.random.default_rng(k)
    c, hgt, wid, oc = 3, 20, 17, 4
    oh, ow = (hgt - k) // s + 1, (wid - k) // s + 1
    n_out = oc * oh * ow
    layers = [(CONV, oc, k, s), (LIN, n_out, 0, 0)]
    l = orc.Learner(layers, (c, hgt, wid), obs_dtype="u8")
    W, b = rng.standard_normal((oc, c, k, k)), rng.standard_normal(oc)
    l.set_state(orc.PARAMS, np.concatenate([W.ravel(), b, np.eye(n_out).ravel(), np.zeros(n_out)]))
    x = rng.integers(0, 256, (2, c, hgt, wid)).astype(np.uint8)
    got = l.forward(0, x.reshape(2, -1)).reshape(2, oc, oh, ow)
    want = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(x).double() / 255.0,
                                                 torch.from_numpy(W), torch.from_numpy(b), stride=s))
    np.testing.assert_allclose(got, want.numpy(), rtol=1e-12, atol=1e-12)


# ---------------------------------------------------------------- backward

def _fd_check(orc, layers, in_chw, obs_dtype, b, seed):
    """Central differences of L(theta) = mean Huber(Q_theta(s_j,a_j) - y_j) with y
    held fixed, the loss rebuilt here from the oracle's forward pass."""
    l, theta, _ = _make(orc, layers, in_chw, seed=seed, obs_dtype=obs_dtype, lr=0.0, gamma=0.9)
    rng = np.random.default_rng(seed)
    mb = _rand_batch(rng, b, in_chw, l.n_actions, obs_dtype)
    mb["reward"] *= np.float32(2.5)                           # reach both Huber branches
    loss = l.step(**mb)
    y, grads = l.last(orc.LAST_Y), l.get_state(orc.GRADS)
    delta = l.last(orc.LAST_DELTA)
    assert np.abs(np.abs(delta) - 1.0).min() > 1e-3          # away from the Huber kink
    assert (np.abs(delta) > 1).any() and (np.abs(delta) < 1).any()

    def frozen_loss(par):
        l.set_state(orc.PARAMS, par)
        q = l.forward(0, mb["obs"])
        return _huber(q[np.arange(b), mb["action"]] - y, 1.0).mean()

    assert frozen_loss(theta) == pytest.approx(loss, rel=1e-13)
    h = 1e-5
    fd = np.zeros_like(theta)
    for p in range(theta.size):
        tp = theta.copy(); tp[p] += h; up = frozen_loss(tp)
        tp[p] -= 2 * h; dn = frozen_loss(tp)
        fd[p] = (up - dn) / (2 * h)
    scale = np.abs(fd).max()
    assert np.abs(grads - fd).max() / scale < 1e-6
    return l, theta, mb, y, grads, frozen_loss


def test_finite_differences_mlp(orc):
    _fd_check(orc, [(LIN, 8, 0, 0), (LIN, 8, 0, 0), (LIN, 2, 0, 0)], (4, 1, 1), "f32", 6, seed=11)


def test_finite_differences_conv(orc):
    _fd_check(orc, [(CONV, 2, 3, 1), (CONV, 3, 4, 2), (LIN, 6, 0, 0), (LIN, 3, 0, 0)], (1, 12, 12),
              "u8", 4, seed=12)


def test_semi_gradient_stops_at_the_target(orc):
    """y is a constant of the step: the analytic gradient equals the finite
    difference with y frozen (checked in _fd_check) and differs from the finite
    difference that re-evaluates y through Q_online(s'); the target network
    changes the loss but receives no gradient."""
    layers = [(LIN, 8, 0, 0), (LIN, 2, 0, 0)]
    in_chw = (4, 1, 1)
    l, theta, mb, y, grads, _ = _fd_check(orc, layers, in_chw, "f32", 6, seed=21)
    target = l.get_state(orc.TARGET)
    mb = dict(mb)
    mb["next_obs"] = mb["obs"] + np.float32(0.01)             # s' close to s: strong coupling
    mb["done"] = np.zeros_like(mb["done"])

    def full_loss(par):
        l.set_state(orc.PARAMS, par); l.set_state(orc.TARGET, par); l.t = 0
        return l.step(**mb)

    full_loss(theta)
    semi = l.get_state(orc.GRADS)
    h = 1e-6
    fd_full = np.zeros_like(theta)
    for p in range(theta.size):
        tp = theta.copy(); tp[p] += h; up = full_loss(tp)
        tp[p] -= 2 * h; dn = full_loss(tp)
        fd_full[p] = (up - dn) / (2 * h)
    assert np.abs(semi - fd_full).max() > 0.05 * np.abs(semi).max()
    # perturbing the target changes the loss; the step produces no target gradient
    l.set_state(orc.PARAMS, theta); l.set_state(orc.TARGET, target)
    l0 = l.step(**mb)
    l.set_state(orc.PARAMS, theta); l.set_state(orc.TARGET, target + 0.1)
    assert l.step(**mb) != l0
    np.testing.assert_array_equal(l.get_state(orc.TARGET), target + 0.1)


# ---------------------------------------------------------------- Adam

def test_adam_closed_forms(orc):
    """Q = w*s + b on one sample with |delta| > kappa, so g = (+-kappa*s, +-kappa) is
    the same at every step while |delta| stays above kappa.  Step 1: the bias
    corrections cancel, update = -lr*g/(|g|+eps).  Constant g: m_hat = g,
    v_hat = g^2 at every t, so every step moves by the same amount."""
    lr, eps = 1e-3, 1e-8
    l = orc.Learner([(LIN, 1, 0, 0)], (1, 1, 1), gamma=0.0, kappa=1.0, lr=lr, eps=eps,
                    target_interval=1000)
    l.set_state(orc.PARAMS, [1.0, 0.5]); l.set_state(orc.TARGET, [0.0, 0.0])
    s = np.array([[4.0]], np.float32)
    one = dict(obs=s, next_obs=s, action=np.zeros(1, np.int32), reward=np.zeros(1, np.float32),
               done=np.zeros(1, np.uint8))
    prev = np.array([1.0, 0.5])
    g = np.array([4.0, 1.0])
    for t in range(1, 6):
        l.step(**one)
        np.testing.assert_allclose(l.get_state(orc.GRADS), g, rtol=1e-15)
        cur = l.get_state(orc.PARAMS)
        np.testing.assert_allclose(cur - prev, -lr * g / (np.abs(g) + eps), rtol=1e-9)
        np.testing.assert_allclose(l.get_state(orc.ADAM_M), (1 - 0.9 ** t) * g, rtol=1e-12)
        np.testing.assert_allclose(l.get_state(orc.ADAM_V), (1 - 0.999 ** t) * g * g, rtol=1e-12)
        prev = cur
    assert l.t == 5
    # zero gradient: parameters stay put (delta = 0 exactly)
    l2 = orc.Learner([(LIN, 1, 0, 0)], (1, 1, 1), gamma=0.0, lr=lr)
    l2.set_state(orc.PARAMS, [1.0, 0.0]); l2.set_state(orc.TARGET, [0.0, 0.0])
    one0 = dict(one); one0["reward"] = np.array([4.0], np.float32)
    l2.step(**one0)
    np.testing.assert_array_equal(l2.get_state(orc.PARAMS), [1.0, 0.0])


def test_target_sync_period(orc):
    layers = [(LIN, 4, 0, 0), (LIN, 2, 0, 0)]
    l, theta, target = _make(orc, layers, (3, 1, 1), seed=4, target_interval=3)
    rng = np.random.default_rng(0)
    for t in range(1, 8):
        l.step(**_rand_batch(rng, 4, (3, 1, 1), 2))
        same = np.array_equal(l.get_state(orc.TARGET), l.get_state(orc.PARAMS))
        assert same == (t % 3 == 0)
        if t < 3:
            np.testing.assert_array_equal(l.get_state(orc.TARGET), target)


# ---------------------------------------------------------------- whole steps against torch (fp64)

def _torch_net(layers, in_chw, flat):
    mods, off = [], 0
    for kind, ws, _, _, _ in synth.layer_shapes(layers, in_chw):
        n = int(np.prod(ws))
        w = torch.tensor(flat[off:off + n].reshape(ws), dtype=torch.float64, requires_grad=True); off += n
        b = torch.tensor(flat[off:off + ws[0]], dtype=torch.float64, requires_grad=True); off += ws[0]
        mods.append((kind, w, b))
    return mods


def _torch_forward(mods, layers, x):
    h = x
    for i, ((kind, w, b), (_, _, k, s)) in enumerate(zip(mods, layers)):
        if kind == CONV:
            h = torch.nn.functional.conv2d(h, w, b, stride=s)
        else:
            h = torch.nn.functional.linear(h.reshape(h.shape[0], -1), w, b)
        if i < len(mods) - 1:
            h = torch.relu(h)
    return h


@pytest.mark.parametrize("case", ["mlp", "conv"])
def test_whole_steps_against_torch_autograd_and_adam(orc, case):
    if case == "mlp":
        layers, in_chw, dt, b = [(LIN, 16, 0, 0), (LIN, 16, 0, 0), (LIN, 3, 0, 0)], (5, 1, 1), "f32", 12
    else:
        layers, in_chw, dt, b = [(CONV, 4, 4, 2), (CONV, 6, 3, 1), (LIN, 10, 0, 0), (LIN, 4, 0, 0)], \
            (2, 14, 14), "u8", 6
    gamma, kappa, lr, interval = 0.97, 0.8, 3e-3, 3
    l, theta, target = _make(orc, layers, in_chw, seed=31, obs_dtype=dt, gamma=gamma, kappa=kappa,
                             lr=lr, target_interval=interval)
    on, tg = _torch_net(layers, in_chw, theta), _torch_net(layers, in_chw, target)
    params = [t for _, w, bb in on for t in (w, bb)]
    opt = torch.optim.Adam(params, lr=lr, betas=(0.9, 0.999), eps=1e-8)
    rng = np.random.default_rng(77)
    for t in range(1, 8):
        mb = _rand_batch(rng, b, in_chw, l.n_actions, dt)
        loss = l.step(**mb)

        def prep(a):
            x = torch.from_numpy(a.astype(np.float64)).reshape(b, *in_chw)
            return x / 255.0 if dt == "u8" else x

        s, sn = prep(mb["obs"]), prep(mb["next_obs"])
        with torch.no_grad():
            a_star = _torch_forward(on, layers, sn).argmax(1)
            q_t = _torch_forward(tg, layers, sn).gather(1, a_star[:, None])[:, 0]
            y = torch.from_numpy(mb["reward"].astype(np.float64)) + \
                gamma * (1 - torch.from_numpy(mb["done"].astype(np.float64))) * q_t
        q = _torch_forward(on, layers, s).gather(1, torch.from_numpy(mb["action"]).long()[:, None])[:, 0]
        tl = torch.nn.functional.huber_loss(q, y, delta=kappa)
        opt.zero_grad(); tl.backward()
        flat_g = torch.cat([p.grad.reshape(-1) for p in params]).numpy()
        opt.step()
        if t % interval == 0:
            with torch.no_grad():
                for (_, w, bb), (_, wt, bt) in zip(on, tg):
                    wt.copy_(w); bt.copy_(bb)
        assert loss == pytest.approx(tl.item(), rel=1e-12)
        np.testing.assert_array_equal(l.last_astar(), a_star.numpy())
        g = l.get_state(orc.GRADS)
        np.testing.assert_allclose(g, flat_g, rtol=1e-9, atol=1e-13 * np.abs(flat_g).max())
        flat_p = torch.cat([p.detach().reshape(-1) for p in params]).numpy()
        np.testing.assert_allclose(l.get_state(orc.PARAMS), flat_p, rtol=1e-9, atol=1e-12)
        flat_t = torch.cat([p.detach().reshape(-1) for _, w, bb in tg for p in (w, bb)]).numpy()
        np.testing.assert_allclose(l.get_state(orc.TARGET), flat_t, rtol=1e-9, atol=1e-12)


# ---------------------------------------------------------------- bf16 rounding mode

def test_bf16_rounding_helper_and_mode_within_bound(orc):
    """The rounding mode equals the exact mode up to the bf16 rounding of GEMM
    operands: a value representable in bf16 passes through a one-layer net
    unchanged, and on a small MLP loss / gradients stay within 2e-2 of the exact
    mode (greedy actions taken from the exact mode, so an argmax near-tie cannot
    turn rounding noise into a jump)."""
    lin = [(LIN, 1, 0, 0)]
    l = orc.Learner(lin, (1, 1, 1), emulate_bf16=True)
    l.set_state(orc.PARAMS, [1.0, 0.0])
    xs = np.array([[1.0], [1.00390625], [1.005859375], [1.01171875], [3.0e38], [-0.3]], np.float32)
    got = l.forward(0, xs)[:, 0]
    want = torch.from_numpy(xs[:, 0]).to(torch.bfloat16).double().numpy()   # library RNE rounding
    np.testing.assert_array_equal(got, want)

    layers = [(LIN, 64, 0, 0), (LIN, 64, 0, 0), (LIN, 4, 0, 0)]
    in_chw = (16, 1, 1)
    exact, theta, target = _make(orc, layers, in_chw, seed=5, lr=1e-3)
    rnd = orc.Learner(layers, in_chw, lr=1e-3, emulate_bf16=True)
    rnd.set_state(orc.PARAMS, theta); rnd.set_state(orc.TARGET, target)
    mb = _rand_batch(np.random.default_rng(9), 512, in_chw, 4)
    le = exact.step(**mb)
    lr_ = rnd.step(**mb, astar_override=exact.last_astar())
    assert abs(le - lr_) / abs(le) < 2e-2
    # a hidden unit whose pre-activation changes sign under rounding flips one row's
    # ReLU mask, a jump of size 1/B in single entries: compare in the L2 norm
    ge, gr = exact.get_state(orc.GRADS), rnd.get_state(orc.GRADS)
    assert np.linalg.norm(ge - gr) / np.linalg.norm(ge) < 2e-2
    assert np.abs(ge - gr).max() > 0
    qe, qr = exact.last(orc.LAST_Q_S), rnd.last(orc.LAST_Q_S)
    assert np.abs(qe - qr).max() / np.abs(qe).max() < 2e-2
