"""GPU: the learner's load folded into its update (Section 3.1, learner loop: load trajectories,
then learn).  tj_sample can leave the observations where they are (indices and scalar fields only)
and tj_learner_step can read them out of the ring through those indices.  What is checked:

 - the indices and scalar fields of such a sample equal the oracle's, bit for bit;
 - a learner fed that way ends, bit for bit, where a learner fed dense copies of the same rows ends
   (same kernels, same values: only the address of each row differs), for every input path of the
   learners: fp32 and bf16 MLP, the u8 first-layer kernels of the pixel networks, and the plain
   image-layout kernels (fp32 pixels, u8 pixels of a network outside the fused kernel's shapes);
 - the first step of one such learner against the oracle itself (sample + update from the ring rows);
 - an empty eligible set leaves a readable state behind (indices are clamped, the status says so);
 - a concurrent insert issued after tj_buffer_reads_done does not disturb the update before it."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2502_20190_amd import synth
from paper_2502_20190_amd.synth import CONV, LIN
from parity_util import rel_max, rel_scalar

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def _mlp(*outs):
    return tuple((LIN, o, 0, 0) for o in outs)


_CASES = {
    "mlp-fp32": dict(base="c2", capacity=20_000, batch=200, layers=_mlp(64, 64, 18)),
    # rows of 7 floats: no 16-byte vector fits a row
    "mlp-fp32-odd": dict(base="c1", capacity=3_000, batch=50, obs_shape=(7,), layers=_mlp(16, 16, 2)),
    "mlp-bf16": dict(base="c3", capacity=30_000, batch=1024, layers=_mlp(256, 256, 32)),
    "mlp-bf16-ragged": dict(base="c3", capacity=9_000, batch=333, layers=_mlp(128, 64, 32)),
    # 84 x 84 u8 stacks, the first-layer kernels that read the frames themselves (forward and weight gradient)
    "pixel-bf16-fused": dict(base="c4", capacity=600, batch=96,
                             layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6),
    # u8 pixels through the channels-last layout kernel (16 output channels: outside the fused kernel)
    "pixel-bf16-plain": dict(base="c4", capacity=500, batch=40, obs_shape=(4, 20, 20),
                             layers=((CONV, 16, 4, 2), (CONV, 16, 3, 1), (LIN, 24, 0, 0), (LIN, 6, 0, 0)), n_actions=6),
    "pixel-fp32-u8": dict(base="c4", capacity=500, batch=40, obs_shape=(3, 18, 18), precision="fp32",
                          layers=((CONV, 8, 4, 2), (CONV, 16, 3, 1), (LIN, 32, 0, 0), (LIN, 5, 0, 0)), n_actions=5),
    "pixel-fp32-f32": dict(base="c4", capacity=500, batch=40, obs_shape=(3, 18, 18), precision="fp32", obs_dtype="f32",
                           layers=((CONV, 8, 4, 2), (CONV, 16, 3, 1), (LIN, 32, 0, 0), (LIN, 5, 0, 0)), n_actions=5),
}


def _workload(case):
    c = dict(_CASES[case])
    wl = synth.small_variant(synth.WORKLOADS[c.pop("base")], c.pop("capacity"), c.pop("batch"))
    return replace(wl, **c)


def _run(tj, wl, rows, theta, target, steps, indirect):
    import torch

    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    buf.insert_host(rows)
    lrn = tj.learner_for_workload(wl, theta, target)
    mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=buf if indirect else None)
    losses, idx = [], []
    for i in range(steps):
        assert buf.sample(mb, wl.current_version, wl.max_staleness, 500 + i) == tj.TJ_OK
        assert lrn.step(mb) == tj.TJ_OK
        losses.append(lrn.read_stats()[0])
        idx.append(mb.host())
    torch.cuda.synchronize()
    st, info = buf.status()
    assert st == tj.TJ_OK and info.sticky_error == 0
    return [lrn.get_state(w) for w in (tj.TJ_STATE_PARAMS, tj.TJ_STATE_ADAM_M, tj.TJ_STATE_ADAM_V)], losses, idx


@pytest.mark.parametrize("case", sorted(_CASES))
def test_update_from_ring_rows_equals_update_from_copies(tj, orc, case):
    wl = _workload(case)
    rows = synth.make_chunk(wl, 11, 0, wl.capacity)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    target = synth.xavier_init(wl.layers, wl.in_chw, 4)
    steps = 3
    dense = _run(tj, wl, rows, theta, target, steps, indirect=False)
    ring = _run(tj, wl, rows, theta, target, steps, indirect=True)
    for a, b in zip(dense[0], ring[0]):
        assert np.array_equal(a, b)
    assert dense[1] == ring[1]
    assert not np.array_equal(dense[0][0], theta)
    for i in range(steps):
        st, oidx, _ = orc.sample(rows["version"], wl.capacity, wl.current_version, wl.max_staleness, 500 + i, wl.batch)
        assert st == 0
        got = ring[2][i]
        assert "obs" not in got
        assert np.array_equal(got["idx"], oidx)
        for f in ("action", "reward", "done"):
            assert np.array_equal(got[f], rows[f][oidx])
            assert np.array_equal(got[f], dense[2][i][f])


@pytest.mark.parametrize("case", ["mlp-fp32", "pixel-bf16-fused"])
def test_first_update_from_ring_rows_against_the_oracle(tj, orc, case):
    wl = _workload(case)
    rows = synth.make_chunk(wl, 12, 0, wl.capacity)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 5)
    target = synth.xavier_init(wl.layers, wl.in_chw, 6)
    got, losses, _ = _run(tj, wl, rows, theta, target, 1, indirect=True)
    st, oidx, _ = orc.sample(rows["version"], wl.capacity, wl.current_version, wl.max_staleness, 500, wl.batch)
    assert st == 0
    bf16 = wl.precision == "bf16"
    o = orc.Learner(wl.layers, wl.in_chw, obs_dtype=wl.obs_dtype, gamma=wl.gamma, kappa=wl.kappa, lr=wl.lr,
                    beta1=wl.beta1, beta2=wl.beta2, eps=wl.eps, target_interval=wl.target_interval,
                    emulate_bf16=bf16)
    o.set_state(orc.PARAMS, theta.astype(np.float64))
    o.set_state(orc.TARGET, target.astype(np.float64))
    loss = o.step(**{f: rows[f][oidx] for f in ("obs", "next_obs", "action", "reward", "done")})
    tol = 2e-2 if bf16 else 1e-4
    assert rel_scalar(losses[0], loss) < tol
    # m = (1 - beta1) g after the first step: the gradient itself
    assert rel_max(got[1], o.get_state(orc.ADAM_M)) < tol
    assert rel_max(got[2], o.get_state(orc.ADAM_V)) < 2 * tol


def test_empty_eligible_set_with_ring_rows_reads_in_bounds(tj):
    """K = 0: the indices are all ones; the update clamps them to the table's last row, runs to the
    end, and the buffer reports that nothing was eligible."""
    import torch

    wl = _workload("mlp-fp32")
    rows = synth.make_chunk(wl, 13, 0, wl.capacity)
    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    buf.insert_host(rows)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    lrn = tj.learner_for_workload(wl, theta, theta)
    mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=buf)
    mb.action.zero_(); mb.reward.zero_(); mb.done.zero_()
    assert buf.sample(mb, wl.current_version + 10_000, 0, 1) == tj.TJ_OK     # nothing that fresh exists
    assert lrn.step(mb) == tj.TJ_OK
    torch.cuda.synchronize()
    st, info = buf.status()
    assert st == tj.TJ_ERR_NO_ELIGIBLE and info.last_n_eligible == 0
    assert np.all(mb.host()["idx"] == 0xFFFFFFFF)
    assert np.all(np.isfinite(lrn.get_state(tj.TJ_STATE_PARAMS)))


def test_indirect_minibatch_needs_a_table_size(tj):
    wl = _workload("mlp-fp32")
    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    lrn = tj.learner_for_workload(wl, theta, theta)
    mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=buf)
    mb.c_step.n_rows = 0
    assert lrn.step(mb) == tj.TJ_ERR_INVALID_ARG
    half = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype)
    half.c.next_obs = None                                   # one destination without the other
    assert buf.sample(half, wl.current_version, wl.max_staleness, 1) == tj.TJ_ERR_INVALID_ARG


def test_insert_after_reads_done_waits_for_the_update(tj):
    """A full ring, every slot eligible; right after the update has been enqueued, a concurrent
    insert replaces every row.  With tj_buffer_reads_done between the two, the update must have
    seen the old rows: its result equals that of the same update with no insert at all."""
    import torch

    wl = replace(_workload("mlp-bf16"), capacity=4096, max_staleness=10_000)
    rows = synth.make_chunk(wl, 21, 0, wl.capacity)
    fresh = synth.make_chunk(wl, 22, 0, wl.capacity)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    target = synth.xavier_init(wl.layers, wl.in_chw, 4)
    ref, _, _ = _run(tj, wl, rows, theta, target, 1, indirect=True)

    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    buf.insert_host(rows)
    lrn = tj.learner_for_workload(wl, theta, target)
    mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=buf)
    dev = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in fresh.items()}
    s_ins = torch.cuda.Stream()
    torch.cuda.synchronize()
    assert buf.sample(mb, wl.current_version, wl.max_staleness, 500) == tj.TJ_OK
    assert lrn.step(mb) == tj.TJ_OK
    buf.reads_done()
    buf.insert_concurrent(dev["obs"], dev["next_obs"], dev["action"], dev["reward"], dev["done"], dev["version"],
                          s_ins)
    torch.cuda.synchronize()
    assert np.array_equal(lrn.get_state(tj.TJ_STATE_PARAMS), ref[0])
    assert torch.equal(buf.field("obs"), dev["obs"])         # and the insert did run


# ---------------------------------------------------------------- frame ring: indirect by planes

def _frame_stream(rng, n, frame_elems, done_p, t0=0):
    frames = rng.integers(0, 256, (n, frame_elems)).astype(np.uint8)
    done = (rng.random(n) < done_p).astype(np.uint8)
    return (frames, rng.integers(0, 18, n).astype(np.int32), rng.uniform(-1, 1, n).astype(np.float32), done,
            ((t0 + np.arange(n)) // 50).astype(np.int32))


def _fill_frame_rings(tj, orc, rng, frame_elems, cap, total, k):
    """The same ragged, wrapping inserts into the library's ring, the oracle's ring and a plain
    host mirror of the frame slots."""
    g = tj.FrameBuffer(cap, frame_elems, k)
    o = orc.FrameBuffer(cap, frame_elems, k) if orc is not None else None
    mirror = np.zeros((cap, frame_elems), np.uint8)
    pos = 0
    while pos < total:
        n = int(min(total - pos, rng.integers(1, min(900, cap) + 1)))
        rows = _frame_stream(rng, n, frame_elems, 0.02, pos)
        assert g.insert_host(*rows) == tj.TJ_OK
        if o is not None:
            assert o.insert(*rows) == 0
        mirror[(pos + np.arange(n)) % cap] = rows[0]
        pos += n
    return g, o, mirror


@pytest.mark.parametrize("frame_elems,cap,total,k", [(7056, 1500, 5300, 4), (100, 4096, 9000, 4), (37, 700, 2500, 3)])
def test_frame_plane_slots_against_the_oracle(tj, orc, frame_elems, cap, total, k):
    """A frame sample without stack destinations: the frames its plane slots name, read from a host
    mirror of the ring, are the oracle's rebuilt stacks (so every slot, with its look-back clamped
    at episode starts and wrapped around the ring, is the right one)."""
    rng = np.random.default_rng(frame_elems + cap + 1)
    g, o, mirror = _fill_frame_rings(tj, orc, rng, frame_elems, cap, total, k)
    cur = (total - 1) // 50
    for seed, max_st, batch in ((1, 3, 64), (2, 0, 17), (3, 1000, 256)):
        mb = tj.Minibatch(batch, frame_elems * k, "u8", ring=g)
        assert g.sample(mb, cur, max_st, seed) == tj.TJ_OK
        st, info = g.status()
        ost, oidx, oK = o.sample(batch, cur, max_st, seed)
        assert st == ost == 0 and info.last_n_eligible == oK
        got = mb.host()
        np.testing.assert_array_equal(got["idx"], oidx)
        want = o.gather(oidx)
        for f in ("action", "reward", "done"):
            np.testing.assert_array_equal(got[f], want[f], err_msg=f)
        planes = got["planes"]
        assert planes.shape == (batch, 2 * k) and planes.max() < cap
        np.testing.assert_array_equal(mirror[planes[:, :k]].reshape(batch, -1), want["obs"])
        np.testing.assert_array_equal(mirror[planes[:, k:]].reshape(batch, -1), want["next_obs"])


_FRAME_CASES = {
    # the u8 first-layer kernels (forward and weight gradient) reading single frames
    "fused-84": dict(hw=(84, 84), k=4, cap=700, total=1900, batch=96, precision="bf16",
                     layers=((CONV, 32, 8, 4), (CONV, 64, 4, 2), (LIN, 24, 0, 0), (LIN, 18, 0, 0))),
    # the channels-last layout kernels: four u8 planes at a time, and the general one (three planes, fp32 net)
    "plain-u8c4": dict(hw=(20, 20), k=4, cap=600, total=1500, batch=40, precision="bf16",
                       layers=((CONV, 16, 4, 2), (CONV, 16, 3, 1), (LIN, 24, 0, 0), (LIN, 18, 0, 0))),
    "plain-fp32": dict(hw=(18, 18), k=3, cap=600, total=1500, batch=40, precision="fp32",
                       layers=((CONV, 8, 4, 2), (CONV, 16, 3, 1), (LIN, 32, 0, 0), (LIN, 18, 0, 0))),
}


@pytest.mark.parametrize("case", sorted(_FRAME_CASES))
def test_update_from_frame_planes_equals_update_from_stacks(tj, case):
    import torch

    c = _FRAME_CASES[case]
    (H, W), k = c["hw"], c["k"]
    wl = replace(synth.small_variant(synth.WORKLOADS["c4"], c["cap"], c["batch"]), obs_shape=(k, H, W),
                 layers=c["layers"], precision=c["precision"], n_actions=18)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    target = synth.xavier_init(wl.layers, wl.in_chw, 4)
    cur = (c["total"] - 1) // 50
    out = []
    for indirect in (False, True):
        g, _, _ = _fill_frame_rings(tj, None, np.random.default_rng(5), H * W, c["cap"], c["total"], k)
        lrn = tj.learner_for_workload(wl, theta, target)
        mb = tj.Minibatch(wl.batch, wl.obs_elems, "u8", ring=g if indirect else None)
        losses = []
        for i in range(3):
            assert g.sample(mb, cur, 5, 900 + i) == tj.TJ_OK
            assert lrn.step(mb) == tj.TJ_OK
            losses.append(lrn.read_stats()[0])
        torch.cuda.synchronize()
        assert g.status()[0] == tj.TJ_OK
        out.append(([lrn.get_state(w) for w in (tj.TJ_STATE_PARAMS, tj.TJ_STATE_ADAM_M, tj.TJ_STATE_ADAM_V)], losses))
    for a, b in zip(out[0][0], out[1][0]):
        assert np.array_equal(a, b)
    assert out[0][1] == out[1][1]
    assert not np.array_equal(out[0][0][0], theta)


def test_frame_planes_argument_checks(tj):
    g, _, _ = _fill_frame_rings(tj, None, np.random.default_rng(6), 64, 64, 40, 4)
    mb = tj.Minibatch(8, 256, "u8", ring=g)
    mb.c.plane_index = None                                  # no stacks and nowhere to put the slots
    assert g.sample(mb, 0, 10, 1) == tj.TJ_ERR_INVALID_ARG
    wl = _workload("mlp-fp32")                               # planes are image channels: not for an MLP
    theta = synth.xavier_init(wl.layers, wl.in_chw, 3)
    lrn = tj.learner_for_workload(wl, theta, theta)
    m2 = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype))
    m2.c_step.plane_index = m2.idx.data_ptr()
    assert lrn.step(m2) == tj.TJ_ERR_INVALID_ARG
