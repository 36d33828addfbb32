"""GPU: one iteration of the learner loop of Section 3.1 (tj_sample + tj_learner_step) recorded in a
HIP graph replays to exactly what the eager calls give.

A captured launch freezes its host arguments: the seed, the current version and the step count
(with it Adam's bias correction and the target-sync decision).  The eager counterpart of every
replay is therefore the same pair of calls with the step count set back to what it was at capture;
optimizer state and weights carry on from replay to replay on both sides.  Between replays the
program does eager work of its own on the same handles (state reads, an eager sample into another
minibatch) and synchronizes, and every replay is compared, bit for bit: weights, both Adam
moments, the target network, loss and step count, sampled indices."""
import numpy as np
import pytest

from paper_2502_20190_amd import synth

pytestmark = pytest.mark.gpu

STATES = ("TJ_STATE_PARAMS", "TJ_STATE_TARGET", "TJ_STATE_ADAM_M", "TJ_STATE_ADAM_V")


def _reset(tj, lrn, theta, target):
    zero = np.zeros_like(theta)
    lrn.set_state(tj.TJ_STATE_PARAMS, theta)
    lrn.set_state(tj.TJ_STATE_TARGET, target)
    lrn.set_state(tj.TJ_STATE_ADAM_M, zero)
    lrn.set_state(tj.TJ_STATE_ADAM_V, zero)
    lrn.t = 0


@pytest.mark.parametrize("cfg,capacity,batch,indirect", [("c1", 10_000, 32, False), ("c2", 30_000, 512, True),
                                                         ("c3", 40_000, 2048, True), ("c4", 600, 64, False)])
def test_graph_replays_equal_eager_iterations(cfg, capacity, batch, indirect):
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding as tj

    wl = synth.small_variant(synth.WORKLOADS[cfg], capacity, batch)
    rows = synth.make_chunk(wl, 5, 0, wl.capacity)
    theta = synth.xavier_init(wl.layers, wl.in_chw, 1)
    target = synth.xavier_init(wl.layers, wl.in_chw, 2)
    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    buf.insert_host(rows)
    ring = buf if indirect else None
    eager, graphed = (tj.learner_for_workload(wl, theta, target) for _ in range(2))
    mb_e, mb_g, mb_other = (tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=ring) for _ in range(3))
    seed, cur, max_st = 77, wl.current_version, wl.max_staleness
    s = torch.cuda.Stream()

    def iteration(lrn, mb, stream):
        assert buf.sample(mb, cur, max_st, seed, stream=stream) == tj.TJ_OK
        assert lrn.step(mb, stream=stream) == tj.TJ_OK

    # every kernel of the iteration has run once on the capturing stream before the capture starts
    for lrn, mb in ((eager, mb_e), (graphed, mb_g)):
        iteration(lrn, mb, s)
    torch.cuda.synchronize()
    for lrn in (eager, graphed):
        _reset(tj, lrn, theta, target)
    torch.cuda.synchronize()

    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        g.capture_begin()
        iteration(graphed, mb_g, s)
        g.capture_end()
    torch.cuda.synchronize()
    assert graphed.t == 1                     # the host count moved with the recorded call; nothing has run yet
    assert np.array_equal(graphed.get_state(tj.TJ_STATE_PARAMS, stream=s), theta)

    for replay in range(4):
        g.replay()
        torch.cuda.synchronize()
        eager.t = 0
        iteration(eager, mb_e, s)
        torch.cuda.synchronize()
        assert np.array_equal(mb_g.host()["idx"], mb_e.host()["idx"]), f"replay {replay}: indices"
        for name in STATES:
            a, b = (l.get_state(getattr(tj, name), stream=s) for l in (graphed, eager))
            assert np.array_equal(a, b), f"replay {replay}: {name}"
        assert graphed.read_stats() == eager.read_stats() and eager.read_stats()[1] == 1
        # eager work of the program's own between replays, on the handles the graph uses
        assert buf.sample(mb_other, cur, max_st, 1000 + replay, stream=s) == tj.TJ_OK
        torch.cuda.synchronize()
    st, info = buf.status()
    assert st == tj.TJ_OK and info.sticky_error == 0
    assert not np.array_equal(graphed.get_state(tj.TJ_STATE_PARAMS, stream=s), theta)
