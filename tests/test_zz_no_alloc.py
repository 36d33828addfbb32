"""GPU test of tj_sample_noalloc (the sampler with its scratch in the library's own device image):
same indices, rows and status as tj_sample, on two calls in a row that share the scratch, the
second on a smaller ring and batch; rings beyond the limit are refused."""
from dataclasses import replace

import numpy as np
import pytest

from paper_2502_20190_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def _filled(tj, wl, seed):
    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    buf.insert_host(synth.make_chunk(wl, seed, 0, wl.capacity))
    return buf


def _both(tj, buf, wl, batch, seed):
    """(tj_sample, tj_sample_noalloc) results of one draw: minibatch fields, K, status."""
    out = []
    for call in (buf.sample, buf.sample_noalloc):
        mb = tj.Minibatch(batch, wl.obs_elems, wl.obs_dtype)
        assert call(mb, wl.current_version, wl.max_staleness, seed) == tj.TJ_OK
        st, info = buf.status()
        out.append((mb.host(), info.last_n_eligible, st))
    return out


def test_two_calls_in_a_row_equal_tj_sample(tj):
    big = replace(synth.WORKLOADS["c2"], capacity=300_000 + 77, obs_shape=(24,))
    small = replace(synth.WORKLOADS["c1"], capacity=5_000)
    bufs = [(_filled(tj, big, 3), big, 4096 + 5, 11), (_filled(tj, small, 4), small, 96, 12)]
    want = []
    for buf, wl, batch, seed in bufs:      # tj_sample first, for both rings
        mb = tj.Minibatch(batch, wl.obs_elems, wl.obs_dtype)
        assert buf.sample(mb, wl.current_version, wl.max_staleness, seed) == tj.TJ_OK
        st, info = buf.status()
        want.append((mb.host(), info.last_n_eligible, st))
    got = []
    mbs = [tj.Minibatch(batch, wl.obs_elems, wl.obs_dtype) for _, wl, batch, _ in bufs]
    for (buf, wl, batch, seed), mb in zip(bufs, mbs):   # then the two allocation-free calls back to back
        assert buf.sample_noalloc(mb, wl.current_version, wl.max_staleness, seed) == tj.TJ_OK
    for (buf, wl, batch, seed), mb in zip(bufs, mbs):
        st, info = buf.status()
        got.append((mb.host(), info.last_n_eligible, st))
    for (w, wk, wst), (g, gk, gst) in zip(want, got):
        assert wst == gst == tj.TJ_OK and wk == gk and wk > 0
        for f in ("idx", "obs", "next_obs", "action", "reward", "done"):
            assert np.array_equal(w[f], g[f]), f
    # a third call on the small ring with nothing eligible: same reporting as tj_sample
    buf, wl, batch, seed = bufs[1]
    mb = tj.Minibatch(batch, wl.obs_elems, wl.obs_dtype)
    assert buf.sample_noalloc(mb, 10_000, 0, 1) == tj.TJ_OK
    st, info = buf.status()
    assert st == tj.TJ_ERR_NO_ELIGIBLE and info.last_n_eligible == 0
    assert (mb.host()["idx"] == 0xFFFFFFFF).all()


def test_limit_and_arguments(tj):
    import ctypes as C

    L = tj.lib()
    wl = replace(synth.WORKLOADS["c1"], capacity=(1 << 22) + 1, obs_shape=(1,))
    buf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    mb = tj.Minibatch(8, wl.obs_elems, wl.obs_dtype)
    assert buf.sample_noalloc(mb, 99, 10, 0) == tj.TJ_ERR_SCRATCH_LIMIT
    assert b"scratch" in L.tj_strerror(tj.TJ_ERR_SCRATCH_LIMIT)
    ok = tj.Buffer(1 << 22, 1, "f32")                     # the largest ring it accepts
    rows = synth.make_chunk(replace(wl, capacity=1 << 22), 5, 0, 1000)
    ok.insert_host(rows)
    assert ok.sample_noalloc(mb, 99, 10, 0) == tj.TJ_OK
    assert ok.status()[0] == tj.TJ_OK
    assert L.tj_sample_noalloc(None, 8, 0, 0, 0, C.byref(mb.c), None) == tj.TJ_ERR_INVALID_ARG
    assert L.tj_sample_noalloc(ok.h, 9, 0, 0, 0, C.byref(mb.c), None) == tj.TJ_ERR_INVALID_ARG
