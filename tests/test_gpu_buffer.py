"""GPU parity: ring insert, staleness-gated sampling and gather against the CPU
oracle, through the C ABI.  Indices and gathered rows must be bit-exact."""
import ctypes

import numpy as np
import pytest

from paper_2502_20190_amd import synth

pytestmark = pytest.mark.gpu
FIELDS = ("obs", "next_obs", "action", "reward", "done")


@pytest.fixture(scope="module")
def tj():
    import torch

    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2502_20190_amd import binding

    binding.lib()
    return binding


def _sync():
    import torch

    torch.cuda.synchronize()


def _fill_both(tj, orc, wl, seed, chunk_rows, total_rows):
    gbuf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    obuf = orc.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    done_rows, c = 0, 0
    while done_rows < total_rows:
        n = min(chunk_rows, total_rows - done_rows)
        rows = synth.make_chunk(wl, seed, c, n)
        gbuf.insert_host(rows)
        assert obuf.insert(**rows) == 0
        done_rows += n
        c += 1
    return gbuf, obuf


def _compare_sample(tj, gbuf, obuf, batch, cur, max_st, seed):
    mb = tj.Minibatch(batch, gbuf.obs_elems, gbuf.obs_dtype)
    assert gbuf.sample(mb, cur, max_st, seed) == tj.TJ_OK
    st, info = gbuf.status()
    ost, oidx, oK = obuf.sample(batch, cur, max_st, seed)
    assert info.last_n_eligible == oK and st == ost
    got = mb.host()
    np.testing.assert_array_equal(got["idx"], oidx)
    if ost == 0:
        want = obuf.gather(oidx)
        for f in FIELDS:
            np.testing.assert_array_equal(got[f], want[f], err_msg=f)
        ver = obuf.versions()[oidx].astype(np.int64)
        assert ((cur - ver >= 0) & (cur - ver <= max_st)).all() and (oidx < obuf.count).all()
    return got, oK


def test_c1_tiny_whole_ring_and_samples(tj, orc):
    wl = synth.WORKLOADS["c1"]
    gbuf, obuf = _fill_both(tj, orc, wl, synth.MASTER_SEED, 3000, wl.capacity)
    _, info = gbuf.status()
    assert (info.count, info.head) == (obuf.count, obuf.head) == (wl.capacity, 0)
    for seed in range(5):
        _, K = _compare_sample(tj, gbuf, obuf, wl.batch, wl.current_version, wl.max_staleness, seed)
        assert 900 < K < 1300
    # determinism and the prefix property
    a, _ = _compare_sample(tj, gbuf, obuf, 64, 99, 10, 7)
    b, _ = _compare_sample(tj, gbuf, obuf, 64, 99, 10, 7)
    c, _ = _compare_sample(tj, gbuf, obuf, 9, 99, 10, 7)
    np.testing.assert_array_equal(a["idx"], b["idx"])
    np.testing.assert_array_equal(a["idx"][:9], c["idx"])


def test_wraparound_inserts_match_ring_contents(tj, orc):
    wl = synth.small_variant(synth.WORKLOADS["c2"], capacity=5000, batch=64)
    gbuf, obuf = _fill_both(tj, orc, wl, 11, 1777, 5000 * 2 + 1234)     # wraps twice, ragged chunks
    _, info = gbuf.status()
    assert (info.count, info.head) == (obuf.count, obuf.head)
    everything = obuf.gather(np.arange(wl.capacity, dtype=np.uint32))
    for f in FIELDS:
        np.testing.assert_array_equal(gbuf.field(f).cpu().numpy(), everything[f], err_msg=f)
    np.testing.assert_array_equal(gbuf.field("version").cpu().numpy(), obuf.versions())
    for seed in (1, 2):
        _compare_sample(tj, gbuf, obuf, 64, 999, 32, seed)


@pytest.mark.parametrize("obs_elems,obs_dtype,capacity", [
    (3, "f32", 700),        # 12-byte rows: 4-byte lanes
    (7, "u8", 1500),        # 7-byte rows: byte lanes
    (256, "f32", 4100),     # 1 KiB rows: one wave per row
    (1100, "f32", 300),     # 4.4 KiB rows: wide path, 2 vectors per thread
    (4 * 84 * 84, "u8", 70),  # pixel rows: wide path, 8 vectors per thread
    (2400, "f32", 130),     # 9.6 KiB rows: wide path, 4 vectors per thread
])
def test_row_shapes(tj, orc, obs_elems, obs_dtype, capacity):
    from dataclasses import replace

    wl = replace(synth.WORKLOADS["c2"], capacity=capacity, obs_shape=(obs_elems,), obs_dtype=obs_dtype,
                 version_max=20, current_version=20)
    gbuf, obuf = _fill_both(tj, orc, wl, 5, min(97, capacity), capacity + 50)
    everything = obuf.gather(np.arange(capacity, dtype=np.uint32))
    for f in FIELDS:
        np.testing.assert_array_equal(gbuf.field(f).cpu().numpy(), everything[f], err_msg=f)
    for batch, max_st in ((1, 20), (33, 3), (300, 0)):
        _compare_sample(tj, gbuf, obuf, batch, 20, max_st, batch)


def test_edge_cases(tj, orc):
    import torch

    wl = synth.small_variant(synth.WORKLOADS["c1"], capacity=3000)
    gbuf, obuf = _fill_both(tj, orc, wl, 3, 1000, 2500)          # partially filled: count < N
    _, info = gbuf.status()
    assert info.count == 2500 and info.head == 2500
    _compare_sample(tj, gbuf, obuf, 32, 99, 10, 1)
    _compare_sample(tj, gbuf, obuf, 32, 99, 0, 2)                # only the current version
    _compare_sample(tj, gbuf, obuf, 32, 99, 1000, 3)             # every valid slot
    _compare_sample(tj, gbuf, obuf, 32, 50, 5, 4)                # tags ahead of cur are ineligible
    # nothing eligible: sticky status, idx = 0xFFFFFFFF, minibatch left alone
    mb = tj.Minibatch(16, wl.obs_elems, wl.obs_dtype)
    mb.obs.fill_(7.0)
    assert gbuf.sample(mb, 5000, 3, 1) == tj.TJ_OK
    st, info = gbuf.status()
    assert st == tj.TJ_ERR_NO_ELIGIBLE and info.last_n_eligible == 0
    assert (mb.host()["idx"] == 0xFFFFFFFF).all() and (mb.obs == 7.0).all().item()
    st, info = gbuf.status()
    assert st == tj.TJ_OK                                        # cleared once reported
    # empty ring
    empty = tj.Buffer(100, 4, "f32")
    mb4 = tj.Minibatch(4, 4, "f32")
    assert empty.sample(mb4, 0, 100, 1) == tj.TJ_OK
    st, info = empty.status()
    assert st == tj.TJ_ERR_NO_ELIGIBLE and info.count == 0
    # argument errors are synchronous and change nothing
    L = tj.lib()
    n = 101
    z = torch.zeros((n, 4), device="cuda:0")
    zi = torch.zeros(n, dtype=torch.int32, device="cuda:0")
    zb = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    rc = L.tj_buffer_insert(empty.h, n, z.data_ptr(), z.data_ptr(), zi.data_ptr(), z.data_ptr(),
                            zb.data_ptr(), zi.data_ptr(), None)
    assert rc == tj.TJ_ERR_CAPACITY
    assert L.tj_buffer_insert(empty.h, 0, None, None, None, None, None, None, None) == tj.TJ_OK
    assert L.tj_buffer_insert(empty.h, 1, None, None, None, None, None, None, None) == tj.TJ_ERR_INVALID_ARG
    st, info = empty.status()
    assert info.count == 0 and info.head == 0
    assert L.tj_sample(empty.h, 8, 0, 0, 0, ctypes.byref(mb4.c), None) == tj.TJ_ERR_INVALID_ARG  # batch mismatch
    _sync()


def test_k_equals_one_and_extreme_tags(tj, orc):
    import torch

    cap = 2100
    gbuf = tj.Buffer(cap, 4, "f32")
    obuf = orc.Buffer(cap, 4, "f32")
    rng = np.random.default_rng(1)
    ver = np.full(cap, 3, np.int32)
    ver[1777] = 9
    ver[0], ver[1] = -2**31, 2**31 - 1
    rows = dict(obs=rng.standard_normal((cap, 4)).astype(np.float32),
                next_obs=rng.standard_normal((cap, 4)).astype(np.float32),
                action=np.arange(cap, dtype=np.int32), reward=np.zeros(cap, np.float32),
                done=np.zeros(cap, np.uint8), version=ver)
    gbuf.insert_host(rows)
    obuf.insert(**rows)
    got, K = _compare_sample(tj, gbuf, obuf, 50, 9, 0, 1)
    assert K == 1 and (got["idx"] == 1777).all()
    _compare_sample(tj, gbuf, obuf, 50, 2**31 - 1, 2**40, 2)
    _compare_sample(tj, gbuf, obuf, 50, 0, 2**31, 3)
    _compare_sample(tj, gbuf, obuf, 50, -2**31, 0, 4)


def test_c2_full_size_ring(tj, orc):
    """Config 2 at its real size (10^6 x 128 fp32) in the launch shape the benchmark uses."""
    wl = synth.WORKLOADS["c2"]
    gbuf, obuf = _fill_both(tj, orc, wl, synth.MASTER_SEED, 250_000, wl.capacity)
    for seed in (1, 2, 3):
        _, K = _compare_sample(tj, gbuf, obuf, wl.batch, wl.current_version, wl.max_staleness, seed)
        assert abs(K - 33_000) < 1500
    probe = np.random.default_rng(0).integers(0, wl.capacity, 4096).astype(np.uint32)
    want = obuf.gather(probe)
    import torch

    pi = torch.from_numpy(probe.astype(np.int64)).cuda()
    for f in FIELDS:
        np.testing.assert_array_equal(gbuf.field(f)[pi].cpu().numpy(), want[f], err_msg=f)


@pytest.mark.parametrize("name", ["c3", "c5"])
def test_full_size_device_filled_ring(tj, orc, name):
    """Configs 3 and 5 at full size: the ring is filled on the device from the
    seeded device generator (8 / 113 GB do not pass through host memory).  The
    oracle gets the version tags, computes its own indices; the rows at those
    indices are regenerated chunk by chunk (never read through the gather) and
    must equal the gathered minibatch bit for bit."""
    import torch

    wl = synth.WORKLOADS[name]
    chunk_rows = 65_536 if name == "c3" else 16_384
    gbuf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    versions = np.empty(wl.capacity, np.int32)
    n_chunks = (wl.capacity + chunk_rows - 1) // chunk_rows
    for c in range(n_chunks):
        n = min(chunk_rows, wl.capacity - c * chunk_rows)
        rows = synth.make_chunk_device(wl, synth.MASTER_SEED, c, n)
        gbuf.insert(rows["obs"], rows["next_obs"], rows["action"], rows["reward"], rows["done"],
                    rows["version"])
        versions[c * chunk_rows:c * chunk_rows + n] = rows["version"].cpu().numpy()
    _sync()
    sweeps = wl.staleness_sweep or (wl.max_staleness,)
    for max_st in sweeps:
        mb = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype)
        assert gbuf.sample(mb, wl.current_version, max_st, 77 + max_st) == tj.TJ_OK
        st, info = gbuf.status()
        ost, oidx, oK = orc.sample(versions, wl.capacity, wl.current_version, max_st, 77 + max_st, wl.batch)
        assert st == ost == 0 and info.last_n_eligible == oK
        got = mb.host()
        np.testing.assert_array_equal(got["idx"], oidx)
        stale = wl.current_version - versions[oidx]
        assert ((stale >= 0) & (stale <= max_st)).all()
        # expected rows: regenerate the chunks that hold the first 64 sampled slots
        for j in range(64):
            c, r = divmod(int(oidx[j]), chunk_rows)
            n = min(chunk_rows, wl.capacity - c * chunk_rows)
            rows = synth.make_chunk_device(wl, synth.MASTER_SEED, c, n)
            for f in FIELDS:
                np.testing.assert_array_equal(got[f][j], rows[f][r].cpu().numpy(), err_msg=f"{f} row {j}")
        # all rows: the gathered minibatch equals the ring rows read back with plain indexing
        pi = torch.from_numpy(oidx.astype(np.int64)).cuda()
        for f in FIELDS:
            assert torch.equal(getattr(mb, f), gbuf.field(f)[pi]), f
    # The update at this size and in the launch configuration bench.py times: a learner that reads the
    # sampled rows out of the full ring through the indices (byte offsets far beyond 4 GiB) ends bit for
    # bit where a learner fed the dense minibatch checked above ends.
    theta = synth.xavier_init(wl.layers, wl.in_chw, 1)
    target = synth.xavier_init(wl.layers, wl.in_chw, 2)
    seed = 77 + sweeps[-1]
    mbi = tj.Minibatch(wl.batch, wl.obs_elems, wl.obs_dtype, ring=gbuf)
    assert gbuf.sample(mbi, wl.current_version, sweeps[-1], seed) == tj.TJ_OK
    assert torch.equal(mbi.idx, mb.idx)
    states = []
    for m in (mb, mbi):
        lrn = tj.learner_for_workload(wl, theta, target)
        assert lrn.step(m) == tj.TJ_OK
        _sync()
        states.append((lrn.get_state(tj.TJ_STATE_PARAMS), lrn.get_state(tj.TJ_STATE_ADAM_V), lrn.read_stats()))
        del lrn
    assert np.array_equal(states[0][0], states[1][0]) and np.array_equal(states[0][1], states[1][1])
    assert states[0][2] == states[1][2] and not np.array_equal(states[0][0], theta)


# ---------------------------------------------------------------- inserts concurrent with sampling

def _busy(stream, ms_target=3.0):
    """Keeps `stream` occupied for a few milliseconds with ordinary torch work, so that what is
    queued behind it is still pending when the host goes on."""
    import torch

    with torch.cuda.stream(stream):
        a = torch.empty(256 * 1024 * 1024 // 4, device="cuda", dtype=torch.float32)
        for _ in range(int(ms_target / 0.15) + 1):   # ~0.15 ms per 256 MiB fill
            a.fill_(1.0)
    return a


def test_sampling_leaves_out_slots_under_an_unfinished_insert(tj, orc):
    """An insert queued on a second stream behind other work is still pending when tj_sample is
    issued: the sample must skip exactly the arc reported by tj_buffer_status, and agree bit for
    bit with the oracle's sampler given that arc and the ring contents from before the insert.
    Once the insert stream has drained, the new rows are visible."""
    import torch

    wl = synth.small_variant(synth.WORKLOADS["c2"], capacity=6000, batch=256)
    gbuf, obuf = _fill_both(tj, orc, wl, 21, 2000, 6000 + 1500)      # full ring, head = 1500
    side = torch.cuda.Stream()
    cur, max_st = wl.current_version, 40
    new_rows = [synth.make_chunk(wl, 22, c, n) for c, n in ((0, 700), (1, 4300))]   # the second one wraps
    dev_rows = [{k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in r.items()} for r in new_rows]
    _sync()
    keep = _busy(side)
    for r in dev_rows:
        gbuf.insert_concurrent(r["obs"], r["next_obs"], r["action"], r["reward"], r["done"], r["version"], side)
    mb = tj.Minibatch(wl.batch, gbuf.obs_elems, gbuf.obs_dtype)
    assert gbuf.sample(mb, cur, max_st, 5) == tj.TJ_OK
    st, info = gbuf.status()
    assert st == tj.TJ_OK
    ex_begin, ex_len = int(info.last_excluded_begin), int(info.last_excluded_len)
    assert (ex_begin, ex_len) == (1500, 5000), "both inserts should still have been pending"
    assert (info.head, info.count) == ((1500 + 5000) % 6000, 6000)
    ost, oidx, oK = orc.sample_excluding(obuf.versions(), obuf.count, wl.capacity, ex_begin, ex_len, cur, max_st,
                                         5, wl.batch)
    assert ost == 0 and info.last_n_eligible == oK
    got = mb.host()
    np.testing.assert_array_equal(got["idx"], oidx)
    want = obuf.gather(oidx)                       # contents from before the inserts
    for f in FIELDS:
        np.testing.assert_array_equal(got[f], want[f], err_msg=f)
    side.synchronize()
    del keep
    for r in new_rows:
        assert obuf.insert(**r) == 0
    _compare_sample(tj, gbuf, obuf, wl.batch, cur, max_st, 6)
    _, info = gbuf.status()
    assert info.last_excluded_len == 0
    whole = obuf.gather(np.arange(wl.capacity, dtype=np.uint32))
    for f in ("obs", "next_obs", "done"):
        np.testing.assert_array_equal(gbuf.field(f).cpu().numpy().reshape(wl.capacity, -1),
                                      whole[f].reshape(wl.capacity, -1), err_msg=f)
    np.testing.assert_array_equal(gbuf.field("version").cpu().numpy(), obuf.versions())


def test_insert_stream_races_sampling_stream(tj, orc):
    """Inserts stream in on a second stream, unsynchronised with the host, while the first stream
    samples: every sample must equal the oracle's for the arc it reports (rows outside the arc are
    fully determined by the inserts issued so far), whatever the interleaving was."""
    import torch

    wl = synth.small_variant(synth.WORKLOADS["c2"], capacity=20000, batch=512)
    gbuf, obuf = _fill_both(tj, orc, wl, 31, 5000, 20000)
    side = torch.cuda.Stream()
    cur, max_st = wl.current_version, 60
    mbs = [tj.Minibatch(wl.batch, gbuf.obs_elems, gbuf.obs_dtype) for _ in range(2)]
    arcs_seen = 0
    for it in range(24):
        rows = synth.make_chunk(wl, 32, it, 1111 + 37 * it)
        dev = {k: torch.from_numpy(np.ascontiguousarray(v)).cuda() for k, v in rows.items()}
        _sync()                                     # the upload is done; from here on no host sync
        if it % 3 == 0:
            keep = _busy(side, 3.0)
        gbuf.insert_concurrent(dev["obs"], dev["next_obs"], dev["action"], dev["reward"], dev["done"],
                               dev["version"], side)
        mb = mbs[it % 2]
        assert gbuf.sample(mb, cur, max_st, 100 + it) == tj.TJ_OK   # issued with no host work in between
        assert obuf.insert(**rows) == 0             # the oracle's ring: state after the insert
        st, info = gbuf.status()                    # synchronises the sampling stream only
        ex_begin, ex_len = int(info.last_excluded_begin), int(info.last_excluded_len)
        arcs_seen += ex_len > 0
        ost, oidx, oK = orc.sample_excluding(obuf.versions(), obuf.count, wl.capacity, ex_begin, ex_len, cur,
                                             max_st, 100 + it, wl.batch)
        assert st == ost == 0 and info.last_n_eligible == oK
        got = mb.host()
        np.testing.assert_array_equal(got["idx"], oidx)
        want = obuf.gather(oidx)
        for f in FIELDS:
            np.testing.assert_array_equal(got[f], want[f], err_msg=f"{f} at iteration {it}")
    side.synchronize()
    assert arcs_seen > 0, "no sample ever overlapped an unfinished insert"


# ---------------------------------------------------------------- frame ring (one frame per slot)

def _frame_stream(rng, n, frame_elems, done_p, t0=0):
    frames = rng.integers(0, 256, (n, frame_elems)).astype(np.uint8)
    done = (rng.random(n) < done_p).astype(np.uint8)
    return (frames, rng.integers(0, 18, n).astype(np.int32), rng.uniform(-1, 1, n).astype(np.float32), done,
            ((t0 + np.arange(n)) // 50).astype(np.int32))


@pytest.mark.parametrize("frame_elems,cap,total,k", [(7056, 3000, 2200, 4), (7056, 1500, 5300, 4), (100, 4096, 9000, 4),
                                                      (37, 700, 2500, 3), (64, 64, 64, 2)])
def test_frame_ring_against_the_oracle(tj, orc, frame_elems, cap, total, k):
    """Inserts in ragged chunks (wrapping), ages, eligibility, indices and rebuilt stacks: bit-exact."""
    rng = np.random.default_rng(frame_elems + cap)
    g = tj.FrameBuffer(cap, frame_elems, k)
    o = orc.FrameBuffer(cap, frame_elems, k)
    pos = 0
    while pos < total:
        n = int(min(total - pos, rng.integers(1, min(900, cap) + 1)))
        rows = _frame_stream(rng, n, frame_elems, 0.02, pos)
        assert g.insert_host(*rows) == tj.TJ_OK and o.insert(*rows) == 0
        pos += n
    st, info = g.status()
    assert (info.head, info.count) == (o.head, o.count)
    np.testing.assert_array_equal(g.ages()[:o.count], o.ages()[:o.count])
    cur = (total - 1) // 50
    for seed, max_st, batch in ((1, 3, 64), (2, 0, 17), (3, 1000, 256)):
        mb = tj.Minibatch(batch, frame_elems * k, "u8")
        assert g.sample(mb, cur, max_st, seed) == tj.TJ_OK
        st, info = g.status()
        ost, oidx, oK = o.sample(batch, cur, max_st, seed)
        assert st == ost and info.last_n_eligible == oK
        got = mb.host()
        np.testing.assert_array_equal(got["idx"], oidx)
        if ost == 0:
            want = o.gather(oidx)
            for f in FIELDS:
                np.testing.assert_array_equal(got[f], want[f], err_msg=f)
    # too many rows at once: refused, nothing changes
    rows = _frame_stream(rng, cap + 1, frame_elems, 0.0)
    assert g.insert_host(*rows) == tj.TJ_ERR_CAPACITY and o.insert(*rows) == -5
    _, info = g.status()
    assert (info.head, info.count) == (o.head, o.count)


def test_frame_ring_edge_cases(tj, orc):
    g = tj.FrameBuffer(16, 8, 4)
    mb = tj.Minibatch(4, 32, "u8")
    assert g.sample(mb, 0, 10, 0) == tj.TJ_OK
    assert g.status()[0] == tj.TJ_ERR_NO_ELIGIBLE                 # empty
    rng = np.random.default_rng(0)
    g.insert_host(*_frame_stream(rng, 1, 8, 0.0))
    assert g.sample(mb, 0, 10, 0) == tj.TJ_OK
    assert g.status()[0] == tj.TJ_ERR_NO_ELIGIBLE                 # one row: no successor
    g.insert_host(*_frame_stream(rng, 1, 8, 0.0))
    assert g.sample(mb, 0, 10, 0) == tj.TJ_OK
    st, info = g.status()
    assert st == tj.TJ_OK and info.last_n_eligible == 1 and (mb.host()["idx"] == 0).all()
    L = tj.lib()
    bad = tj.tj_frame_buffer_desc(4, 8, 4)                        # capacity below two stacks
    assert L.tj_frame_buffer_arena_bytes(ctypes.byref(bad)) == 0


def test_ring_with_more_tiles_than_one_block_scans(tj, orc):
    """9 M slots = 8790 tiles of 1024: beyond the 8192 tile counts that the select kernel's blocks
    prefix-sum for themselves in LDS, so the scan runs as a kernel of its own.  Partly filled ring,
    ragged last tile, batches on both sides of the draws-per-block steps."""
    from dataclasses import replace

    wl = replace(synth.WORKLOADS["c2"], capacity=9_000_000, obs_shape=(1,))
    total = 8_800_000 + 321
    gbuf = tj.Buffer(wl.capacity, wl.obs_elems, wl.obs_dtype)
    rows = synth.make_chunk(wl, 77, 0, total)
    gbuf.insert_host(rows)
    for batch, cur, max_st, seed in ((1000, 999, 3, 1), (37, 500, 0, 2), (5000, 999, 999, 3)):
        mb = tj.Minibatch(batch, wl.obs_elems, wl.obs_dtype)
        assert gbuf.sample(mb, cur, max_st, seed) == tj.TJ_OK
        st, info = gbuf.status()
        ost, oidx, oK = orc.sample(rows["version"], total, cur, max_st, seed, batch)
        assert st == ost == 0 and info.last_n_eligible == oK
        got = mb.host()
        np.testing.assert_array_equal(got["idx"], oidx)
        for f in FIELDS:
            np.testing.assert_array_equal(got[f], rows[f][oidx], err_msg=f)
