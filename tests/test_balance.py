"""Production / consumption balance (Section 3.3, Eq. 2-3; Appendix D.1): the oracle's plan is pinned
to the paper's serial ratio and Lag-k setting and to a simulation through the oracle's own ring and
sampler; the library's host routine is then compared with the oracle value by value."""
import numpy as np
import pytest


def test_balanced_case_is_lag_k(orc):
    # TR_L = TR_A and B = B_s: the asynchronous pool must equal the serial buffer (Appendix D.1: a
    # buffer of k batches is Lag-k), so k versions stay eligible and the share is exactly P (Eq. 2)
    for k in (1, 2, 4, 8):
        st, p = orc.balance_plan(5000.0, 5000.0, 256, 256, 256 * k, 1 << 20)
        assert st == 0 and p["max_staleness"] == k - 1
        assert p["rows_per_version"] == 256 and p["window"] == 256 * k
        assert p["ratio"] == p["target_ratio"] == 1.0 / k and p["throughput"] == 5000.0 and p["cut"] == 0


def test_rates_scale_the_gate(orc):
    # actors four times faster than the learner: each version tags 4 B rows, a quarter of the versions
    st, p = orc.balance_plan(1000.0, 4000.0, 128, 128, 128 * 16, 1 << 20)
    assert (p["max_staleness"], p["rows_per_version"], p["window"]) == (3, 512, 2048)
    assert p["ratio"] == p["target_ratio"] == 1 / 16 and p["throughput"] == 1000.0
    # actors four times slower: four times as many versions
    st, p = orc.balance_plan(4000.0, 1000.0, 128, 128, 128 * 16, 1 << 20)
    assert (p["max_staleness"], p["rows_per_version"], p["window"]) == (63, 32, 2048) and p["throughput"] == 1000.0
    # never fewer than one version, and the ring bounds the pool
    assert orc.balance_plan(10.0, 1e6, 64, 64, 64, 1 << 30)[1]["max_staleness"] == 0
    st, p = orc.balance_plan(1000.0, 1000.0, 100, 100, 100 * 50, 1234)
    assert p["cut"] == 1 and p["max_staleness"] == 11 and p["window"] == 1200
    # more production never widens the gate
    gates = [orc.balance_plan(1000.0, a, 64, 64, 64 * 32, 1 << 20)[1]["max_staleness"] for a in (250, 500, 1000, 2000, 8000)]
    assert gates == sorted(gates, reverse=True)
    for bad in ((0.0, 1.0, 8, 8, 8, 8), (1.0, -1.0, 8, 8, 8, 8), (1.0, 1.0, 0, 8, 8, 8), (1.0, 1.0, 8, 9, 8, 8)):
        assert orc.balance_plan(*bad)[0] != 0


@pytest.mark.parametrize("tr_l,tr_a,batch,k", [(3000.0, 3000.0, 64, 4), (2000.0, 6000.0, 32, 9), (9000.0, 3000.0, 96, 2)])
def test_plan_against_a_simulated_ring(orc, tr_l, tr_a, batch, k):
    """Steady state through the oracle's ring and sampler: R rows arrive per policy version; with
    the planned gate the eligible count is the planned pool, so one batch is the share P of it."""
    st, p = orc.balance_plan(tr_l, tr_a, batch, batch, batch * k, 1 << 16)
    R = int(p["rows_per_version"])
    assert R == p["rows_per_version"]
    n_versions = int(p["max_staleness"]) + 12
    buf = orc.Buffer(1 << 16, 1, "f32")
    for ver in range(n_versions):
        z = np.zeros((R, 1), np.float32)
        buf.insert(z, z, np.zeros(R, np.int32), np.zeros(R, np.float32), np.zeros(R, np.uint8),
                   np.full(R, ver, np.int32))
    st, idx, K = buf.sample(batch, n_versions - 1, int(p["max_staleness"]), 1)
    assert st == 0 and K == p["window"]
    assert abs(batch / K - p["target_ratio"]) <= 0.5 / (k * tr_l / tr_a) * p["target_ratio"] + 1e-12


def test_library_routine_equals_the_oracle(orc):
    _library_routine_equals_the_oracle(orc)


@pytest.mark.gpu
def test_library_routine_equals_the_oracle_in_the_gpu_run(orc):
    """The same comparison in the GPU run (host arithmetic of the library, as loaded there)."""
    _library_routine_equals_the_oracle(orc)


def _library_routine_equals_the_oracle(orc):
    from paper_2502_20190_amd import binding as tj

    rng = np.random.default_rng(4)
    for _ in range(300):
        tr_l, tr_a = float(rng.uniform(10, 1e7)), float(rng.uniform(10, 1e7))
        batch, bs = int(rng.integers(1, 10000)), int(rng.integers(1, 4096))
        ns, cap = bs * int(rng.integers(1, 200)), int(rng.integers(1, 1 << 22))
        st, want = orc.balance_plan(tr_l, tr_a, batch, bs, ns, cap)
        gst, got = tj.balance_plan(tr_l, tr_a, batch, bs, ns, cap)
        assert st == gst == 0
        assert got.max_staleness == want["max_staleness"] and got.window_exceeds_capacity == want["cut"]
        for name in ("rows_per_version", "window", "ratio", "target_ratio", "throughput"):
            assert abs(getattr(got, name) - want[name]) <= 1e-12 * abs(want[name]), name
        rel = abs(tr_l - tr_a) / max(tr_l, tr_a)
        assert got.bottleneck == (0 if rel <= 0.05 else (1 if tr_a < tr_l else 2))
    assert tj.balance_plan(0.0, 1.0, 8, 8, 8, 8)[0] == tj.TJ_ERR_INVALID_ARG
    assert tj.balance_plan(1.0, 1.0, 8, 9, 8, 8)[0] == tj.TJ_ERR_INVALID_ARG
