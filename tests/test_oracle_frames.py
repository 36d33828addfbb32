"""Pins of the oracle's frame ring (one frame per slot, stacks rebuilt at sampling) against an
independent, explicit construction: the environment stream is kept as Python lists of episodes, every
transition's two stacks are assembled the long way (repeat the episode's first frame while fewer than
k frames exist), and a slot of the ring is usable iff all frames of both stacks are still stored."""
import numpy as np
import pytest


def _stream(rng, n, frame_elems, done_p):
    frames = rng.integers(0, 256, (n, frame_elems)).astype(np.uint8)
    done = (rng.random(n) < done_p).astype(np.uint8)
    action = rng.integers(0, 6, n).astype(np.int32)
    reward = rng.uniform(-1, 1, n).astype(np.float32)
    version = (np.arange(n) // 7).astype(np.int32)            # a new policy version every 7 rows
    return frames, action, reward, done, version


def _explicit(frames, done, k):
    """Per time step t: (list of k frame times of s, list of k frame times of s')."""
    n = len(done)
    start, starts = 0, []
    for t in range(n):
        starts.append(start)
        if done[t]:
            start = t + 1
    stack = lambda t: [max(starts[t], t - (k - 1 - p)) for p in range(k)]
    return [(stack(t), stack(t + 1) if t + 1 < n else None) for t in range(n)]


@pytest.mark.parametrize("seed,cap,total,k", [(0, 64, 40, 4), (1, 64, 64, 4), (2, 50, 173, 4), (3, 33, 400, 3), (4, 16, 16, 2)])
def test_frame_ring_against_explicit_stacks(orc, seed, cap, total, k):
    rng = np.random.default_rng(seed)
    fe = 5
    frames, action, reward, done, version = _stream(rng, total, fe, 0.15)
    buf = orc.FrameBuffer(cap, fe, k)
    pos = 0
    while pos < total:                                          # ragged chunks, wrap-around
        n = int(min(total - pos, rng.integers(1, 12)))
        assert buf.insert(frames[pos:pos + n], action[pos:pos + n], reward[pos:pos + n], done[pos:pos + n],
                          version[pos:pos + n]) == 0
        pos += n
    ref = _explicit(frames, done, k)
    oldest = max(0, total - cap)                                # time steps still stored: [oldest, total)
    usable = {}
    for t in range(oldest, total):
        s, sn = ref[t]
        if sn is not None and min(s) >= oldest:                 # successor stored, look-back stored
            usable[t % cap] = t
    cur, max_st = int(version[-1]), 3
    E = sorted(slot for slot, t in usable.items() if 0 <= cur - version[t] <= max_st)
    st, idx, K = buf.sample(32, cur, max_st, seed)
    assert K == len(E)
    if not E:
        assert st == -4
        return
    assert st == 0
    for j in range(32):
        assert idx[j] == E[(orc.rng64(seed, j) * len(E)) >> 64]
    got = buf.gather(idx)
    for j, slot in enumerate(idx):
        t = usable[int(slot)]
        s, sn = ref[t]
        np.testing.assert_array_equal(got["obs"][j], np.concatenate([frames[u] for u in s]))
        np.testing.assert_array_equal(got["next_obs"][j], np.concatenate([frames[u] for u in sn]))
        assert (got["action"][j], got["reward"][j], got["done"][j]) == (action[t], reward[t], done[t])
    # every usable slot, not only the sampled ones
    all_slots = np.array(sorted(usable), np.uint32)
    full = buf.gather(all_slots)
    for j, slot in enumerate(all_slots):
        s, sn = ref[usable[int(slot)]]
        np.testing.assert_array_equal(full["obs"][j], np.concatenate([frames[u] for u in s]))
        np.testing.assert_array_equal(full["next_obs"][j], np.concatenate([frames[u] for u in sn]))


def test_frame_ring_edge_cases(orc):
    buf = orc.FrameBuffer(8, 2, 4)
    z = lambda n: (np.zeros((n, 2), np.uint8), np.zeros(n, np.int32), np.zeros(n, np.float32))
    assert buf.sample(4, 0, 10, 0)[0] == -4                     # empty
    f, a, r = z(1)
    buf.insert(f, a, r, np.zeros(1, np.uint8), np.zeros(1, np.int32))
    assert buf.sample(4, 0, 10, 0)[0] == -4                     # a single row has no successor
    f, a, r = z(1)
    buf.insert(f, a, r, np.zeros(1, np.uint8), np.zeros(1, np.int32))
    st, idx, K = buf.sample(4, 0, 10, 0)
    assert (st, K) == (0, 1) and (idx == 0).all()
    assert orc.FrameBuffer(4, 2, 4).insert(*z(5), np.zeros(5, np.uint8), np.zeros(5, np.int32)) == -5
    # ages: capped at stack - 1, reset after done
    buf = orc.FrameBuffer(16, 1, 4)
    done = np.array([0, 0, 0, 0, 0, 1, 0, 0, 1, 1, 0], np.uint8)
    n = len(done)
    buf.insert(np.zeros((n, 1), np.uint8), np.zeros(n, np.int32), np.zeros(n, np.float32), done, np.zeros(n, np.int32))
    np.testing.assert_array_equal(buf.ages()[:n], [0, 1, 2, 3, 3, 3, 0, 1, 2, 0, 0])
