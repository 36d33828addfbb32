"""The C-ABI library loads and exports every function include/tianji.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "tianji.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tj_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2502_20190_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        from paper_2502_20190_amd.build import build_hip
        build_hip()
    names = _declared()
    assert len(names) >= 17
    lib = ctypes.CDLL(binding.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_host_side_argument_checks_need_no_gpu():
    from paper_2502_20190_amd import binding as b

    L = b.lib()
    assert b.tj_strerror(b.TJ_ERR_NO_ELIGIBLE).startswith("no eligible")
    bad = b.tj_buffer_desc(0, 4, 0)
    assert L.tj_buffer_arena_bytes(ctypes.byref(bad)) == 0
    ok = b.tj_buffer_desc(10_000, 4, 0)
    n = L.tj_buffer_arena_bytes(ctypes.byref(ok))
    # two obs fields + action + reward + done + version, each padded to 256 bytes, plus scratch
    assert n >= 10_000 * (2 * 16 + 4 + 4 + 1 + 4) and n % 256 == 0
    d = b.make_learner_desc([(0, 64, 0, 0), (0, 64, 0, 0), (0, 2, 0, 0)], (4, 1, 1), "f32", "fp32", 32,
                            0.99, 1.0, 1e-3, 0.9, 0.999, 1e-8, 100)
    assert L.tj_learner_num_params(ctypes.byref(d)) == 4 * 64 + 64 + 64 * 64 + 64 + 64 * 2 + 2
    assert L.tj_learner_arena_bytes(ctypes.byref(d)) > 0
    h = ctypes.c_void_p()
    assert L.tj_buffer_create(ctypes.byref(ok), None, n, None, ctypes.byref(h)) == b.TJ_ERR_INVALID_ARG
    assert L.tj_buffer_create(ctypes.byref(ok), 4096, 16, None, ctypes.byref(h)) == b.TJ_ERR_ARENA_TOO_SMALL
    assert L.tj_sample(None, 4, 0, 0, 0, None, None) == b.TJ_ERR_INVALID_ARG
    assert L.tj_learner_step(None, None, None, None) == b.TJ_ERR_INVALID_ARG


def test_synth_param_count_matches_library():
    from paper_2502_20190_amd import binding as b, synth

    for wl in synth.WORKLOADS.values():
        d = b.make_learner_desc(wl.layers, wl.in_chw, wl.obs_dtype, wl.precision, wl.batch, wl.gamma,
                                wl.kappa, wl.lr, wl.beta1, wl.beta2, wl.eps, wl.target_interval)
        assert b.lib().tj_learner_num_params(ctypes.byref(d)) == synth.num_params(wl.layers, wl.in_chw)
    assert synth.num_params(synth.WORKLOADS["c3"].layers, (256, 1, 1)) == 2_395_168
    assert synth.num_params(synth.WORKLOADS["c4"].layers, (4, 84, 84)) == 1_693_362
