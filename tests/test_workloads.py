"""Host-side checks of the seeded input generators and the workload catalogue (no GPU)."""
import numpy as np
import pytest

import workloads as wl


def test_splitmix64_known_sequence():
    """First outputs of the splitmix64 generator started at state 0 (Vigna's reference
    implementation adds the golden-ratio increment before mixing): published test vector."""
    state = np.uint64(0)
    inc = np.uint64(0x9E3779B97F4A7C15)
    outs = []
    with np.errstate(over="ignore"):
        for _ in range(3):
            outs.append(int(wl.splitmix64(np.array([state]))[0]))
            state = state + inc
    assert outs == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_field_is_deterministic_and_in_range():
    a = wl.uniform_field((33, 65), -1.0, 1.0, 5, np.float64)
    b = wl.uniform_field((33, 65), -1.0, 1.0, 5, np.float64)
    c = wl.uniform_field((33, 65), -1.0, 1.0, 6, np.float64)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    assert a.min() >= -1.0 and a.max() < 1.0
    assert abs(a.mean()) < 0.05 and abs(a.std() - 1 / np.sqrt(3)) < 0.03


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_window_equals_slice_of_field(dtype):
    full = wl.uniform_field((9, 20, 31), 0.0, 1.0, 3, dtype)
    win = wl.uniform_window((9, 20, 31), (2, 5, 7), (4, 6, 11), 0.0, 1.0, 3, dtype)
    assert np.array_equal(win, full[2:6, 5:11, 7:18])
    full2 = wl.uniform_field((40, 50), -1.0, 1.0, 9, dtype)
    win2 = wl.uniform_window((40, 50), (38, 0), (2, 50), -1.0, 1.0, 9, dtype)
    assert np.array_equal(win2, full2[38:40])


def test_shapes_have_the_catalogue_tap_counts():
    assert wl.mask_star(1, 1).sum() == 5 and wl.mask_star(4, 4).sum() == 17
    assert wl.mask_box(1, 1).sum() == 9 and wl.mask_box(2, 2).sum() == 25
    assert wl.mask_star(1, 1, 1).sum() == 7 and wl.mask_box(1, 1, 1).sum() == 27
    assert wl.mask_faces_edges().sum() == 19 and wl.mask_star(4, 4, 4).sum() == 25


def test_config_catalogue():
    cfg = wl.all_configs()
    assert [c.taps for c in cfg["config1"]] == [5]
    assert [(c.coef.shape[1], c.coef.shape[0]) for c in cfg["config2"]] == wl.CONV_SHAPES
    assert [c.taps for c in cfg["config3"]] == [9, 25, 17]
    assert [c.taps for c in cfg["config4"]] == [7, 27, 19]
    assert [c.taps for c in cfg["config5"]] == [25, 25]
    for name in ("config3", "config4", "config5"):
        for c in cfg[name]:
            assert np.all(c.coef >= 0) and abs(float(c.coef.astype(np.float64).sum()) - 1.0) < 1e-6
    c5 = cfg["config5"][1].coef
    assert np.array_equal(c5, c5[::-1, :, :]) and np.array_equal(c5, c5[:, ::-1, :]) \
        and np.array_equal(c5, c5[:, :, ::-1])
    assert [c.coef.shape for c in cfg["filter_sweep"]] == [(m, m) for m in range(2, 21)]
    t3 = {c.name: c.taps for c in cfg["table3"]}
    assert t3["t3_2d5pt_f32"] == 5 and t3["t3_2ds25pt_f64"] == 25 and t3["t3_2d121pt_f32"] == 121
    assert t3["t3_3d13pt_f64"] == 13 and t3["t3_3d125pt_f32"] == 125 and t3["t3_poisson_f64"] == 19
    assert t3["t3_2d64pt_f32"] == 64 and t3["t3_2d64pt_f64"] == 64
    c1 = cfg["config1"][0]
    assert c1.coef.max() < 0.25 and c1.coef[c1.coef != 0].min() > 0
    assert cfg["config2"][0].boundary == "clamp" and cfg["config3"][0].steps == 100


def test_oracle_and_generators_match_the_committed_lock_file():
    """tests/golden/oracle_lock.txt is written by tests/golden/make_golden.py (oracle only)."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_golden", os.path.join(here, "golden", "make_golden.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert mod.render() == open(os.path.join(here, "golden", "oracle_lock.txt")).read()


def test_device_generator_matches_host_generator():
    """uniform_field_on (torch integer arithmetic) reproduces uniform_field bit for bit, including
    counters beyond 2^31 (a window of a grid of almost 2^31 elements)."""
    torch = pytest.importorskip("torch")
    for dt in (np.float32, np.float64):
        for seed in (0, 5, 123456):
            host = wl.uniform_field((37, 1001), -1.0, 1.0, seed, dt)
            assert np.array_equal(host, wl.uniform_field_on("cpu", (37, 1001), -1.0, 1.0, seed, dt).numpy())
    big = (3, 46340, 46340)   # flat indices up to 6.4e9
    tail = wl.uniform_window(big, (2, 46339, 46000), (1, 1, 340), 0.0, 1.0, 9, np.float32)
    flat0 = (2 * 46340 + 46339) * 46340 + 46000
    z = wl.uniform_at(np.arange(flat0, flat0 + 340, dtype=np.uint64), 0.0, 1.0, 9, np.float32)
    assert np.array_equal(tail.ravel(), z)
