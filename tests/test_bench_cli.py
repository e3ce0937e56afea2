"""Host-side checks of bench.py and of the evidence files it reads (no GPU)."""
import glob
import json
import os
import re
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                         timeout=120)
    assert res.returncode != 0
    assert "ONE GPU" in (res.stdout + res.stderr)
    assert not res.stdout.strip().startswith("{")      # no result line


def test_measured_traffic_file_is_what_bench_expects():
    """profiles/measured_traffic.json: '<instance>@<grid>' -> HBM bytes per launch, written by the profiling
    summariser from the counter runs; every figure lies between 1x and 1.3x the algorithmic bytes."""
    table = json.load(open(os.path.join(ROOT, "profiles", "measured_traffic.json")))["bytes_per_launch"]
    assert len(table) >= 20
    for key, entry in table.items():
        inst, grid = key.split("@")
        dims = [int(d) for d in grid.split("x")]
        points = 1
        for d in dims:
            points *= d
        esz = 8 if inst.startswith("double") or inst.endswith("_f64") else 4
        assert 0.99 * 2 * esz * points <= entry <= 1.3 * 2 * esz * points, key


def test_every_profile_summary_names_the_command_that_made_it():
    """Each summary under profiles/ gives a full command line made of committed files only."""
    for path in glob.glob(os.path.join(ROOT, "profiles", "*.md")):
        text = open(path).read()
        cmds = re.findall(r"^\s{4}(.*(?:bench\.py|python -m paper_1907_06154_amd\.\w+).*)$", text, flags=re.M)
        assert cmds, os.path.basename(path)
        for c in cmds:
            assert "_work/" not in c and "tune.py" not in c, (os.path.basename(path), c)
            for module in re.findall(r"python -m paper_1907_06154_amd\.(\w+)", c):
                assert os.path.exists(os.path.join(ROOT, "paper_1907_06154_amd", module + ".py")), (os.path.basename(path), c)


def test_every_workload_of_the_generators_can_be_named_on_the_command_line():
    """bench.py --workload accepts every key of workloads.all_configs() (plus the default line and the scan)."""
    sys.path.insert(0, ROOT)
    import workloads as wl
    res = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0
    choices = re.search(r"--workload \{([^}]*)\}", res.stdout.replace("\n", " "))
    assert choices, res.stdout
    names = {c.strip() for c in choices.group(1).split(",")}
    assert set(wl.all_configs()) | {"default", "scan"} == names, names
    for cases in wl.all_configs().values():
        assert len({c.name for c in cases}) == len(cases)          # case names are unique within a workload
        for c in cases:
            assert c.kind in ("conv2d", "conv3d", "stencil2d", "stencil3d"), c.name
            assert c.coef.ndim == (2 if c.kind == "conv2d" else 3), c.name
            assert len(c.shape) == (2 if c.kind in ("conv2d", "stencil2d") else 3), c.name
