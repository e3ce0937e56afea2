"""GPU parity of ssam_scan (inclusive prefix sums, Sec. 3.6) against the CPU oracle, element by
element, through the C ABI.  Tolerance, per element i: |gpu_i - oracle_i| <= tol * (|a_0| + ... +
|a_i|) with tol = 2e-6 for fp32 and 1e-13 for fp64.  It follows from the kernel's arithmetic: sums
inside one step of 64 lanes are formed in the element type (at most 3 + 6 + 1 additions on the way
to any output), everything carried across steps is fp64, and the result is rounded once."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

KNOBS = ("scan_segments", "scan_order", "scan_chained", "scan_spin_limit", "scan_one_group")
TOL = {np.dtype(np.float32): 2e-6, np.dtype(np.float64): 1e-13}


@pytest.fixture(scope="module")
def ssam():
    import paper_1907_06154_amd as s
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    s.lib()
    yield s
    for name in KNOBS:
        s.ssam_set_tuning(name, -1)


def check(got, a, what):
    want = oracle.scan(a)
    bound = np.cumsum(np.abs(a.astype(np.float64)))
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    ratio = float(np.max(err / np.maximum(bound, np.finfo(np.float64).tiny))) if a.size else 0.0
    assert ratio <= TOL[a.dtype], f"{what}: error / sum of magnitudes = {ratio:.3e}"


SIZES = [1, 2, 3, 63, 64, 65, 127, 128, 255, 256, 257, 511, 1023, 1024, 1025, 2047, 4096, 4099,
         65536, 100003, (1 << 20) + 17, (1 << 23) + 5]


@pytest.mark.parametrize("one_group", [-1, 0, 1 << 22])
@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_scan_matches_oracle(ssam, dtype, one_group):
    """one_group: the built-in limit of the one-workgroup launch (128 KiB), never, or up to 4 Mi elements."""
    ssam.ssam_set_tuning("scan_one_group", one_group)
    for k, n in enumerate(SIZES):
        lo = -1.0 if k % 2 == 0 else 0.0
        a = wl.uniform_field((n,), lo, 1.0, 900 + k, dtype)
        print(f"scan {np.dtype(dtype).name} n={n} range [{lo}, 1)", flush=True)
        got = ssam.ssam_scan(torch.from_numpy(a).cuda())
        torch.cuda.synchronize()
        check(got.cpu().numpy(), a, f"n={n}")
        if n <= 70000:                       # in place
            x = torch.from_numpy(a).cuda()
            ssam.ssam_scan(x, x)
            torch.cuda.synchronize()
            check(x.cpu().numpy(), a, f"in place n={n}")
    ssam.ssam_set_tuning("scan_one_group", -1)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_scan_of_integers_is_exact(ssam, dtype):
    """Small integers: every partial sum is an integer the element type holds, so any grouping of
    the additions gives the same bits."""
    n = (1 << 22) + 3
    ones = torch.ones(n, dtype=torch.from_numpy(np.zeros(1, dtype)).dtype, device="cuda")
    print(f"scan ones {np.dtype(dtype).name} n={n}", flush=True)
    got = ssam.ssam_scan(ones)
    torch.cuda.synchronize()
    assert torch.equal(got, torch.arange(1, n + 1, device="cuda").to(got.dtype))
    vals = (wl.uniform_field((n,), -4.0, 5.0, 921, np.float64)).astype(np.int64)
    a = vals.astype(dtype)
    got = ssam.ssam_scan(torch.from_numpy(a).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(got.cpu().numpy(), np.cumsum(vals).astype(dtype))


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_scan_segment_overrides_unaligned_and_in_place(ssam, dtype):
    n = 300007
    a = wl.uniform_field((n + 3,), -1.0, 1.0, 930, dtype)
    for segs, order in [(1, -1), (3, 0), (7, 1), (100, 0), (4096, 1), (-1, 0)]:
        ssam.ssam_set_tuning("scan_chained", 0)
        ssam.ssam_set_tuning("scan_segments", segs)
        ssam.ssam_set_tuning("scan_order", order)
        print(f"scan {np.dtype(dtype).name} n={n} segments<={segs} order={order}", flush=True)
        need = ssam.ssam_scan_workspace_bytes(n, dtype)
        assert need <= 8 * (segs if segs > 0 else 4096) and (segs != 1 or need == 0)
        d = torch.from_numpy(a).cuda()
        # element-aligned only: input shifted by one element, output by three
        out = torch.full((n + 3,), 7.0, dtype=d.dtype, device="cuda")
        ssam.ssam_scan(d[1:n + 1], out[3:])
        torch.cuda.synchronize()
        assert float(out[0]) == 7.0 and float(out[2]) == 7.0
        check(out[3:].cpu().numpy(), a[1:n + 1], f"unaligned, segments<={segs}")
        # in place, with a workspace the caller owns
        work = torch.empty(max(need, 8), dtype=torch.uint8, device="cuda")
        x = d[:n].clone()
        ssam.ssam_scan(x, x, work)
        torch.cuda.synchronize()
        check(x.cpu().numpy(), a[:n], f"in place, segments<={segs}")
        # in place never takes the one-pass schedule, also when it is forced for the size
        ssam.ssam_set_tuning("scan_chained", 1)
        x = d[:n].clone()
        ssam.ssam_scan(x, x)
        torch.cuda.synchronize()
        check(x.cpu().numpy(), a[:n], f"in place with one pass requested, segments<={segs}")
    for name in KNOBS:
        ssam.ssam_set_tuning(name, -1)


def gave_up(work) -> int:
    """Word 16 of the workspace of a one-pass call: nonzero if a wave ran out of polls and the
    fallback kernel redid the array."""
    torch.cuda.synchronize()
    return int(work.view(torch.int64)[16])


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_one_pass_scan_matches_oracle(ssam, dtype):
    """The one-pass schedule, forced on short arrays too: one segment, ragged last segments, several
    groups of 64 segments, and more than 64 groups (the third level of published sums)."""
    short = 16 * 64 * (4 if dtype == np.float32 else 2)   # segment with element-wise accesses (16 wave-rounds)
    per = (32 * 64 * 4) if dtype == np.float32 else (26 * 64 * 2)   # with 16-byte accesses: 32 or 26 wave-rounds
    ssam.ssam_set_tuning("scan_chained", 1)
    sizes = [1, per - 1, per, per + 1, 5 * per + 77, 64 * per, 64 * per + 1, 200 * per + 13, 4100 * per + 3]
    for k, n in enumerate(sizes):
        a = wl.uniform_field((n + 1,), -1.0, 1.0, 950 + k, dtype)
        need = ssam.ssam_scan_workspace_bytes(n, dtype)
        assert need >= 8 * (5152 + -(-n // short))
        work = torch.empty(need, dtype=torch.uint8, device="cuda")
        d = torch.from_numpy(a).cuda()
        for off in (0, 1):                       # 16-byte aligned, then element-aligned only
            print(f"one-pass scan {np.dtype(dtype).name} n={n} offset={off}", flush=True)
            out = torch.empty(n + 1, dtype=d.dtype, device="cuda")
            ssam.ssam_scan(d[off:off + n], out[off:off + n], work)
            assert gave_up(work) == 0
            check(out[off:off + n].cpu().numpy(), a[off:off + n], f"one pass n={n} offset={off}")
    # by default arrays of 128 MiB and more take the one-pass schedule, shorter ones do not
    ssam.ssam_set_tuning("scan_chained", -1)
    n = (160 << 20) // np.dtype(dtype).itemsize + 3
    assert ssam.ssam_scan_workspace_bytes(n, dtype) >= 8 * (5152 + n // short)
    assert ssam.ssam_scan_workspace_bytes(n // 2, dtype) <= 8 * 4096
    a = wl.uniform_field((n,), 0.0, 1.0, 970, dtype)
    got = ssam.ssam_scan(torch.from_numpy(a).cuda())
    torch.cuda.synchronize()
    check(got.cpu().numpy(), a, "one pass by default")
    # twice the same bits: the sums are combined in a fixed order whatever the timing
    again = ssam.ssam_scan(torch.from_numpy(a).cuda())
    torch.cuda.synchronize()
    assert torch.equal(got, again)


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
def test_one_pass_scan_that_gives_up_is_redone(ssam, dtype):
    """A poll limit of 0 set from the host makes every wave that would have to wait give up at
    once (no wave spins); the one-workgroup kernel behind the pass then produces the result."""
    per = (32 * 64 * 4) if dtype == np.float32 else (26 * 64 * 2)
    n = 300 * per + 5
    a = wl.uniform_field((n,), -1.0, 1.0, 980, dtype)
    ssam.ssam_set_tuning("scan_chained", 1)
    ssam.ssam_set_tuning("scan_spin_limit", 0)
    work = torch.empty(ssam.ssam_scan_workspace_bytes(n, dtype), dtype=torch.uint8, device="cuda")
    print(f"one-pass scan with poll limit 0, {np.dtype(dtype).name} n={n}", flush=True)
    got = ssam.ssam_scan(torch.from_numpy(a).cuda(), None, work)
    assert gave_up(work) == 1
    check(got.cpu().numpy(), a, "redone after giving up")
    ssam.ssam_set_tuning("scan_spin_limit", -1)
    got = ssam.ssam_scan(torch.from_numpy(a).cuda(), None, work)
    assert gave_up(work) == 0
    check(got.cpu().numpy(), a, "same workspace, normal limit")
    ssam.ssam_set_tuning("scan_chained", -1)


@pytest.mark.parametrize("chained", [0, 1])
def test_scan_can_be_captured_in_a_hip_graph(ssam, chained):
    """Both schedules only enqueue kernels on the caller's stream (the workspace is cleared by a
    kernel, not a memset), so a call can be captured and replayed; every replay is checked against
    the eager result, with eager work and synchronisations in between."""
    n = 3_000_017
    a = wl.uniform_field((n,), -1.0, 1.0, 990, np.float32)
    ssam.ssam_set_tuning("scan_chained", chained)
    d = torch.from_numpy(a).cuda()
    out = torch.empty_like(d)
    work = torch.empty(ssam.ssam_scan_workspace_bytes(n, np.float32), dtype=torch.uint8, device="cuda")
    ssam.ssam_scan(d, out, work)
    torch.cuda.synchronize()
    eager = out.cpu().numpy().copy()
    check(eager, a, "eager")
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        ssam.ssam_scan(d, out, work)
    for replay in range(4):
        print(f"scan graph replay {replay}, one pass {chained}", flush=True)
        out.fill_(float("nan"))
        work.fill_(255)                         # whatever the workspace holds is cleared by the call
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy(), eager), f"replay {replay} differs from the eager run"
        other = ssam.ssam_scan(d[: n // 3])      # unrelated eager work between replays
        torch.cuda.synchronize()
        check(other.cpu().numpy(), a[: n // 3], "eager between replays")
    ssam.ssam_set_tuning("scan_chained", -1)


def test_scan_random_sizes_offsets_and_schedules(ssam):
    """Seeded random lengths, element offsets of input and output, segment limits and schedules."""
    rng = np.random.default_rng(20240607)
    pool = {dt: wl.uniform_field((3_000_000 + 8,), -1.0, 1.0, 960 + k, dt) for k, dt in enumerate((np.float32, np.float64))}
    dev_pool = {dt: torch.from_numpy(a).cuda() for dt, a in pool.items()}
    for case in range(48):
        dt = (np.float32, np.float64)[case % 2]
        n = int(rng.choice([rng.integers(1, 300), rng.integers(300, 70_000), rng.integers(70_000, 3_000_000)]))
        off_in, off_out = int(rng.integers(0, 8)), int(rng.integers(0, 8))
        chained, segs = int(rng.integers(0, 2)), int(rng.choice([-1, 1, 2, 5, 64, 1000, 4096]))
        ssam.ssam_set_tuning("scan_chained", chained)
        ssam.ssam_set_tuning("scan_segments", segs)
        print(f"scan case {case}: {np.dtype(dt).name} n={n} offsets {off_in}/{off_out} one pass {chained} segments<={segs}", flush=True)
        src = dev_pool[dt][off_in:off_in + n]
        out = torch.full((n + 16,), -3.0, dtype=src.dtype, device="cuda")
        ssam.ssam_scan(src, out[off_out:off_out + n])
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert np.all(got[:off_out] == -3.0) and np.all(got[off_out + n:] == -3.0), "wrote outside the output"
        check(got[off_out:off_out + n], pool[dt][off_in:off_in + n], f"case {case}")
    for name in KNOBS:
        ssam.ssam_set_tuning(name, -1)


def test_one_pass_scans_on_two_streams_at_once(ssam):
    """Two one-pass scans in flight on their own streams with their own workspaces: the waves of one
    only ever wait for waves of the same launch that already run, so sharing the device costs time,
    not correctness; neither gives up."""
    n = (96 << 20) // 4 + 11
    ssam.ssam_set_tuning("scan_chained", 1)
    jobs = []
    for k, dtype in enumerate((np.float32, np.float64)):
        a = wl.uniform_field((n // (k + 1),), -1.0, 1.0, 985 + k, dtype)
        d = torch.from_numpy(a).cuda()
        work = torch.empty(ssam.ssam_scan_workspace_bytes(a.size, dtype), dtype=torch.uint8, device="cuda")
        jobs.append((a, d, torch.empty_like(d), work, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(6):
        print(f"two streams, repetition {rep}", flush=True)
        for a, d, out, work, st in jobs:
            ssam.ssam_scan(d, out, work, stream=st)
    torch.cuda.synchronize()
    for a, d, out, work, st in jobs:
        assert gave_up(work) == 0
        check(out.cpu().numpy(), a, f"two streams, {a.dtype}")
    ssam.ssam_set_tuning("scan_chained", -1)


def test_scan_of_a_gibibyte(ssam):
    """2^28 fp32 elements, generated on the device with the shared counter-based generator, the
    default (one-pass) schedule, every element against the oracle."""
    n = 1 << 28
    d = wl.uniform_field_on("cuda", (n,), -1.0, 1.0, 995, np.float32)
    print(f"scan f32 n={n}", flush=True)
    work = torch.empty(ssam.ssam_scan_workspace_bytes(n, np.float32), dtype=torch.uint8, device="cuda")
    got = ssam.ssam_scan(d, None, work)
    assert gave_up(work) == 0
    a = d.cpu().numpy()
    want = oracle.scan(a)
    bound = np.cumsum(np.abs(a), dtype=np.float64)
    err = np.abs(got.cpu().numpy().astype(np.float64) - want)
    assert float(np.max(err / np.maximum(bound, 1e-300))) <= TOL[np.dtype(np.float32)]


def test_scan_edges_and_errors(ssam):
    L = ssam.lib()
    empty = torch.empty(0, dtype=torch.float32, device="cuda")
    assert ssam.ssam_scan(empty).numel() == 0
    a = torch.ones(1 << 16, dtype=torch.float32, device="cuda")
    b = torch.zeros_like(a)
    work = torch.empty(1 << 18, dtype=torch.uint8, device="cuda")
    n, need = a.numel(), ssam.ssam_scan_workspace_bytes(a.numel(), torch.float32)
    assert need > 0
    p = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)
    assert L.ssam_scan(p(a), p(b), n, 0, p(work), need - 8, None) == 2       # workspace too small
    assert L.ssam_scan(p(a), p(b), n, 0, None, 0, None) == 1                 # workspace missing
    assert L.ssam_scan(p(a), p(b), n, 7, p(work), need, None) == 4           # dtype
    assert L.ssam_scan(p(a), p(b), -1, 0, p(work), need, None) == 2
    assert L.ssam_scan(p(a), p(a, 64), n - 16, 0, p(work), need, None) == 5  # partial overlap
    assert L.ssam_scan(p(a), p(b), n, 0, p(a), need, None) == 5              # workspace inside the input
    assert L.ssam_scan(p(a, 2), p(b), n - 1, 0, p(work), need, None) == 2    # misaligned element
    assert L.ssam_scan(None, p(b), n, 0, p(work), need, None) == 1
    torch.cuda.synchronize()
    assert float(b.abs().sum()) == 0.0                                       # nothing was launched
