"""ssam_scan_static, the entry point that allocates nothing (its workspace is an array the library
holds in device memory), checked through the C ABI against ssam_scan on the same inputs: same
kernels and schedules, so the results must agree to the scan's tolerance (|x_i - y_i| <= tol *
(|a_0| + ... + |a_i|), 2e-6 fp32 / 1e-13 fp64), and against the CPU oracle.  Each case makes two calls in a
row, the second on a smaller input, so that whatever the first left in the shared array is there
when the second starts.  Collected last on purpose: it must pass alone and after the other tests."""
import ctypes

import numpy as np
import pytest

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

TOL = {np.dtype(np.float32): 2e-6, np.dtype(np.float64): 1e-13}
CODE = {np.dtype(np.float32): 0, np.dtype(np.float64): 1}
KNOBS = ("scan_segments", "scan_order", "scan_chained", "scan_spin_limit", "scan_one_group")


@pytest.fixture(scope="module")
def L():
    import paper_1907_06154_amd as s
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = s.lib()
    for name in KNOBS:
        s.ssam_set_tuning(name, -1)
    yield lib
    for name in KNOBS:
        s.ssam_set_tuning(name, -1)


def scan_both(L, a):
    """(ssam_scan_static result, ssam_scan result) for host array a, both through the C ABI."""
    code = CODE[a.dtype]
    n = a.size
    d_in = torch.from_numpy(a).cuda()
    out_static = torch.full_like(d_in, float("nan"))
    out_ref = torch.full_like(d_in, float("nan"))
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    st = L.ssam_scan_static(d_in.data_ptr(), out_static.data_ptr(), n, code, stream)
    assert st == 0, L.ssam_status_string(st)
    need = int(L.ssam_scan_workspace_bytes(n, code))
    work = torch.empty(max(need, 8), dtype=torch.uint8, device="cuda")
    st = L.ssam_scan(d_in.data_ptr(), out_ref.data_ptr(), n, code, work.data_ptr(), work.numel(), stream)
    assert st == 0, L.ssam_status_string(st)
    torch.cuda.synchronize()
    return out_static.cpu().numpy(), out_ref.cpu().numpy()


def check(L, a, what):
    got, ref = scan_both(L, a)
    bound = np.maximum(np.cumsum(np.abs(a.astype(np.float64))), np.finfo(np.float64).tiny)
    tol = TOL[a.dtype]
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    r1 = float(np.max(np.abs(got.astype(np.float64) - ref.astype(np.float64)) / bound))
    assert r1 <= tol, f"{what}: differs from ssam_scan by {r1:.3e} of the sum of magnitudes"
    r2 = float(np.max(np.abs(got.astype(np.float64) - oracle.scan(a).astype(np.float64)) / bound))
    assert r2 <= tol, f"{what}: differs from the oracle by {r2:.3e} of the sum of magnitudes"


# (first call, second and smaller call); "scan_chained" 1 makes every out-of-place array that the
# one-pass schedule can hold take it (ticket counter, flag and published sums live in the workspace),
# -1 leaves the built-in choice: three launches at these sizes (segment sums in the workspace)
CASES = [(-1, 3_000_017, 1_000_003), (1, 5_000_011, 2_500_007), (1, 4_200_000, 70_001), (-1, 300_000, 40_000)]


@pytest.mark.parametrize("dtype", [np.float32, np.float64])
@pytest.mark.parametrize("chained,n1,n2", CASES)
def test_static_scan_two_calls_in_a_row(L, dtype, chained, n1, n2):
    import paper_1907_06154_amd as s
    s.ssam_set_tuning("scan_chained", chained)
    try:
        for k, n in enumerate((n1, n2)):
            print(f"ssam_scan_static {np.dtype(dtype).name} chained={chained} n={n}", flush=True)
            a = wl.uniform_field((n,), -1.0, 1.0, 1300 + k, dtype)
            check(L, a, f"n={n} call {k + 1}")
    finally:
        s.ssam_set_tuning("scan_chained", -1)


def test_static_scan_rejects_without_touching_the_gpu(L):
    big = (1 << 32) + 1
    assert L.ssam_scan_static(ctypes.c_void_p(16), ctypes.c_void_p(32), big, 0, None) == 2      # SSAM_ERR_DIM
    assert L.ssam_scan_static(ctypes.c_void_p(16), ctypes.c_void_p(32), -1, 0, None) == 2
    assert L.ssam_scan_static(ctypes.c_void_p(16), ctypes.c_void_p(32), 10, 7, None) == 4       # SSAM_ERR_ENUM
    assert L.ssam_scan_static(None, ctypes.c_void_p(32), 10, 0, None) == 1                      # SSAM_ERR_NULL
    assert L.ssam_scan_static(None, None, 0, 0, None) == 0                                      # nothing to do
