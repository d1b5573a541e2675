"""The entry point that allocates nothing (imunpack_percentile_static: its counters live in a fixed
device array of the library) against the entry point it is a variant of (imunpack_percentile with a
caller workspace), through the C ABI: the same bits, on two calls in a row, the second with a smaller
input, so that whatever the first call left in the shared array would show."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def imu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_07339_amd import binding
    return binding


def test_static_scratch_percentile_matches_the_workspace_one(imu):
    g = torch.Generator().manual_seed(5)
    big = (torch.randn((1536, 2048), generator=g) * 3.0)
    big[torch.rand(big.shape, generator=g) < 0.001] *= 500.0
    small = torch.randn((77, 130), generator=g) * 0.02          # smaller, other magnitudes, scalar-load path
    alpha = torch.empty(1, dtype=torch.float32, device="cuda")
    status = torch.empty(1, dtype=torch.int32, device="cuda")
    for X, p in ((big, 95.0), (small, 95.0), (small.t(), 50.0), (big, 99.9), (small, 100.0)):
        Xd = X.to("cuda")
        want, want_status = imu.imunpack_percentile(Xd, p)
        alpha.fill_(-1.0)
        status.fill_(-1)
        imu.imunpack_percentile_static(Xd, p, alpha, status)
        torch.cuda.synchronize()
        assert int(status.item()) == int(want_status.item()) == 0
        assert alpha.cpu().numpy().view(np.uint32)[0] == want.cpu().numpy().view(np.uint32)[0]
        # and against the definition: the k-th smallest magnitude, k = ceil(p N / 100)
        mags = np.sort(np.abs(X.contiguous().numpy()).ravel())
        k = min(mags.size, max(1, int(np.ceil(p * mags.size / 100.0))))
        assert alpha.item() == mags[k - 1]
    # a NaN raises the flag through this entry point too
    bad = small.clone()
    bad[3, 4] = float("nan")
    imu.imunpack_percentile_static(bad.to("cuda"), 95.0, alpha, status)
    assert int(status.item()) == 1


def test_static_scratch_percentile_rejects_what_its_counters_cannot_hold(imu):
    alpha = torch.empty(1, dtype=torch.float32, device="cuda")
    x = torch.zeros((4, 4), device="cuda")
    import ctypes as C
    lib = C.CDLL(imu.LIB_PATH)
    lib.imunpack_percentile_static.restype = C.c_int
    lib.imunpack_percentile_static.argtypes = [C.c_void_p, C.c_int64, C.c_int64, C.c_int64, C.c_int64, C.c_double,
                                               C.c_void_p, C.c_void_p, C.c_void_p]
    # 2^16 x 2^16 entries: one more than the counters hold; rejected on the host, nothing is launched
    assert lib.imunpack_percentile_static(x.data_ptr(), 1 << 16, 1 << 16, 1 << 16, 1, 95.0, alpha.data_ptr(), None, None) == imu.ERANGE
    assert lib.imunpack_percentile_static(x.data_ptr(), 4, 4, 4, 1, 0.0, alpha.data_ptr(), None, None) == imu.EINVAL
