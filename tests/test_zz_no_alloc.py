"""conqur_score_rows_static (the entry point for callers that cannot allocate) against conqur_quant_error /
conqur_quant_error_zp, through the C ABI: two calls in a row on one GPU, the second with a smaller input, so that what
the first call left in the library's static array must not leak into the second result."""
import numpy as np
import pytest

from paper_2605_10793_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL_REL = 1e-3      # the bar of the int4 error (relative); the two paths run the same kernels, so far closer is expected


@pytest.fixture(scope="module")
def B():
    import torch
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a HIP device")
    from paper_2605_10793_amd import binding
    binding.load()
    return binding


@pytest.mark.parametrize("dtype,d", [("bf16", 512), ("f32", 192)])
def test_static_score_matches_quant_error_twice_in_a_row(B, dtype, d):
    import torch
    w = I.small_workload(d, 300, n_batches=2, dtype=dtype, seed=4242, massive_frac=0.01)
    R0 = I.initial_rotation(w)
    cal = B.Calibrator(d, 1, dtype, R0, max_tokens=300)
    out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda:0")
    try:
        for b, T in ((0, 300), (1, 77)):                      # the second call is the smaller one
            Xd = B.to_device(I.batch(w, b, T), dtype)
            Y = cal.rotate(Xd)
            for zp, clip in ((False, 1.0), (True, 0.9)):
                ref = cal.quant_error_zp(Xd, 4, clip) if zp else cal.quant_error(Xd, 4)
                out.fill_(-1.0)
                B.score_rows_static(Y, out, 4, zp, clip)
                torch.cuda.synchronize()
                got = out.cpu().numpy()
                print(f"  static score {dtype} T={T} zp={zp}: sse {got[0]:.9e} vs {ref[0]:.9e}  energy {got[1]:.9e} vs {ref[1]:.9e}",
                      flush=True)
                assert abs(got[0] - ref[0]) <= TOL_REL * ref[0] and abs(got[1] - ref[1]) <= TOL_REL * ref[1]
                assert abs(got[0] - ref[0]) <= 1e-9 * ref[0] and abs(got[1] - ref[1]) <= 1e-9 * ref[1]   # same kernels, same rows
        # a wider buffer than d (row stride), and the error paths
        Ybuf = torch.zeros((77, d + 16), dtype=Y.dtype, device="cuda:0")
        Ybuf[:, :d] = Y
        out.fill_(-1.0)
        B.score_rows_static(Ybuf, out, 4, False, 1.0, d=d)
        torch.cuda.synchronize()
        ref = cal.quant_error(Xd, 4)
        assert abs(out[0].item() - ref[0]) <= 1e-9 * ref[0]
        lib = B.load()
        big = 65537
        assert lib.conqur_score_rows_static(Y.data_ptr(), B.BF16 if dtype == "bf16" else B.F32, big, d, d, 4, 0, 1.0,
                                            out.data_ptr(), None) == B.EINVAL          # more rows than the static array holds
        assert lib.conqur_score_rows_static(Y.data_ptr(), 7, 77, d, d, 4, 0, 1.0, out.data_ptr(), None) == B.EINVAL
        assert lib.conqur_score_rows_static(Y.data_ptr(), B.BF16, 77, d, d, 9, 0, 1.0, out.data_ptr(), None) == B.EINVAL
        assert lib.conqur_score_rows_static(Y.data_ptr(), B.BF16, 77, d, d, 4, 1, 0.0, out.data_ptr(), None) == B.EINVAL
        assert lib.conqur_score_rows_static(None, B.BF16, 77, d, d, 4, 0, 1.0, out.data_ptr(), None) == B.EINVAL
        assert lib.conqur_score_rows_static(Y.data_ptr(), B.BF16, 77, d, d - 8, 4, 0, 1.0, out.data_ptr(), None) == B.EINVAL
    finally:
        cal.close()
