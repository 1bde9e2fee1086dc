"""GPU: the peak micro-benchmarks behind the roofline denominators return plausible rates."""
import pytest

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible():
    import torch
    from paper_1705_09786_amd import binding as B
    buf = torch.zeros(1 << 30, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    lds_cu, hbm = B.measure_peaks(buf.data_ptr(), buf.numel(), torch.cuda.current_stream().cuda_stream)
    # nominal: 128 B/clk/CU at 2.4 GHz = 307 GB/s per CU; 8 TB/s of HBM
    assert 100e9 < lds_cu < 700e9, lds_cu
    assert 1e12 < hbm < 9e12, hbm


def test_measure_peaks_rejects_bad_arguments():
    import ctypes as ct
    from paper_1705_09786_amd import binding as B
    a, b = ct.c_double(), ct.c_double()
    assert B.lib().amp_measure_peaks(None, 1 << 30, None, ct.byref(a), ct.byref(b)) == B.AMP_EINVAL
