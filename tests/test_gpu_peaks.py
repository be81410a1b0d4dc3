"""spec_measure_peaks: the two microkernels give rates a MI355X can have, below its published peaks
(8 TB/s, 2.5 PFLOP/s for f16 MFMA), and the call refuses a buffer too small to stream."""
import ctypes as C

import pytest
import torch

pytestmark = pytest.mark.gpu


def test_measured_peaks_are_plausible_and_below_nominal():
    from paper_2310_18813_amd import binding as B
    hbm, mfma = B.spec_measure_peaks("cuda:0", 1 << 30)
    assert 2000.0 < hbm < 8000.0, hbm
    assert 800.0 < mfma < 2520.0, mfma
    # a second call agrees within 10 %
    hbm2, mfma2 = B.spec_measure_peaks("cuda:0", 1 << 30)
    assert abs(hbm2 - hbm) / hbm < 0.1 and abs(mfma2 - mfma) / mfma < 0.1


def test_too_small_a_buffer_is_refused():
    from paper_2310_18813_amd import binding as B
    buf = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    g, t = C.c_double(0.0), C.c_double(0.0)
    st = torch.cuda.current_stream()
    rc = B.lib.spec_measure_peaks(C.c_void_p(st.cuda_stream), C.c_void_p(buf.data_ptr()), 4096, C.byref(g), C.byref(t))
    assert rc == B.ERR_CAPACITY
    rc = B.lib.spec_measure_peaks(C.c_void_p(st.cuda_stream), None, 4096, C.byref(g), C.byref(t))
    assert rc == B.ERR_INVALID_ARG
