"""The measuring aid pack_measure_ceiling: plausible figures on an MI355X and clean errors."""
import ctypes as C

import pytest

from paper_2002_02885_amd import binding

pytestmark = pytest.mark.gpu


def test_measured_ceilings_lie_between_a_floor_and_the_published_peaks():
    hbm = binding.measure_ceiling("hbm_copy")
    bf16 = binding.measure_ceiling("mfma_bf16")
    fp32 = binding.measure_ceiling("mfma_fp32")
    # published: 8 TB/s, 2.5 PFLOP/s bf16, 157.3 TFLOP/s fp32; a healthy card reaches well over a third of each
    assert 2500.0 < hbm <= 8000.0
    assert 800.0 < bf16 <= 2500.0 * 1.02
    assert 50.0 < fp32 <= 157.3 * 1.02


def test_unknown_ceiling_is_rejected():
    out = C.c_double(-1.0)
    assert binding.lib().pack_measure_ceiling(7, None, C.byref(out)) == binding.PACK_EINVAL
    assert binding.lib().pack_measure_ceiling(0, None, None) == binding.PACK_EINVAL
    assert out.value == -1.0
