"""CPU-side checks of the C ABI: the library loads, exports every symbol the header declares, and
rejects bad specifications with the documented status codes (no compute without a GPU)."""
import os
import re

import numpy as np
import pytest

import workloads as wl
from paper_2002_02885_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "pack.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pack_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = _declared_symbols()
    assert len(names) >= 12
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def _status(models, B=4, in_shape=(1, 1, 8), dtype="f32", batch=None):
    try:
        binding.Pack(B, in_shape, dtype, models, batch).destroy()
    except binding.PackError as e:
        return e.status
    return binding.PACK_OK


def test_bad_specifications_are_rejected_before_any_device_work():
    mlp = wl.mlp([4], 3)
    assert _status([]) == binding.PACK_EINVAL                                  # K < 1
    assert _status([mlp] * 257) == binding.PACK_EINVAL                         # K > PACK_MAX_MODELS
    assert _status([mlp], batch=[0]) == binding.PACK_EINVAL
    assert _status([mlp], batch=[5]) == binding.PACK_EINVAL                    # b_k > B
    assert _status([[("conv3x3", 4, 3), ("gap",), ("linear", 3)]], in_shape=(4, 4, 2)) == binding.PACK_EINVAL
    assert _status([[(9, 4), ("linear", 3)]]) == binding.PACK_EINVAL           # unknown op
    assert _status([[("linear", 0)]]) == binding.PACK_EINVAL
    assert _status([[("relu",), ("linear", 3)]]) == binding.PACK_ESHAPE
    assert _status([[("linear", 3), ("relu",)]]) == binding.PACK_ESHAPE        # must end in logits
    assert _status([[("conv3x3", 4, 1), ("relu",)]], in_shape=(4, 4, 2)) == binding.PACK_ESHAPE
    assert _status([[("res_begin",), ("linear", 3)]]) == binding.PACK_ESHAPE   # unmatched
    assert _status([[("conv3x3", 4, 1), ("res_end",), ("gap",), ("linear", 3)]], in_shape=(4, 4, 2)) == binding.PACK_ESHAPE
    bad_shortcut = [("conv3x3", 4, 1), ("relu",), ("res_begin",), ("conv3x3", 3, 1), ("res_end",), ("gap",), ("linear", 3)]
    assert _status([bad_shortcut], in_shape=(4, 4, 2)) == binding.PACK_ESHAPE  # 4 -> 3 channels
    assert binding.lib().pack_last_error().decode() != ""


def test_null_handles_are_harmless():
    lib = binding.lib()
    assert lib.pack_num_params(None, 0) == 0
    assert lib.pack_num_classes(None, 0) == 0
    assert lib.pack_num_launches(None) == 0
    lib.pack_destroy(None)
    assert lib.pack_step(None, None, None, None) == binding.PACK_EINVAL


@pytest.mark.skipif(__import__("torch").cuda.is_available(), reason="only meaningful without a GPU")
def test_valid_specification_without_a_device_fails_loudly():
    assert _status([wl.mlp([4], 3)]) == binding.PACK_EDEVICE
