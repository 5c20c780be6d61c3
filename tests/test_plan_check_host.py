"""Plan verification on the host (pack_plan_check): the planner's real launch plans of the convolution
configurations, at full size, walked through the address rules of the halo kernels (weight gradient;
stride-1 forward pass and input gradient) without a GPU: every load of every thread of every chunk of
every tile (prefetches beyond the reduction included) must stay inside its tensor or be cut off by the
range check, and every matrix-instruction operand slot must hold the element the definition of the
product puts there."""
import pytest

import workloads as wl
from paper_2002_02885_amd import binding


def _check(w, **kw):
    walked, skipped, loads = binding.plan_check(w.B, w.in_shape, w.dtype, w.models, w.batch, **kw)
    assert walked >= 1 and loads > 0
    return walked, skipped, loads


def test_full_size_plans_of_all_five_configurations():
    """Every matrix-product launch of the real plans is walked: the staged-tile kernels by running their
    fetchers on the CPU, the halo kernels by their address rules.  Nothing is skipped."""
    expect = {"c1": 2, "c2": 4, "c3": 8, "c4": 8, "c5": 22}     # matrix-product launches per step
    loads = {}
    for name, n in expect.items():
        w = wl.CONFIGS[name]()
        walked, skipped, loads[name] = _check(w)
        assert walked == n and skipped == 0, (name, walked, skipped)
    assert loads["c5"] > 10 * loads["c3"] > 10 ** 9


@pytest.mark.parametrize("make", [
    lambda: wl.config5(K=2, B=8, size=16, steps=1),
    lambda: wl.config5(K=2, B=3, size=32, widths=(64, 128, 192), n_classes=10, steps=1),
    lambda: wl.config5(K=1, B=2, size=64, widths=(64, 128), n_classes=10, steps=1, dtype=wl.F32),
    lambda: wl.config3(K=3, B=5, size=32, widths=(64, 64, 64), steps=1, dtype=wl.BF16),
    lambda: wl.config5(K=1, B=2, size=24, widths=(64, 64), n_classes=10, steps=1),     # 24-pixel rows: not a power of two, stays on the staged tiles
])
def test_reduced_and_odd_shapes(make):
    w = make()
    walked, skipped, loads = binding.plan_check(w.B, w.in_shape, w.dtype, w.models, w.batch)
    assert walked >= 1 and loads > 0


def test_members_on_their_own_batches_and_argument_errors():
    w = wl.config5(K=2, B=4, size=16, widths=(64, 64), n_classes=10, steps=1)
    _check(w, per_member_input=True)
    with pytest.raises(binding.PackError):
        binding.plan_check(4, (16, 16, 3), "bf16", [[("relu",)]], [4])
    with pytest.raises(binding.PackError):
        binding.plan_check(4, (16, 16, 3), "bf16", w.models, [5, 4])


def test_the_walk_notices_planted_mistakes(tmp_path):
    """The host-side walk is compiled (host code only) as it is and with one address rule deliberately wrong:
    halo rows one too low, the two channel halves of a fragment swapped, the right padding column fetched
    instead of zeroed, stride-2 taps reading neighbouring instead of every second pixel.  The clean build
    must pass on every case, each planted mistake must fail on at least one."""
    import os
    import shutil
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc to compile the driver with")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2002_02885_amd", "csrc")
    cases = [("1", "1", "2", "16", "16", "64", "64"), ("1", "2", "2", "32", "32", "64", "128"),
             ("0", "1", "1", "16", "16", "64", "64"), ("0", "2", "1", "32", "32", "64", "64"),
             ("0", "1", "1", "32", "32", "32", "64"), ("1", "1", "1", "16", "16", "96", "64")]      # 32 input channels per tile

    def build(plant):
        exe = str(tmp_path / f"walk{plant}")
        subprocess.run([hipcc, "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", f"-DPACK_HALO_PLANT={plant}", "-I", csrc,
                        os.path.join(csrc, "conv_dw_halo_check.cpp"), os.path.join(root, "tests", "halo_walk_driver.cpp"), "-o", exe],
                       check=True, capture_output=True)
        return exe

    clean = build(0)
    for c in cases:
        r = subprocess.run([clean, *c], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.startswith("OK"), (c, r.stdout)
    for plant in (1, 2, 3, 4):
        exe = build(plant)
        results = [subprocess.run([exe, *c], capture_output=True, text=True) for c in cases]
        assert any(r.returncode == 1 and "FAIL" in r.stdout for r in results), plant


def test_the_walk_of_the_stride_1_forward_and_input_gradient_form_notices_planted_mistakes(tmp_path):
    """Same for the halo form of the stride-1 forward pass and input gradient: input-gradient taps displaced
    the forward way, halo columns fetched one pixel to the right."""
    import os
    import shutil
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc to compile the driver with")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2002_02885_amd", "csrc")
    # bf16, dx, B, H, W, Cin, Cout: rows of 64, 32, 16 and 8 pixels (whole images per tile from 16 down); both
    # directions; one and several channel blocks; the 32-column form
    cases = [("1", "0", "1", "64", "64", "64", "64"), ("1", "1", "2", "32", "32", "128", "128"), ("1", "0", "4", "16", "16", "256", "64"),
             ("1", "1", "8", "8", "8", "64", "512"), ("0", "0", "1", "32", "32", "64", "64"), ("0", "1", "2", "32", "32", "32", "64")]

    def build(plant):
        exe = str(tmp_path / f"rows{plant}")
        subprocess.run([hipcc, "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", f"-DPACK_HALO_PLANT={plant}", "-I", csrc,
                        os.path.join(csrc, "conv_rows_halo_check.cpp"), os.path.join(root, "tests", "rows_walk_driver.cpp"), "-o", exe],
                       check=True, capture_output=True)
        return exe

    clean = build(0)
    for c in cases:
        r = subprocess.run([clean, *c], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.startswith("OK"), (c, r.stdout)
    for plant in (5, 6):
        exe = build(plant)
        results = [subprocess.run([exe, *c], capture_output=True, text=True) for c in cases]
        assert any(r.returncode == 1 and "FAIL" in r.stdout for r in results), plant


def test_the_walk_of_the_staged_tile_fetchers_notices_planted_mistakes(tmp_path):
    """Same for the fetchers of the aligned staged-tile kernels, which the walk runs on the CPU as they are: the
    gathered pixels one column to the right, rows beyond the problem loaded instead of cut off."""
    import os
    import shutil
    import subprocess
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc to compile the driver with")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    csrc = os.path.join(root, "paper_2002_02885_amd", "csrc")
    # bf16, stride, B, H, W, Cin, Cout (the last case: 96 output channels, a ragged column tile)
    cases = [("1", "1", "2", "16", "16", "64", "64"), ("1", "2", "3", "16", "16", "64", "128"), ("0", "1", "2", "8", "8", "32", "96"),
             ("0", "2", "1", "12", "12", "32", "64")]

    def build(plant):
        exe = str(tmp_path / f"fetch{plant}")
        subprocess.run([hipcc, "-x", "hip", "--cuda-host-only", "-std=c++17", "-O1", f"-DPACK_HALO_PLANT={plant}", "-I", csrc,
                        os.path.join(csrc, "gemm_fetch_check.cpp"), os.path.join(root, "tests", "fetch_walk_driver.cpp"), "-o", exe],
                       check=True, capture_output=True)
        return exe

    clean = build(0)
    for c in cases:
        r = subprocess.run([clean, *c], capture_output=True, text=True)
        assert r.returncode == 0 and r.stdout.startswith("OK"), (c, r.stdout)
    for plant in (7, 8):
        exe = build(plant)
        results = [subprocess.run([exe, *c], capture_output=True, text=True) for c in cases]
        assert any(r.returncode == 1 and "FAIL" in r.stdout for r in results), plant
