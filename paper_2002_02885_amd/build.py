"""Builds libpack.so for gfx950 with hipcc (cross-compiles without a GPU)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpack.so")
SOURCES = ["pack_kernels.hip", "pack_conv_dw.hip", "conv_dw_halo_check.cpp", "conv_rows_halo_check.cpp", "gemm_fetch_check.cpp", "pack_api.cpp", "pack_schedule.cpp", "pack_search.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-pthread",
         # do not generate packed-fp32 instructions (v_pk_*_f32)
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         # per-kernel register report, checked below
         "-Rpass-analysis=kernel-resource-usage"]


def check_no_spills(report: str) -> int:
    """The GEMM kernels issue their operand loads as assembly statements whose completion the
    compiler does not track.  That is only sound while no register such a load targets is
    spilled or copied before the hand-placed wait, so the build refuses kernels that spill:
    scratch must be 0 and the accumulation registers (AGPRs) must hold the MFMA accumulators
    only: 16 per 32x32 block, (BM/64) * (BN/64) blocks per wave.  Returns the number of GEMM
    kernels checked."""
    import re
    name, checked = None, 0
    agprs = None
    for line in report.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name, agprs = m.group(1), None
            continue
        if name is None or not any(k in name for k in ("gemm_kernel", "conv_dw_halo_kernel", "conv_rows_halo_kernel")):
            continue
        m = re.search(r"AGPRs: (\d+)", line)
        if m:
            agprs = int(m.group(1))
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m:
            t = re.search(r"gemm_kernelILi\d+E[tf]Li(\d+)ELi(\d+)E", name)
            # halo form of the convolution weight gradient: nine 32x32 blocks (one per tap) per wave
            want = 16 * (int(t.group(1)) // 64) * (int(t.group(2)) // 64) if t else 16 * 9
            if not t and agprs == 0:
                want = 0   # these keep their accumulator blocks in ordinary registers (no more than five, or four, per wave)
            r = re.search(r"conv_rows_halo_kernelILi\d+E[tf]Li\d+ELi\d+ELi(\d+)E", name)
            if r:   # two blocks of pixels x TN blocks of columns per wave, in AGPRs or all in ordinary registers
                want = 0 if agprs == 0 else 32 * int(r.group(1))
            if int(m.group(1)) != 0 or agprs != want:
                raise RuntimeError(f"{name}: scratch {m.group(1)} bytes, {agprs} AGPRs (accumulators need {want}): "
                                   "the kernel spills; the assembly-load pipeline would be unsound")
            checked += 1
            name = None
    return checked


def build(verbose: bool = False) -> str:
    """Compiles every source to an object (in parallel, keeping the device assembly), checks the register
    report and the assembly of the kernels with hand-placed waits, and links the library."""
    import concurrent.futures
    import shutil
    import tempfile
    from . import isa_check
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = tempfile.mkdtemp(prefix="libpack_build_")
    noise = ("is not a recognized feature for this target", "-Rpass-analysis=kernel-resource-usage")

    def compile_one(src):
        obj = os.path.join(tmp, os.path.splitext(src)[0] + ".o")
        cmd = [hipcc] + [f for f in FLAGS if f not in ("-shared", "-pthread")] + ["-save-temps=obj", "-c", os.path.join(CSRC, src), "-o", obj]
        res = subprocess.run(cmd, capture_output=True, text=True, cwd=tmp)
        err = "\n".join(l for l in res.stderr.splitlines() if not any(n in l for n in noise))
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n" + err)
        return obj, res.stderr, err

    try:
        with concurrent.futures.ThreadPoolExecutor(max_workers=len(SOURCES)) as ex:
            results = list(ex.map(compile_one, SOURCES))
        n = sum(check_no_spills(report) for _, report, _ in results)
        if n < 48 + 6 + 8:
            raise RuntimeError(f"register report covered only {n} matrix-product kernels")
        n_asm = 0
        for f in sorted(os.listdir(tmp)):
            if f.endswith("gfx950.s"):
                n_asm += isa_check.check_assembly(open(os.path.join(tmp, f)).read())
        if n_asm < n:
            raise RuntimeError(f"assembly check covered only {n_asm} of {n} matrix-product kernels")
        if verbose:
            for _, _, err in results:
                for line in err.splitlines():
                    if "warning:" in line or "error:" in line:
                        print(line, file=sys.stderr)
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-pthread"] + [o for o, _, _ in results] + ["-o", LIB + ".tmp"]
        res = subprocess.run(link, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n" + res.stderr)
        os.replace(LIB + ".tmp", LIB)
    finally:
        shutil.rmtree(tmp, ignore_errors=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
