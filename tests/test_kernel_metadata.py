"""The paper's register-budget lesson (Sec. 5.4 and the spilling experiment of
Sec. 6.3): a GEMM kernel must never spill.  Checked on the compiled code object
without a GPU: every gemm kernel has zero scratch and zero spilled registers,
and fits the 256-register budget that lets two waves share a SIMD."""
import os
import re
import subprocess

import pytest

import paper_1611_08035_amd as xg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
READELF = "/opt/rocm/llvm/bin/llvm-readelf"
BUNDLER = "/opt/rocm/llvm/bin/clang-offload-bundler"


def kernel_metadata():
    """Parse the AMDGPU metadata note of the gfx950 code object embedded in libxgemm.so."""
    lib = xg.library_path()
    if not (os.path.exists(READELF) and os.path.exists(BUNDLER) and os.path.exists(lib)):
        pytest.skip("llvm tools or library not available")
    import tempfile
    notes = ""
    with tempfile.TemporaryDirectory() as td:
        fat = os.path.join(td, "fat.bin")
        subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", lib, fat], check=True)
        blob = open(fat, "rb").read()
        magic = b"__CLANG_OFFLOAD_BUNDLE__"
        starts = [m.start() for m in re.finditer(re.escape(magic), blob)]
        assert starts, "no offload bundle in the library"
        # one bundle per translation unit, concatenated in the section
        for n, (a, b) in enumerate(zip(starts, starts[1:] + [len(blob)])):
            part = os.path.join(td, f"bundle{n}.bin")
            co = os.path.join(td, f"gfx950_{n}.co")
            open(part, "wb").write(blob[a:b])
            r = subprocess.run([BUNDLER, "--list", "--type=o", "--input=" + part], capture_output=True, text=True)
            targets = [t for t in r.stdout.split() if "gfx950" in t]
            if not targets:
                continue
            subprocess.run([BUNDLER, "--unbundle", "--type=o", "--input=" + part, "--targets=" + targets[0],
                            "--output=" + co], check=True)
            notes += subprocess.run([READELF, "--notes", co], capture_output=True, text=True, check=True).stdout
    kernels = []
    for blk in notes.split("- .agpr_count:")[1:]:
        d = {"agpr_count": int(blk.split("\n")[0].strip())}
        for key in ("name", "vgpr_count", "vgpr_spill_count", "sgpr_spill_count", "private_segment_fixed_size"):
            m = re.search(r"\.%s:\s+(\S+)" % key, blk)
            d[key] = m.group(1) if m else None
        kernels.append(d)
    return kernels


def test_gemm_kernels_never_spill():
    ks = [k for k in kernel_metadata() if k["name"] and "gemm_kernel" in k["name"]]
    assert len(ks) >= 40, "expected every tile variant x transpose pair (+ the fallback path)"
    for k in ks:
        assert int(k["vgpr_spill_count"]) == 0, k
        assert int(k["sgpr_spill_count"] or 0) == 0, k
        assert int(k["private_segment_fixed_size"]) == 0, k
        assert int(k["vgpr_count"]) <= 256 and k["agpr_count"] == 0, k


def test_no_kernel_of_the_library_uses_scratch_memory():
    """The block kernels of the level-3 routines hold whole tiles and panels in registers;
    none of them (nor any other kernel) may fall back to scratch memory for them."""
    ks = [k for k in kernel_metadata() if k["name"]]
    assert len(ks) >= 80
    for k in ks:
        assert int(k["vgpr_spill_count"]) == 0, k
        assert int(k["private_segment_fixed_size"]) == 0, k
