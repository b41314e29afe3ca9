"""What the grouped contraction assumes of the code the compiler makes from it, checked on the generated assembly
(no GPU: hipcc cross-compiles gfx950).

* M0 holds the LDS base of the direct-to-LDS tile loads and is written once per four loads, by assembly statements:
  the compiler must have no use of its own for it in these kernels.
* The statistics kernel keeps everything in registers: no scratch memory (a scratch reload would count on the same
  in-order counter as the tile loads and stall the K loop's waits).
* The K loop of a full tile holds its accumulators still: no copies between accumulation and vector registers,
  128 MFMAs per K tile, one barrier.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2508_02322_amd", "csrc")


@pytest.fixture(scope="module")
def gemm_asm(tmp_path_factory):
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not found")
    from paper_2508_02322_amd import build
    out = tmp_path_factory.mktemp("asm") / "gemm.s"
    flags = [f for f in build.FLAGS if f != "-fPIC"]
    cmd = [hipcc, *flags, "-I" + os.path.join(ROOT, "include"), "--cuda-device-only", "-S",
           os.path.join(CSRC, "gemm.hip"), "-o", str(out)]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr[-2000:]
    return out.read_text()


def _functions(asm):
    """name -> body of every bf16 contraction kernel."""
    out = {}
    for chunk in re.split(r"\n(?=_Z\w+:\s)", asm):
        m = re.match(r"(_Z\w+):", chunk)
        if m and "grouped_gemm_bf16" in m.group(1):
            out[m.group(1)] = chunk
    return out


def test_m0_is_written_by_the_tile_loads_only(gemm_asm):
    kernels = _functions(gemm_asm)
    assert len(kernels) >= 6
    for name, body in kernels.items():
        inside = False
        for line in body.splitlines():
            if "#ASMSTART" in line:
                inside = True
            elif "#ASMEND" in line:
                inside = False
            elif not inside and re.search(r"\bm0\b", line.split(";")[0]):
                raise AssertionError(f"{name}: the compiler touches M0 outside the tile loads: {line.strip()}")


def test_statistics_kernel_uses_no_scratch(gemm_asm):
    found = 0
    for m in re.finditer(r"\.name:\s+(\S+).*?\.private_segment_fixed_size:\s+(\d+)", gemm_asm, re.S):
        name, scratch = m.group(1), int(m.group(2))
        if "grouped_gemm_bf16_kernel" in name and re.search(r"Lb[01]ELi0E", name):   # <TAIL, epilogue 0>
            found += 1
            assert scratch == 0, f"{name}: {scratch} bytes of scratch per lane"
    assert found == 2


def test_full_tile_loop_keeps_its_accumulators_in_place(gemm_asm):
    for name, body in _functions(gemm_asm).items():
        if "compact" in name or "Lb0ELi0E" not in name:      # the scoring kernel, K a multiple of the K tile
            continue
        blocks = re.split(r"\n(?=\.LBB\d+_\d+:)", body)
        loop = max(blocks, key=lambda b: len(re.findall(r"\bv_mfma", b)))
        assert len(re.findall(r"\bv_mfma_f32_16x16x32_bf16", loop)) == 128
        assert len(re.findall(r"\bs_barrier", loop)) == 1
        assert not re.search(r"\bv_accvgpr_(read|write|mov)", loop), "accumulator copies inside the K loop"
        assert not re.search(r"\bscratch_", loop)
        assert len(re.findall(r"\bglobal_load_lds_dwordx4", loop)) == 16
        assert len(re.findall(r"s_mov_b32 m0", loop)) == 4
        return
    raise AssertionError("scoring kernel not found")
