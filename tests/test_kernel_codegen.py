"""The many-row GEMM places loads, waits and MFMAs by hand: activation fragments are read from LDS by
instructions the compiler does not know to be loads, and the register a read lands in must stay that value's
register until the hand-placed wait.  That holds as long as the compiler neither spills in that kernel nor copies
registers inside its tile loop.  This test compiles the bf16 kernels to assembly with the library's flags and
checks exactly that for every instantiation (no GPU needed)."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2408_08146_amd", "csrc")
OUT = os.path.join(ROOT, "_build", "kernels_bf16.s")


def _assembly():
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(hipcc):
        pytest.skip("hipcc not available")
    from paper_2408_08146_amd.build import FLAGS
    src = os.path.join(CSRC, "kernels_bf16.hip")
    deps = [src, os.path.join(CSRC, "koala_internal.h"), os.path.join(ROOT, "include", "koala.h")]
    if not os.path.exists(OUT) or os.path.getmtime(OUT) < max(os.path.getmtime(d) for d in deps):
        os.makedirs(os.path.dirname(OUT), exist_ok=True)
        flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
        res = subprocess.run([hipcc, *flags, "--cuda-device-only", "-S", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
                              src, "-o", OUT], capture_output=True, text=True)
        assert res.returncode == 0, res.stderr[-2000:]
    return open(OUT).read().splitlines()


def test_many_row_gemm_has_no_spills_and_no_register_copies_in_its_tile_loop():
    lines = _assembly()
    starts = [i for i, l in enumerate(lines) if re.match(r"^_ZN\S*k_gemm_big\S*:", l)]
    assert len(starts) >= 8, "the many-row GEMM's instantiations were not found in the assembly"
    for s in starts:
        name = lines[s].split(":")[0]
        end = next(i for i in range(s, len(lines)) if lines[i].startswith("\t.amdhsa_kernel " + name))
        desc = lines[end:end + 80]
        scratch = next(int(l.split()[-1]) for l in desc if ".amdhsa_private_segment_fixed_size" in l)
        assert scratch == 0, f"{name} spills {scratch} bytes per lane"
        body = lines[s:end]
        assert not any("scratch_" in l for l in body), f"{name} uses scratch memory"
        # a tile = the code from its barrier to the last of its 2 * U * MTW MFMAs (the kernel's name carries U, MTW)
        U, MTW = (int(v) for v in re.search(r"k_gemm_bigILi(\d+)ELi(\d+)E", name).groups())
        per_tile = 2 * U * MTW
        tiles = 0
        for b in (i for i, l in enumerate(body) if l.strip() == "s_barrier"):
            seen, e = 0, b + 1
            while e < len(body) and seen < per_tile and body[e].strip() != "s_barrier":
                seen += "v_mfma_f32_16x16x32_f16" in body[e]
                e += 1
            if seen < per_tile:
                continue                      # the barrier before the epilogue
            tiles += 1
            tile = body[b:e]
            assert sum("ds_read_b128" in l for l in tile) == 2 * MTW
            copies = [l.strip() for l in tile
                      if re.match(r"^\s*v_mov_b32(_e32)?\s+v\d+,\s*v\d+", l)
                      or re.match(r"^\s*v_accvgpr_read", l)
                      or re.match(r"^\s*v_accvgpr_write_b32\s+a\d+,\s*v\d+", l)]
            assert not copies, f"{name} copies registers inside a tile: {copies[:4]}"
        assert tiles >= 4, f"{name}: found {tiles} tile bodies"
