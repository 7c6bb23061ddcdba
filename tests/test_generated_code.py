"""A scan of the device code the compiler generates for the kernels (no GPU needed).

gfx950 returned garbage from a 64-bit shift whose amount sat in the last VGPR of the wave's register
allocation while other waves shared the SIMD (the erratum the compiler rewrites for gfx90a; it does
not for this target), and which register holds the amount is the register allocator's choice.  So
the kernels contain no 64-bit shift by a register amount at all, and this test keeps it that way."""
import re
import shutil
import subprocess

import pytest

from paper_2502_20566_amd import build as Bld


@pytest.mark.skipif(shutil.which(Bld.HIPCC) is None, reason="hipcc not installed")
def test_no_64_bit_shift_by_a_register_amount(tmp_path):
    out = tmp_path / "device.s"
    flags = [f for f in Bld.FLAGS if f not in ("-shared", "-fPIC")]
    subprocess.run([Bld.HIPCC, *flags, "--cuda-device-only", "-S", *Bld.SOURCES, "-o", str(out)],
                   check=True, capture_output=True)
    text = out.read_text()
    assert text.count("s_endpgm") > 20                       # the kernels are all there
    shifts = re.findall(r"^\s*(v_(?:lshl|lshr|ashr)rev_b64)\s+v\[\d+:\d+\],\s*([^,\s]+),", text, flags=re.M)
    assert shifts, "expected the constant-amount shifts of the address arithmetic"
    by_register = [(op, amt) for op, amt in shifts if not re.fullmatch(r"-?\d+|0x[0-9a-fA-F]+", amt)]
    assert by_register == []
