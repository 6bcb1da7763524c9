"""Build hygiene for the device code.

On MI355X a kernel of this library returned wrong words now and then when a 64-bit shift
(v_lshlrev_b64 / v_lshrrev_b64 / v_ashrrev_i64) took its amount from the last vector register of the
kernel's allocation (v47 of 48; registers are handed out eight at a time): the shift then behaved as
if the amount were the lane number, which is what the register after it holds when a newly started
wavefront is its neighbour in the register file.  The same shifts by other registers of the same
kernel were always right.  The kernel has been restructured since and no longer shows the pattern,
but nothing in the source can forbid it: this test reads the generated code of every kernel, so that a
later change of the register allocation cannot bring it back unnoticed.
"""
import os
import re
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import __graft_entry__ as entry  # noqa: E402

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SHIFT = re.compile(r"\bv_(?:lshlrev_b64|lshrrev_b64|ashrrev_i64)(?:_e64)? v\[\d+:\d+\], v(\d+),")


def device_listing(src, out):
    flags = [f for f in entry.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    cmd = [HIPCC] + flags + ["--cuda-device-only", "-S", "-o", out, os.path.join(entry.CSRC, src)]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout
    return open(out).read()


def kernels_of(listing):
    for part in re.split(r"\n(?=\t\.globl\t)", listing):
        name = re.search(r"\.globl\t(\S+)", part)
        nvgpr = re.search(r"\.amdhsa_next_free_vgpr (\d+)", part)
        if name and nvgpr:
            yield name.group(1), int(nvgpr.group(1)), part


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not installed")
def test_no_wide_shift_takes_its_amount_from_the_last_vector_register():
    with tempfile.TemporaryDirectory() as tmp:
        with ThreadPoolExecutor(max_workers=4) as pool:
            listings = list(pool.map(lambda s: device_listing(s, os.path.join(tmp, s + ".s")), entry.SOURCES))
    seen = 0
    for src, listing in zip(entry.SOURCES, listings):
        for name, nvgpr, body in kernels_of(listing):
            seen += 1
            amounts = {int(m.group(1)) for m in SHIFT.finditer(body)}
            last = (nvgpr + 7) // 8 * 8 - 1              # last register of the allocation, in eights
            assert last not in amounts, f"{src}: {name} shifts 64 bits by v{last}, the last register it holds"
    assert seen >= 10          # the listings were parsed: the library has more kernels than that
