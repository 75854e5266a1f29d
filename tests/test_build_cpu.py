"""Checks on the compiled device code that need no GPU."""
import re

import pytest

from paper_2502_12784_amd import build


@pytest.fixture(scope="module")
def asm():
    return build.device_assembly()[0]


def test_every_direct_lds_load_carries_its_hazard_guard(asm):
    """The global->LDS loads are inline assembly, invisible to the compiler's hazard handling: each
    must be preceded by the five wait states that separate it from a VALU write of the scalar
    registers (descriptor, offset, M0) it reads."""
    loads = re.findall(r"buffer_load_dword(?:x4)? .* lds", asm)
    assert len(loads) > 500          # every attention kernel uses them
    assert build.unguarded_lds_loads(asm) == []


def test_no_packed_fp32_arithmetic(asm):
    """The library is built with packed fp32 operations switched off."""
    assert not re.search(r"\bv_pk_(add|mul|fma)_f32\b", asm)


def test_tile_loops_do_not_spill():
    table = build.kernel_resources()
    rows = [l.split() for l in table.splitlines() if l.startswith("mha_")]
    assert len(rows) > 60
    assert all(r[-1] == "0" for r in rows), [r for r in rows if r[-1] != "0"]
