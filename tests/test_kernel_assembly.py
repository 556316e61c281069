"""Host-side check of the compiled kernels: registers that the dense path loads behind the compiler's
back (queued between asynchronous copies, waited for by hand) are named by no instruction between their
load and the statement that releases them, on any path through the generated gfx950 assembly."""
import re

import pytest

from paper_2505_17694_amd import check_pending_loads as chk


@pytest.fixture(scope="module")
def assembly():
    return chk.assembly()


def test_no_instruction_touches_a_register_that_is_still_being_loaded(assembly):
    asm = assembly
    loads, marks, bad = chk.check(asm)
    # per instantiation of the dense path (2 element types x 2 live roles x 2 strides): 8 loads, 1 release
    assert loads == 64 and marks == 8, (loads, marks)
    assert not bad, bad[:10]


def test_the_check_sees_a_planted_copy(assembly):
    """A copy of a pending register planted behind the first label after a load sequence is reported."""
    asm = assembly.splitlines()
    is_load = lambda i: chk._LOAD.match(asm[i]) and asm[i - 1].strip() == ";;#ASMSTART"
    first = next(i for i in range(1, len(asm)) if is_load(i))
    reg = int(re.match(r"v\[(\d+):", chk._LOAD.match(asm[first]).group(1)).group(1))
    j, seen = first, 0
    while seen < 8:
        seen += bool(is_load(j))
        j += 1
    while not asm[j].startswith(".LBB"):
        j += 1
    asm.insert(j + 1, f"\tv_mov_b32_e32 v250, v{reg}")
    _, _, bad = chk.check("\n".join(asm))
    assert [code for _, code in bad] == [f"v_mov_b32_e32 v250, v{reg}"]
