"""The build's guard for linear_skinny_2bit (csrc/linear_skinny.hip): that kernel retires its LDS-DMA copies with a
counted s_waitcnt, which is right only while copies and weight loads are issued in source order.  The guard reads the
device assembly the shipped object was assembled from; here its parser is run on canned text, good and bad, and on the
assembly of the current build."""
import os

import pytest

from paper_2402_17764_amd import build as Bld


def _kernel(params, prologue, loops, name="linear_skinny_2bit"):
    mangled = "_ZN6bitnet%d%sILi%sE" % (len(name), name, "ELi".join(str(p) for p in params))
    copy = "\tbuffer_load_dwordx4 v1, s[4:7], 0 offen lds\n"
    weight = "\tbuffer_load_dwordx4 v[2:5], v6, s[8:11], 0 offen\n"
    emit = lambda seq: "".join(copy if c == "L" else weight for c in seq)
    text = mangled + "EvPKaPKfPK15HIP_vector_typeIjLj4EES4_iilliiiPvNS_7OutTypeE:\n\ts_load_dwordx2 s[0:1], s[4:5], 0x0\n"
    text += emit(prologue) + "\ts_waitcnt vmcnt(3)\n"
    for seg in loops:
        text += "\ts_barrier\n" + emit(seg) + "\tv_mfma_i32_16x16x64_i8 v[0:3], v[4:7], v[8:11], v[0:3]\n"
    return text + "\ts_barrier\n\ts_endpgm\n"


def test_issue_order_parser_accepts_source_order_and_rejects_everything_else():
    p = (2, 2, 2, 4, 2, 2)                      # kMT, kR, kW, kS, kD, kLx: 4 copies then 2 weight loads per step, prologue of 2
    unit = "LLLL" + "WW"
    good = _kernel(p, unit * 2, [unit, unit])
    assert Bld.check_issue_order(good, [p]) == [p]
    # a weight load hoisted above the last copy of the prologue, and one in the loop
    for bad in (_kernel(p, "LLLWLW" + unit, [unit]), _kernel(p, unit * 2, [unit, "LLWLLW"]), _kernel(p, unit, [unit]),
                _kernel(p, unit * 2, [])):
        with pytest.raises(RuntimeError):
            Bld.check_issue_order(bad, [p])
    # an expected instantiation that the assembly does not hold, one it holds unasked, and a truncated kernel
    with pytest.raises(RuntimeError):
        Bld.check_issue_order(good, [p, (1, 1, 1, 8, 2, 2)])
    with pytest.raises(RuntimeError):
        Bld.check_issue_order(good + _kernel((1, 1, 1, 8, 2, 2), "LLLLW" * 2, ["LLLLW"]), [p])
    with pytest.raises(RuntimeError):
        Bld.check_issue_order(good.replace("\ts_endpgm\n", ""), [p])
    with pytest.raises(RuntimeError):
        Bld.check_issue_order("", [p])
    # other kernels in the same file are not its business
    other = _kernel(p, "WWLL", ["WL"], name="linear_skinny_ws_2bit")
    assert Bld.check_issue_order(other + good, [p]) == [p]


def test_dispatched_instantiations_are_read_from_the_launcher():
    src = open(os.path.join(Bld.CSRC, "linear_skinny.hip")).read()
    inst = Bld.skinny_instantiations(src)
    assert len(inst) >= 10 and all(len(t) == 6 for t in inst)
    assert Bld.skinny_instantiations("if (a) SKINNY(1, 2, 3, 4, 5, 6); else SKINNY(1, 2, 3, 4, 5, 6);") == [(1, 2, 3, 4, 5, 6)]


def test_current_build_passes_the_guard():
    asm = os.path.join(Bld.BUILD, "linear_skinny-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(asm):
        pytest.skip("no build directory here (the library was built elsewhere)")
    src = open(os.path.join(Bld.CSRC, "linear_skinny.hip")).read()
    checked = Bld.check_issue_order(open(asm).read(), Bld.skinny_instantiations(src))
    assert sorted(checked) == Bld.skinny_instantiations(src)
