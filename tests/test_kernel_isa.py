"""Build-time checks of the compiled GEMM kernels (gfx950 assembly as hipcc emits it for the library's own
sources with the library's own flags; nothing runs on a GPU).

The 4-wave GEMM kernel writes its MFMAs as inline assembly, so the compiler no longer sees their data
hazards, and both GEMM sources write the M0 register behind the compiler's back for their asynchronous
global -> LDS copies.  What the source guarantees by construction is checked here in the instruction stream
of every instantiation, so that a compiler upgrade or a changed flag that breaks an assumption fails the
test suite instead of corrupting results:

  1. every MFMA of gemm_kernel4 accumulates in place in the accumulation registers (destination = addend,
     the form whose back-to-back dependency the hardware interlocks) and no two MFMAs use overlapping but
     different accumulator ranges;
  2. the same accumulator is not touched again by anything but its own MFMA inside the main loop (no copies
     in and out of the accumulation registers around the MFMAs);
  3. on every control-flow path from the last MFMA, at least 19 wait states (the requirement for the
     longest, 16-pass, matrix instruction; the 16x16x32 bf16 one needs fewer) pass before the first
     instruction other than an MFMA that reads or writes an accumulation register;
  4. M0 is written only by the copy sequence (s_mov_b32 m0 / s_nop 0 / global_load_lds_*) and read by
     nothing else, in gemm.hip and mx.hip;
  5. no vector memory instruction reads a scalar register that a vector instruction (v_readlane,
     v_readfirstlane, a compare with a scalar destination) wrote fewer than 5 wait states earlier.  The
     compiler keeps that distance for its own instructions but does not look into inline assembly, and the
     copies take their base address in scalar registers: a spilled scalar restored right in front of one
     would make it read a stale address.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2407_00952_amd import build as libbuild

CSRC = libbuild.CSRC
MIN_WAIT_STATES = 19


def _assembly(src):
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "k.s")
        cmd = ["hipcc", *[f for f in libbuild.FLAGS if f != "-fPIC"], "--cuda-device-only", "-S",
               os.path.join(CSRC, src), "-o", out]
        p = subprocess.run(cmd, capture_output=True, text=True)
        assert p.returncode == 0, p.stderr[-2000:]
        return open(out).read()


def _functions(text):
    """{mangled name: [instruction lines]} for every kernel in an assembly file (labels kept, comments dropped)."""
    funcs, name, body = {}, None, []
    for line in text.splitlines():
        m = re.match(r"^(_Z\w+):", line)
        if m:
            name, body = m.group(1), []
            continue
        if name is None:
            continue
        if line.startswith(".Lfunc_end"):
            funcs[name] = body
            name = None
            continue
        code = line.split(";")[0].rstrip()
        if not code.strip() or code.strip().startswith((".", "//")) and not re.match(r"^\.L\w+:", code.strip()):
            continue
        body.append(code.strip())
    return funcs


def _is_label(ins):
    return ins.endswith(":")


def _wait_states(ins):
    if _is_label(ins):
        return 0
    m = re.match(r"s_nop\s+(\d+)", ins)
    return int(m.group(1)) + 1 if m else 1


_AGPR = re.compile(r"\ba(\d+)\b|\ba\[(\d+):(\d+)\]")


def _agprs(ins):
    regs = set()
    for m in _AGPR.finditer(ins):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


@pytest.fixture(scope="module")
def gemm_asm():
    return _assembly("gemm.hip")


def test_four_wave_gemm_mfma_hazards(gemm_asm):
    funcs = {n: b for n, b in _functions(gemm_asm).items() if "gemm_kernel4" in n}
    assert len(funcs) == 10, sorted(funcs)         # five epilogues x two tile heights
    for name, body in funcs.items():
        ni = int(re.search(r"gemm_kernel4ILi\d+ELi(\d+)E", name).group(1))      # 16-row MFMA tiles per wave along M
        assert ni in (4, 8), name
        mf = [(i, ins) for i, ins in enumerate(body) if ins.startswith("v_mfma")]
        # the unrolled loop body: 2 k-steps x (ni x 8) MFMAs
        assert len(mf) == 2 * 8 * ni, (name, len(mf))
        ranges = []
        for _, ins in mf:
            m = re.match(r"v_mfma_f32_16x16x32_bf16 a\[(\d+):(\d+)\], v\[\d+:\d+\], v\[\d+:\d+\], a\[(\d+):(\d+)\]$", ins)
            assert m, (name, ins)
            d0, d1, c0, c1 = map(int, m.groups())
            assert (d0, d1) == (c0, c1) and d1 - d0 == 3 and d0 % 4 == 0, (name, ins)      # (1) in place, aligned
            ranges.append(d0)
        # ni x 8 distinct accumulators per k-step, the same ones in both: a register is written again that many
        # MFMAs later at the earliest and ranges never overlap partially
        half = 8 * ni
        assert sorted(ranges[:half]) == sorted(ranges[half:]) and len(set(ranges[:half])) == half, name
        first, last = mf[0][0], mf[-1][0]
        # (2) nothing else touches an accumulation register between the first and the last MFMA
        for ins in body[first:last + 1]:
            if not ins.startswith("v_mfma"):
                assert not _agprs(ins), (name, ins)
        # (3) every path from the last MFMA to an access of an accumulation register that is not an MFMA
        worst, where = _min_wait_states_to_acc_access(body, last)
        assert worst >= MIN_WAIT_STATES, (name, worst, where)


def _min_wait_states_to_acc_access(body, start):
    """Follow every control-flow path from the instruction after body[start]; a path ends at the next MFMA
    (inside the loop nothing else touches the accumulators, check 2), at s_endpgm, or once it has collected
    the required wait states.  Returns the fewest wait states in front of any other instruction that reads
    or writes an accumulation register, and that instruction."""
    labels = {ins[:-1]: i for i, ins in enumerate(body) if _is_label(ins)}
    best = {}
    worst, where = 10 ** 9, None
    todo = [(start + 1, 0)]
    while todo:
        i, ws = todo.pop()
        while i < len(body):
            if ws >= MIN_WAIT_STATES or best.get(i, 10 ** 9) <= ws:
                break
            best[i] = ws
            ins = body[i]
            if ins.startswith("v_mfma") or ins.startswith("s_endpgm"):
                break
            if _agprs(ins):
                if ws < worst:
                    worst, where = ws, ins
                break
            m = re.match(r"s_(c?)branch\w*\s+(\S+)", ins)
            ws += _wait_states(ins)
            if m:
                assert m.group(2) in labels, ins
                todo.append((labels[m.group(2)], ws))
                if not m.group(1):                  # unconditional: no fall-through
                    break
            i += 1
    return (worst if where is not None else MIN_WAIT_STATES), where


def _check_m0(text, what):
    for name, body in _functions(text).items():
        code = [ins for ins in body if not _is_label(ins)]
        for i, ins in enumerate(code):
            if not re.search(r"\bm0\b", ins):
                continue
            if re.match(r"s_mov_b32 m0, s\d+$", ins):
                assert code[i + 1] == "s_nop 0" and code[i + 2].startswith("global_load_lds_dword"), \
                    (what, name, code[i:i + 3])
            else:
                raise AssertionError("%s: %s: M0 used outside the copy sequence: %s" % (what, name, ins))
        # the copies read M0 implicitly: each one must be preceded by the write that belongs to it
        for i, ins in enumerate(code):
            if ins.startswith("global_load_lds_dword"):
                assert i >= 2 and code[i - 1] == "s_nop 0" and code[i - 2].startswith("s_mov_b32 m0,"), \
                    (what, name, code[max(i - 2, 0):i + 1])


def test_m0_is_only_used_by_the_async_copies(gemm_asm):
    _check_m0(gemm_asm, "gemm.hip")
    _check_m0(_assembly("mx.hip"), "mx.hip")


_SREG = re.compile(r"\bs(\d+)\b|\bs\[(\d+):(\d+)\]")
_VMEM = ("global_load", "global_store", "global_atomic", "buffer_load", "buffer_store", "scratch_load", "scratch_store")


def _sregs(text):
    regs = set()
    for m in _SREG.finditer(text):
        if m.group(1) is not None:
            regs.add(int(m.group(1)))
        else:
            regs.update(range(int(m.group(2)), int(m.group(3)) + 1))
    return regs


def _valu_scalar_dest(ins):
    """Scalar registers written by a vector instruction (empty for everything else)."""
    op = ins.split()[0]
    if op.startswith(("v_readlane_b32", "v_readfirstlane_b32")) or (op.startswith("v_cmp") and op.endswith("_e64")):
        return _sregs(ins.split(None, 1)[1].split(",")[0])
    return set()


def _check_valu_sgpr_to_vmem(text, what):
    for name, body in _functions(text).items():
        code = [ins for ins in body if not _is_label(ins)]
        for i, ins in enumerate(code):
            if not ins.startswith(_VMEM):
                continue
            used = _sregs(ins)
            if not used:
                continue
            ws, j = 0, i - 1
            while j >= 0 and ws < 5:
                hit = _valu_scalar_dest(code[j]) & used
                assert not hit, (what, name, code[j], ins, "only %d wait states between" % ws)
                ws += _wait_states(code[j])
                j -= 1


def test_vector_written_scalars_are_settled_before_vector_memory_reads_them(gemm_asm):
    _check_valu_sgpr_to_vmem(gemm_asm, "gemm.hip")
    _check_valu_sgpr_to_vmem(_assembly("mx.hip"), "mx.hip")
    _check_valu_sgpr_to_vmem(_assembly("attention.hip"), "attention.hip")


def test_the_scalar_hazard_check_sees_a_planted_hazard():
    bad = ("_Z3foov:\n\tv_readlane_b32 s0, v255, 16\n\tv_readlane_b32 s1, v255, 17\n\tv_readlane_b32 s51, v255, 19\n"
           "\tglobal_load_dwordx4 v[178:181], v221, s[0:1]\n\ts_endpgm\n.Lfunc_end0:\n")
    with pytest.raises(AssertionError):
        _check_valu_sgpr_to_vmem(bad, "planted")
    _check_valu_sgpr_to_vmem(bad.replace("\tglobal_load", "\ts_nop 4\n\tglobal_load"), "planted, with wait states")
