"""Static check of the pipelined attention kernel's machine code (no GPU needed).

The pipelined steps issue their matrix and vector instructions through inline assembly, so the
compiler's hazard recogniser does not see them.  On gfx950 the result of a 32x32x16 matrix
instruction (8 passes) must not be read by a vector instruction, nor copied out of an accumulation
register, for 11 wait states after issue, and the hardware does not interlock this.  The source
keeps every such pair three or more slots apart; this test compiles the kernel to assembly and
verifies it on what the compiler actually emitted: between a matrix instruction and the first
non-matrix instruction that reads (or overwrites) any register of its result there are at least
`MIN_GAP` issued instructions (an `s_nop n` counts n + 1), along every path of the control flow."""
import os
import re
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(ROOT, "paper_2601_08743_amd", "csrc", "prefill_attn_bf16.hip")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
MIN_GAP = 12
KERNEL = "attn_bf16_pipe_kernel"

_REG = re.compile(r"\b([va])\[(\d+):(\d+)\]|\b([va])(\d+)\b")


def _regs(text):
    """Set of (file, index) registers named in an operand string."""
    out = set()
    for m in _REG.finditer(text):
        if m.group(1):
            out.update((m.group(1), i) for i in range(int(m.group(2)), int(m.group(3)) + 1))
        else:
            out.add((m.group(4), int(m.group(5))))
    return out


def _kernel_instructions(asm_text):
    """(op, operands) list of the kernel, and a map label -> index of the instruction that follows it."""
    lines = asm_text.splitlines()
    start = next(i for i, l in enumerate(lines) if re.match(r"^_ZN2tc\d+%s\w*:" % KERNEL, l))
    end = next(i for i in range(start, len(lines)) if lines[i].startswith(".Lfunc_end"))
    ins, labels = [], {}
    for l in lines[start + 1:end]:
        l = l.split(";")[0].strip()
        if not l or l.startswith("."):
            m = re.match(r"^(\.LBB\d+_\d+):", l)
            if m:
                labels[m.group(1)] = len(ins)
            continue
        if l.endswith(":"):
            continue
        op, _, rest = l.partition(" ")
        ins.append((op, rest.strip()))
    return ins, labels


@pytest.fixture(scope="module")
def instructions():
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC),
               "-S", "--cuda-device-only", SRC, "-o", out]
        subprocess.check_call(cmd, stderr=subprocess.DEVNULL)
        return _kernel_instructions(open(out).read())


def test_matrix_results_are_not_read_too_early(instructions):
    """Every path of the control-flow graph is followed from each matrix instruction (both ways at a
    conditional branch) until MIN_GAP wait states have passed, a barrier is met or the kernel ends."""
    ins, labels = instructions
    n_mfma, tightest = 0, [None]

    def walk(i0, op, rest, dst, j, gap, seen):
        while j < len(ins) and gap < MIN_GAP:
            if (j, gap) in seen:
                return
            seen.add((j, gap))
            op2, rest2 = ins[j]
            if op2.startswith("v_mfma"):
                gap += 1            # accumulating into the same registers is forwarded by the hardware
            elif op2 == "s_nop":
                gap += int(rest2) + 1
            elif op2 in ("s_endpgm", "s_barrier"):
                return              # a barrier or the end: far more than MIN_GAP cycles away
            elif op2 == "s_branch":
                j = labels[rest2.strip()]
                gap += 1
                continue
            elif op2.startswith("s_cbranch"):
                walk(i0, op, rest, dst, labels[rest2.strip()], gap + 1, seen)
                gap += 1
            elif _regs(rest2) & dst:
                assert gap >= MIN_GAP, "instruction %d (%s %s): result touched by '%s %s' after %d wait states" % (
                    i0, op, rest, op2, rest2, gap)
                return
            else:
                gap += 1
            j += 1

    for i, (op, rest) in enumerate(ins):
        if not op.startswith("v_mfma"):
            continue
        n_mfma += 1
        walk(i, op, rest, _regs(rest.split(",")[0]), i + 1, 0, set())
    assert n_mfma >= 32 * 5, "the pipelined steps were not found in the kernel"
    print("matrix instructions checked on all paths: %d" % n_mfma)


def test_pipelined_steps_keep_their_slot_structure(instructions):
    """In the two steady-state step bodies (one per parity) every matrix instruction is followed
    by the vector work of exactly one score before the next one: 31 gaps per body with exactly one
    `v_exp_f32` (the hand-placed one; the compiler's own are spelled v_exp_f32_e32).  This guards
    against the slots collapsing into blocks of matrix instructions, which would still compute the
    right thing but lose the overlap the schedule exists for."""
    gaps, cur, seen_mfma = [], 0, False
    for op, _ in instructions[0]:
        if op.startswith("v_mfma"):
            if seen_mfma:
                gaps.append(cur)
            cur, seen_mfma = 0, True
        elif op == "v_exp_f32":
            cur += 1
        elif op == "s_barrier":
            seen_mfma = False
    one = sum(1 for g in gaps if g == 1)
    print("gaps between matrix instructions holding exactly one hand-placed exp: %d" % one)
    assert one >= 2 * 31


def test_no_vector_write_right_in_front_of_a_hand_placed_matrix_instruction():
    """A matrix instruction must not read a register that a vector instruction wrote less than 2
    wait states earlier; the compiler keeps that rule for its own matrix instructions and cannot
    for those inside inline assembly.  The hand-written steps keep every such pair far apart, but
    the compiler's own moves can land there: a build of this kernel once reloaded a Q fragment from
    accumulation registers (v_accvgpr_read, a spill under register pressure) directly in front of
    the first QK instruction of a key-tile half, and short pipelined runs returned launch-dependent
    rows; two idle slots in front of the matrix instructions made them right again.  Checked on the
    emitted code of all kernels in the file: every matrix instruction inside an assembly statement,
    its three source operands, the two wait states in front of it."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(SRC),
                               "-S", "--cuda-device-only", SRC, "-o", out], stderr=subprocess.DEVNULL)
        raw = open(out).read().splitlines()
    ins, in_asm = [], False                     # (text, inside an assembly statement)
    for l in raw:
        t = l.strip()
        if t.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if t.startswith(";;#ASMEND"):
            in_asm = False
            continue
        t = t.split(";")[0].strip()
        if not t or t.startswith(".") or t.endswith(":"):
            continue
        ins.append((t, in_asm))
    n = 0
    for i, (t, in_asm) in enumerate(ins):
        if not (in_asm and t.startswith("v_mfma")):
            continue
        n += 1
        src = set()
        for part in t.split(None, 1)[1].split(",")[1:]:
            src |= _regs(part)
        gap, j = 0, i - 1
        while j >= 0 and gap < 2:
            op, _, rest = ins[j][0].partition(" ")
            if op == "s_nop":
                gap += int(rest) + 1
            else:
                if op.startswith("v_") and not op.startswith("v_mfma") and not op.startswith("v_cmp"):
                    assert not (_regs(rest.split(",")[0]) & src), "'%s' writes a source of '%s' %d wait states ahead of it" % (
                        ins[j][0], t, gap)
                gap += 1
            j -= 1
    assert n >= 32 * 5
    print("hand-placed matrix instructions checked: %d" % n)


def _sregs(text):
    out = set()
    for m in re.finditer(r"\bs\[(\d+):(\d+)\]|\bs(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def _device_asm(src):
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    path = os.path.join(ROOT, "paper_2601_08743_amd", "csrc", src)
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(path),
                               "-S", "--cuda-device-only", path, "-o", out], stderr=subprocess.DEVNULL)
        lines = [l.split(";")[0].strip() for l in open(out)]
    return [l for l in lines if l and not l.startswith(".")]


@pytest.mark.parametrize("src", ["prefill_attn_bf16.hip", "prefill_attn_pp_bf16.hip", "decode_attn_bf16.hip"])
def test_lds_loads_read_no_freshly_vector_written_scalar(src):
    """A vector-memory instruction must not read a scalar register that a vector instruction wrote
    less than 5 wait states earlier (no interlock), and the compiler cannot keep that rule for a load
    hidden in inline assembly (csrc/lds_dma.h): it puts the v_readfirstlane of a per-lane base right in
    front of the statement.  The statement copies the base with a scalar move of its own, so the
    nearest writer of every such load's base pair must be a scalar instruction (a scalar-written
    register may be used at once).  Checked on the emitted code."""
    lines = _device_asm(src)
    loads = [i for i, l in enumerate(lines) if l.startswith("global_load_lds")]
    assert loads, "no direct-to-LDS loads found in %s" % src
    for i in loads:
        base = _sregs(lines[i].split(None, 1)[1])
        assert len(base) == 2, lines[i]
        gap, writer = 0, None
        for j in range(i - 1, max(i - 12, -1), -1):
            if lines[j].endswith(":"):
                break
            op, _, rest = lines[j].partition(" ")
            if op == "s_nop":
                gap += int(rest) + 1
                continue
            if _sregs(rest.split(",")[0]) & base and not op.startswith(("s_cmp", "s_cbranch", "s_waitcnt")):
                writer = (op, gap)
                break
            gap += 1
        assert writer is not None, "base of '%s' has no writer in sight" % lines[i]
        assert writer[0].startswith("s_") or writer[1] >= 5, (lines[i], writer)
    print("%s: %d direct-to-LDS loads, every base written by a scalar instruction" % (src, len(loads)))


@pytest.mark.parametrize("src", ["prefill_attn_bf16.hip", "prefill_attn_pp_bf16.hip", "decode_attn_bf16.hip"])
def test_compiler_keeps_nothing_in_m0(src):
    """The direct-to-LDS loads (csrc/lds_dma.h) set M0 in inline assembly and cannot declare it as
    clobbered (the compiler reserves the register).  That is sound only while the compiler itself
    never keeps a value in M0 in these kernels: every mention of m0 in the emitted code must be one
    of the hand-written `s_mov_b32 m0, ...` that directly precede a global_load_lds."""
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    path = os.path.join(ROOT, "paper_2601_08743_amd", "csrc", src)
    with tempfile.TemporaryDirectory() as d:
        out = os.path.join(d, "k.s")
        subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                               "-packed-fp32-ops", "-I", os.path.join(ROOT, "include"), "-I", os.path.dirname(path),
                               "-S", "--cuda-device-only", path, "-o", out], stderr=subprocess.DEVNULL)
        lines = [l.split(";")[0].strip() for l in open(out)]
    lines = [l for l in lines if l and not l.startswith(".")]
    uses = [i for i, l in enumerate(lines) if re.search(r"\bm0\b", l)]
    assert uses, "no direct-to-LDS loads found in %s" % src
    for i in uses:
        assert re.match(r"^s_mov_b32 m0, ", lines[i]), lines[i]
        nxt = [l for l in lines[i + 1:i + 4] if not l.startswith("s_nop")]
        assert nxt and nxt[0].startswith("global_load_lds_dwordx4"), (lines[i], nxt[:1])
    print("%s: %d uses of m0, all hand-written" % (src, len(uses)))
