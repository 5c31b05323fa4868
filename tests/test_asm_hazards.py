"""Static check of the generated code of the kernels that issue loads from inline assembly (no GPU needed).

attn_bf16.hip (row numbers of the next tile, LDS fragment reads) and colmass_bf16.hip (LDS fragment and
log-sum-exp reads) issue some loads from inline assembly, which the compiler takes for ordinary
instructions whose result is there at once.  Two
things must therefore hold in the generated code, and neither is visible in the source:

  * nothing reads or overwrites the destination registers of such a load before a wait that
    covers it (a register copy placed right behind the load would copy the old content);
  * the registers are not given to another value while the load is in flight;
  * m0, which the gathers of a tile share as their LDS base, is not written by anything else
    between the first and the last of them.

The test compiles the file to assembly and walks every attention kernel: it keeps the vector
memory and the LDS operations in issue order, retires them at each s_waitcnt the way the
hardware counters do (both kinds complete in order), and reports every instruction that touches
the destination of an assembly-issued load still in flight.  Control flow is followed along
fall-through edges only; the state is dropped behind an unconditional branch.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2605_20813_amd", "csrc")

REG = re.compile(r"\b([va])(?:(\d+)|\[(\d+):(\d+)\])")
ASYNC_ASM_LOAD = re.compile(r"^(global_load_dword(?:x[234])?|ds_read_b128|ds_read_b64_tr_b16|ds_read_b64|ds_read_b32)\s")
VMEM = re.compile(r"^(global_|buffer_|scratch_|flat_)")
LDS = re.compile(r"^ds_")


def regs_of(text):
    out = set()
    for kind, single, lo, hi in REG.findall(text):
        if single:
            out.add((kind, int(single)))
        else:
            out.update((kind, r) for r in range(int(lo), int(hi) + 1))
    return out


def wait_counts(ins):
    vm = re.search(r"vmcnt\((\d+)\)", ins)
    lgkm = re.search(r"lgkmcnt\((\d+)\)", ins)
    return (int(vm.group(1)) if vm else None), (int(lgkm.group(1)) if lgkm else None)


def check_function(lines):
    """lines: assembly lines of one kernel.  Returns a list of (line number, instruction, registers)."""
    vm, lgkm = [], []            # in-flight operations, oldest first: sets of guarded registers
    bad = []
    in_asm = False
    m0_from_asm = False          # m0 holds the LDS base that an assembly statement put there
    for no, raw in lines:
        ins = raw.split(";")[0].strip() if not raw.strip().startswith(";;#") else raw.strip()
        if ins.startswith(";;#ASMSTART"):
            in_asm = True
            continue
        if ins.startswith(";;#ASMEND"):
            in_asm = False
            continue
        if not ins or ins.startswith(".") or ins.endswith(":"):
            continue
        op = ins.split()[0]
        if op == "s_waitcnt":
            nvm, nlgkm = wait_counts(ins)
            if nvm is not None:
                del vm[:max(0, len(vm) - nvm)]
            if nlgkm is not None:
                del lgkm[:max(0, len(lgkm) - nlgkm)]
            continue
        if op in ("s_branch", "s_endpgm", "s_setpc_b64"):
            vm, lgkm = [], []
            continue
        # The gathers of a tile share one LDS base in m0: written by the first assembly statement,
        # used by the later loads through their instruction offsets.  Nothing else may write m0 in
        # between.
        if re.match(r"^s_\w+\s+m0\b", ins):
            m0_from_asm = in_asm
        if in_asm and op.startswith("global_load_lds") and not m0_from_asm:
            bad.append((no, ins, ["m0 not set by the gather's own code"]))
        touched = regs_of(ins)
        pending = set().union(*vm, *lgkm) if (vm or lgkm) else set()
        hit = touched & pending
        if hit:
            bad.append((no, ins, sorted(hit)))
        is_lds_dma = op.startswith("global_load_lds") or " lds" in ins
        if VMEM.match(op):
            guarded = set()
            if in_asm and ASYNC_ASM_LOAD.match(ins) and not is_lds_dma:
                guarded = regs_of(ins.split(",")[0])
            vm.append(guarded)
        elif LDS.match(op):
            guarded = set()
            if in_asm and ASYNC_ASM_LOAD.match(ins):
                guarded = regs_of(ins.split(",")[0])
            lgkm.append(guarded)
    return bad


def kernels_of(asm_text, name_part):
    lines = asm_text.split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"^_Z\w*%s\w*:" % name_part, l)]
    for s in starts:
        e = next(i for i in range(s, len(lines)) if lines[i].startswith(".Lfunc_end"))
        yield lines[s].split(":")[0], [(i + 1, lines[i]) for i in range(s + 1, e)]


def test_checker_sees_a_copy_behind_an_asynchronous_load():
    sample = """
        ;;#ASMSTART
        global_load_dwordx4 v[90:93], v75, s[52:53]
        ;;#ASMEND
        v_mov_b32_e32 v0, v91
        s_waitcnt vmcnt(0)
        v_mov_b32_e32 v1, v92
    """.split("\n")
    bad = check_function(list(enumerate(sample)))
    assert len(bad) == 1 and "v0, v91" in bad[0][1]
    reuse = """
        ;;#ASMSTART
        ds_read_b128 v[4:7], v9 offset:16
        ;;#ASMEND
        ;;#ASMSTART
        ds_read_b128 v[10:13], v9 offset:32
        ;;#ASMEND
        s_waitcnt lgkmcnt(1)
        v_add_f32_e32 v20, v4, v5
        v_mov_b32_e32 v11, 0
    """.split("\n")
    bad = check_function(list(enumerate(reuse)))
    assert len(bad) == 1 and "v11" in bad[0][1]
    base_lost = """
        ;;#ASMSTART
        s_add_i32 m0, s5, 0x4000
        v_mad_u32_u24 v3, v1, s2, v2
        ;;#ASMEND
        ;;#ASMSTART
        global_load_lds_dwordx4 v3, s[8:9] offset:0
        ;;#ASMEND
        s_mov_b32 m0, s7
        ;;#ASMSTART
        global_load_lds_dwordx4 v4, s[10:11] offset:0x400
        ;;#ASMEND
    """.split("\n")
    bad = check_function(list(enumerate(base_lost)))
    assert len(bad) == 1 and "offset:0x400" in bad[0][1]


def _assembly_of(source):
    from paper_2605_20813_amd import build
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    flags = [f for f in build.HIPCC_FLAGS if f not in ("-fPIC", "-fvisibility=hidden")]
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "kernel.s")
        subprocess.run([hipcc, *flags, "-S", "--cuda-device-only", "-o", out, os.path.join(CSRC, source)],
                       check=True, capture_output=True)
        return open(out).read()


# file, kernel name, instantiations expected (attention: three modes x two head dimensions; column pass: two
# head dimensions)
CHECKED = [("attn_bf16.hip", "attn_bf16_kernel", 6), ("colmass_bf16.hip", "colmass_bf16_kernel", 2)]


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="needs hipcc")
@pytest.mark.parametrize("source,kernel,count", CHECKED)
def test_no_instruction_touches_an_assembly_issued_load_in_flight(source, kernel, count):
    text = _assembly_of(source)
    found = 0
    for name, lines in kernels_of(text, kernel):
        found += 1
        bad = check_function(lines)
        assert not bad, "%s: %d hazards, first: line %d `%s` touches %s" % (name, len(bad), bad[0][0], bad[0][1], bad[0][2])
    assert found >= count
