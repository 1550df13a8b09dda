"""Static checks over the compiled gfx950 ISA of the kernels that keep memory operations in flight behind the
compiler's back (CPU only: hipcc cross-compiles to assembly, nothing runs).

Two kernels issue loads as inline assembly and wait for them by hand, because the compiler's own counter
bookkeeping cost too much there: the mid-batch kernel (global loads of the weight stages, retired by one
`s_waitcnt vmcnt(n)` per stage) and the big-tile kernel (LDS reads of the A operands, retired by
`s_waitcnt lgkmcnt(n)`).  The compiler does not know that the destination registers of such a load are still
pending: if it copied, reused or overwrote them between the load and the wait that retires it, a result would be
wrong only now and then.  Memory operations of one kind retire in order, so a linear scan in layout order can tell.
"""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_2511_19438_amd import build as B

VM_PREFIXES = ("global_load", "global_store", "global_atomic", "buffer_", "scratch_", "flat_")


def compile_to_asm(src, defines, out_dir):
    out = os.path.join(out_dir, os.path.basename(src) + "".join(defines).replace("=", "_").replace("-D", ".") + ".s")
    cmd = [B.HIPCC, *B.COMMON, *defines, "--cuda-device-only", "-S", os.path.join(B.CSRC, src), "-o", out]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr[-2000:]
    return out


def kernels(path):
    """{kernel name: instruction lines (labels, directives and comments removed; asm markers kept)}"""
    text = open(path).read()
    out = {}
    for m in re.finditer(r"^(_Z\w+):.*?\n(.*?)\.end_amdhsa_kernel", text, re.S | re.M):
        lines = []
        for raw in m.group(2).split("\n"):
            t = raw.strip()
            if t.startswith(";;#ASM"):
                lines.append(t)
                continue
            t = t.split(";")[0].strip()
            if not t or t.startswith(".") or t.endswith(":"):
                continue
            lines.append(t)
        out[m.group(1)] = lines
    return out


def vregs(operand):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", operand):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


def check_pending(lines, is_tracked, is_counted, wait_re, what):
    """Scans `lines` twice (the second pass stands for the loop's next trip and for the code after it): an
    instruction for which is_tracked(op, in_asm) holds puts its destination registers in flight; instructions for
    which is_counted(op) holds take a place in the in-order queue; `wait_re` extracts n from the waits.  No other
    instruction may name a register in flight."""
    problems = []
    queue = []  # [dest regs or None, text]
    in_asm = False
    for trip in range(2):
        for t in lines:
            if t.startswith(";;#ASMSTART"):
                in_asm = True
                continue
            if t.startswith(";;#ASMEND"):
                in_asm = False
                continue
            op = t.split()[0]
            m = wait_re.search(t) if op == "s_waitcnt" else None
            if op == "s_waitcnt":
                if m:
                    n = int(m.group(1))
                    queue = queue[len(queue) - n:] if n else []
                continue
            if op == "s_endpgm":
                queue = []
                continue
            named = vregs(t.split(None, 1)[1]) if " " in t else set()
            for dest, text in queue:
                if dest and dest & named and not (is_tracked(op, in_asm) and text == t):
                    problems.append(f"{what}: '{t}' names v{sorted(dest & named)} while '{text}' is in flight")
            if is_counted(op):
                dest = vregs(t.split(None, 1)[1].split(",")[0]) if is_tracked(op, in_asm) else None
                queue.append([dest, t])
    return problems


@pytest.fixture(scope="module")
def asm_files():
    if not os.path.exists(B.HIPCC):
        pytest.skip("no hipcc")
    tmp = tempfile.mkdtemp(prefix="gptq_isa_")
    jobs = [("mid.hip", [])] + [("prefill_tile.hip", [f"-DGPTQ_PREFILL_TILE={t}"]) for t in B.PREFILL_TILES]
    with ThreadPoolExecutor(max_workers=5) as pool:
        files = list(pool.map(lambda j: compile_to_asm(j[0], j[1], tmp), jobs))
    return {"mid": files[0], "prefill": files[1:]}


def test_mid_batch_kernel_leaves_registers_of_pending_weight_loads_alone(asm_files):
    ks = {k: v for k, v in kernels(asm_files["mid"]).items() if "mid_kernel" in k}
    assert len(ks) >= 5
    wait = re.compile(r"vmcnt\((\d+)\)")
    for name, lines in ks.items():
        tracked = lambda op, in_asm: in_asm and op.startswith("global_load_dword")  # noqa: E731
        counted = lambda op: op.startswith(VM_PREFIXES)  # noqa: E731
        n_asm = sum(1 for i, t in enumerate(lines) if t.startswith("global_load_dword") and i and
                    lines[i - 1].startswith(";;#ASMSTART"))
        assert n_asm >= 18, f"{name}: expected the loop's weight loads as inline assembly, found {n_asm}"
        problems = check_pending(lines, tracked, counted, wait, name)
        assert not problems, "\n".join(problems[:10])


def test_big_tile_kernel_leaves_registers_of_pending_lds_reads_alone(asm_files):
    wait = re.compile(r"lgkmcnt\((\d+)\)")
    seen = 0
    for path in asm_files["prefill"]:
        for name, lines in kernels(path).items():
            if "prefill_pipelined_kernel" not in name:
                continue
            seen += 1
            tracked = lambda op, in_asm: in_asm and op.startswith("ds_read")  # noqa: E731
            counted = lambda op: op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load")  # noqa: E731
            problems = check_pending(lines, tracked, counted, wait, name)
            assert not problems, "\n".join(problems[:10])
    assert seen >= 4


def test_the_checker_itself_flags_a_planted_violation():
    wait = re.compile(r"vmcnt\((\d+)\)")
    tracked = lambda op, in_asm: in_asm and op.startswith("global_load_dword")  # noqa: E731
    counted = lambda op: op.startswith(VM_PREFIXES)  # noqa: E731
    good = [";;#ASMSTART", "global_load_dwordx4 v[4:7], v1, s[2:3]", ";;#ASMEND",
            "global_load_lds_dwordx4 v2, s[4:5]",
            "v_add_u32 v8, v9, v10",
            ";;#ASMSTART", "s_waitcnt vmcnt(1)", ";;#ASMEND",
            "v_mov_b32 v11, v4",
            "s_waitcnt vmcnt(0)"]
    assert check_pending(good, tracked, counted, wait, "good") == []
    early_use = list(good)
    early_use[4] = "v_add_u32 v8, v5, v10"   # reads a register whose load has not been waited for
    assert len(check_pending(early_use, tracked, counted, wait, "early use")) >= 1
    clobber = list(good)
    clobber[4] = "v_mov_b32 v6, v10"          # hands a pending destination to something else
    assert len(check_pending(clobber, tracked, counted, wait, "clobber")) >= 1
    late_wait = list(good)
    late_wait[6] = "s_waitcnt vmcnt(2)"       # a wait that does not retire the load
    assert len(check_pending(late_wait, tracked, counted, wait, "late wait")) >= 1
