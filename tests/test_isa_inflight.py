"""Static check of the compiled scan kernel (no GPU needed): the registers that receive the
hand-issued code, norm and centroid loads of ivfpq_scan_bank_kernel, and the code and query loads
of ivfpq_scan_listmajor_kernel (the same pipeline, two queries at a time), are in flight between the
load and a counted wait that the compiler knows nothing about.  A copy, spill or any other
compiler-generated instruction that touches such a register inside the pipelined loop would read
it before the data has arrived (or clobber it afterwards) without any error at run time -- so the
generated assembly is checked here: inside the loop, from its first request (the third code load:
two requests precede the loop) to the drain after the loop, those registers are read only by the look-up address instructions (v_perm_b32),
by the hand-written asm itself and, for the stored-norm form, by the addition that consumes a norm,
and they are written only by the hand-issued loads."""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2401_08281_amd", "csrc", "kernels_ivfpq.hip")


def vgprs(token):
    """VGPR numbers named by one operand: v12 or v[12:15]."""
    m = re.fullmatch(r"v(\d+)", token)
    if m:
        return {int(m.group(1))}
    m = re.fullmatch(r"v\[(\d+):(\d+)\]", token)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    return set()


def operands(line):
    body = line.split(";")[0].strip()
    parts = body.split(None, 1)
    if len(parts) < 2:
        return parts[0] if parts else "", []
    ops = [o.strip() for o in re.split(r",\s*(?![^\[]*\])", parts[1])]
    return parts[0], ops


@pytest.fixture(scope="module")
def kernels(tmp_path_factory):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    from paper_2401_08281_amd import build as b
    out = str(tmp_path_factory.mktemp("isa") / "kernels_ivfpq.s")
    flags = [f for f in b.FLAGS if f not in ("-fPIC",)]
    subprocess.run([hipcc] + flags + ["-S", "--cuda-device-only", SRC, "-o", out], check=True,
                   stdout=subprocess.DEVNULL, stderr=subprocess.DEVNULL)
    text = open(out).read().splitlines()
    funcs, cur, name = {}, None, None
    for line in text:
        m = re.match(r"^(_ZN\S*ivfpq_scan_(?:bank|listmajor)_kernel\S*):", line)
        if m:
            name, cur = m.group(1), []
            continue
        if cur is not None:
            cur.append(line)
            if "s_endpgm" in line:
                funcs[name] = cur
                cur = None
    return funcs


def test_every_instantiation_is_present(kernels):
    # three shapes x four table forms x three selection widths, and the list-major kernel of every shape
    assert len(kernels) == 39, sorted(kernels)


def test_no_compiler_instruction_touches_a_register_in_flight(kernels):
    """For every register that a hand-issued load writes inside the pipelined loop: from that load
    to the last legitimate read before the register is loaded again (a v_perm_b32 of the look-ups,
    a line of hand-written asm, the norm's addition), nothing else reads or writes it.  The loop
    body (three unrolled steps) is walked twice in text order so that a set requested in the last
    step and consumed in the first is covered."""
    for name, lines in kernels.items():
        metric2 = re.search(r"ivfpq_scan_bank_kernelILi\d+ELi\d+ELi2E", name) is not None
        code_blocks, drains = [], []
        for n, line in enumerate(lines):
            if "#ASMSTART" in line and re.search(r"global_load_dwordx[24]\b", lines[n + 1]):
                code_blocks.append(n)
            if "#ASMSTART" in line and "vmcnt(0)" in lines[n + 1]:
                drains.append(n)
        assert len(code_blocks) == 5 and drains, (name, code_blocks)   # 2 in the prologue, 3 in the loop
        # (the list-major kernel's pipelined loop sits inside two outer loops, and its drain is laid
        # out ahead of it in the text: there the body runs to the end of the function)
        after = [d for d in drains if d > code_blocks[4]]
        body = lines[code_blocks[2]:min(after) if after else len(lines)]
        seq = body + body
        loads, allowed, other = {}, {}, {}
        in_asm = False
        for n, line in enumerate(seq):
            if "#ASMSTART" in line:
                in_asm = True
                continue
            if "#ASMEND" in line:
                in_asm = False
                continue
            if not line.startswith("\t") or line.strip().startswith((";", ".")):
                continue
            op, ops = operands(line)
            regs = [vgprs(o) for o in ops]
            if in_asm and op.startswith("global_load_dword"):
                for r in regs[0]:
                    loads.setdefault(r, []).append(n)
                continue
            touched = set().union(*regs) if regs else set()
            ok = in_asm or (op.startswith("v_perm_b32") and not (regs[0] & touched - regs[0])) or \
                (metric2 and op.startswith("v_add_f32"))
            reads_only = not regs or not regs[0] or op.startswith(("ds_write", "global_store", "scratch_store"))
            for r in touched:
                wrote = (not reads_only) and r in regs[0]
                if ok and not (wrote and not in_asm):
                    allowed.setdefault(r, []).append(n)
                else:
                    other.setdefault(r, []).append((n, line.strip()))
        assert len(loads) >= 6, (name, sorted(loads))
        for r, ls in loads.items():
            for i, l in enumerate(ls):
                if l >= len(body):
                    break
                nxt = ls[i + 1] if i + 1 < len(ls) else len(seq)
                reads = [a for a in allowed.get(r, []) if l < a < nxt]
                assert reads, "%s: v%d is loaded (line %d) and never consumed" % (name, r, l)
                end = max(reads)
                bad = [(n, t) for n, t in other.get(r, []) if l < n < end]
                assert not bad, "%s: v%d is in flight from line %d to %d, touched by %s" % (name, r, l, end, bad[:3])
