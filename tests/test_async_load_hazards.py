"""Static check of the tiled kernel's generated code (no GPU needed).

The tiled GEMM issues its main-loop loads from inline assembly and waits for them with
explicit s_waitcnt instructions.  The compiler therefore does not know that a destination
register is "in flight" between the load and the wait.  If it considered such a register dead
it could hand it to another value, which the late-arriving load would then overwrite (for an
address register that is an out-of-bounds access).  This test compiles the kernel to assembly
and verifies, instruction by instruction, that no register is read or written while an
asynchronous load into it can still be outstanding, using the in-order completion of vector
loads to interpret every `s_waitcnt vmcnt(N)`.
"""
import os
import re
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2310_04836_amd", "csrc", "linear_tiled.hip")


def _regs(tok):
    tok = tok.split(" ")[0]
    m = re.match(r"[va]\[(\d+):(\d+)\]$", tok)
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def _scan(lines, pending, problems, name):
    """Walks `lines` in order; `pending` is the issue-ordered list of in-flight destination sets."""
    for t in lines:
        m = re.match(r"(\S+)\s*(.*)", t)
        op, args = m.group(1), m.group(2)
        toks = [a.strip() for a in args.split(",")]
        if op == "s_waitcnt":
            mm = re.search(r"vmcnt\((\d+)\)", args)
            if mm:
                n = int(mm.group(1))
                del pending[: max(0, len(pending) - n)]   # all but the n youngest have landed
            continue
        touched = set()
        for a in toks:
            touched |= _regs(a)
        if op.startswith("global_load_lds"):
            pending.append(set())
            continue
        if op.startswith("global_load") or op.startswith("buffer_load"):
            dst = _regs(toks[0])
            for rs in pending:
                if rs & touched:
                    problems.append("%s: %s" % (name, t))
            pending.append(dst)
            continue
        if op.startswith("global_store") or op.startswith("global_atomic"):
            pending.append(set())            # stores also occupy a vmcnt slot on this target
        for rs in pending:
            if rs & touched:
                problems.append("%s: %s" % (name, t))
                break


def check_asm(text, kernel_substr):
    problems, kernels = [], 0
    for km in re.finditer(r"^(_Z\w*%s\w*):[^\n]*\n(.*?)s_endpgm" % kernel_substr, text, re.S | re.M):
        kernels += 1
        name = km.group(1)[-48:]
        body = [l.strip() for l in km.group(2).split("\n")]
        body = [l for l in body if l and not l.startswith(";")]
        labels = {l[:-1].split(":")[0]: i for i, l in enumerate(body) if l.startswith(".LBB")}
        insts = [(i, l) for i, l in enumerate(body)
                 if not l.startswith(".") and not l.startswith("s_branch")]
        pending = []
        _scan([l for _, l in insts if not l.startswith("s_cbranch")], pending, problems, name)
        # loops: replay every backward-branch region once more with the state at its end
        for i, l in insts:
            if l.startswith("s_cbranch"):
                tgt = l.split()[-1]
                j = labels.get(tgt)
                if j is not None and j < i:
                    region = [x for k, x in insts if j <= k < i and not x.startswith("s_cbranch")]
                    carried = []
                    _scan(region, carried, [], name)          # state at the end of one trip
                    _scan(region, carried, problems, name)    # second trip sees the carried loads
    return kernels, problems


@pytest.fixture(scope="module")
def tiled_asm(tmp_path_factory):
    from paper_2310_04836_amd import build as b
    out = tmp_path_factory.mktemp("asm") / "linear_tiled.s"
    flags = [f for f in b.FLAGS if f != "-fPIC"]
    subprocess.check_call([b.HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(out), SRC],
                          stderr=subprocess.DEVNULL)
    return out.read_text()


def test_no_register_is_touched_while_an_async_load_into_it_is_in_flight(tiled_asm):
    kernels, problems = check_asm(tiled_asm, "linear_tiled_kernel")
    assert kernels == 8
    assert not problems, "\n".join(problems[:10])


def test_checker_sees_a_planted_hazard():
    asm = """_Zfake_linear_tiled_kernel_x:   ; @x
	global_load_dwordx4 v[4:7], v[0:1], off
	global_load_dwordx4 v[8:11], v[0:1], off offset:512
	s_waitcnt vmcnt(1)
	v_add_u32_e32 v2, v4, v5
	v_add_u32_e32 v3, v8, v2
	s_waitcnt vmcnt(0)
	v_add_u32_e32 v3, v9, v2
	s_endpgm
"""
    kernels, problems = check_asm(asm, "linear_tiled_kernel")
    assert kernels == 1 and len(problems) == 1 and "v8" in problems[0]
