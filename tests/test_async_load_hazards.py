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
    m = re.match(r"v\[(\d+):(\d+)\]$", tok)   # accumulation registers a[...] are another file; no load targets them
    if m:
        return set(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    return {int(m.group(1))} if m else set()


def _step(t, pending, problems, name):
    """Applies instruction `t` to `pending`, the issue-ordered list of in-flight destination sets."""
    m = re.match(r"(\S+)\s*(.*)", t)
    op, args = m.group(1), m.group(2)
    toks = [a.strip() for a in args.split(",")]
    if op == "s_waitcnt":
        mm = re.search(r"vmcnt\((\d+)\)", args)
        if mm:
            n = int(mm.group(1))
            del pending[: max(0, len(pending) - n)]   # all but the n youngest have landed
        return
    touched = set()
    for a in toks:
        touched |= _regs(a)
    hit = any(rs & touched for rs in pending)
    if op.startswith("global_load_lds"):
        pending.append(frozenset())
    elif op.startswith("global_load") or op.startswith("buffer_load") or op.startswith("scratch_load"):
        pending.append(frozenset(_regs(toks[0])))
    elif op.startswith("global_store") or op.startswith("global_atomic") or op.startswith("scratch_store"):
        pending.append(frozenset())            # stores also occupy a vmcnt slot on this target
    if hit:
        problems.add("%s: %s" % (name, t))


def _canon(pending):
    """State key: the oldest entries that name no register (stores, copies into LDS) can be dropped;
    a wait counts from the youngest end, so they never decide which register loads remain."""
    k = 0
    while k < len(pending) and not pending[k]:
        k += 1
    return tuple(pending[k:])


def check_asm(text, kernel_substr):
    """Follows every path of the control flow graph of each matching kernel (state = the pending
    loads; a (block, state) pair is expanded once) and returns (kernels, sorted problems)."""
    problems, kernels = set(), 0
    for km in re.finditer(r"^(_Z\w*%s\w*):[^\n]*\n(.*?)\.end_amdhsa_kernel" % kernel_substr, text, re.S | re.M):
        kernels += 1
        name = km.group(1)[-48:]
        body = [l.strip() for l in km.group(2).split("\n")]
        body = [l for l in body if l and not l.startswith(";")]
        labels = {l.split(":")[0]: i for i, l in enumerate(body) if re.match(r"\.LBB\w+:", l)}
        is_label = [bool(re.match(r"\.LBB\w+:", l)) for l in body]
        work, seen = [(0, ())], set()
        while work:
            i, state = work.pop()
            if (i, state) in seen:
                continue
            seen.add((i, state))
            assert len(seen) < 20000, "state explosion in %s" % name
            pending = list(state)
            first = True
            while i < len(body):
                l = body[i]
                if is_label[i] and not first:
                    work.append((i, _canon(pending)))   # a block start: expanded once per state
                    break
                first = False
                if l.startswith(".") or l.endswith(":"):
                    i += 1
                    continue
                if l.startswith("s_endpgm"):
                    break
                if l.startswith("s_branch"):
                    work.append((labels[l.split()[-1]], _canon(pending)))
                    break
                if l.startswith("s_cbranch"):
                    work.append((labels[l.split()[-1]], _canon(pending)))
                    work.append((i + 1, _canon(pending)))
                    break
                _step(l, pending, problems, name)
                i += 1
    return kernels, sorted(problems)


@pytest.fixture(scope="module")
def tiled_asm(tmp_path_factory):
    from paper_2310_04836_amd import build as b
    out = tmp_path_factory.mktemp("asm") / "linear_tiled.s"
    flags = [f for f in b.FLAGS if f != "-fPIC"]
    subprocess.check_call([b.HIPCC, *flags, "-S", "--cuda-device-only", "-o", str(out), SRC],
                          stderr=subprocess.DEVNULL)
    return out.read_text()


def test_no_register_is_touched_while_an_async_load_into_it_is_in_flight(tiled_asm):
    # signed-nibble and zero-point forms, without and with the K of a tile split over workgroups
    for name in ("linear_tiled_kernel", "linear_tiled_zp_kernel", "linear_tiled_cols_kernel", "linear_tiled_cols_zp_kernel",
                 "linear_tiled_splitk_kernel", "linear_tiled_splitk_zp_kernel"):
        kernels, problems = check_asm(tiled_asm, name)
        assert kernels == 12, (name, kernels)      # two group sizes x three tile shapes x {fp16, INT32 test hook}
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
	.end_amdhsa_kernel
"""
    kernels, problems = check_asm(asm, "linear_tiled_kernel")
    assert kernels == 1 and len(problems) == 1 and "v8" in problems[0]


def test_checker_follows_branches_and_loops():
    # the hazard exists only on the path that skips the wait, and only in the second loop trip
    asm = """_Zfake_linear_tiled_kernel_y:   ; @y
	s_cbranch_scc1 .LBB0_2
	global_load_dwordx4 v[4:7], v[0:1], off
	s_branch .LBB0_3
.LBB0_2:
	v_mov_b32_e32 v4, 0
.LBB0_3:
	v_add_u32_e32 v20, v21, v22
	s_cbranch_scc1 .LBB0_5
	s_waitcnt vmcnt(0)
.LBB0_5:
	v_add_u32_e32 v2, v4, v2
.LBB0_6:
	v_add_u32_e32 v3, v12, v2
	global_load_dwordx4 v[12:15], v[0:1], off
	s_waitcnt vmcnt(1)
	s_cbranch_scc1 .LBB0_6
	s_waitcnt vmcnt(0)
	s_endpgm
.LBB0_9:
	s_endpgm
	.end_amdhsa_kernel
"""
    kernels, problems = check_asm(asm, "linear_tiled_kernel")
    assert kernels == 1
    # also flagged: the second trip's load into v[12:15] while the first trip's may be outstanding
    assert len(problems) == 3 and any("v4, v2" in p for p in problems) and any("v12, v2" in p for p in problems)
