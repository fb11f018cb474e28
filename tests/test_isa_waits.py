"""Static check of the ISA hipcc generates for the GEMM kernels (CPU only: cross-compiles, runs nothing).

The kernels read their MFMA fragments from LDS with inline-assembly ds_read instructions, which the compiler does
not track in lgkmcnt: the waits are written by hand and kept in place with scheduling fences.  A compiler that
moved an MFMA above its wait would not fail to build and might not fail a numerical test either (the data usually
has landed), so the instruction stream itself is checked: on every path, between an LDS read and an MFMA that
uses its destination registers there must be an s_waitcnt lgkmcnt small enough to cover it (LDS operations of a
wave complete in order).
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _regs(tok):
    m = re.match(r"v\[(\d+):(\d+)\]", tok)
    if m:
        return frozenset(range(int(m.group(1)), int(m.group(2)) + 1))
    m = re.match(r"v(\d+)$", tok)
    if m:
        return frozenset({int(m.group(1))})
    return frozenset()


def _merge(a, b):
    """Join of two pending lists (oldest first): aligned at the youngest end, united element by element."""
    out = []
    for i in range(1, max(len(a), len(b)) + 1):
        x = a[-i] if i <= len(a) else frozenset()
        y = b[-i] if i <= len(b) else frozenset()
        out.append(x | y)
    return tuple(reversed(out))


def _transfer(state, instructions, hazards, where):
    st = list(state)
    for t in instructions:
        op = t.split()[0]
        if op.startswith("ds_read"):
            st.append(_regs(t.split()[1].rstrip(",")))
        elif op.startswith("ds_") or op.startswith("s_load") or op.startswith("s_buffer_load"):
            st.append(frozenset())          # counted in lgkmcnt, delivers nothing an MFMA reads
        elif op == "s_waitcnt":
            m = re.search(r"lgkmcnt\((\d+)\)", t)
            if m and int(m.group(1)) < len(st):
                st = st[len(st) - int(m.group(1)):]
        elif op.startswith("v_mfma"):
            toks = [x.rstrip(",") for x in t.split()[1:]]
            srcs = _regs(toks[1]) | _regs(toks[2])
            if any(p & srcs for p in st) and hazards is not None:
                hazards.append((where, t))
        st = st[-16:]                       # the counter holds 15; older ones have been waited for by the hardware
    return tuple(st)


def lint_kernel(lines):
    blocks = [("entry", [])]
    for line in lines:
        t = line.strip()
        if not t or t.startswith(";"):
            continue
        m = re.match(r"^(\.LBB\w+):", t)
        if m:
            blocks.append((m.group(1), []))
        else:
            blocks[-1][1].append(t)
    index = {name: i for i, (name, _) in enumerate(blocks)}
    succ = []
    for i, (_, ins) in enumerate(blocks):
        s, fall = set(), True
        for t in ins:
            op = t.split()[0]
            if op.startswith("s_cbranch"):
                s.add(index[t.split()[1]])
            elif op == "s_branch":
                s.add(index[t.split()[1]])
                fall = False
            elif op == "s_endpgm":
                fall = False
        if fall and i + 1 < len(blocks):
            s.add(i + 1)
        succ.append(s)
    state = [None] * len(blocks)
    state[0] = tuple()
    work = [0]
    while work:
        i = work.pop()
        out = _transfer(state[i], blocks[i][1], None, None)
        for j in succ[i]:
            new = out if state[j] is None else _merge(state[j], out)
            if new != state[j]:
                state[j] = new
                work.append(j)
    hazards = []
    for i, (name, ins) in enumerate(blocks):
        if state[i] is not None:
            _transfer(state[i], ins, hazards, name)
    return hazards


def test_lint_flags_a_planted_hazard():
    planted = ["ds_read_b128 v[2:5], v9 offset:0", "ds_read_b128 v[6:9], v9 offset:16", "s_waitcnt lgkmcnt(1)",
               "v_mfma_f32_32x32x16_bf16 a[0:15], v[6:9], v[2:5], a[0:15]", "s_endpgm"]
    assert len(lint_kernel(planted)) == 1
    planted[2] = "s_waitcnt lgkmcnt(0)"
    assert lint_kernel(planted) == []
    # across a back edge: the read at the bottom of the loop body is still pending at its top
    loop = [".LBB0_1:", "v_mfma_f32_32x32x16_bf16 a[0:15], v[6:9], v[2:5], a[0:15]", "ds_read_b128 v[2:5], v9 offset:0",
            "s_cbranch_scc1 .LBB0_1", "s_endpgm"]
    assert len(lint_kernel(loop)) == 1


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_no_mfma_reads_a_fragment_before_its_wait(tmp_path):
    stage = tmp_path / "paper" / "csrc"
    stage.mkdir(parents=True)
    (tmp_path / "include").mkdir()
    csrc = os.path.join(ROOT, "paper_2603_22276_amd", "csrc")
    for f in os.listdir(csrc):
        shutil.copy(os.path.join(csrc, f), stage / f)
    for f in os.listdir(os.path.join(ROOT, "include")):
        shutil.copy(os.path.join(ROOT, "include", f), tmp_path / "include" / f)
    asm = tmp_path / "gemm.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-S", "--cuda-device-only", "-o", str(asm), str(stage / "gemm_bf16.hip")]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout[-2000:]
    kernels, current = {}, None
    for line in asm.read_text().split("\n"):
        m = re.match(r"^(_ZN\S*gemm_bf16_kernel\S*):", line)
        if m:
            current = m.group(1)
            kernels[current] = []
            continue
        if current is not None:
            if line.startswith(".Lfunc_end"):   # blocks may follow the first s_endpgm; the function ends here
                current = None
            else:
                kernels[current].append(line)
    assert len(kernels) >= 20, "expected every GEMM instantiation in the assembly"
    assert sum("v_mfma" in l for ls in kernels.values() for l in ls) > 500
    bad = {k: h for k, h in ((k, lint_kernel(v)) for k, v in kernels.items()) if h}
    assert not bad, "MFMA issued before the LDS read feeding it is covered by a wait: %r" % (
        {k[-60:]: h[:3] for k, h in bad.items()},)
