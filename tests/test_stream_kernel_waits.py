"""Host-side checks of the streaming projection kernel (`csrc/gemm_stream.hip`), whose weight loads are
inline assembly that the compiler does not track: every wait of its main loop is a hand-written count,
and registers with a load in flight must stay allocated until a wait covers them.  No GPU needed:

* the wait counts of the source are re-derived from the issue order of a wave's memory instructions;
* the compiled kernel (gfx950 ISA of this repository's own source) is read back: between the last
  weight loads of the main loop and the wait that covers them, and between the first weight loads and
  theirs, no instruction may touch a register those loads write.
"""
import os
import re
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "paper_2505_24791_amd", "csrc", "gemm_stream.hip")

CKS, PD = 16, 8     # k-steps per chunk, look-ahead of the weight fragments in k-steps


def _constants():
    text = open(SRC).read()
    ck = int(re.search(r"S_CK = (\d+)", text).group(1))
    pd = int(re.search(r"S_PD = (\d+)", text).group(1))
    return ck // 16, pd, text


def test_source_constants_are_the_ones_checked_here():
    cks, pd, text = _constants()
    assert (cks, pd) == (CKS, PD)
    assert "wait_vm(15 + 2 * pieces_window(ks))" in text
    assert "wait_vm(14 + 2 * pieces_window(ks) + (ks < 8 ? 2 : 0))" in text
    assert "vmcnt(16)" in text and "0x4070" in text


def _window(ks):
    return sum(1 for d in range(1, 8) if ((ks - d + CKS) % CKS) < 8)


def test_wait_counts_cover_the_loads_they_are_for():
    """Issue order of one wave: prologue (sixteen weight fragments, sixteen pieces of chunk 0), then per
    k-step [wait, two pieces in k-steps 0-7], ..., [wait, fragment 0], ..., fragment 1.  A wait for "at
    most n outstanding" guarantees a load only if at least n younger operations were issued after it."""
    order, pos = [], {}

    def issue(label):
        pos[label] = len(order)
        order.append(label)

    for p in range(PD):
        for j in range(2):
            issue(("w", p, j))
    for q in range(16):
        issue(("a", 0, q))
    exact = 0
    for c in range(6):
        for ks in range(CKS):
            kg = c * CKS + ks
            n0 = 15 + 2 * _window(ks)
            younger = len(order) - 1 - pos[("w", kg, 0)]
            assert younger >= n0, (c, ks, younger, n0)
            exact += younger == n0
            if ks < 8:
                issue(("a", c + 1, 2 * ks))
                issue(("a", c + 1, 2 * ks + 1))
            n1 = 14 + 2 * _window(ks) + (2 if ks < 8 else 0)
            younger = len(order) - 1 - pos[("w", kg, 1)]
            assert younger >= n1, (c, ks, younger, n1)
            exact += younger == n1
            issue(("w", kg + PD, 0))
            issue(("w", kg + PD, 1))
            if ks == CKS - 2:      # the wait in front of the chunk's last k-step: every piece of chunk c + 1
                assert len(order) - 1 - pos[("a", c + 1, 15)] >= 16
    # in the steady state the counts are exact (no look-ahead is given away); only chunk 0 waits longer
    assert exact >= 2 * CKS * 5


def _regs(text):
    out = set()
    for m in re.finditer(r"\bv\[(\d+):(\d+)\]|\bv(\d+)\b", text):
        if m.group(1):
            out.update(range(int(m.group(1)), int(m.group(2)) + 1))
        else:
            out.add(int(m.group(3)))
    return out


@pytest.fixture(scope="module")
def kernel_isa(tmp_path_factory):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("no hipcc")
    d = tmp_path_factory.mktemp("isa")
    from paper_2505_24791_amd.build import HIPCC_FLAGS
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
    r = subprocess.run([hipcc, *flags, "--save-temps", "-c", SRC, "-o", str(d / "gemm_stream.o")], cwd=d,
                       stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert r.returncode == 0, r.stdout[-2000:]
    asm = (d / "gemm_stream-hip-amdgcn-amd-amdhsa-gfx950.s").read_text().splitlines()
    kernels = {}
    name = None
    for line in asm:
        m = re.match(r"(_ZN3sjd\S*gemm_stream_resid_kernel\S*):", line)
        if m:
            name = m.group(1)
            kernels[name] = []
        if name:
            kernels[name].append(line)
            if "s_endpgm" in line:
                name = None
    assert len(kernels) == 2, list(kernels)       # float16 and bfloat16
    return kernels


def _main_loop(lines):
    labels = {l.split(":")[0]: i for i, l in enumerate(lines) if re.match(r"\.LBB\d+_\d+:", l)}
    best = None
    for i, l in enumerate(lines):
        m = re.search(r"s_cbranch\w+ (\.LBB\d+_\d+)", l)
        if m and labels.get(m.group(1), i) < i:
            n = sum("v_mfma" in x for x in lines[labels[m.group(1)]:i])
            if best is None or n > best[2]:
                best = (labels[m.group(1)], i, n)
    return best


def test_compiled_kernel_keeps_in_flight_registers_untouched(kernel_isa):
    load = re.compile(r"\s+global_load_dwordx4 v\[(\d+):(\d+)\]")
    for name, lines in kernel_isa.items():
        start, end, n_mfma = _main_loop(lines)
        assert n_mfma == 256, (name, n_mfma)          # two chunks of sixteen k-steps of eight
        body = lines[start:end]
        assert not [l for l in body if re.search(r"s_waitcnt vmcnt\(0\)", l)], "a full wait inside the main loop"
        ring = set()
        for l in body:
            m = load.match(l)
            if m:
                ring.update(range(int(m.group(1)), int(m.group(2)) + 1))
        assert len(ring) >= 64
        # inside the loop, from a weight load to the first matrix instruction that takes its registers as
        # second source, nothing else may touch them: a copy or a spill there would move data that has not
        # arrived.  (Outside that span the allocator may use the registers for anything.)  The body is
        # walked twice: the last loads of an iteration are consumed at the start of the next one.
        in_flight = set()
        for l in body + body:
            if not re.match(r"\s+(v_|ds_|global_|buffer_|scratch_)", l):
                continue
            m = load.match(l)
            if m:
                dst = set(range(int(m.group(1)), int(m.group(2)) + 1))
                assert not (_regs(l.split(",", 1)[1]) & in_flight), (name, l.strip())   # the address operands
                assert not (dst & in_flight), (name, l.strip())
                in_flight |= dst
                continue
            mm = re.match(r"\s+v_mfma\w+ a\[\d+:\d+\], (v\[\d+:\d+\]), (v\[\d+:\d+\]), a\[", l)
            if mm:
                assert not (_regs(mm.group(1)) & in_flight), (name, l.strip())
                in_flight -= _regs(mm.group(2))
                continue
            assert not (_regs(l) & in_flight), (name, l.strip())
        # after the loop: nothing writes or reads a register that may still have a load in flight
        wait = next(i for i in range(end, len(lines)) if re.search(r"s_waitcnt vmcnt\(0\)", lines[i]))
        for l in lines[end:wait]:
            if re.match(r"\s+(v_|ds_|global_|buffer_)", l):
                assert not (_regs(l) & ring), (name, l.strip())
        # the prologue: the first sixteen fragments are not touched before the wait that covers them
        first_mfma = next(i for i, l in enumerate(lines) if "v_mfma" in l)
        loads = [(i, load.match(l)) for i, l in enumerate(lines[:first_mfma])]
        loads = [(i, set(range(int(m.group(1)), int(m.group(2)) + 1))) for i, m in loads if m]
        assert len(loads) == 16, (name, len(loads))
        wait = next(i for i in range(loads[-1][0], len(lines)) if re.search(r"s_waitcnt vmcnt\(0\)", lines[i]))
        issued = set()
        at = dict(loads)
        for i in range(loads[0][0], wait):
            l = lines[i]
            if i in at:
                assert not (_regs(l.split(",", 1)[1]) & issued), (name, l.strip())    # the address operands
                issued |= at[i]
            elif re.match(r"\s+(v_|ds_|global_|buffer_)", l):
                assert not (_regs(l) & issued), (name, l.strip())
