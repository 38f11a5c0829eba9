"""Host-side check of the streaming projection kernel (`csrc/gemm_stream.hip`), whose weight loads are
inline assembly that the compiler does not track: every wait of its main loop is a hand-written count.
The counts of the source are re-derived here from the issue order of a wave's memory instructions.
(That the registers of loads in flight stay allocated until their wait holds by construction in the
source: every wait takes the registers it covers as in/out operands.)  No GPU needed.
"""
import os
import re

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
    assert "wait_vm_for(bq[slot][0], 15 + 2 * pieces_window(ks))" in text
    assert "wait_vm_for(bq[slot][1], 14 + 2 * pieces_window(ks) + (ks < 8 ? 2 : 0))" in text
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
