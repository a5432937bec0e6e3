"""The fused kernels must draw every dealer word that the protocol consumes (no GPU needed: compiles a probe).

The output shares of hb_relu depend on less than the protocol computes: the P shares of the adder enter only through
openings, and the B2A share r^A_0 cancels in the opened value delta of the multiply.
A compiler that sees this algebra deletes the SplitMix64 evaluations behind those values, and throughput figures would
then be those of a shortened protocol.  The kernels are written so that it cannot; this test counts the SplitMix64
evaluations in the machine code of the bounds-check-free tile body (one copy of the arithmetic) and compares them
with the protocol's count per wavefront lane: the words of one group (5 per evaluated gate, + the B2A word) plus the
arithmetic words of the L elements a lane finishes.
"""
import os
import re
import shutil
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def _expected(w, op, shared):
    R = 0 if w == 1 else (w - 1).bit_length()
    L = min(64 // w, 32)
    if shared:      # gate 0: 5 words; a round: 8 words, 5 in the last round (no P-update)
        group = 5 + (8 * (R - 1) + 5 if R else 0)
    else:           # 5 words per evaluated gate: gate 0 and two per round but the last P-update
        group = 5 * (2 * R if R else 1)
    per_element = {"relu": 6, "drelu": 1}[op]
    return group + 1 + per_element * L


def _expected_mp(w, op, parties):
    R = 0 if w == 1 else (w - 1).bit_length()
    L = min(64 // w, 64 // parties)
    gates = 2 * R if R else 1                               # per adder: gate 0 and two per round but the last P-update
    group = (parties - 1) * gates * (3 * parties - 1) + 1   # p - 1 adders, 3p - 1 words per gate, + the B2A word
    per_element = {"relu": 4 * parties - 2, "drelu": parties - 1}[op]
    return group + per_element * L


@pytest.fixture(scope="module")
def probe_asm():
    if not os.path.exists(HIPCC):
        pytest.skip("hipcc not available")
    tmp = tempfile.mkdtemp(prefix="hb_probe_")
    try:
        out = os.path.join(tmp, "probe.s")
        cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
               "-packed-fp32-ops", "-I" + os.path.join(ROOT, "paper_2309_04875_amd", "csrc"), "-S", "--cuda-device-only",
               "-o", out, os.path.join(ROOT, "tests", "probes", "dealer_words_probe.hip")]
        subprocess.run(cmd, check=True, stdout=subprocess.PIPE, stderr=subprocess.PIPE)
        with open(out) as f:
            return f.read()
    finally:
        shutil.rmtree(tmp, ignore_errors=True)


def _mix64_count(asm, kernel):
    start = asm.index("\n%s:" % kernel)
    body = asm[start:asm.index("s_endpgm", start)]
    # each SplitMix64 evaluation has exactly one 64-bit logical right shift by 30, by 27 and by 31
    counts = [len(re.findall(r"v_lshrrev_b64 v\[\d+:\d+\], %d, v\[\d+:\d+\]" % s, body)) for s in (30, 27, 31)]
    assert counts[0] == counts[1] == counts[2], counts
    return counts[0]


@pytest.mark.parametrize("kernel,w,op,shared", [
    ("probe_w8_relu", 8, "relu", False),
    ("probe_w8_drelu", 8, "drelu", False),
    ("probe_w8_relu_shared", 8, "relu", True),
    ("probe_w16_relu", 16, "relu", False),
    ("probe_w6_relu", 6, "relu", False),
])
def test_every_dealer_word_is_drawn(probe_asm, kernel, w, op, shared):
    assert _mix64_count(probe_asm, kernel) == _expected(w, op, shared)


@pytest.mark.parametrize("kernel,w,op,parties", [
    ("probe_p3_w8_relu", 8, "relu", 3),
    ("probe_p3_w8_drelu", 8, "drelu", 3),
    ("probe_p4_w8_relu", 8, "relu", 4),
])
def test_every_dealer_word_is_drawn_multi_party(probe_asm, kernel, w, op, parties):
    assert _mix64_count(probe_asm, kernel) == _expected_mp(w, op, parties)
