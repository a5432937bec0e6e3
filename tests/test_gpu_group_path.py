"""The thread-per-group kernels serve slice widths above 32 by default; with HB_KERNEL=group in the environment
(read once, when the library is loaded) they serve every width.  This runs a parity sweep in a child process
that has the variable set, so that those kernels stay covered for all widths."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import numpy as np, torch, oracle
from paper_2309_04875_amd import hb
rng = np.random.default_rng(31)
dev = "cuda"
for w in list(range(1, 17)) + [21, 31, 32, 33, 64]:
    L = min(64 // w, 32)
    for n in (1, L + 1, 256 * L, 3 * 256 * L + L // 2 + 1):
        k = int(rng.integers(0, 64 - w + 1)); m = k + w; seed = int(rng.integers(0, 1 << 63))
        sh = [rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64) for _ in range(4)]
        d = [torch.from_numpy(s).to(dev) for s in sh]
        for layout in (0, 1):
            g0, g1, _ = hb.hb_relu_ex(d[0], d[1], k, m, seed, layout)
            e0, e1, _ = oracle.relu(sh[0], sh[1], k, m, seed, variant=layout)
            assert np.array_equal(g0.cpu().numpy(), e0) and np.array_equal(g1.cpu().numpy(), e1), ("relu", w, n, layout)
        g0, g1, _ = hb.hb_drelu(d[0], d[1], k, m, seed)
        e0, e1, _ = oracle.drelu(sh[0], sh[1], k, m, seed)
        assert np.array_equal(g0.cpu().numpy(), e0) and np.array_equal(g1.cpu().numpy(), e1), ("drelu", w, n)
        for parties in (3, 4):
            outs, _ = hb.hb_relu_mp(d[:parties], k, m, seed)
            exp, _ = oracle.mp_relu(sh[:parties], k, m, seed)
            for q in range(parties):
                assert np.array_equal(outs[q].cpu().numpy(), exp[q]), ("mp", parties, w, n, q)
print("group path ok")
"""


def test_every_width_through_the_group_kernels():
    env = dict(os.environ, HB_KERNEL="group", PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    proc = subprocess.run([sys.executable, "-c", CHILD], env=env, cwd=ROOT, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)
    assert proc.returncode == 0 and "group path ok" in proc.stdout, proc.stdout[-2000:]
