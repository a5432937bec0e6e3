"""GPU parity of the prepared-set entry points (hb_plan_create / hb_plan_run / hb_plan_destroy) and of the two
wave-tile shapes against the oracle, bit for bit.

Short launches take the small wave-tile kernels and long ones the large wave-tile kernels; the environment
variable HB_SMALL_TILE_LIMIT (read once, when the library is loaded) moves the switch-over, so child processes
run the same parity sweep with the small tiles switched off (0) and forced on for every size (a huge limit).
"""
import ctypes
import os
import subprocess
import sys

import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb, workloads

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SEED = 0x2309048750000001
DEV = "cuda"


def _dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def _set(specs, root):
    items, host = [], []
    for spec in specs:
        _, s0, s1 = workloads.materialize(spec)
        d0, d1 = _dev(s0), _dev(s1)
        items.append((d0, d1, torch.zeros_like(d0), torch.zeros_like(d1), spec.k, spec.m,
                      hb.hb_tensor_seed(root, spec.tensor_id)))
        host.append((s0, s1))
    return items, host


@pytest.mark.parametrize("relu", [True, False])
@pytest.mark.parametrize("dealer", [hb.HB_DEALER_PER_GATE, hb.HB_DEALER_SHARED_MASK])
def test_plan_matches_oracle_on_the_one_image_set_and_mixed_widths(relu, dealer):
    specs = workloads.resnet18_cifar()
    kms = [(12, 20), (8, 14), (0, 64), (5, 12), (3, 4), (8, 40), (2, 3), (8, 18)]
    specs = specs + [workloads.TensorSpec("mixed", 100 + i, (n,), k, m, 2.0, "normal", 500 + i)
                     for i, ((k, m), n) in enumerate(zip(kms, (1000, 1, 513, 4097, 77, 2049, 300, 0)))]
    items, host = _set(specs, SEED)
    plan = hb.hb_plan_create(items, relu, dealer)
    fn = oracle.relu if relu else oracle.drelu
    for rep in range(2):                       # a plan is run many times: the second run after fresh inputs
        bits = hb.hb_plan_run(plan)
        ebits = 0
        for (d0, d1, o0, o1, k, m, seed), (s0, s1) in zip(items, host):
            e0, e1, b = fn(s0, s1, k, m, seed, variant=dealer)
            assert np.array_equal(o0.cpu().numpy(), e0) and np.array_equal(o1.cpu().numpy(), e1), (k, m, rep)
            ebits += b
        assert bits == ebits
        rng = np.random.default_rng(rep)
        for i, (d0, d1, o0, o1, k, m, seed) in enumerate(items):
            s0 = rng.integers(0, 1 << 64, d0.numel(), dtype=np.uint64).view(np.int64)
            host[i] = (s0, host[i][1])
            d0.copy_(_dev(s0))
            o0.zero_()
            o1.zero_()
    hb.hb_plan_destroy(plan)
    hb.hb_plan_destroy(plan)                   # closing twice is harmless in the binding


def test_plan_in_a_hip_graph_and_on_a_side_stream():
    items, host = _set(workloads.resnet18_cifar(), SEED + 1)
    plan = hb.hb_plan_create(items, True)
    hb.hb_plan_run(plan)
    torch.cuda.synchronize()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            hb.hb_plan_run(plan)
    torch.cuda.synchronize()
    for rep in range(3):
        for (d0, d1, o0, o1, k, m, seed) in items:
            o0.zero_()
            o1.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (d0, d1, o0, o1, k, m, seed), (s0, s1) in zip(items, host):
            e0, e1, _ = oracle.relu(s0, s1, k, m, seed)
            assert np.array_equal(o0.cpu().numpy(), e0) and np.array_equal(o1.cpu().numpy(), e1), (k, m, rep)


def test_plan_errors():
    n = 512
    t = [torch.zeros(n, dtype=torch.int64, device=DEV) for _ in range(8)]
    good = [(t[0], t[1], t[2], t[3], 12, 20, 1), (t[4], t[5], t[6], t[7], 8, 14, 2)]
    handle = ctypes.c_void_p(1)
    arr = hb.make_batch(good)
    arr[1].m = 8                                            # bad slice
    assert hb.raw("hb_plan_create", arr, 2, 1, 0, ctypes.byref(handle)) == hb.HB_EINVAL and not handle.value
    arr = hb.make_batch(good)
    arr[1].out0 = arr[0].share0                             # output over another tensor's input
    assert hb.raw("hb_plan_create", arr, 2, 1, 0, ctypes.byref(handle)) == hb.HB_EINVAL and not handle.value
    arr = hb.make_batch(good)
    assert hb.raw("hb_plan_create", arr, 2, 1, 7, ctypes.byref(handle)) == hb.HB_EINVAL     # unknown dealer layout
    assert hb.raw("hb_plan_create", arr, 2, 1, 0, None) == hb.HB_EINVAL
    assert hb.raw("hb_plan_run", None, None, None) == hb.HB_EINVAL
    hb.raw("hb_plan_destroy", None)
    empty = hb.hb_plan_create([], True)
    assert hb.hb_plan_run(empty) == 0
    plan = hb.hb_plan_create(good, True)
    assert hb.hb_plan_run(plan) == n * (241 + 213)
    torch.cuda.synchronize()


CHILD = r"""
import numpy as np, torch, oracle
from paper_2309_04875_amd import hb
rng = np.random.default_rng(41)
dev = "cuda"
for w in list(range(1, 33)):
    L = min(64 // w, 32)
    for n in (1, L + 1, 16 * L - 1, 16 * L, 16 * L + 1, 64 * L + 3, 3 * 256 * L + L // 2 + 1, 70001):
        k = int(rng.integers(0, 64 - w + 1)); m = k + w; seed = int(rng.integers(0, 1 << 63))
        sh = [rng.integers(0, 1 << 64, n + 1, dtype=np.uint64).view(np.int64) for _ in range(2)]
        for off in (0, 1):                                   # 16-byte and 8-byte aligned buffers
            d = [torch.from_numpy(s).to(dev)[off:] for s in sh]
            g0, g1, _ = hb.hb_relu(d[0], d[1], k, m, seed)
            e0, e1, _ = oracle.relu(sh[0][off:], sh[1][off:], k, m, seed)
            assert np.array_equal(g0.cpu().numpy(), e0) and np.array_equal(g1.cpu().numpy(), e1), ("relu", w, n, off)
            g0, g1, _ = hb.hb_drelu(d[0], d[1], k, m, seed)
            e0, e1, _ = oracle.drelu(sh[0][off:], sh[1][off:], k, m, seed)
            assert np.array_equal(g0.cpu().numpy(), e0) and np.array_equal(g1.cpu().numpy(), e1), ("drelu", w, n, off)
# a batch with more tensors of one width than one launch holds, ragged sizes, in place
items, host = [], []
for i in range(30):
    n = 100 + 37 * i
    s0 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64); s1 = rng.integers(0, 1 << 64, n, dtype=np.uint64).view(np.int64)
    d0, d1 = torch.from_numpy(s0).to(dev), torch.from_numpy(s1).to(dev)
    items.append((d0, d1, d0, d1, 12, 20, 900 + i)); host.append((s0, s1))
hb.hb_relu_batch(items)
for (d0, d1, o0, o1, k, m, seed), (s0, s1) in zip(items, host):
    e0, e1, _ = oracle.relu(s0, s1, k, m, seed)
    assert np.array_equal(o0.cpu().numpy(), e0) and np.array_equal(o1.cpu().numpy(), e1), ("batch", seed)
print("tile shapes ok")
"""


@pytest.mark.parametrize("limit", ["0", "1000000000"])
def test_every_width_on_large_tiles_only_and_on_small_tiles_only(limit):
    env = dict(os.environ, HB_SMALL_TILE_LIMIT=limit, PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    proc = subprocess.run([sys.executable, "-c", CHILD], env=env, cwd=ROOT, stdout=subprocess.PIPE,
                          stderr=subprocess.STDOUT, text=True, timeout=600)
    assert proc.returncode == 0 and "tile shapes ok" in proc.stdout, proc.stdout[-2000:]
