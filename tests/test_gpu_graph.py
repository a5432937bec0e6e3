"""The calls enqueue kernels and nothing else, so a set of ReLU layers can be captured in a HIP graph and replayed
(the one-image ResNet18 set is launch-bound: 17 small tensors).  The graph is replayed several times, with eager
work and synchronisations between the replays and fresh inputs written into the captured buffers, and every replay
is compared with the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2309_04875_amd import hb, workloads

pytestmark = pytest.mark.gpu

SEED = 0x2309048750000001
DEV = "cuda"


def test_batched_relu_set_in_a_hip_graph():
    specs = workloads.resnet18_cifar()
    host, items = [], []
    for spec in specs:
        _, s0, s1 = workloads.materialize(spec)
        d0, d1 = torch.from_numpy(s0).to(DEV), torch.from_numpy(s1).to(DEV)
        host.append((s0, s1))
        items.append((d0, d1, torch.empty_like(d0), torch.empty_like(d1), spec.k, spec.m,
                      hb.hb_tensor_seed(SEED, spec.tensor_id)))
    counts = torch.zeros(64, dtype=torch.int64, device=DEV)
    batch = hb.make_batch(items)
    hb.hb_relu_batch(batch)                       # eager once (also warms up the module)
    torch.cuda.synchronize()

    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        with torch.cuda.graph(graph, stream=stream):
            hb.hb_relu_batch(batch)               # one launch per slice width
            hb.hb_drelu(items[0][0], items[0][1], specs[0].k, specs[0].m, items[0][6], items[1][2], items[1][3])
            hb.hb_eco_scan(items[0][0], items[0][1], counts)     # clears its counters with a kernel, not a memset
    torch.cuda.synchronize()

    rng = np.random.default_rng(5)
    for replay in range(3):
        if replay:                                # new shares in the captured input buffers
            for t, (spec, (s0, s1)) in enumerate(zip(specs, host)):
                s0[:] = rng.integers(0, 1 << 64, spec.n, dtype=np.uint64).view(np.int64)
                s1[:] = rng.integers(0, 1 << 64, spec.n, dtype=np.uint64).view(np.int64)
                items[t][0].copy_(torch.from_numpy(s0))
                items[t][1].copy_(torch.from_numpy(s1))
        for it in items:                          # eager work between replays: wipe the outputs
            it[2].zero_()
            it[3].zero_()
        counts.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for t, (spec, (s0, s1)) in enumerate(zip(specs, host)):
            if t == 1:                            # its outputs were overwritten by the captured hb_drelu of tensor 0
                e0, e1, _ = oracle.drelu(host[0][0], host[0][1], specs[0].k, specs[0].m, items[0][6])
            else:
                e0, e1, _ = oracle.relu(s0, s1, spec.k, spec.m, items[t][6])
            assert np.array_equal(items[t][2].cpu().numpy(), e0), (replay, t)
            assert np.array_equal(items[t][3].cpu().numpy(), e1), (replay, t)
        expect = oracle.eco_scan(host[0][0], host[0][1])
        assert np.array_equal(counts.cpu().numpy().view(np.uint64), np.asarray(expect, dtype=np.uint64)), replay
