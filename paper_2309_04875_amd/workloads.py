"""Seeded synthetic inputs for the secret-shared ReLU path.

This module only makes inputs: plaintext activations, their 2^16 fixed-point encoding
(paper Sec. 2.2, "Operation of CrypTen": x = round(D * x_f), D = 2^16 per Sec. 3.1) and a
2-party additive sharing on Z_2^64.  It contains none of the protocol's arithmetic and no
dealer randomness, so both the GPU library's tests and the CPU oracle's tests draw from it.

The tensors stand in for ResNet18 activations on CIFAR-sized (3x32x32) and ImageNet-sized
(3x224x224) inputs (paper Sec. 2.3 and Sec. 5): only the shapes and the fixed-point scale are
taken from the paper; values are Gaussian / Laplace noise.
"""
from dataclasses import dataclass
from typing import Iterator, List, Tuple

import numpy as np

FIXED_POINT_BITS = 16
SCALE = float(1 << FIXED_POINT_BITS)

# ReLU input shapes (C, H, W) of ResNet18 for one image.
RESNET18_32 = [(64, 32, 32)] * 5 + [(128, 16, 16)] * 4 + [(256, 8, 8)] * 4 + [(512, 4, 4)] * 4
RESNET18_224 = [(64, 112, 112)] + [(64, 56, 56)] * 4 + [(128, 28, 28)] * 4 + [(256, 14, 14)] * 4 + [(512, 7, 7)] * 4


@dataclass(frozen=True)
class TensorSpec:
    """One ReLU input tensor of a workload."""
    workload: str
    tensor_id: int
    shape: Tuple[int, ...]
    k: int              # lowest kept bit
    m: int              # one past the highest kept bit
    sigma: float        # scale of the plaintext distribution (float units)
    dist: str           # "normal" or "laplace"
    data_seed: int      # seed of the value / share streams

    @property
    def n(self) -> int:
        return int(np.prod(self.shape, dtype=np.int64))

    @property
    def w(self) -> int:
        return self.m - self.k


def _rng(*key) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([int(v) for v in key])))


def encode_fixed_point(v: np.ndarray) -> np.ndarray:
    """round-half-even(v * 2^16) as int64."""
    return np.rint(v * SCALE).astype(np.int64)


def share_additively(x: np.ndarray, rng: np.random.Generator) -> Tuple[np.ndarray, np.ndarray]:
    """share0 uniform on Z_2^64, share1 = x - share0 (mod 2^64); both returned as int64."""
    share0 = rng.integers(0, 1 << 64, size=x.shape, dtype=np.uint64)
    share1 = x.view(np.uint64) - share0          # unsigned arithmetic wraps mod 2^64
    return share0.view(np.int64), share1.view(np.int64)


def plaintext(spec: TensorSpec, chunk: int = 1 << 24) -> Iterator[np.ndarray]:
    """Yield the fixed-point plaintext of `spec` in flat chunks (deterministic in the chunk size)."""
    rng = _rng(spec.data_seed, 0)
    left = spec.n
    while left > 0:
        c = min(chunk, left)
        if spec.dist == "normal":
            v = rng.standard_normal(c) * spec.sigma
        elif spec.dist == "laplace":
            v = rng.laplace(0.0, spec.sigma, c)
        else:
            raise ValueError(spec.dist)
        yield encode_fixed_point(v)
        left -= c


def materialize(spec: TensorSpec, chunk: int = 1 << 24) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """(x, share0, share1) of a tensor, flat int64 arrays.  The chunk size is part of the recipe."""
    share_rng = _rng(spec.data_seed, 1)
    xs, s0s, s1s = [], [], []
    for x in plaintext(spec, chunk):
        s0, s1 = share_additively(x, share_rng)
        xs.append(x)
        s0s.append(s0)
        s1s.append(s1)
    if not xs:
        e = np.empty(0, dtype=np.int64)
        return e, e.copy(), e.copy()
    return np.concatenate(xs), np.concatenate(s0s), np.concatenate(s1s)


def flat_normal(n: int = 65536, k: int = 0, m: int = 64, seed: int = 1) -> TensorSpec:
    """Flat tensor, v ~ N(0, sigma = 2) at 2^16 scale."""
    return TensorSpec("flat_normal", 0, (n,), k, m, 2.0, "normal", seed)


def _per_tensor(workload: str, shapes, batch: int, seed: int, k_range, widths, single_km=None) -> List[TensorSpec]:
    """Per-tensor sigma is log-uniform in [0.5, 4]; k and w are drawn per tensor unless fixed."""
    meta = _rng(seed, 12345)
    specs = []
    for t, chw in enumerate(shapes):
        sigma = float(np.exp(meta.uniform(np.log(0.5), np.log(4.0))))
        k = int(meta.integers(k_range[0], k_range[1] + 1))
        w = int(widths[int(meta.integers(0, len(widths)))])
        if single_km is not None:
            k, w = single_km[0], single_km[1] - single_km[0]
        shape = ((batch,) if batch > 1 else ()) + tuple(chw)
        specs.append(TensorSpec(workload, t, shape, k, k + w, sigma, "normal", seed * 1000 + t))
    return specs


def resnet18_cifar(batch: int = 1, seed: int = 2, single_km=None) -> List[TensorSpec]:
    """17 ReLU inputs of ResNet18 on 3x32x32 images; k in [8,14], m = k + 8 unless single_km."""
    return _per_tensor("resnet18_cifar_b%d" % batch, RESNET18_32, batch, seed, (8, 14), (8,), single_km)


def resnet18_cifar_batch512(seed: int = 3) -> List[TensorSpec]:
    """The headline throughput set: batch 512, one (k, m) = (12, 20) for every tensor."""
    return _per_tensor("resnet18_cifar_b512_k12_m20", RESNET18_32, 512, seed, (8, 14), (8,), (12, 20))


def width_sweep(n: int = 1 << 26, seed: int = 4, widths=(64, 32, 16, 8, 6, 4)) -> List[TensorSpec]:
    """Flat Laplace(0,1) tensor at k = 8 for each width; w = 64 cannot start at bit 8 and uses (0, 64)."""
    out = []
    for t, w in enumerate(widths):
        k = 8 if 8 + w <= 64 else 0
        out.append(TensorSpec("width_sweep_w%d" % w, t, (n,), k, k + w, 1.0, "laplace", seed))
    return out


def resnet18_imagenet(batch: int = 64, seed: int = 5) -> List[TensorSpec]:
    """17 ReLU inputs of ResNet18 on 3x224x224 images; k in [6,16], w in {6, 8, 10} per tensor."""
    return _per_tensor("resnet18_imagenet_b%d" % batch, RESNET18_224, batch, seed, (6, 16), (6, 8, 10))


def materialize_on_device(spec: TensorSpec, device="cuda"):
    """(x, share0, share1) as flat int64 tensors generated on the GPU with torch's seeded generator.

    Same distributions as `materialize` (different random streams); used where the host generator
    would dominate the run time (the batch-512 and 224x224 sets, the 2^26 sweep).
    """
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(spec.data_seed))
    n = spec.n
    if spec.dist == "normal":
        v = torch.randn(n, generator=g, device=device, dtype=torch.float64) * spec.sigma
    elif spec.dist == "laplace":
        u = torch.rand(n, generator=g, device=device, dtype=torch.float64) - 0.5
        v = -spec.sigma * torch.sign(u) * torch.log1p(-2.0 * u.abs())
        del u
    else:
        raise ValueError(spec.dist)
    x = torch.round(v * SCALE).to(torch.int64)
    del v
    hi = torch.randint(0, 1 << 32, (n,), generator=g, device=device, dtype=torch.int64)
    lo = torch.randint(0, 1 << 32, (n,), generator=g, device=device, dtype=torch.int64)
    share0 = (hi << 32) | lo
    del hi, lo
    share1 = x - share0           # int64 arithmetic wraps mod 2^64
    return x, share0, share1
