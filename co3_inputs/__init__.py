"""Seeded synthetic gradient generators and workload descriptors.

Shared by the oracle-side and HIP-side tests and by the benchmark.  This
module holds none of the codec's arithmetic: it only draws i.i.d. generalised
normal samples (the paper's statistical model of DNN gradients, Sec. II-C) in
the shapes of the five benchmark workloads.

Sampler: x = alpha * s * G**(1/beta), G ~ Gamma(1/beta, 1), s = +-1 fair, so
that the density is proportional to exp(-(|x|/alpha)**beta).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

BASE_SEED = 20220309


def rng_for(cfg: int, point: int = 0, u: int = 0, t: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence([BASE_SEED, cfg, point, u, t])))


def gennorm(rng: np.random.Generator, n: int, beta: float, alpha: float) -> np.ndarray:
    """n samples of GenNorm(beta, scale alpha), drawn in float64, returned as float32."""
    g = rng.standard_gamma(1.0 / beta, size=n)
    s = rng.integers(0, 2, size=n).astype(np.float64) * 2.0 - 1.0
    return (alpha * s * g ** (1.0 / beta)).astype(np.float32)


def gennorm_outliers(rng, n: int, beta: float, alpha: float, frac: float, factor: float) -> np.ndarray:
    """GenNorm(beta, alpha) with a fraction ``frac`` of samples drawn at ``factor`` times the scale."""
    x = gennorm(rng, n, beta, alpha)
    mask = rng.random(n) < frac
    x[mask] *= np.float32(factor)
    return x


def resnet18_cifar_tensor_sizes() -> List[int]:
    """Parameter-tensor sizes of the CIFAR-stem ResNet-18, in network order (62 tensors)."""
    sizes: List[int] = [3 * 64 * 9, 64, 64]                     # stem conv + its norm scale/shift
    cin = 64
    for cout, first_stride in ((64, 1), (128, 2), (256, 2), (512, 2)):
        for block in range(2):
            c_in = cin if block == 0 else cout
            sizes += [c_in * cout * 9, cout, cout, cout * cout * 9, cout, cout]
            if block == 0 and (first_stride != 1 or c_in != cout):
                sizes += [c_in * cout, cout, cout]              # 1x1 projection shortcut + norm
        cin = cout
    sizes += [512 * 10, 10]                                     # classifier weight, bias
    assert len(sizes) == 62 and sum(sizes) == 11_173_962
    return sizes


def seg_offsets(sizes: Sequence[int]) -> np.ndarray:
    return np.concatenate([[0], np.cumsum(np.asarray(sizes, dtype=np.int64))]).astype(np.int64)


def group_small_tensors(sizes: Sequence[int], min_elems: int = 16384) -> Tuple[int, ...]:
    """Sizes of groups of consecutive tensors in which every tensor below ``min_elems`` elements joins the
    large tensor before it (leading small tensors join the first large one): the groups that share a code
    when one code per tensor would give tables to tensors of a few hundred elements."""
    groups = []
    pending = 0
    for s in sizes:
        if s >= min_elems:
            groups.append(s + pending)
            pending = 0
        elif groups:
            groups[-1] += s
        else:
            pending += s
    if pending:
        groups.append(pending)
    return tuple(groups)


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: U clients x n elements, format E/M, T iterations."""
    name: str
    cfg: int
    U: int
    n: int
    E: int
    M: int
    T: int
    sizes: Optional[Tuple[int, ...]] = None        # tensor sizes (None: one segment)
    table: str = "empirical"
    note: str = ""

    @property
    def seg_off(self) -> np.ndarray:
        return seg_offsets(self.sizes if self.sizes is not None else [self.n])


def c1() -> Workload:
    return Workload("C1", 1, 1, 65_536, 3, 1, 5)


def c2() -> Workload:
    sz = tuple(resnet18_cifar_tensor_sizes())
    return Workload("C2", 2, 1, sum(sz), 4, 3, 100, sizes=sz)


def c3(n: int = 11_173_962, U: int = 10) -> Workload:
    return Workload("C3", 3, U, n, 3, 0, 50)


def c4(n: int = 100_000_000) -> Workload:
    return Workload("C4", 4, 1, n, 5, 2, 20, table="model+empirical")


C5_FORMATS = ((2, 0), (3, 1), (4, 3), (5, 2))
C5_BETAS = (0.5, 1.0, 2.0)


def c5(point: int, n: int = 25_000_000, U: int = 16) -> Workload:
    E, M = C5_FORMATS[point // len(C5_BETAS)]
    return Workload(f"C5[{point}]", 5, U, n, E, M, 10, note=f"beta={C5_BETAS[point % len(C5_BETAS)]}")


# ---------------------------------------------------------------------------
# per-workload parameter draws (fixed once per workload) and gradient draws
# ---------------------------------------------------------------------------
def c2_tensor_scales() -> np.ndarray:
    """Per-tensor scale alpha = 10**Uniform(-5, -2), drawn once."""
    r = rng_for(2, 0, 0, 10_000)
    return 10.0 ** r.uniform(-5.0, -2.0, size=62)


def c3_client_betas(U: int = 10) -> np.ndarray:
    r = rng_for(3, 0, 0, 10_000)
    return r.uniform(0.5, 1.5, size=U)


def host_gradient(w: Workload, u: int, t: int, n: Optional[int] = None, point: int = 0) -> np.ndarray:
    """Gradient of client ``u`` at iteration ``t`` (1-based) for workload ``w``, drawn on the host.

    ``n`` overrides the element count (reduced-size parity cases keep the distribution).
    """
    n = w.n if n is None else n
    r = rng_for(w.cfg, point, u, t)
    if w.cfg == 1:
        return gennorm(r, n, 1.0, 1e-3)
    if w.cfg == 2:
        assert n == w.n
        scales = c2_tensor_scales()
        return np.concatenate([gennorm(r, s, 0.8, a) for s, a in zip(w.sizes, scales)])
    if w.cfg == 3:
        return gennorm(r, n, float(c3_client_betas(max(w.U, 10))[u]), 1e-3)
    if w.cfg == 4:
        return gennorm_outliers(r, n, 1.0, 1e-4, 1e-4, 100.0)
    if w.cfg == 5:
        return gennorm(r, n, C5_BETAS[point % len(C5_BETAS)], 1e-3)
    raise ValueError(w.cfg)


def device_gennorm(n: int, beta: float, alpha: float, seed: int, device="cuda"):
    """Same sampler on the GPU (torch generator), for inputs too large to draw on the host quickly."""
    import torch
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    conc = torch.full((n,), 1.0 / beta, dtype=torch.float32, device=device)
    g = torch._standard_gamma(conc, generator=gen)
    s = torch.randint(0, 2, (n,), generator=gen, device=device, dtype=torch.int8).to(torch.float32) * 2.0 - 1.0
    x = (alpha * s.double() * g.double() ** (1.0 / beta)).to(torch.float32)
    return x


def device_gennorm_outliers(n: int, beta: float, alpha: float, frac: float, factor: float, seed: int, device="cuda"):
    """device_gennorm with a fraction ``frac`` of the samples at ``factor`` times the scale (the C4 recipe)."""
    import torch
    x = device_gennorm(n, beta, alpha, seed, device)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 1)
    mask = torch.rand(n, device=device, generator=gen) < frac
    return torch.where(mask, x * factor, x)
