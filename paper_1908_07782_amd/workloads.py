"""Seeded synthetic workloads for the segmented-gossip round.

This module only describes shapes and draws random inputs; it contains none of the
method's arithmetic, so both the GPU library's tests and the CPU oracle's tests may
use it.  The aggregation round is value-oblivious (no data-dependent branch), so
independent draws with the shapes of flattened model parameter vectors stand in for
the trained CNN parameters of the paper's experiments (Sec. 5.1).

Each configuration: N workers, P parameters per worker, S segments, R replicas,
T rounds, value distribution of the parameters (second number = standard deviation,
or half-width for the uniform case), the peer-hash seed, and for the fused
local-step workload the learning rate and gradient standard deviation.
"""
from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    N: int
    P: int
    S: int
    R: int
    rounds: int
    dist: str            # "normal" or "uniform"
    scale: float         # std for normal, half-width for uniform
    data_seed: int = 0
    hash_seed: int = 0
    fused: bool = False
    lr: float = 0.0
    grad_std: float = 0.0

    @property
    def ld(self):
        return row_pitch(self.P)

    @property
    def algorithmic_bytes_per_round(self):
        # (R+1) reads + 1 write of 4 bytes per element per worker
        return 4 * (self.R + 2) * self.N * self.P


def row_pitch(P, multiple=64):
    """Row pitch in elements: P rounded up to a multiple of 64 floats (256 bytes)."""
    return (P + multiple - 1) // multiple * multiple


WORKLOADS = {
    # tiny: fits in cache, launch-latency bound
    "c1_tiny": Workload("c1_tiny", N=4, P=65_536, S=8, R=2, rounds=1,
                        dist="normal", scale=0.05),
    # ResNet-18-sized flat vector; last segment takes the remainder
    "c2_resnet18": Workload("c2_resnet18", N=32, P=11_689_512, S=32, R=4, rounds=10,
                            dist="normal", scale=0.02),
    # ResNet-50-sized; the paper's default (S, R) = (10, 2) at about 30 workers
    "c3_resnet50": Workload("c3_resnet50", N=32, P=25_557_032, S=10, R=2, rounds=10,
                            dist="normal", scale=0.02, hash_seed=7),
    # prime P, fused local SGD step then gossip
    "c4_prime_fused": Workload("c4_prime_fused", N=100, P=1_000_003, S=7, R=3, rounds=20,
                               dist="uniform", scale=0.1, fused=True, lr=0.01, grad_std=1e-3),
    # BERT-large-sized, the model size the paper's introduction cites
    "c5_bertlarge": Workload("c5_bertlarge", N=16, P=335_141_888, S=16, R=4, rounds=5,
                             dist="normal", scale=0.02),
}


def _generator(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def fill_params(buf, wl, P=None):
    """Fill buf[:, :P] (a (N, ld) float32 tensor on any device) with the workload's
    parameter distribution, one independent row per worker, row by row so that peak
    temporary memory is one row.  Padding columns are left as they are."""
    P = wl.P if P is None else P
    g = _generator(wl.data_seed, buf.device)
    for w in range(buf.shape[0]):
        row = buf[w, :P]
        if wl.dist == "normal":
            row.normal_(0.0, wl.scale, generator=g)
        elif wl.dist == "uniform":
            row.uniform_(-wl.scale, wl.scale, generator=g)
        else:
            raise ValueError(wl.dist)
    return buf


def fill_grads(buf, wl, rnd, P=None):
    """Fill buf[:, :P] with the round's synthetic gradients g ~ N(0, grad_std),
    redrawn every round from seed (data_seed + 1000003 * (rnd + 1))."""
    P = wl.P if P is None else P
    g = _generator(wl.data_seed + 1000003 * (int(rnd) + 1), buf.device)
    for w in range(buf.shape[0]):
        buf[w, :P].normal_(0.0, wl.grad_std, generator=g)
    return buf


def dataset_sizes(N, seed=0, device="cpu"):
    """Synthetic per-worker dataset sizes |D_j|: integers in [100, 2000) as float32."""
    g = _generator(seed + 77, "cpu")
    d = torch.randint(100, 2000, (N,), generator=g).to(torch.float32)
    return d.to(device)


def small_case(N, P, S, R, seed=0, dist="normal", scale=0.05, hash_seed=0, **kw):
    return Workload(f"small_N{N}_P{P}_S{S}_R{R}", N=N, P=P, S=S, R=R, rounds=1,
                    dist=dist, scale=scale, data_seed=seed, hash_seed=hash_seed, **kw)
