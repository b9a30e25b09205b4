"""Seeded synthetic workloads shared by the tests, the benchmark and the CPU oracle.

This module holds no arithmetic of the method: only parameter sets (ring degree, RNS primes,
plaintext modulus), communication graphs, the grouping of nodes by closed neighbourhood
(index sets only) and float32 gradient vectors drawn from ``numpy.random.default_rng``.
The gradients stand in for the MNIST / CIFAR-10 model updates of the paper's evaluation
(Sec. 6): ciphertext cost depends only on vector length, not on the values.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

SEED = 0x0123456789ABCDEF      # Philox key used by every configuration
RNG_BASE = 20220704            # numpy generator seed = RNG_BASE + configuration number
CBD_ETA = 21


@dataclass
class Config:
    name: str
    number: int
    log2_n: int
    q: List[int]
    t: int
    parties: int
    n_values: int
    frac_bits: int
    topology: str               # "complete" | "circulant" | "circulant-permuted" | "none"
    offsets: tuple = ()
    dist: str = "normal"        # "normal" | "laplace"
    dist_scale: float = 0.01
    batch: int = 0              # transform micro-benchmark only
    seed: int = SEED
    eta: int = CBD_ETA
    _perm: np.ndarray = field(default=None, repr=False)

    @property
    def N(self) -> int:
        return 1 << self.log2_n

    @property
    def L(self) -> int:
        return len(self.q)

    @property
    def C(self) -> int:
        return (self.n_values + self.N - 1) // self.N

    def rng(self) -> np.random.Generator:
        return np.random.default_rng(RNG_BASE + self.number)

    # -- graph ---------------------------------------------------------------------------
    def adjacency(self) -> List[List[int]]:
        """Neighbour lists N_i (without i itself), sorted."""
        P = self.parties
        if self.topology == "complete":
            return [[j for j in range(P) if j != i] for i in range(P)]
        if self.topology in ("circulant", "circulant-permuted"):
            base = [sorted({(i + d) % P for d in self.offsets} | {(i - d) % P for d in self.offsets})
                    for i in range(P)]
            if self.topology == "circulant":
                return base
            perm = self.rng().permutation(P)          # first draw of the generator
            adj = [None] * P
            for i in range(P):
                adj[int(perm[i])] = sorted(int(perm[j]) for j in base[i])
            return adj
        return []

    def groups(self) -> List[List[int]]:
        """Distinct closed neighbourhoods {i} u N_i, ordered by their smallest owner i;
        members sorted by party id."""
        return closed_neighbourhood_groups(self.adjacency())[0]

    def receivers(self) -> List[List[int]]:
        """For every group, the nodes whose closed neighbourhood it is: the receivers of its sum
        (one node per group on the circulant graphs, every node on a complete graph)."""
        groups, owner = closed_neighbourhood_groups(self.adjacency())
        out = [[] for _ in groups]
        for i, g in enumerate(owner):
            out[g].append(i)
        return out

    @property
    def max_group(self) -> int:
        gs = self.groups()
        return max(len(g) for g in gs) if gs else 1

    # -- gradients -----------------------------------------------------------------------
    def gradients(self, parties=None, n_values=None) -> List[np.ndarray]:
        """float32 vectors, one per party, in party order from one generator stream."""
        rng = self.rng()
        if self.topology == "circulant-permuted":
            rng.permutation(self.parties)             # keep the stream aligned with adjacency()
        P = self.parties if parties is None else parties
        n = self.n_values if n_values is None else n_values
        out = []
        for _ in range(P):
            if self.dist == "normal":
                g = rng.normal(0.0, self.dist_scale, size=n)
            else:
                g = rng.laplace(0.0, self.dist_scale, size=n)
            out.append(g.astype(np.float32))
        return out


def closed_neighbourhood_groups(adj):
    """Return (groups, owner_of_node): nodes with the same closed neighbourhood share a group."""
    groups, index, owner = [], {}, []
    for i, nb in enumerate(adj):
        key = tuple(sorted(set(nb) | {i}))
        if key not in index:
            index[key] = len(groups)
            groups.append(list(key))
        owner.append(index[key])
    return groups, owner


_Q30_1024 = [1073707009]
_Q36_4096 = [68719403009, 68719230977, 68719206401]
_Q54_8192 = [18014398508400641, 18014398508138497, 18014398507892737, 18014398507794433]
_Q54_16384 = [18014398508400641, 18014398508138497, 18014398507614209, 18014398507220993,
              18014398506827777, 18014398506729473, 18014398505943041, 18014398504206337]
_K60_65536 = [2, 62, 75, 83, 107, 110, 129, 155, 177, 194, 198, 215, 218, 222, 224, 275]
_Q60_65536 = [(1 << 60) - k * (1 << 17) + 1 for k in _K60_65536]

CONFIGS = {
    "C1": Config("C1", 1, 10, _Q30_1024, 12289, 4, 4096, 8, "complete"),
    "C2": Config("C2", 2, 12, _Q36_4096, 65537, 16, 101770, 10, "circulant", (1, 2)),
    "C3": Config("C3", 3, 13, _Q54_8192, 65537, 32, 1250000, 12, "circulant-permuted", (1, 2, 3),
                 dist="laplace", dist_scale=0.005),
    "C4": Config("C4", 4, 14, _Q54_16384, 65537, 8, 11200000, 14, "complete", dist_scale=0.001),
    "C5": Config("C5", 5, 16, _Q60_65536, 0, 0, 0, 0, "none", batch=64),
}


def toy_config(log2_n: int, q, t, parties: int, n_values: int, frac_bits: int = 4,
               topology: str = "complete", offsets=(), number: int = 99) -> Config:
    """A small parameter set for tests (same recipe, reduced sizes)."""
    return Config("toy", number, log2_n, list(q), t, parties, n_values, frac_bits, topology,
                  tuple(offsets))
