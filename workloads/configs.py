"""The five synthetic workload shapes (single job, Q = K, one batch per r-subset).

Each stands in for a shape the method is meant for; the paper itself measures
on no dataset, so these seeded synthetic tensors are the whole workload.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import comb


@dataclass(frozen=True)
class Workload:
    name: str
    K: int          # nodes
    r: int          # replication mu*K
    Q: int          # functions
    N: int          # files
    T: int          # elements per intermediate value
    sigma: float    # std of the fp32 values
    modes: tuple    # payload modes the shape is run in

    @property
    def c(self):
        return self.Q // self.K

    @property
    def W(self):
        return self.c * self.T

    @property
    def G(self):
        return comb(self.K, self.r + 1)

    @property
    def m(self):
        return self.N // comb(self.K, self.r)

    @property
    def v_elems(self):
        return self.Q * self.N * self.T

    @property
    def v_bytes(self):
        return 4 * self.v_elems


CONFIGS = {
    "cfg1_tiny": Workload("cfg1_tiny", 4, 2, 4, 12, 256, 1.0, ("f32", "u32")),
    "cfg2_k10": Workload("cfg2_k10", 10, 3, 10, 120, 4096, 1.0, ("f32", "u32")),
    "cfg3_gradient": Workload("cfg3_gradient", 8, 2, 8, 28, 3_200_000, 0.01, ("f32",)),
    "cfg4_k16": Workload("cfg4_k16", 16, 3, 16, 560, 4096, 1.0, ("f32",)),
    "cfg5_k24": Workload("cfg5_k24", 24, 4, 24, 10626, 2048, 1.0, ("f32", "u32")),
}


def get(name: str) -> Workload:
    return CONFIGS[name]
