"""The synthetic workload shapes.

The first five are single-job shapes (Q = K, one batch per r-subset of the
cluster).  Each stands in for a shape the method is meant for; the paper itself
measures on no dataset, so these seeded synthetic tensors are the whole
workload.  `jobs_k8` is the paper's own schedule (J = C(K, r+1) jobs, two
stages per subset, Sec. IV) at a size that fills the device.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import comb


@dataclass(frozen=True)
class Workload:
    name: str
    K: int          # nodes
    r: int          # replication mu*K
    Q: int          # functions per job
    N: int          # files per job
    T: int          # elements per intermediate value
    sigma: float    # std of the fp32 values
    modes: tuple    # payload modes the shape is run in
    jobs: bool = False   # True: the paper's J-job schedule; False: one job over the whole cluster
    compression: bool = False   # True: the uncoded compression-only comparison scheme (appendix)

    @property
    def c(self):
        return self.Q // self.K

    @property
    def W(self):
        return self.c * self.T

    @property
    def J(self):
        return comb(self.K, self.r + 1) if self.jobs else 1

    @property
    def G(self):
        """Rounds: one per (r+1)-subset, times K-r for the J-job schedule."""
        g = comb(self.K, self.r + 1)
        return g * (self.K - self.r) if self.jobs else g

    @property
    def m(self):
        return self.N // ((self.r + 1) if self.jobs else comb(self.K, self.r))

    @property
    def v_elems(self):
        return self.J * self.Q * self.N * self.T

    @property
    def v_bytes(self):
        return 4 * self.v_elems


CONFIGS = {
    "cfg1_tiny": Workload("cfg1_tiny", 4, 2, 4, 12, 256, 1.0, ("f32", "u32", "h32", "bf16", "f16")),
    "cfg2_k10": Workload("cfg2_k10", 10, 3, 10, 120, 4096, 1.0, ("f32", "u32", "h32")),
    "cfg3_gradient": Workload("cfg3_gradient", 8, 2, 8, 28, 3_200_000, 0.01, ("f32", "h32", "bf16")),
    "cfg4_k16": Workload("cfg4_k16", 16, 3, 16, 560, 4096, 1.0, ("f32",)),
    "cfg5_k24": Workload("cfg5_k24", 24, 4, 24, 10626, 2048, 1.0, ("f32", "u32", "h32", "bf16", "f16")),
    "jobs_k8": Workload("jobs_k8", 8, 2, 8, 9, 150_000, 1.0, ("f32", "u32"), jobs=True),
    # the gradient shape through the compression-only comparison scheme (4 batches of 7 files)
    "comp_gradient": Workload("comp_gradient", 8, 2, 8, 28, 3_200_000, 0.01, ("f32",), compression=True),
}


def get(name: str) -> Workload:
    return CONFIGS[name]
