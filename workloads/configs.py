"""The five benchmark workloads (synthetic stand-ins shaped after the paper's Table 2 datasets).

Each entry fixes graph family and size, feature width and distribution, number of
augmentation hops, layer widths, penalties and (for the quantised variant) the grid.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional, Tuple

BASE_SEED = 20210509


@dataclass(frozen=True)
class Workload:
    name: str
    cfg_id: int                      # enters the seed: BASE_SEED + 1000*cfg_id + stream
    n_nodes: int
    graph: str                       # "er" | "pa"
    graph_param: Tuple[int, ...]     # er: (avg_degree,) ; pa: attachment counts cycled per new node
    feat_dim: int
    feat_kind: str                   # "bernoulli01" | "normal"
    hops: int                        # highest adjacency power; blocks = hops + 1
    hidden: int
    n_layers: int
    n_classes: int
    rho: float
    nu: float
    iters: int
    quant: Optional[Tuple[float, float, int]] = None   # (lo, hi, levels) of the uniform grid
    quant_q: bool = False                               # q_l is kept on the grid as well (needs quant)
    slope: float = 0.0                                  # negative-side slope of the activation (0 = ReLU)
    risk: str = "ce"                                    # risk on the output layer: "ce" cross-entropy, "ls" least squares

    @property
    def n0(self) -> int:
        return (self.hops + 1) * self.feat_dim

    @property
    def dims(self) -> Tuple[int, ...]:
        """(n_0, n_1, ..., n_L)."""
        return (self.n0,) + (self.hidden,) * (self.n_layers - 1) + (self.n_classes,)

    def seed(self, stream: int) -> int:
        return BASE_SEED + 1000 * self.cfg_id + stream


WORKLOADS = {
    "C1": Workload("C1", 1, 2_000, "er", (4,), 500, "bernoulli01", 2, 100, 4, 7, 0.01, 0.01, 10),
    "C2": Workload("C2", 2, 20_000, "pa", (3,), 500, "normal", 3, 500, 10, 3, 1e-3, 1e-3, 20),
    "C3": Workload("C3", 3, 170_000, "pa", (3, 4), 128, "normal", 3, 1000, 10, 40, 1e-3, 1e-3, 20),
    "C4": Workload("C4", 4, 20_000, "pa", (3,), 500, "normal", 2, 500, 50, 10, 1e-3, 1e-3, 20),
    "C5": Workload("C5", 5, 100_000, "pa", (5,), 256, "normal", 3, 1000, 16, 20, 1e-3, 1e-3, 20,
                   quant=(-1.0, 1.0, 256)),
}
# C5 with p and q both on the grid (the variant at the end of Appendix B)
WORKLOADS["C5pq"] = replace(WORKLOADS["C5"], name="C5pq", quant_q=True)
# C5 on a grid of 65536 levels (the 16-bit case of Section 5.5)
WORKLOADS["C5x16"] = replace(WORKLOADS["C5"], name="C5x16", quant=(-1.0, 1.0, 65536))


def get_workload(name: str) -> Workload:
    return WORKLOADS[name]


def scaled_workload(name: str, n_nodes: int, hidden: Optional[int] = None,
                    n_layers: Optional[int] = None, feat_dim: Optional[int] = None) -> Workload:
    """A reduced copy of a workload (same family, same seeds' cfg_id) for oracle-speed tests."""
    w = WORKLOADS[name]
    return replace(w, name=f"{name}@{n_nodes}", n_nodes=n_nodes,
                   hidden=hidden if hidden is not None else w.hidden,
                   n_layers=n_layers if n_layers is not None else w.n_layers,
                   feat_dim=feat_dim if feat_dim is not None else w.feat_dim)
