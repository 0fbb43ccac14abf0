"""Workload recipes: shapes, seeds and generators of the benchmark configurations.

``c0`` .. ``c4`` are the five configurations of the benchmark definition; the ``*_s``
entries are the same recipes shrunk until a CPU oracle finishes in seconds (they keep
the degree skew, a ragged tail and several tiles per launch).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

from . import graphs


@dataclass
class Workload:
    name: str
    kind: str                  # "er" | "rmat"
    n: int
    seed: int
    dims: List[int]            # L_s + 1 level widths
    n_chunks: int
    variant: str = "gcn"       # "gcn" | "gcnii"
    dtype: str = "f32"         # "f32" | "bf16" (storage of levels; accumulation is fp32)
    level0_f32: bool = False   # bf16 stages may take fp32 level-0 features (first stage)
    avg_degree: float = 0.0    # ER only
    n_candidates: int = 0      # R-MAT draws (calibrated so that nnz lands near the target)
    gcnii_alpha: float = 0.1
    gcnii_first_layer: int = 1  # global 1-based index of the stage's first layer
    relabel: bool = True
    rmat_abc: tuple = (0.57, 0.19, 0.19)
    first_stage: Optional[bool] = None  # None: GCN-type stages are first stages (features in, no input gradient)
    note: str = ""

    @property
    def n_layers(self) -> int:
        return len(self.dims) - 1


def make_graph(w: Workload):
    if w.kind == "er":
        return graphs.erdos_renyi(w.n, w.avg_degree, w.seed)
    if w.kind == "rmat":
        a, b, c = w.rmat_abc
        return graphs.rmat(w.n, w.n_candidates, w.seed, a=a, b=b, c=c, relabel=w.relabel)
    raise ValueError(w.kind)


CONFIGS = {
    # configs[0]: tiny Erdos-Renyi, fp32 everywhere
    "c0": Workload("c0", "er", 4096, 2308100870, [64] * 5, 4, avg_degree=10.0),
    # configs[1]: Reddit-shaped (Table 2: 233.0K vertices, 114.6M edges, 602 features)
    "c1": Workload("c1", "rmat", 232_965, 2308100871, [602, 256, 256, 256, 256], 8,
                   dtype="bf16", level0_f32=True, n_candidates=92_300_000),
    # configs[2]: sparser and larger, 8-layer stage at hidden 128
    "c2": Workload("c2", "rmat", 2_450_000, 2308100872, [100] + [128] * 8, 16,
                   dtype="bf16", level0_f32=True, n_candidates=96_700_000, rmat_abc=(0.46, 0.21, 0.21)),
    # configs[3]: 16-layer GCNII stage (layers 17..32 of a 64-layer model)
    "c3": Workload("c3", "rmat", 169_343, 2308100873, [256] * 17, 8, variant="gcnii",
                   dtype="bf16", n_candidates=1_450_000, gcnii_first_layer=17),
    # configs[4]: large, HBM-bound
    "c4": Workload("c4", "rmat", 10_000_000, 2308100874, [256] * 5, 32,
                   dtype="bf16", n_candidates=133_400_000, rmat_abc=(0.54, 0.19, 0.19)),
    # c1's graph under a middle stage (bf16 level 0, input gradient wanted) of each layer type, same width
    "c1_mid": Workload("c1_mid", "rmat", 232_965, 2308100871, [256] * 5, 8, dtype="bf16", n_candidates=92_300_000,
                       first_stage=False),
    "c1_sage": Workload("c1_sage", "rmat", 232_965, 2308100871, [256] * 5, 8, variant="sage", dtype="bf16",
                        n_candidates=92_300_000, first_stage=False),
    "c1_res": Workload("c1_res", "rmat", 232_965, 2308100871, [256] * 5, 8, variant="resgcn", dtype="bf16",
                       n_candidates=92_300_000, first_stage=False),
    # shrunk versions for element-by-element parity against the oracle
    "c1_s": Workload("c1_s", "rmat", 6_007, 2308100881, [602, 256, 256, 256, 256], 8,
                     dtype="bf16", level0_f32=True, n_candidates=260_000),
    "c2_s": Workload("c2_s", "rmat", 20_011, 2308100882, [100] + [128] * 8, 16,
                     dtype="bf16", level0_f32=True, n_candidates=330_000, rmat_abc=(0.46, 0.21, 0.21)),
    "c3_s": Workload("c3_s", "rmat", 5_003, 2308100883, [256] * 17, 8, variant="gcnii",
                     dtype="bf16", n_candidates=34_000, gcnii_first_layer=17),
    "c4_s": Workload("c4_s", "rmat", 30_011, 2308100884, [256] * 5, 32,
                     dtype="bf16", n_candidates=310_000, rmat_abc=(0.54, 0.19, 0.19)),
}
