"""The five synthetic workload shapes (stand-ins for the paper's Table 1 datasets).

Index 0 is the small case the CPU oracle finishes in seconds; index 2 has the shape of
the 111M-node citation graph the paper's per-mini-batch table (Table 6) is measured on.
The datasets themselves are not available: R-MAT graphs of the same node count, edge
count and feature width stand in for them.
"""
from dataclasses import dataclass, field
from typing import List, Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    num_nodes: int            # V
    num_edges: int            # nominal directed edges before (u,v) de-duplication
    feat_dim: int             # d_0
    feat_dtype: str           # "f32" | "bf16"
    hidden: int
    num_classes: int          # output width of the last layer
    fanouts: Tuple[int, ...]  # ordered away from the targets (Section 7.1 of the paper)
    batch: int                # number of target nodes
    direction: int = 0        # 0 = out-edges (CSR by source), 1 = in-edges, 2 = both
    train_fraction: float = 1.0
    graph_seed: int = 1
    feat_seed: int = 2
    weight_seed: int = 3
    target_seed: int = 4
    # link prediction (0 = node-classification workload): positive edges per batch, edges per chunk that
    # share one list of negatives, negatives per chunk, relation types (Zipf(1.1)-distributed)
    lp_edges: int = 0
    lp_chunk: int = 0
    lp_negatives: int = 0
    num_relations: int = 0

    @property
    def num_layers(self) -> int:
        return len(self.fanouts)

    @property
    def dims(self) -> List[int]:
        k = self.num_layers
        return [self.feat_dim] + [self.hidden] * (k - 1) + [self.num_classes]

    def capacity(self) -> Tuple[int, int]:
        """Upper bounds (nodes, neighbour slots) for one mini-batch of `batch` targets."""
        mult = 2 if self.direction == 2 else 1
        level = self.batch
        nodes, slots = level, 0
        for f in self.fanouts:
            level = level * f * mult
            slots += level
            nodes += min(level, self.num_nodes)
        return min(nodes, self.num_nodes), slots


CONFIGS = [
    WorkloadConfig("rmat16k", 16_384, 262_144, 32, "f32", 32, 10, (10, 5), 256),
    WorkloadConfig("rmat1m", 1 << 20, 16_777_216, 128, "f32", 256, 64, (15, 10, 5), 1000),
    WorkloadConfig("rmat111m", 111_000_000, 1_620_000_000, 128, "f32", 256, 172, (15, 10, 5), 1000,
                   train_fraction=0.011),
    WorkloadConfig("rmat122m", 122_000_000, 1_300_000_000, 768, "bf16", 256, 153, (15, 10, 5), 1000),
    WorkloadConfig("rmat86m_lp", 86_000_000, 338_000_000, 100, "f32", 100, 100, (20,), 150_000,
                   direction=2, lp_edges=50_000, lp_chunk=1000, lp_negatives=1000, num_relations=1000),
]


def get_config(name_or_index) -> WorkloadConfig:
    if isinstance(name_or_index, int):
        return CONFIGS[name_or_index]
    for c in CONFIGS:
        if c.name == name_or_index:
            return c
    raise KeyError(name_or_index)
