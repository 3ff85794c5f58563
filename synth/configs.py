"""The synthetic workload configurations: five two-tier ones, a three-tier cascade and a boosted-tree one.

Each mirrors one regime the paper discusses: a handful of first packets as
context (Section 3.1), a tree model as the fast tier and a heavier model as the
slow tier (Sections 3.1, 4.4), an assigned portion between a few per cent and a
half of the flows (Section 5.3), and raw header bits as the slow tier's input
(Section 4.1).
"""
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple


@dataclass(frozen=True)
class WorkloadConfig:
    name: str
    n_flows: int
    # packets per flow: fixed count, or None for ragged geometric(p) clipped to [1, max_pkts]
    pkts_per_flow: Optional[int]
    geom_p: float = 0.1
    max_pkts: int = 64
    depths: Tuple[int, ...] = (8,)          # prefix windows, strictly increasing
    n_trees: int = 16
    tree_depth: int = 8
    n_classes: int = 4
    # gate: either a vote-fraction threshold theta, an explicit vmin, or target escalated fractions
    theta: Optional[float] = None
    vmin: Optional[int] = None
    target_fracs: Tuple[float, ...] = ()
    mlp_dims: Tuple[int, int, int, int] = (32, 128, 128, 4)
    mlp_dtype: str = "f32"                   # "f32" | "bf16"
    raw_pkts: int = 0                        # slow model reads raw header bits if > 0
    raw_bits: int = 0
    hdr_words: int = 0
    n_batches: int = 1
    data_seed: int = 1000
    model_seed: int = 2000
    calib_flows: int = 4096                  # flows whose features feed thresholds / standardisation
    # three-tier cascade (Section 3.1): a single decision tree in front of the forest; 0 = none
    tree0_depth: int = 0
    tree0_features: int = 0                  # the tree and the forest split on the first this-many columns
    theta0: Optional[float] = None           # the tree escalates a flow iff max_y P(y|x) < theta0
    # boosted-tree form of the fast model (Section 4.1): leaves hold margins, softmax gives P(y|x)
    fast_kind: str = "votes"                 # "votes" (hard-voting forest) | "gbdt"
    score: str = "lc"                        # uncertainty score of the gbdt gate: "lc" | "entropy" (Section 3.2)

    @property
    def n_features(self) -> int:
        return 32 * len(self.depths)

    def scaled(self, n_flows: int) -> "WorkloadConfig":
        """Same workload at a different flow count (parity tests use small ones)."""
        return replace(self, n_flows=n_flows)


CONFIGS = {
    1: WorkloadConfig(
        name="cfg1_small", n_flows=4096, pkts_per_flow=8, depths=(8,),
        n_trees=16, tree_depth=8, n_classes=4, theta=0.75,
        mlp_dims=(32, 128, 128, 4), mlp_dtype="f32",
        data_seed=1001, model_seed=2001),
    2: WorkloadConfig(
        name="cfg2_1m_stats", n_flows=1 << 20, pkts_per_flow=16, depths=(8, 16),
        n_trees=100, tree_depth=12, n_classes=10, target_fracs=(0.25,),
        mlp_dims=(64, 512, 512, 10), mlp_dtype="bf16",
        data_seed=1002, model_seed=2002),
    3: WorkloadConfig(
        name="cfg3_1m_rawbits", n_flows=1 << 20, pkts_per_flow=10, depths=(5, 10),
        n_trees=100, tree_depth=10, n_classes=10, target_fracs=(0.20,),
        mlp_dims=(4800, 1024, 512, 10), mlp_dtype="bf16",
        raw_pkts=10, raw_bits=480, hdr_words=15,
        data_seed=1003, model_seed=2003),
    4: WorkloadConfig(
        name="cfg4_stream_ragged", n_flows=65536, pkts_per_flow=None, geom_p=0.1, max_pkts=64,
        depths=(8, 64), n_trees=200, tree_depth=10, n_classes=16, vmin=18,
        mlp_dims=(64, 1024, 1024, 16), mlp_dtype="bf16", n_batches=200,
        data_seed=1004, model_seed=2004),
    5: WorkloadConfig(
        name="cfg5_sweep", n_flows=1 << 22, pkts_per_flow=32, depths=(8, 16, 24, 32),
        n_trees=500, tree_depth=10, n_classes=32, target_fracs=(0.05, 0.25, 0.50),
        mlp_dims=(128, 2048, 2048, 32), mlp_dtype="bf16",
        data_seed=1005, model_seed=2005),
    # the cascade the paper evaluates (decision tree, then a boosted/bagged ensemble, then the
    # slow model; Section 5.2): config 2's shape with a depth-10 tree on the first window
    6: WorkloadConfig(
        name="cfg6_three_tier", n_flows=1 << 20, pkts_per_flow=16, depths=(8, 16),
        n_trees=100, tree_depth=12, n_classes=10, vmin=14,
        mlp_dims=(64, 512, 512, 10), mlp_dtype="bf16",
        tree0_depth=10, tree0_features=32, theta0=0.6,
        data_seed=1006, model_seed=2006),
    # the fast model as gradient-boosted trees (20 rounds x 10 classes, 256 leaves each), gated by
    # the entropy of its softmax; threshold from Algorithm 1's quantile rule at the target portion
    7: WorkloadConfig(
        name="cfg7_gbdt_entropy", n_flows=1 << 20, pkts_per_flow=16, depths=(8, 16),
        n_trees=200, tree_depth=8, n_classes=10, target_fracs=(0.25,),
        mlp_dims=(64, 512, 512, 10), mlp_dtype="bf16", fast_kind="gbdt", score="entropy",
        data_seed=1007, model_seed=2007),
}


def get_config(idx: int) -> WorkloadConfig:
    return CONFIGS[idx]
