"""Seeded synthetic workloads shaped like the paper's flow-classification tasks.

This package only *draws inputs*: packet records (CSR by flow), random-split
forests and Xavier-initialised MLP weights.  It holds none of the method's
arithmetic (no feature statistics, no tree walks, no gating, no matmuls), so
the CPU oracle and the HIP library can both be fed from it without sharing any
code of the method itself.  Anything that depends on feature values (split
thresholds, standardisation constants) takes a feature sample as an *argument*;
the caller decides which side computed that sample.

The synthetic flows stand in for the paper's three datasets (service
recognition, device identification, VCA QoE; Section 5.1), which need the
authors' captures: context lengths of 1-20 packets, 4-32 classes, thousands of
header-bit features and 5-60 % escalated flows follow Sections 3.1, 4.4, 5.3.
"""
from .configs import CONFIGS, WorkloadConfig, get_config
from .packets import make_packets, PacketBatch
from .models import make_forest, make_mlp, make_tree, make_gbdt, make_truth, Forest, Gbdt, Mlp, Tree, round_to_bf16

__all__ = [
    "CONFIGS", "WorkloadConfig", "get_config",
    "make_packets", "PacketBatch",
    "make_forest", "make_mlp", "make_tree", "make_gbdt", "make_truth", "Gbdt", "Forest", "Mlp", "Tree", "round_to_bf16",
]
