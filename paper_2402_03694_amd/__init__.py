"""Batched fast-slow flow classification on AMD MI355X (gfx950).

The product is the HIP library libserveflow_hip.so (C ABI in include/serveflow.h); this
package is its thin Python binding.  Build the library with ``python -m
paper_2402_03694_amd.build``; importing ``binding`` without it fails loudly (there is no
CPU fallback).
"""
from .binding import (DeviceJoinTable, sf_join_table_bytes, sf_join_workspace_bytes, SF_BF16, SF_F32, SF_SCORE_ENTROPY, SF_SCORE_LC, DeviceGbdt, DeviceForest, DeviceMlp, DevicePackets, DeviceTree, ServeFlow, ServeFlowError,
                      sf_per_class_thresholds, sf_universal_thresholds, sf_vmin_for_target, sf_vmin_from_theta, sf_workspace_bytes)
from .upload import forest_to_device, mlp_to_device, packets_to_device, tree_to_device, gbdt_to_device

__all__ = ["DeviceJoinTable", "sf_join_table_bytes", "sf_join_workspace_bytes", "SF_BF16", "SF_F32", "SF_SCORE_LC", "SF_SCORE_ENTROPY", "DeviceGbdt", "gbdt_to_device", "DeviceForest", "DeviceMlp", "DevicePackets", "DeviceTree", "tree_to_device", "ServeFlow", "ServeFlowError",
           "sf_vmin_from_theta", "sf_workspace_bytes", "sf_universal_thresholds", "sf_per_class_thresholds", "sf_vmin_for_target", "forest_to_device", "mlp_to_device", "packets_to_device"]
