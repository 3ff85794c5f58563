"""ctypes binding of libserveflow_hip.so: argument marshalling only.

Every step of the path (featurize, fast model, gate, slow model) runs in the library's HIP
kernels; this module turns torch device tensors into the pointers and sizes of the C ABI
declared in include/serveflow.h.  torch is used for device memory and the stream, nothing
else.  There is no CPU fallback: if the library is missing the import fails.
"""
import ctypes
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# SERVEFLOW_LIB names another build of the same library (the host-sanitized one of build.build_host_sanitized)
LIB_PATH = os.environ.get("SERVEFLOW_LIB") or os.path.join(_HERE, "libserveflow_hip.so")

SF_OK, SF_EINVAL, SF_ENOMEM, SF_EHIP, SF_EUNSUPPORTED, SF_EDATA = 0, -1, -2, -3, -4, -5
SF_F32, SF_BF16 = 0, 1
SF_MAX_WINDOWS = 4

EXPORTS = ("sf_workspace_bytes", "sf_create", "sf_destroy", "sf_last_error", "sf_featurize",
           "sf_validate_packets", "sf_fast_infer", "sf_validate_forest", "sf_route",
           "sf_vmin_from_theta", "sf_slow_infer", "sf_score_histogram", "sf_universal_thresholds",
           "sf_vmin_for_target", "sf_fastest_infer", "sf_validate_tree", "sf_route_ratio",
           "sf_fast_infer_subset", "sf_route_subset", "sf_gbdt_infer", "sf_route_score", "sf_score_quantiles",
           "sf_class_score_histogram", "sf_per_class_thresholds", "sf_join_table_bytes", "sf_join_workspace_bytes",
           "sf_join_step", "sf_join_pending", "sf_slow_infer_pairs", "sf_forest_packed_bytes", "sf_forest_pack",
           "sf_gbdt_pack", "sf_mlp_ordered_bytes", "sf_mlp_order", "sf_route_static", "sf_probe_gather", "sf_classify", "sf_featurize_fast_infer")


class SfPackets(ctypes.Structure):
    _fields_ = [("n_flows", ctypes.c_uint32), ("n_pkts", ctypes.c_uint64),
                ("flow_off", ctypes.c_void_p), ("pkt_size", ctypes.c_void_p),
                ("pkt_iat", ctypes.c_void_p), ("pkt_dir", ctypes.c_void_p),
                ("pkt_hdr", ctypes.c_void_p), ("hdr_words", ctypes.c_uint32)]


class SfFeatCfg(ctypes.Structure):
    _fields_ = [("n_windows", ctypes.c_uint32), ("depth", ctypes.c_uint32 * SF_MAX_WINDOWS),
                ("raw_pkts", ctypes.c_uint32), ("raw_bits", ctypes.c_uint32)]


class SfForest(ctypes.Structure):
    _fields_ = [("n_trees", ctypes.c_uint32), ("depth", ctypes.c_uint32),
                ("n_classes", ctypes.c_uint32), ("n_features", ctypes.c_uint32),
                ("node_feat", ctypes.c_void_p), ("node_thr", ctypes.c_void_p),
                ("leaf_label", ctypes.c_void_p), ("packed", ctypes.c_void_p)]


class SfTree(ctypes.Structure):
    _fields_ = [("depth", ctypes.c_uint32), ("n_classes", ctypes.c_uint32), ("n_features", ctypes.c_uint32),
                ("node_feat", ctypes.c_void_p), ("node_thr", ctypes.c_void_p), ("leaf_count", ctypes.c_void_p)]


class SfGbdt(ctypes.Structure):
    _fields_ = [("n_trees", ctypes.c_uint32), ("depth", ctypes.c_uint32), ("n_classes", ctypes.c_uint32),
                ("n_features", ctypes.c_uint32), ("node_feat", ctypes.c_void_p), ("node_thr", ctypes.c_void_p),
                ("leaf_value", ctypes.c_void_p), ("base", ctypes.c_void_p), ("packed", ctypes.c_void_p)]


class SfJoinTable(ctypes.Structure):
    _fields_ = [("slots", ctypes.c_void_p), ("cap_log2", ctypes.c_uint32)]


SF_SCORE_LC, SF_SCORE_ENTROPY = 0, 1


class SfMlp(ctypes.Structure):
    _fields_ = [("n_in", ctypes.c_uint32), ("n_h1", ctypes.c_uint32), ("n_h2", ctypes.c_uint32),
                ("n_classes", ctypes.c_uint32), ("dtype", ctypes.c_int),
                ("mu", ctypes.c_void_p), ("inv_sigma", ctypes.c_void_p), ("clamp", ctypes.c_float),
                ("w1", ctypes.c_void_p), ("w2", ctypes.c_void_p), ("w3", ctypes.c_void_p),
                ("b1", ctypes.c_void_p), ("b2", ctypes.c_void_p), ("b3", ctypes.c_void_p),
                ("ordered", ctypes.c_void_p)]


class ServeFlowError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("serveflow error %d: %s" % (code, text))
        self.code = code


def load_library() -> ctypes.CDLL:
    """Load the built library (python -m paper_2402_03694_amd.build makes it).  Raises if absent."""
    if not os.path.exists(LIB_PATH):
        raise ImportError("%s is missing: build it with paper_2402_03694_amd.build.build()" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, sz = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_size_t
    lib.sf_workspace_bytes.restype = sz
    lib.sf_workspace_bytes.argtypes = [u32] * 6
    lib.sf_create.restype = ctypes.c_int
    lib.sf_create.argtypes = [ctypes.POINTER(vp), vp, vp, sz]
    lib.sf_destroy.restype = None
    lib.sf_destroy.argtypes = [vp]
    lib.sf_last_error.restype = ctypes.c_char_p
    lib.sf_last_error.argtypes = [vp]
    lib.sf_featurize.restype = ctypes.c_int
    lib.sf_featurize.argtypes = [vp, ctypes.POINTER(SfPackets), ctypes.POINTER(SfFeatCfg), vp, u32, vp]
    lib.sf_validate_packets.restype = ctypes.c_int
    lib.sf_validate_packets.argtypes = [vp, ctypes.POINTER(SfPackets)]
    lib.sf_fast_infer.restype = ctypes.c_int
    lib.sf_fast_infer.argtypes = [vp, vp, u32, u32, ctypes.POINTER(SfForest), vp, vp, vp, vp]
    lib.sf_validate_forest.restype = ctypes.c_int
    lib.sf_validate_forest.argtypes = [vp, ctypes.POINTER(SfForest)]
    lib.sf_route.restype = ctypes.c_int
    lib.sf_route.argtypes = [vp, vp, vp, u32, ctypes.POINTER(ctypes.c_uint16), u32, vp, vp]
    lib.sf_route_static.restype = ctypes.c_int
    lib.sf_route_static.argtypes = lib.sf_route.argtypes
    lib.sf_classify.restype = ctypes.c_int
    lib.sf_classify.argtypes = [vp, ctypes.POINTER(SfPackets), ctypes.POINTER(SfFeatCfg), ctypes.POINTER(SfForest),
                                ctypes.POINTER(ctypes.c_uint16), u32, ctypes.POINTER(SfMlp), vp, u32, vp, vp, vp, vp, vp, vp]
    lib.sf_featurize_fast_infer.restype = ctypes.c_int
    lib.sf_featurize_fast_infer.argtypes = [vp, ctypes.POINTER(SfPackets), ctypes.POINTER(SfFeatCfg), ctypes.POINTER(SfForest),
                                            ctypes.POINTER(ctypes.c_uint16), u32, vp, u32, vp, vp, vp]
    lib.sf_probe_gather.restype = ctypes.c_int
    lib.sf_probe_gather.argtypes = [vp, ctypes.c_int, u32, u32, u32, vp, vp, ctypes.POINTER(ctypes.c_uint64)]
    lib.sf_vmin_from_theta.restype = u32
    lib.sf_vmin_from_theta.argtypes = [ctypes.c_float, u32]
    lib.sf_slow_infer.restype = ctypes.c_int
    lib.sf_slow_infer.argtypes = [vp, vp, u32, ctypes.POINTER(SfPackets), ctypes.POINTER(SfFeatCfg), vp, vp,
                                  u32, u32, ctypes.POINTER(SfMlp), vp, vp, vp]
    lib.sf_fastest_infer.restype = ctypes.c_int
    lib.sf_fastest_infer.argtypes = [vp, vp, u32, u32, ctypes.POINTER(SfTree), vp, vp, vp, vp]
    lib.sf_validate_tree.restype = ctypes.c_int
    lib.sf_validate_tree.argtypes = [vp, ctypes.POINTER(SfTree)]
    lib.sf_route_ratio.restype = ctypes.c_int
    lib.sf_route_ratio.argtypes = [vp, vp, vp, u32, ctypes.c_float, vp, vp]
    lib.sf_fast_infer_subset.restype = ctypes.c_int
    lib.sf_fast_infer_subset.argtypes = [vp, vp, u32, u32, vp, vp, u32, ctypes.POINTER(SfForest), vp, vp, vp, vp]
    lib.sf_route_subset.restype = ctypes.c_int
    lib.sf_route_subset.argtypes = [vp, vp, vp, vp, vp, u32, ctypes.POINTER(ctypes.c_uint16), u32, vp, vp]
    lib.sf_class_score_histogram.restype = ctypes.c_int
    lib.sf_class_score_histogram.argtypes = [vp, vp, vp, vp, u32, u32, u32, ctypes.POINTER(ctypes.c_uint32)]
    lib.sf_per_class_thresholds.restype = ctypes.c_int
    lib.sf_per_class_thresholds.argtypes = [ctypes.POINTER(ctypes.c_uint32), u32, u32, ctypes.c_double,
                                            ctypes.POINTER(ctypes.c_uint16), ctypes.POINTER(ctypes.c_double)]
    lib.sf_forest_packed_bytes.restype = sz
    lib.sf_forest_packed_bytes.argtypes = [u32, u32]
    lib.sf_forest_pack.restype = ctypes.c_int
    lib.sf_forest_pack.argtypes = [vp, ctypes.POINTER(SfForest), vp]
    lib.sf_gbdt_pack.restype = ctypes.c_int
    lib.sf_gbdt_pack.argtypes = [vp, ctypes.POINTER(SfGbdt), vp]
    lib.sf_mlp_ordered_bytes.restype = sz
    lib.sf_mlp_ordered_bytes.argtypes = [ctypes.POINTER(SfMlp)]
    lib.sf_mlp_order.restype = ctypes.c_int
    lib.sf_mlp_order.argtypes = [vp, ctypes.POINTER(SfMlp), vp]
    lib.sf_slow_infer_pairs.restype = ctypes.c_int
    lib.sf_slow_infer_pairs.argtypes = [vp, vp, u32, u32, vp, vp, vp, u32, u32, ctypes.POINTER(SfMlp), vp, vp]
    lib.sf_join_table_bytes.restype = sz
    lib.sf_join_table_bytes.argtypes = [u32]
    lib.sf_join_workspace_bytes.restype = sz
    lib.sf_join_workspace_bytes.argtypes = [u32]
    lib.sf_join_step.restype = ctypes.c_int
    lib.sf_join_step.argtypes = [vp, ctypes.POINTER(SfJoinTable), u32, u32, vp, vp, u32, vp, vp, u32, vp, vp, u32, vp, vp]
    lib.sf_join_pending.restype = ctypes.c_int
    lib.sf_join_pending.argtypes = [vp, ctypes.POINTER(SfJoinTable), ctypes.c_int, vp, vp, vp, u32, vp]
    lib.sf_gbdt_infer.restype = ctypes.c_int
    lib.sf_gbdt_infer.argtypes = [vp, vp, u32, u32, ctypes.POINTER(SfGbdt), ctypes.c_int, vp, vp, vp, vp]
    lib.sf_route_score.restype = ctypes.c_int
    lib.sf_route_score.argtypes = [vp, vp, u32, ctypes.c_float, vp, vp]
    lib.sf_score_quantiles.restype = ctypes.c_int
    lib.sf_score_quantiles.argtypes = [vp, vp, u32, ctypes.POINTER(ctypes.c_double), u32,
                                       ctypes.POINTER(ctypes.c_float)]
    lib.sf_score_histogram.restype = ctypes.c_int
    lib.sf_score_histogram.argtypes = [vp, vp, u32, u32, ctypes.POINTER(ctypes.c_uint32)]
    lib.sf_universal_thresholds.restype = ctypes.c_int
    lib.sf_universal_thresholds.argtypes = [ctypes.POINTER(ctypes.c_uint32), u32, ctypes.POINTER(ctypes.c_double), u32,
                                            ctypes.POINTER(ctypes.c_uint16)]
    lib.sf_vmin_for_target.restype = u32
    lib.sf_vmin_for_target.argtypes = [ctypes.POINTER(ctypes.c_uint32), u32, ctypes.c_double,
                                       ctypes.POINTER(ctypes.c_double)]
    return lib


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = load_library()
    return _lib


def _ptr(t: Optional[torch.Tensor], dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("expected a device tensor")
    if not t.is_contiguous():
        raise TypeError("expected a contiguous tensor")
    if dtype is not None and t.dtype != dtype:
        raise TypeError("expected dtype %s, got %s" % (dtype, t.dtype))
    return ctypes.c_void_p(t.data_ptr())


def sf_workspace_bytes(max_flows: int, n_trees: int = 0, tree_depth: int = 0, n_in: int = 0, n_h1: int = 0,
                       n_h2: int = 0) -> int:
    return int(lib().sf_workspace_bytes(max_flows, n_trees, tree_depth, n_in, n_h1, n_h2))


def sf_vmin_from_theta(theta: float, n_trees: int) -> int:
    return int(lib().sf_vmin_from_theta(ctypes.c_float(theta), n_trees))


def sf_universal_thresholds(hist, n_trees: int, quantiles):
    """hist: sequence of n_trees+1 counts.  Returns the top_votes value at each quantile (Algorithm 1)."""
    h = (ctypes.c_uint32 * (n_trees + 1))(*[int(x) for x in hist])
    q = (ctypes.c_double * len(quantiles))(*[float(x) for x in quantiles])
    out = (ctypes.c_uint16 * len(quantiles))()
    rc = lib().sf_universal_thresholds(h, n_trees, q, len(quantiles), out)
    if rc != SF_OK:
        raise ServeFlowError(rc, "sf_universal_thresholds: bad arguments or empty histogram")
    return list(out)


def sf_join_table_bytes(cap_log2: int) -> int:
    return int(lib().sf_join_table_bytes(cap_log2))


def sf_join_workspace_bytes(cap_log2: int) -> int:
    return int(lib().sf_join_workspace_bytes(cap_log2))


class DeviceJoinTable:
    """Both queues' hash tables in one zero-filled device buffer."""

    def __init__(self, cap_log2: int, device="cuda:0"):
        self.cap_log2 = cap_log2
        self.buf = torch.zeros(sf_join_table_bytes(cap_log2) // 8, dtype=torch.int64, device=device)

    def c_struct(self) -> SfJoinTable:
        t = SfJoinTable()
        t.slots, t.cap_log2 = self.buf.data_ptr(), self.cap_log2
        return t


def sf_per_class_thresholds(hist, n_trees: int, n_classes: int, target: float):
    """hist: the flat list from ServeFlow.sf_class_score_histogram.  Returns (vmin per class, reached fraction)."""
    h = (ctypes.c_uint32 * len(hist))(*hist)
    out = (ctypes.c_uint16 * n_classes)()
    reached = ctypes.c_double()
    rc = lib().sf_per_class_thresholds(h, n_trees, n_classes, float(target), out, ctypes.byref(reached))
    if rc != SF_OK:
        raise ServeFlowError(rc, "sf_per_class_thresholds: bad arguments")
    return [int(v) for v in out], reached.value


def sf_vmin_for_target(hist, n_trees: int, target: float):
    """Returns (vmin, reached escalated fraction)."""
    h = (ctypes.c_uint32 * (n_trees + 1))(*[int(x) for x in hist])
    reached = ctypes.c_double()
    v = lib().sf_vmin_for_target(h, n_trees, float(target), ctypes.byref(reached))
    return int(v), float(reached.value)


class DevicePackets:
    """Packet records on the device (SoA, CSR by flow)."""

    def __init__(self, flow_off, pkt_size, pkt_iat, pkt_dir, pkt_hdr=None):
        self.flow_off, self.pkt_size, self.pkt_iat, self.pkt_dir, self.pkt_hdr = flow_off, pkt_size, pkt_iat, pkt_dir, pkt_hdr
        self.n_flows = int(flow_off.shape[0]) - 1
        self.n_pkts = int(pkt_size.shape[0])

    def c_struct(self) -> SfPackets:
        # uint16/uint32 tensors are carried as int16/int32 storage of the same bits
        s = SfPackets()
        s.n_flows, s.n_pkts = self.n_flows, self.n_pkts
        s.flow_off = _ptr(self.flow_off, torch.int32).value
        s.pkt_size = _ptr(self.pkt_size, torch.int16).value if self.n_pkts else None
        s.pkt_iat = _ptr(self.pkt_iat, torch.float32).value if self.n_pkts else None
        s.pkt_dir = _ptr(self.pkt_dir, torch.uint8).value if self.n_pkts else None
        if self.pkt_hdr is not None:
            s.pkt_hdr = _ptr(self.pkt_hdr, torch.int32).value
            s.hdr_words = int(self.pkt_hdr.shape[1])
        return s


class DeviceForest:
    def __init__(self, n_trees, depth, n_classes, n_features, node_feat, node_thr, leaf_label):
        self.n_trees, self.depth, self.n_classes, self.n_features = n_trees, depth, n_classes, n_features
        self.node_feat, self.node_thr, self.leaf_label = node_feat, node_thr, leaf_label
        self.packed = None   # set by ServeFlow.sf_forest_pack

    def c_struct(self) -> SfForest:
        s = SfForest()
        s.n_trees, s.depth, s.n_classes, s.n_features = self.n_trees, self.depth, self.n_classes, self.n_features
        s.node_feat = _ptr(self.node_feat, torch.int16).value
        s.node_thr = _ptr(self.node_thr, torch.float32).value
        s.leaf_label = _ptr(self.leaf_label, torch.uint8).value
        s.packed = self.packed.data_ptr() if self.packed is not None else None
        return s


class DeviceTree:
    def __init__(self, depth, n_classes, n_features, node_feat, node_thr, leaf_count):
        self.depth, self.n_classes, self.n_features = depth, n_classes, n_features
        self.node_feat, self.node_thr, self.leaf_count = node_feat, node_thr, leaf_count

    def c_struct(self) -> SfTree:
        s = SfTree()
        s.depth, s.n_classes, s.n_features = self.depth, self.n_classes, self.n_features
        s.node_feat = _ptr(self.node_feat, torch.int16).value
        s.node_thr = _ptr(self.node_thr, torch.float32).value
        s.leaf_count = _ptr(self.leaf_count, torch.int16).value
        return s


class DeviceGbdt:
    def __init__(self, n_trees, depth, n_classes, n_features, node_feat, node_thr, leaf_value, base=None):
        self.n_trees, self.depth, self.n_classes, self.n_features = n_trees, depth, n_classes, n_features
        self.node_feat, self.node_thr, self.leaf_value, self.base = node_feat, node_thr, leaf_value, base
        self.packed = None   # set by ServeFlow.sf_gbdt_pack

    def c_struct(self) -> SfGbdt:
        s = SfGbdt()
        s.n_trees, s.depth, s.n_classes, s.n_features = self.n_trees, self.depth, self.n_classes, self.n_features
        s.node_feat = _ptr(self.node_feat, torch.int16).value
        s.node_thr = _ptr(self.node_thr, torch.float32).value
        s.leaf_value = _ptr(self.leaf_value, torch.float32).value
        s.base = _ptr(self.base, torch.float32).value if self.base is not None else None
        s.packed = self.packed.data_ptr() if self.packed is not None else None
        return s


class DeviceMlp:
    """Weights row-major [out][in]: float32 for SF_F32, bfloat16 for SF_BF16; biases float32."""

    def __init__(self, dims, dtype, w1, b1, w2, b2, w3, b3, mu=None, inv_sigma=None, clamp=8.0):
        self.dims, self.dtype = tuple(dims), dtype
        self.w1, self.b1, self.w2, self.b2, self.w3, self.b3 = w1, b1, w2, b2, w3, b3
        self.mu, self.inv_sigma, self.clamp = mu, inv_sigma, clamp
        self.ordered = None  # set by ServeFlow.sf_mlp_order

    def c_struct(self) -> SfMlp:
        s = SfMlp()
        s.n_in, s.n_h1, s.n_h2, s.n_classes = self.dims
        s.dtype = self.dtype
        wd = torch.float32 if self.dtype == SF_F32 else torch.bfloat16
        s.mu = _ptr(self.mu, torch.float32).value if self.mu is not None else None
        s.inv_sigma = _ptr(self.inv_sigma, torch.float32).value if self.inv_sigma is not None else None
        s.clamp = self.clamp
        s.w1, s.w2, s.w3 = (_ptr(w, wd).value for w in (self.w1, self.w2, self.w3))
        s.b1, s.b2, s.b3 = (_ptr(b, torch.float32).value for b in (self.b1, self.b2, self.b3))
        s.ordered = self.ordered.data_ptr() if self.ordered is not None else None
        return s


def _feat_cfg(depths: Sequence[int], raw_pkts: int = 0, raw_bits: int = 0) -> SfFeatCfg:
    c = SfFeatCfg()
    if len(depths) > SF_MAX_WINDOWS:
        raise ServeFlowError(SF_EINVAL, "more than %d windows" % SF_MAX_WINDOWS)
    c.n_windows = len(depths)
    for i, d in enumerate(depths):
        c.depth[i] = int(d)
    c.raw_pkts, c.raw_bits = raw_pkts, raw_bits
    return c


class ServeFlow:
    """One library context: a HIP stream plus a device workspace (a torch tensor it keeps alive)."""

    def __init__(self, workspace_bytes: int, stream: Optional[torch.cuda.Stream] = None, device="cuda:0"):
        self._h = None
        self._lib = lib()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.stream = stream
        self.workspace = torch.empty(max(int(workspace_bytes), 256) + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        aligned = (base + 255) // 256 * 256
        h = ctypes.c_void_p()
        sptr = ctypes.c_void_p(stream.cuda_stream) if stream is not None else ctypes.c_void_p(
            torch.cuda.current_stream(self.device).cuda_stream)
        rc = self._lib.sf_create(ctypes.byref(h), sptr, ctypes.c_void_p(aligned),
                                 int(self.workspace.numel() - (aligned - base)))
        if rc != SF_OK:
            raise ServeFlowError(rc, self._lib.sf_last_error(None).decode())
        self._h = h

    def close(self):
        if self._h is not None:
            self._lib.sf_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc: int):
        if rc != SF_OK:
            raise ServeFlowError(rc, self._lib.sf_last_error(self._h).decode())

    # ---- the four steps, named as in the C ABI --------------------------------------------
    def sf_featurize(self, pk: DevicePackets, depths: Sequence[int], feat: torch.Tensor,
                     raw: Optional[torch.Tensor] = None, raw_pkts: int = 0, raw_bits: int = 0):
        s, c = pk.c_struct(), _feat_cfg(depths, raw_pkts, raw_bits)
        self._check(self._lib.sf_featurize(self._h, ctypes.byref(s), ctypes.byref(c), _ptr(feat, torch.float32),
                                           int(feat.shape[1]) if feat.dim() == 2 else 0, _ptr(raw, torch.uint8)))

    def sf_validate_packets(self, pk: DevicePackets):
        s = pk.c_struct()
        self._check(self._lib.sf_validate_packets(self._h, ctypes.byref(s)))

    def sf_fast_infer(self, feat: torch.Tensor, forest: DeviceForest, pred: torch.Tensor, top_votes: torch.Tensor,
                      votes: Optional[torch.Tensor] = None, leaf_idx: Optional[torch.Tensor] = None,
                      n_flows: Optional[int] = None):
        f = forest.c_struct()
        n = int(feat.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_fast_infer(self._h, _ptr(feat, torch.float32), int(feat.shape[1]), n, ctypes.byref(f),
                                            _ptr(votes, torch.int16), _ptr(pred, torch.int16),
                                            _ptr(top_votes, torch.int16), _ptr(leaf_idx, torch.int16)))

    def sf_validate_forest(self, forest: DeviceForest):
        f = forest.c_struct()
        self._check(self._lib.sf_validate_forest(self._h, ctypes.byref(f)))

    def sf_route(self, top_votes: torch.Tensor, pred: Optional[torch.Tensor], vmin, esc_idx: torch.Tensor,
                 esc_count: torch.Tensor, n_flows: Optional[int] = None):
        vm = [int(vmin)] if isinstance(vmin, int) else [int(v) for v in vmin]
        arr = (ctypes.c_uint16 * len(vm))(*vm)
        n = int(top_votes.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_route(self._h, _ptr(top_votes, torch.int16), _ptr(pred, torch.int16), n, arr, len(vm),
                                       _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32)))

    def sf_featurize_fast_infer(self, pk: DevicePackets, depths: Sequence[int], forest: DeviceForest, vmin,
                                feat: Optional[torch.Tensor], pred: torch.Tensor, top_votes: torch.Tensor,
                                labels: Optional[torch.Tensor] = None):
        s, c, f = pk.c_struct(), _feat_cfg(depths), forest.c_struct()
        vm = [int(vmin)] if isinstance(vmin, int) else [int(v) for v in vmin]
        arr = (ctypes.c_uint16 * len(vm))(*vm)
        self._check(self._lib.sf_featurize_fast_infer(
            self._h, ctypes.byref(s), ctypes.byref(c), ctypes.byref(f), arr, len(vm), _ptr(feat, torch.float32),
            int(feat.shape[1]) if feat is not None else 0, _ptr(pred, torch.int16), _ptr(top_votes, torch.int16),
            _ptr(labels, torch.int16)))

    def sf_classify(self, pk: DevicePackets, depths: Sequence[int], forest: DeviceForest, vmin, mlp: DeviceMlp,
                    feat: Optional[torch.Tensor], pred: torch.Tensor, top_votes: torch.Tensor, esc_idx: torch.Tensor,
                    esc_count: torch.Tensor, labels: torch.Tensor, logits: Optional[torch.Tensor] = None,
                    raw_pkts: int = 0, raw_bits: int = 0):
        s, c, f, m = pk.c_struct(), _feat_cfg(depths, raw_pkts, raw_bits), forest.c_struct(), mlp.c_struct()
        vm = [int(vmin)] if isinstance(vmin, int) else [int(v) for v in vmin]
        arr = (ctypes.c_uint16 * len(vm))(*vm)
        self._check(self._lib.sf_classify(
            self._h, ctypes.byref(s), ctypes.byref(c), ctypes.byref(f), arr, len(vm), ctypes.byref(m),
            _ptr(feat, torch.float32), int(feat.shape[1]) if feat is not None else 0, _ptr(pred, torch.int16),
            _ptr(top_votes, torch.int16), _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32),
            _ptr(logits, torch.float32), _ptr(labels, torch.int16)))

    def sf_route_static(self, top_votes: torch.Tensor, pred: Optional[torch.Tensor], vmin, esc_idx: torch.Tensor,
                        esc_count: torch.Tensor, n_flows: Optional[int] = None):
        vm = [int(vmin)] if isinstance(vmin, int) else [int(v) for v in vmin]
        arr = (ctypes.c_uint16 * len(vm))(*vm)
        n = int(top_votes.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_route_static(self._h, _ptr(top_votes, torch.int16), _ptr(pred, torch.int16), n, arr,
                                              len(vm), _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32)))

    def sf_probe_gather(self, kind: int, table: torch.Tensor, sink: torch.Tensor, iters: int, blocks: int) -> int:
        """Enqueues one probe launch; returns the number of 64-lane gathers it performs."""
        words = int(table.numel()) * table.element_size() // 16
        log2 = words.bit_length() - 1
        if words != 1 << log2:
            raise ServeFlowError(SF_EINVAL, "probe table must hold a power of two of 16-byte records")
        done = ctypes.c_uint64()
        self._check(self._lib.sf_probe_gather(self._h, int(kind), log2, int(iters), int(blocks), _ptr(table),
                                              _ptr(sink, torch.int32), ctypes.byref(done)))
        return int(done.value)

    # ---- models prepared once instead of per call ---------------------------------------------
    def _aligned_bytes(self, n: int) -> torch.Tensor:
        buf = torch.empty(n + 256, dtype=torch.uint8, device=self.device)
        off = (-buf.data_ptr()) % 256
        return buf[off:off + n]

    def sf_forest_pack(self, forest: DeviceForest):
        forest.packed = None
        f = forest.c_struct()
        buf = self._aligned_bytes(int(self._lib.sf_forest_packed_bytes(forest.n_trees, forest.depth)))
        self._check(self._lib.sf_forest_pack(self._h, ctypes.byref(f), ctypes.c_void_p(buf.data_ptr())))
        forest.packed = buf

    def sf_gbdt_pack(self, model: "DeviceGbdt"):
        model.packed = None
        m = model.c_struct()
        buf = self._aligned_bytes(int(self._lib.sf_forest_packed_bytes(model.n_trees, model.depth)))
        self._check(self._lib.sf_gbdt_pack(self._h, ctypes.byref(m), ctypes.c_void_p(buf.data_ptr())))
        model.packed = buf

    def sf_mlp_order(self, mlp: DeviceMlp):
        mlp.ordered = None
        m = mlp.c_struct()
        n = int(self._lib.sf_mlp_ordered_bytes(ctypes.byref(m)))
        if n == 0:
            return                       # nothing to prepare for this model (binary32)
        buf = self._aligned_bytes(n)
        self._check(self._lib.sf_mlp_order(self._h, ctypes.byref(m), ctypes.c_void_p(buf.data_ptr())))
        mlp.ordered = buf

    # ---- the tier in front of the fast model and the list forms of steps 2-4 ----------------
    def sf_fastest_infer(self, feat: torch.Tensor, tree: DeviceTree, pred: torch.Tensor, top_count: torch.Tensor,
                         leaf_total: torch.Tensor, leaf_idx: Optional[torch.Tensor] = None,
                         n_flows: Optional[int] = None):
        t = tree.c_struct()
        n = int(feat.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_fastest_infer(self._h, _ptr(feat, torch.float32), int(feat.shape[1]), n,
                                               ctypes.byref(t), _ptr(pred, torch.int16), _ptr(top_count, torch.int16),
                                               _ptr(leaf_total, torch.int16), _ptr(leaf_idx, torch.int16)))

    def sf_validate_tree(self, tree: DeviceTree):
        t = tree.c_struct()
        self._check(self._lib.sf_validate_tree(self._h, ctypes.byref(t)))

    def sf_route_ratio(self, top_count: torch.Tensor, leaf_total: torch.Tensor, theta: float, esc_idx: torch.Tensor,
                       esc_count: torch.Tensor, n_flows: Optional[int] = None):
        n = int(top_count.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_route_ratio(self._h, _ptr(top_count, torch.int16), _ptr(leaf_total, torch.int16), n,
                                             ctypes.c_float(theta), _ptr(esc_idx, torch.int32),
                                             _ptr(esc_count, torch.int32)))

    def sf_fast_infer_subset(self, feat: torch.Tensor, idx: torch.Tensor, idx_count: torch.Tensor,
                             forest: DeviceForest, pred: torch.Tensor, top_votes: torch.Tensor,
                             votes: Optional[torch.Tensor] = None, labels: Optional[torch.Tensor] = None,
                             idx_cap: Optional[int] = None):
        f = forest.c_struct()
        cap = int(pred.shape[0]) if idx_cap is None else int(idx_cap)
        self._check(self._lib.sf_fast_infer_subset(
            self._h, _ptr(feat, torch.float32), int(feat.shape[1]), int(feat.shape[0]), _ptr(idx, torch.int32),
            _ptr(idx_count, torch.int32), cap, ctypes.byref(f), _ptr(votes, torch.int16), _ptr(pred, torch.int16),
            _ptr(top_votes, torch.int16), _ptr(labels, torch.int16)))

    def sf_route_subset(self, top_votes: torch.Tensor, pred: Optional[torch.Tensor], idx: torch.Tensor,
                        idx_count: torch.Tensor, vmin, esc_idx: torch.Tensor, esc_count: torch.Tensor,
                        idx_cap: Optional[int] = None):
        vm = [int(vmin)] if isinstance(vmin, int) else [int(v) for v in vmin]
        arr = (ctypes.c_uint16 * len(vm))(*vm)
        cap = int(top_votes.shape[0]) if idx_cap is None else int(idx_cap)
        self._check(self._lib.sf_route_subset(self._h, _ptr(top_votes, torch.int16), _ptr(pred, torch.int16),
                                              _ptr(idx, torch.int32), _ptr(idx_count, torch.int32), cap, arr, len(vm),
                                              _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32)))

    def sf_slow_infer_pairs(self, mlp: DeviceMlp, feat: torch.Tensor, pair_row: torch.Tensor, pair_flow: torch.Tensor,
                            n_pairs: torch.Tensor, labels: torch.Tensor, logits: Optional[torch.Tensor] = None,
                            pair_cap: Optional[int] = None):
        m = mlp.c_struct()
        cap = int(pair_row.shape[0]) if pair_cap is None else int(pair_cap)
        if logits is not None:
            cap = min(cap, int(logits.shape[0]))
        self._check(self._lib.sf_slow_infer_pairs(
            self._h, _ptr(feat, torch.float32), int(feat.shape[1]), int(feat.shape[0]), _ptr(pair_row, torch.int32),
            _ptr(pair_flow, torch.int32), _ptr(n_pairs, torch.int32), cap, int(labels.shape[0]), ctypes.byref(m),
            _ptr(logits, torch.float32), _ptr(labels, torch.int16)))

    # ---- the queues in front of the slow model -----------------------------------------------
    def sf_join_step(self, table: "DeviceJoinTable", now: int, timeout: int, q3_id, q3_val, q2_id, q2_val,
                     pair_q3: torch.Tensor, pair_q2: torch.Tensor, n_pairs: torch.Tensor,
                     stats: Optional[torch.Tensor] = None):
        t = table.c_struct()
        n3 = 0 if q3_id is None else int(q3_id.shape[0])
        n2 = 0 if q2_id is None else int(q2_id.shape[0])
        self._check(self._lib.sf_join_step(
            self._h, ctypes.byref(t), int(now) & 0xFFFFFFFF, int(timeout), _ptr(q3_id, torch.int64) if n3 else None,
            _ptr(q3_val, torch.int32) if n3 else None, n3, _ptr(q2_id, torch.int64) if n2 else None,
            _ptr(q2_val, torch.int32) if n2 else None, n2, _ptr(pair_q3, torch.int32), _ptr(pair_q2, torch.int32),
            int(pair_q3.shape[0]), _ptr(n_pairs, torch.int32), _ptr(stats, torch.int32)))

    def sf_join_pending(self, table: "DeviceJoinTable", queue: int, ids: torch.Tensor, vals: Optional[torch.Tensor],
                        stamps: Optional[torch.Tensor], count: torch.Tensor):
        t = table.c_struct()
        self._check(self._lib.sf_join_pending(self._h, ctypes.byref(t), int(queue), _ptr(ids, torch.int64),
                                              _ptr(vals, torch.int32), _ptr(stamps, torch.int32), int(ids.shape[0]),
                                              _ptr(count, torch.int32)))

    # ---- boosted trees as the fast model, real-valued scores --------------------------------
    def sf_gbdt_infer(self, feat: torch.Tensor, model: DeviceGbdt, score_kind: int, pred: torch.Tensor,
                      score: torch.Tensor, margins: Optional[torch.Tensor] = None,
                      leaf_idx: Optional[torch.Tensor] = None, n_flows: Optional[int] = None):
        m = model.c_struct()
        n = int(feat.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_gbdt_infer(self._h, _ptr(feat, torch.float32), int(feat.shape[1]), n, ctypes.byref(m),
                                            int(score_kind), _ptr(margins, torch.float32), _ptr(pred, torch.int16),
                                            _ptr(score, torch.float32), _ptr(leaf_idx, torch.int16)))

    def sf_route_score(self, score: torch.Tensor, threshold: float, esc_idx: torch.Tensor, esc_count: torch.Tensor,
                       n_flows: Optional[int] = None):
        n = int(score.shape[0]) if n_flows is None else n_flows
        self._check(self._lib.sf_route_score(self._h, _ptr(score, torch.float32), n, ctypes.c_float(threshold),
                                             _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32)))

    def sf_score_quantiles(self, score: torch.Tensor, quantiles, n_flows: Optional[int] = None):
        n = int(score.shape[0]) if n_flows is None else n_flows
        q = (ctypes.c_double * len(quantiles))(*[float(v) for v in quantiles])
        out = (ctypes.c_float * len(quantiles))()
        self._check(self._lib.sf_score_quantiles(self._h, _ptr(score, torch.float32), n, q, len(quantiles), out))
        return [float(v) for v in out]

    def sf_class_score_histogram(self, top_votes: torch.Tensor, pred: torch.Tensor, truth: torch.Tensor, n_trees: int,
                                 n_classes: int, n_flows: Optional[int] = None):
        n = int(top_votes.shape[0]) if n_flows is None else n_flows
        hist = (ctypes.c_uint32 * (n_classes * (n_trees + 1) * 2))()
        self._check(self._lib.sf_class_score_histogram(self._h, _ptr(top_votes, torch.int16), _ptr(pred, torch.int16),
                                                       _ptr(truth, torch.int16), n, n_trees, n_classes, hist))
        return list(hist)

    def sf_score_histogram(self, top_votes: torch.Tensor, n_trees: int, n_flows: Optional[int] = None):
        n = int(top_votes.shape[0]) if n_flows is None else n_flows
        hist = (ctypes.c_uint32 * (n_trees + 1))()
        self._check(self._lib.sf_score_histogram(self._h, _ptr(top_votes, torch.int16), n, n_trees, hist))
        return list(hist)

    def sf_slow_infer(self, mlp: DeviceMlp, esc_idx: torch.Tensor, esc_count: torch.Tensor, labels: torch.Tensor,
                      feat: Optional[torch.Tensor] = None, raw_src: Optional[DevicePackets] = None,
                      raw_pkts: int = 0, raw_bits: int = 0, logits: Optional[torch.Tensor] = None,
                      esc_cap: Optional[int] = None, pred: Optional[torch.Tensor] = None):
        m = mlp.c_struct()
        n = int(labels.shape[0])
        cap = n if esc_cap is None else int(esc_cap)
        if logits is not None:
            cap = min(cap, int(logits.shape[0]))
        s = raw_src.c_struct() if raw_src is not None else None
        c = _feat_cfg([1], raw_pkts, raw_bits) if raw_src is not None else None
        self._check(self._lib.sf_slow_infer(
            self._h, _ptr(feat, torch.float32), int(feat.shape[1]) if feat is not None else 0,
            ctypes.byref(s) if s is not None else None, ctypes.byref(c) if c is not None else None,
            _ptr(esc_idx, torch.int32), _ptr(esc_count, torch.int32), cap, n, ctypes.byref(m),
            _ptr(pred, torch.int16), _ptr(logits, torch.float32), _ptr(labels, torch.int16)))
