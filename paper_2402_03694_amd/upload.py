"""Host arrays -> device tensors for the binding (copies and dtype reinterpretation only)."""
import numpy as np
import torch

from .binding import SF_BF16, SF_F32, DeviceForest, DeviceMlp, DeviceGbdt, DevicePackets, DeviceTree


def _dev(a: np.ndarray, device) -> torch.Tensor:
    """Upload keeping the bits: unsigned 16/32-bit arrays travel as the signed type of the same width."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    elif a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).to(device)


def packets_to_device(pk, device="cuda:0", with_hdr: bool = True) -> DevicePackets:
    """pk: any object with flow_off, pkt_size, pkt_iat, pkt_dir and optionally pkt_hdr numpy arrays."""
    hdr = getattr(pk, "pkt_hdr", None)
    return DevicePackets(_dev(pk.flow_off, device), _dev(pk.pkt_size, device), _dev(pk.pkt_iat, device),
                         _dev(pk.pkt_dir, device), _dev(hdr, device) if (hdr is not None and with_hdr) else None)


def forest_to_device(f, device="cuda:0") -> DeviceForest:
    return DeviceForest(f.n_trees, f.depth, f.n_classes, f.n_features, _dev(f.node_feat, device),
                        _dev(f.node_thr, device), _dev(f.leaf_label, device))


def tree_to_device(t, device="cuda:0") -> DeviceTree:
    return DeviceTree(t.depth, t.n_classes, t.n_features, _dev(t.node_feat, device), _dev(t.node_thr, device),
                      _dev(t.leaf_count, device))


def gbdt_to_device(g, device="cuda:0") -> DeviceGbdt:
    return DeviceGbdt(g.n_trees, g.depth, g.n_classes, g.n_features, _dev(g.node_feat, device), _dev(g.node_thr, device),
                      _dev(g.leaf_value, device), _dev(g.base, device) if g.base is not None else None)


def mlp_to_device(m, device="cuda:0") -> DeviceMlp:
    """m.dtype "bf16": weights must already be bfloat16-representable float32; they are narrowed exactly."""
    bf = m.dtype == "bf16"

    def w(a):
        t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
        if bf:
            tb = t.to(torch.bfloat16)
            if not torch.equal(tb.to(torch.float32), t):
                raise ValueError("weights are not bfloat16-representable")
            return tb.contiguous()
        return t

    def v(a):
        return None if a is None else torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)

    return DeviceMlp(m.dims, SF_BF16 if bf else SF_F32, w(m.w1), v(m.b1), w(m.w2), v(m.b2), w(m.w3), v(m.b3),
                     v(m.mu), v(m.inv_sigma), float(m.clamp))
