"""Seeded packet records, stored SoA and CSR by flow.

Per packet: size (uint16), inter-arrival time (float32 seconds), direction
(uint8 in {0, 1}) and, optionally, the first ``raw_bits`` header bits packed
into ``hdr_words`` little-endian uint32 words (header byte k sits in word k//4
at bit offset 8*(k%4); header bit b is bit 7-(b%8) of byte b//8, i.e. bits are
numbered MSB-first as on the wire).  These are the flow-level quantities the
paper names as inputs (packet sizes, inter-arrival times, direction: Section
3.1; all header bits per packet: Section 4.1).
"""
from dataclasses import dataclass
from typing import Optional

import numpy as np

from .configs import WorkloadConfig


@dataclass
class PacketBatch:
    flow_off: np.ndarray            # uint32 [n_flows + 1]
    pkt_size: np.ndarray            # uint16 [n_pkts]
    pkt_iat: np.ndarray             # float32 [n_pkts]
    pkt_dir: np.ndarray             # uint8 [n_pkts]
    pkt_hdr: Optional[np.ndarray]   # uint32 [n_pkts, hdr_words] or None
    hidden_class: Optional[np.ndarray]  # uint8 [n_flows]: the label the header bits encode

    @property
    def n_flows(self) -> int:
        return int(self.flow_off.shape[0] - 1)

    @property
    def n_pkts(self) -> int:
        return int(self.pkt_size.shape[0])


def _sizes(rng: np.random.Generator, n: int) -> np.ndarray:
    """60 % uniform 40..100, 25 % uniform 500..1000, 15 % exactly 1500 bytes."""
    mode = rng.random(n, dtype=np.float32)
    small = rng.integers(40, 101, size=n, dtype=np.uint16)
    large = rng.integers(500, 1001, size=n, dtype=np.uint16)
    out = np.where(mode < 0.60, small, np.where(mode < 0.85, large, np.uint16(1500)))
    return out.astype(np.uint16)


def _iats(rng: np.random.Generator, n: int) -> np.ndarray:
    """lognormal(mu=-6, sigma=2) seconds, stored as float32."""
    return np.exp(rng.normal(-6.0, 2.0, size=n)).astype(np.float32)


def _flow_lengths(cfg: WorkloadConfig, rng: np.random.Generator, n_flows: int) -> np.ndarray:
    if cfg.pkts_per_flow is not None:
        return np.full(n_flows, cfg.pkts_per_flow, dtype=np.uint32)
    n = rng.geometric(cfg.geom_p, size=n_flows)
    return np.clip(n, 1, cfg.max_pkts).astype(np.uint32)


def _header_words(cfg: WorkloadConfig, seed: int, lens: np.ndarray, hidden: np.ndarray,
                  model_rng: np.random.Generator) -> np.ndarray:
    """Bernoulli(0.3) header bits (a 16-bit uniform below 19661, i.e. p = 0.300003); 64 fixed bit
    positions carry a per-class constant pattern (a stand-in for protocol fields that identify the
    service).  Packets are drawn in chunks of 32,768, chunk c from its own stream (the data seed's
    generator jumped c+1 times), so chunks can be drawn by a few threads and the result does not
    depend on how many."""
    n_bits = cfg.raw_bits
    n_pkts = int(lens.sum())
    fixed_pos = model_rng.choice(n_bits, size=64, replace=False)
    patterns = (model_rng.random((cfg.n_classes, 64)) < 0.5)
    pkt_class = np.repeat(hidden, lens)
    words = np.empty((n_pkts, cfg.hdr_words), dtype=np.uint32)
    chunk = 1 << 15
    pad = cfg.hdr_words * 32 - n_bits

    def draw(c: int) -> None:
        s, e = c * chunk, min(n_pkts, (c + 1) * chunk)
        rng = np.random.Generator(np.random.PCG64(seed).jumped(c + 1))
        bits = rng.integers(0, 65536, size=(e - s, n_bits), dtype=np.uint16) < 19661
        bits[:, fixed_pos] = patterns[pkt_class[s:e]]
        if pad:
            bits = np.concatenate([bits, np.zeros((e - s, pad), bool)], axis=1)
        by = np.packbits(bits, axis=1, bitorder="big")       # MSB-first within each byte
        words[s:e] = np.ascontiguousarray(by).view("<u4")

    n_chunks = (n_pkts + chunk - 1) // chunk
    if n_chunks <= 1:
        for c in range(n_chunks):
            draw(c)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(min(8, n_chunks)) as pool:
            list(pool.map(draw, range(n_chunks)))
    return words


def make_packets(cfg: WorkloadConfig, batch: int = 0, n_flows: Optional[int] = None) -> PacketBatch:
    """Draw one batch of flows for ``cfg``.  Batch b of a streaming config uses its own seed."""
    n_flows = cfg.n_flows if n_flows is None else n_flows
    seed = cfg.data_seed * 1000 + batch
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = _flow_lengths(cfg, rng, n_flows)
    flow_off = np.zeros(n_flows + 1, dtype=np.uint32)
    csum = np.cumsum(lens, dtype=np.uint64)
    n_pkts = int(csum[-1]) if n_flows else 0
    if n_pkts >= 1 << 32:
        raise ValueError("packet offsets are uint32: a batch holds fewer than 2^32 packets")
    flow_off[1:] = csum.astype(np.uint32)
    size = _sizes(rng, n_pkts)
    iat = _iats(rng, n_pkts)
    direction = (rng.random(n_pkts, dtype=np.float32) < 0.5).astype(np.uint8)
    hdr = None
    hidden = None
    if cfg.raw_pkts > 0:
        hidden = rng.integers(0, cfg.n_classes, size=n_flows, dtype=np.uint8)
        model_rng = np.random.Generator(np.random.PCG64(cfg.model_seed * 1000 + 7))
        hdr = _header_words(cfg, seed, lens, hidden, model_rng)
    return PacketBatch(flow_off, size, iat, direction, hdr, hidden)
