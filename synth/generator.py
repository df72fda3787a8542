"""Structured synthetic attention inputs (stand-in for real long-context prompts).

The paper measures on real prompts pushed through real model weights; neither is
available here.  What the generator keeps from those workloads is their *shape*
(head counts, head_dim, sequence length) and the *structure* the paper describes
in attention maps (Sec. 3-4: attention sinks, vertical lines, block / staircase
patterns that similar heads share):

* every cluster of heads owns a piecewise-constant "topic" sequence; a query and a
  key that carry the same topic get a logit boost (staircase / block pattern shared
  by all heads of the cluster),
* the key of token 0 is a sink (+4 sigma logit for every query),
* a few seeded "heavy vertical" key positions get a large boost for every query,
* values carry a topic-dependent mean so that attention outputs are O(1).

Everything is drawn from counter-based Philox streams keyed by
(seed, tensor id, head), rounded to bfloat16 with round-to-nearest-even, and
returned as uint16 bit patterns.  No attention arithmetic happens here.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np


# --------------------------------------------------------------------------- #
# bf16 <-> f32 bit helpers (data formatting only)
# --------------------------------------------------------------------------- #
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32 exactly."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# --------------------------------------------------------------------------- #
# configurations (the benchmark workloads, in order)
# --------------------------------------------------------------------------- #
@dataclass(frozen=True)
class LayerConfig:
    name: str
    index: int            # 1-based position in the list of benchmark workloads
    seq: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    block: int
    n_clusters: int
    gamma: float
    rank: int             # rank of the shared per-cluster component
    n_heavy: int          # heavy vertical key positions
    cluster_mode: str     # "contig" (c = h // size) or "perm" (seeded permutation)
    n_layers: int = 1
    topic_gain: float = 6.0    # same-topic logit boost (lambda)
    sink_beta: float = 4.0     # query projection on the sink direction
    sink_boost: float = 4.0    # logit boost of key 0
    heavy_boost: float = 10.0  # logit boost of the heavy vertical keys
    value_gain: float = 4.0    # topic-dependent mean of V (nu)
    value_noise: float = 1.0   # std of the i.i.d. part of V (epsilon ~ N(0,1), as the workload statement gives it)
    # Optional spread of head behaviour (entry (cluster * cluster_size + rank of the head inside its cluster, by head
    # index) modulo the tuple's length): a multiplier on the query's topic gain (small = diffuse attention, large =
    # highly sparse) and a shift of the topic ids the query follows (non-zero = a head whose pattern differs from
    # its cluster's).
    query_gain: Optional[tuple] = None
    topic_shift: Optional[tuple] = None

    @property
    def cluster_size(self) -> int:
        return self.n_q_heads // self.n_clusters

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def nqb(self) -> int:
        return self.seq // self.block


CONFIGS: Dict[str, LayerConfig] = {
    "tiny": LayerConfig("tiny", 1, 1024, 4, 4, 64, 64, 2, 0.9, 4, 0, "contig"),
    "llama8b_32k": LayerConfig("llama8b_32k", 2, 32768, 32, 8, 128, 128, 8, 0.95, 8, 16, "contig"),
    "llama8b_128k": LayerConfig("llama8b_128k", 3, 131072, 32, 8, 128, 128, 8, 0.95, 8, 16, "contig"),
    "qwen7b_128k": LayerConfig("qwen7b_128k", 4, 131072, 28, 4, 128, 128, 7, 0.9, 8, 16, "perm"),
    "llama70b_128k": LayerConfig("llama70b_128k", 5, 131072, 64, 8, 128, 128, 16, 0.95, 8, 16, "contig",
                                 n_layers=4),
    # The Llama-3-8B shape with a spread of head sparsities inside every cluster, so that the thresholds the paper
    # states (gamma 0.9, tau 0.2, delta 0.3) split the heads into dense pivots, pattern-sharing heads, heads whose
    # pattern is not similar enough and highly sparse heads that are excluded from sharing.
    "llama8b_128k_regime": LayerConfig("llama8b_128k_regime", 6, 131072, 32, 8, 128, 128, 8, 0.9, 8, 16, "contig",
                                       query_gain=(0.04, 0.05, 0.04, 0.045, 0.04, 0.05, 0.04, 1.0),
                                       topic_shift=(0, 0, 0, 3, 0, 0, 0, 0)),
}


def _rng(seed: int, tensor_id: int, sub: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), (int(tensor_id) << 32) | int(sub)]))


def _clusters(cfg: LayerConfig, seed: int):
    """head_to_cluster[Hq], pivot_heads[C]."""
    Hq, C = cfg.n_q_heads, cfg.n_clusters
    size = cfg.cluster_size
    if cfg.cluster_mode == "contig":
        h2c = np.arange(Hq, dtype=np.int32) // size
        piv = (np.arange(C, dtype=np.int32) * size).astype(np.int32)
    elif cfg.cluster_mode == "perm":
        perm = _rng(seed, 90).permutation(Hq).astype(np.int32)
        h2c = np.empty(Hq, dtype=np.int32)
        for c in range(C):
            h2c[perm[c * size:(c + 1) * size]] = c
        piv = perm[::size][:C].astype(np.int32).copy()
    else:
        raise ValueError(cfg.cluster_mode)
    return h2c, piv


def _topic_sequence(cfg: LayerConfig, rng: np.random.Generator, N: int) -> np.ndarray:
    """Piecewise-constant topic id per token; segment lengths uniform in [2B, 16B]."""
    B = cfg.block
    out = np.empty(N, dtype=np.int64)
    pos = 0
    while pos < N:
        seg = int(rng.integers(2 * B, 16 * B + 1))
        out[pos:pos + seg] = int(rng.integers(0, cfg.rank))
        pos += seg
    return out


def make_layer(cfg: LayerConfig, layer: int = 0, seq: Optional[int] = None,
               heads: Optional[List[int]] = None, structure_layer: Optional[int] = None) -> dict:
    """Generate one layer's inputs.

    Returns a dict with
      q  uint16 [N][Hq][d]   bf16 bits (token-major)
      k  uint16 [N][Hkv][d]
      v  uint16 [N][Hkv][d]
      head_to_cluster int32 [Hq], pivot_heads int32 [C], cfg (with seq applied), seed

    `seq` overrides the sequence length (same recipe, shorter prefix statistics).
    `structure_layer`, if given, takes the prompt-dependent structure (cluster membership, topic
    sequences, heavy vertical positions) from that layer's streams while the projections and the
    noise stay this layer's own: layers of one prompt, whose clusters span the layers.
    """
    if seq is not None and seq != cfg.seq:
        cfg = replace(cfg, seq=int(seq))
    N, Hq, Hkv, d = cfg.seq, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    if N % cfg.block:
        raise ValueError("seq must be a multiple of block")
    seed = 1000 * cfg.index + layer
    sseed = seed if structure_layer is None else 1000 * cfg.index + int(structure_layer)
    G = cfg.group
    h2c, piv = _clusters(cfg, sseed)
    C, r = cfg.n_clusters, cfg.rank

    g = float(np.sqrt(cfg.topic_gain * np.sqrt(d)))
    topics = [_topic_sequence(cfg, _rng(sseed, 10, c), N) for c in range(C)]
    A = [(_rng(seed, 11, c).standard_normal((r, d)) / np.sqrt(d)).astype(np.float32) for c in range(C)]
    A2 = [(_rng(seed, 12, c).standard_normal((r, d)) / np.sqrt(d)).astype(np.float32) for c in range(C)]
    e_s = _rng(seed, 13).standard_normal(d)
    e_s = (e_s / np.linalg.norm(e_s)).astype(np.float32)

    b = np.zeros(N, dtype=np.float32)
    b[0] = cfg.sink_boost
    if cfg.n_heavy > 0 and N > 1:
        heavy = _rng(sseed, 14).choice(np.arange(1, N), size=min(cfg.n_heavy, N - 1), replace=False)
        b[heavy] = cfg.heavy_boost
    else:
        heavy = np.zeros(0, dtype=np.int64)

    q = np.empty((N, Hq, d), dtype=np.uint16)
    k = np.empty((N, Hkv, d), dtype=np.uint16)
    v = np.empty((N, Hkv, d), dtype=np.uint16)

    rank_in_cluster = np.zeros(Hq, dtype=np.int64)
    for c in range(C):
        for pos, h in enumerate(np.nonzero(h2c == c)[0]):
            rank_in_cluster[h] = pos
    for h in range(Hq):
        c = int(h2c[h])
        x = _rng(seed, 1, h).standard_normal((N, d), dtype=np.float32)
        pos = c * cfg.cluster_size + int(rank_in_cluster[h])
        gh = g * float(np.sqrt(cfg.query_gain[pos % len(cfg.query_gain)])) if cfg.query_gain else g
        shift = int(cfg.topic_shift[pos % len(cfg.topic_shift)]) if cfg.topic_shift else 0
        x += (gh * A[c])[(topics[c] + shift) % cfg.rank]
        x += cfg.sink_beta * e_s
        q[:, h, :] = f32_to_bf16_bits(x)
    for kv in range(Hkv):
        cl = sorted({int(h2c[h]) for h in range(kv * G, (kv + 1) * G)})
        x = _rng(seed, 2, kv).standard_normal((N, d), dtype=np.float32)
        y = cfg.value_noise * _rng(seed, 3, kv).standard_normal((N, d), dtype=np.float32)
        for c in cl:
            x += (g * A[c])[topics[c]]
            y += (cfg.value_gain * A2[c])[topics[c]]
        x += (b * (np.sqrt(d) / cfg.sink_beta))[:, None] * e_s[None, :]
        k[:, kv, :] = f32_to_bf16_bits(x)
        v[:, kv, :] = f32_to_bf16_bits(y)

    return {"q": q, "k": k, "v": v, "head_to_cluster": h2c, "pivot_heads": piv,
            "cfg": cfg, "seed": seed, "heavy": np.sort(heavy)}


def random_qkv(seed: int, N: int, Hq: int, Hkv: int, d: int, scale: float = 1.0):
    """Plain N(0, scale^2) bf16 Q/K/V bit patterns for small unit tests."""
    r = _rng(seed, 77)
    q = f32_to_bf16_bits(scale * r.standard_normal((N, Hq, d), dtype=np.float32))
    k = f32_to_bf16_bits(scale * r.standard_normal((N, Hkv, d), dtype=np.float32))
    v = f32_to_bf16_bits(scale * r.standard_normal((N, Hkv, d), dtype=np.float32))
    return q, k, v
