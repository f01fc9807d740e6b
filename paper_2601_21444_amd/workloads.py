"""Seeded synthetic host-share workloads (inputs only; none of the method's arithmetic lives here).

A workload is everything one virtual host of the sequence-parallel prefill holds for one layer:
the query-block probe ``Q_qr``, the local context block ``Q, K, V``, the anchor block ``K_a, V_a`` and
the full context blocks ``K^(p), V^(p)`` of the ``P`` preceding hosts (Sec. 3.2 "Context Splitting",
Sec. 3.3 "Approximate Attention").  The preceding hosts' blocks are handed out uncompressed: whoever
consumes them (the CPU oracle in the tests, the HIP library in the bench) runs its own compression to
obtain the passing block.

The shapes follow the paper's hyper-parameter rule l_a = n/64, l_p = n/128 (Sec. 5.1) on
Qwen2.5-VL-shaped heads; the values are random stand-ins for the paper's video benchmarks, whose data
and weights are not used.

All tensors are returned as numpy ``uint16`` arrays holding bf16 bit patterns, laid out
``[tokens, heads, head_dim]`` with ``head_dim`` contiguous.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Tuple, Union

import numpy as np


@dataclass(frozen=True)
class HostShare:
    """Shape and distribution recipe of one virtual host's share."""

    name: str
    seed: Union[int, Tuple[int, ...]]
    n_q_heads: int          # Hq
    n_kv_heads: int         # Hkv
    head_dim: int           # d
    n_q: int                # query-block (probe) length
    l_a: int                # anchor length
    P: int                  # number of preceding hosts (passing blocks)
    L_prev: int             # length of each preceding host's context block
    l_p: int                # keys kept per block by the compression
    L: int                  # local block length l_b
    key_recipe: str = "normal"   # "normal" | "scaled" | "frames"
    frame_len: int = 4096        # only for key_recipe == "frames"
    frame_rank: int = 16
    frame_noise: float = 0.5

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def s_kv(self) -> int:
        return self.l_a + self.P * self.l_p + self.L

    @property
    def visible_pairs_per_head(self) -> int:
        """(query, key) pairs the mask leaves visible, per query head."""
        return self.L * (self.l_a + self.P * self.l_p) + self.L * (self.L + 1) // 2

    @property
    def attention_flops(self) -> int:
        """4*d flops (QK^T and PV, multiply+add each) per visible pair, over all query heads."""
        return 4 * self.head_dim * self.visible_pairs_per_head * self.n_q_heads

    @property
    def compress_bytes(self) -> int:
        """Algorithmic bytes of one compression call: K read once, l_p rows of K and V read and
        written, and the index list written."""
        row = self.n_kv_heads * self.head_dim * 2
        return self.L * row + 4 * self.l_p * row + 4 * self.l_p * self.n_kv_heads


CONFIGS: Dict[str, HostShare] = {
    c.name: c
    for c in [
        HostShare("tiny", 0, 2, 1, 64, 8, 64, 3, 512, 32, 512),
        HostShare("3b-8k", 1, 16, 2, 128, 64, 1024, 3, 8192, 512, 8192, key_recipe="scaled"),
        HostShare("3b-128k", 2, 16, 2, 128, 64, 2048, 7, 16384, 1024, 16384),
        HostShare("7b-frames", 3, 28, 4, 128, 64, 2048, 7, 16384, 2048, 16384, key_recipe="frames"),
        HostShare("imbalance-h1", (4, 1), 28, 4, 128, 64, 4096, 0, 16384, 512, 16384),
        HostShare("imbalance-h8", (4, 8), 28, 4, 128, 64, 4096, 7, 16384, 512, 16384),
        HostShare("imbalance-h15", (4, 15), 28, 4, 128, 64, 4096, 14, 16384, 512, 16384),
    ]
}

#: The configuration the headline metric is quoted on (16K local block, 128K-token video, 8 hosts).
HEADLINE = "3b-128k"


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (nearest, ties to even) and return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns to float32 (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


@dataclass
class HostShareInputs:
    cfg: HostShare
    q_probe: np.ndarray                 # Q_qr  [n_q, Hq, d]
    q: np.ndarray                       # Q^(h) [L, Hq, d]
    k_anchor: np.ndarray                # [l_a, Hkv, d]
    v_anchor: np.ndarray
    k_prev: List[np.ndarray] = field(default_factory=list)   # P x [L_prev, Hkv, d]
    v_prev: List[np.ndarray] = field(default_factory=list)
    k: np.ndarray = None                # K^(h) [L, Hkv, d]
    v: np.ndarray = None


def _keys(rng: np.random.Generator, cfg: HostShare, tokens: int) -> np.ndarray:
    shape = (tokens, cfg.n_kv_heads, cfg.head_dim)
    if cfg.key_recipe == "normal":
        x = rng.standard_normal(shape, dtype=np.float32)
    elif cfg.key_recipe == "scaled":
        x = rng.standard_normal(shape, dtype=np.float32) * np.float32(1.0 / np.sqrt(cfg.head_dim))
    elif cfg.key_recipe == "frames":
        # Video-like redundancy: the tokens of one frame share a mean direction drawn from a random
        # low-dimensional subspace (unit-variance entries), plus independent noise.
        n_frames = -(-tokens // cfg.frame_len)
        x = np.empty(shape, dtype=np.float32)
        for f in range(n_frames):
            lo, hi = f * cfg.frame_len, min(tokens, (f + 1) * cfg.frame_len)
            basis = rng.standard_normal((cfg.n_kv_heads, cfg.head_dim, cfg.frame_rank), dtype=np.float32)
            z = rng.standard_normal((cfg.n_kv_heads, cfg.frame_rank), dtype=np.float32)
            mu = np.einsum("hdr,hr->hd", basis, z) / np.float32(np.sqrt(cfg.frame_rank))
            eps = rng.standard_normal((hi - lo, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32)
            x[lo:hi] = mu[None] + np.float32(cfg.frame_noise) * eps
    else:
        raise ValueError(cfg.key_recipe)
    return f32_to_bf16_bits(x)


def _normal(rng: np.random.Generator, shape) -> np.ndarray:
    return f32_to_bf16_bits(rng.standard_normal(shape, dtype=np.float32))


def generate(cfg: Union[str, HostShare]) -> HostShareInputs:
    """Draw one workload.  Draw order: Q_qr, Q, K_a, V_a, (K^(p), V^(p)) for p < P, K, V."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    rng = np.random.default_rng(cfg.seed)
    hq, hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    out = HostShareInputs(
        cfg=cfg,
        q_probe=_normal(rng, (cfg.n_q, hq, d)),
        q=_normal(rng, (cfg.L, hq, d)),
        k_anchor=_keys(rng, cfg, cfg.l_a),
        v_anchor=_normal(rng, (cfg.l_a, hkv, d)),
    )
    for _ in range(cfg.P):
        out.k_prev.append(_keys(rng, cfg, cfg.L_prev))
        out.v_prev.append(_normal(rng, (cfg.L_prev, hkv, d)))
    out.k = _keys(rng, cfg, cfg.L)
    out.v = _normal(rng, (cfg.L, hkv, d))
    return out


def custom(name: str, seed, hq: int, hkv: int, d: int, n_q: int, l_a: int, P: int, L_prev: int,
           l_p: int, L: int, key_recipe: str = "normal", **kw) -> HostShare:
    """A host share with arbitrary (e.g. ragged, degenerate) sizes, for shape sweeps."""
    return HostShare(name, seed, hq, hkv, d, n_q, l_a, P, L_prev, l_p, L, key_recipe=key_recipe, **kw)
