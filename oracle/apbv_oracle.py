"""Plain fp64 CPU oracle of one virtual host's share of APB-V's approximate prefill attention.

TEST INFRASTRUCTURE ONLY: slow, obviously-correct numpy written from the paper's definitions.  It
shares no code with the HIP path and must never be imported by it.

What the paper fixes, and what each function follows:

* ``importance_scores`` (and the alternative reductions ``importance_scores_max`` /
  ``importance_scores_softmax_sum`` over ``logit_matrix``) / ``arg_top`` / ``compress_kv`` -- Sec. 3.3 "Approximate Attention" (the
  query-to-context scores Q_qr K^(h)T identify the l_p most important KV pairs) and Alg. 1, steps
  "Identify Essential KVs" and "Send Block 1's Essential KVs" (S_h <- Q_qr K^(h)T;
  (K,V).gather(ArgTop_{l_p}(S_h))).
* ``make_passing_block`` -- Sec. 3.3 (the passing block is the concatenation of the compressed blocks of
  the preceding hosts) and Sec. 4.3 (host h sees h*l_p passing keys).
* ``visibility_mask`` / ``host_attention`` -- Eq. 1 (softmax attention with a mask) applied to the
  concatenated KV of Eq. 4, A_h = Attn(Q^(h), [K_a, K_p^(h), K^(h)], [V_a, V_p^(h), V^(h)]).
* ``merge_lse`` -- Eq. 5, A_qr = Merge({A_qr^(h), lse^(h)}): partial attention results of the same queries over
  disjoint key sets are combined with weights exp(lse^(h)) (the "online softmax" of App. B.1).

Readings taken where the paper is silent (all of them are definitions this build adopts):

* The n_q x l_b score matrix of a GQA group is reduced to one score per key and KV head by SUMMING
  the raw logits over all query-block rows and over the group's query heads.  The sum is linear, so
  it equals the dot product of the key with a pooled query.  **parity unpinned**: the paper gives no
  worked example or closed form for this reduction; the tests pin the arithmetic of the chosen
  definition (linearity against the explicit logit matrix, exact rational evaluation on tiny inputs),
  not the choice itself.
* ArgTop returns indices ordered by descending score; equal scores (compared as real numbers, so
  +0 == -0) are ordered by ascending index.  Selection is per KV head.
* The mask of Eq. 1 is additive: a masked logit is excluded from the softmax.  Anchor and passing
  keys are visible to every local query; local key j is visible to local query i iff j <= i.
* Only strictly preceding hosts contribute to the passing block.
* The softmax scale is 1/sqrt(head_dim), passed in explicitly.

All tensor arguments are numpy ``uint16`` arrays of bf16 bit patterns, ``[tokens, heads, head_dim]``;
they are widened exactly to float64 before any arithmetic.
"""
from __future__ import annotations

from typing import List, Optional, Sequence, Tuple

import numpy as np


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening bf16 -> float64 (bf16 is the upper half of an IEEE float32)."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------- compression (Sec. 3.3)

def pooled_query(q_probe: np.ndarray, n_kv_heads: int) -> np.ndarray:
    """q_bar[v, :] = sum over the query-block rows t and the query heads g of KV head v's group of
    Q_qr[t, v*G+g, :].  Returns float64 ``[Hkv, d]``."""
    q = bf16_bits_to_f64(q_probe)                      # [n_q, Hq, d]
    n_q, hq, d = q.shape
    if hq % n_kv_heads:
        raise ValueError("Hq must be a multiple of Hkv")
    g = hq // n_kv_heads
    return q.reshape(n_q, n_kv_heads, g, d).sum(axis=(0, 2))


def importance_scores(q_probe: np.ndarray, k: np.ndarray) -> np.ndarray:
    """s[v, j] = sum_t sum_g Q_qr[t, v*G+g, :] . K[j, v, :]   (Alg. 1: S_h <- Q_qr K^(h)T, summed
    over the rows of S_h that belong to KV head v).  Returns float64 ``[Hkv, L]``.

    The sum over the head dimension is taken one coordinate at a time, in ascending order and in the
    same order for every key, so that identical key rows get identical scores (exact ties)."""
    kk = bf16_bits_to_f64(k)                           # [L, Hkv, d]
    L, hkv, d = kk.shape
    qbar = pooled_query(q_probe, hkv)                  # [Hkv, d]
    s = np.zeros((hkv, L), dtype=np.float64)
    for v in range(hkv):
        for c in range(d):
            s[v] += qbar[v, c] * kk[:, v, c]
    return s


def logit_matrix(q_probe: np.ndarray, k: np.ndarray, kv_head: int) -> np.ndarray:
    """The rows of S_h = Q_qr K^(h)T (Alg. 1) that belong to KV head ``kv_head``: raw logits
    ``[n_q * G, L]`` float64, row (t, g) = Q_qr[t, kv_head*G+g, :] . K[:, kv_head, :]."""
    q = bf16_bits_to_f64(q_probe)
    kk = bf16_bits_to_f64(k)
    n_q, hq, d = q.shape
    hkv = kk.shape[1]
    if hq % hkv:
        raise ValueError("Hq must be a multiple of Hkv")
    g = hq // hkv
    rows = q[:, kv_head * g:(kv_head + 1) * g, :].reshape(n_q * g, d)
    return rows @ kk[:, kv_head, :].T


def importance_scores_max(q_probe: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Alternative reduction of S_h to one score per key: s[v, j] = max over the query-block rows t and the
    group's query heads g of the raw logit Q_qr[t, v*G+g, :] . K[j, v, :].  Returns float64 ``[Hkv, L]``.
    (A reading of Sec. 3.3 / Alg. 1 other than the sum; **parity unpinned** by the paper like the sum.)"""
    hkv = k.shape[1]
    return np.stack([logit_matrix(q_probe, k, v).max(axis=0) for v in range(hkv)])


def importance_scores_softmax_sum(q_probe: np.ndarray, k: np.ndarray, softmax_scale: float) -> np.ndarray:
    """Alternative reduction of S_h: every query row's scaled logits are normalised by a softmax over the
    block's keys (Eq. 1 without a mask) and the probabilities are summed over the rows:
    s[v, j] = sum_{t, g} softmax_j(softmax_scale * S_h[(t, g), :])[j]  -- the attention mass the query block
    puts on key j (the kind of pruning score App. C names for the FastV baseline, "SnapKV-like").  Returns float64
    ``[Hkv, L]``.  **parity unpinned** by the paper."""
    hkv = k.shape[1]
    out = []
    for v in range(hkv):
        z = softmax_scale * logit_matrix(q_probe, k, v)
        z = z - z.max(axis=1, keepdims=True)
        e = np.exp(z)
        out.append((e / e.sum(axis=1, keepdims=True)).sum(axis=0))
    return np.stack(out)


def arg_top(scores: np.ndarray, l_p: int) -> np.ndarray:
    """Indices of the l_p largest entries of a 1-D score vector, by descending score; equal scores by
    ascending index (a stable sort of 0..L-1 on the negated score)."""
    s = np.asarray(scores, dtype=np.float64)
    if s.ndim != 1:
        raise ValueError("arg_top takes one score vector")
    if not 0 <= l_p <= s.shape[0]:
        raise ValueError("need 0 <= l_p <= L")
    if not np.all(np.isfinite(s)):
        raise ValueError("scores must be finite")
    order = np.argsort(-(s + 0.0), kind="stable")      # s + 0.0 turns -0.0 into +0.0
    return order[:l_p].astype(np.int32)


def compress_kv(q_probe: np.ndarray, k: np.ndarray, v: np.ndarray, l_p: int, reducer: str = "sum",
                softmax_scale: Optional[float] = None
                ) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
    """Compressed block of one context block (Alg. 1: (K,V).gather(ArgTop_{l_p}(S_h))).  ``reducer`` picks how
    S_h becomes one score per key: "sum" (the adopted reading), "max" or "softmax_sum" (needs ``softmax_scale``).

    Returns ``(idx [Hkv, l_p] int32, K_c [l_p, Hkv, d] uint16, V_c [l_p, Hkv, d] uint16,
    scores [Hkv, L] float64)``; row i of K_c for head v is the bit copy of K[idx[v, i], v, :]."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    L, hkv, d = k.shape
    if v.shape != k.shape:
        raise ValueError("K and V must have the same shape")
    if reducer == "sum":
        s = importance_scores(q_probe, k)
    elif reducer == "max":
        s = importance_scores_max(q_probe, k)
    elif reducer == "softmax_sum":
        if softmax_scale is None:
            raise ValueError("softmax_sum needs softmax_scale")
        s = importance_scores_softmax_sum(q_probe, k, softmax_scale)
    else:
        raise ValueError("unknown reducer")
    idx = np.empty((hkv, l_p), dtype=np.int32)
    k_c = np.empty((l_p, hkv, d), dtype=np.uint16)
    v_c = np.empty((l_p, hkv, d), dtype=np.uint16)
    for h in range(hkv):
        idx[h] = arg_top(s[h], l_p)
        k_c[:, h, :] = k[idx[h], h, :]
        v_c[:, h, :] = v[idx[h], h, :]
    return idx, k_c, v_c, s


def make_passing_block(q_probe: np.ndarray, k_prev: Sequence[np.ndarray], v_prev: Sequence[np.ndarray],
                       l_p: int, n_kv_heads: int, head_dim: int) -> Tuple[np.ndarray, np.ndarray]:
    """Passing block of a host: compressed blocks of the strictly preceding hosts, in host order
    (Sec. 3.3).  Returns ``(K_p, V_p)``, each ``[P*l_p, Hkv, d]`` uint16."""
    ks: List[np.ndarray] = [np.empty((0, n_kv_heads, head_dim), dtype=np.uint16)]
    vs: List[np.ndarray] = [np.empty((0, n_kv_heads, head_dim), dtype=np.uint16)]
    for kp, vp in zip(k_prev, v_prev):
        _, k_c, v_c, _ = compress_kv(q_probe, kp, vp, l_p)
        ks.append(k_c)
        vs.append(v_c)
    return np.concatenate(ks, axis=0), np.concatenate(vs, axis=0)


# --------------------------------------------------------------------------- attention (Eq. 1, Eq. 4)

def visibility_mask(rows: np.ndarray, l_a: int, n_pass: int, L: int) -> np.ndarray:
    """Boolean mask ``[len(rows), l_a + n_pass + L]`` over the concatenated keys [anchor | passing |
    local]: anchor and passing keys are visible to every query; local key j is visible to local query
    i iff j <= i."""
    rows = np.asarray(rows, dtype=np.int64)
    m = np.zeros((rows.shape[0], l_a + n_pass + L), dtype=bool)
    m[:, : l_a + n_pass] = True
    m[:, l_a + n_pass:] = np.arange(L, dtype=np.int64)[None, :] <= rows[:, None]
    return m


def host_attention(q: np.ndarray,
                   k_anchor: np.ndarray, v_anchor: np.ndarray,
                   k_pass: np.ndarray, v_pass: np.ndarray,
                   k: np.ndarray, v: np.ndarray,
                   scale: float,
                   rows: Optional[np.ndarray] = None,
                   chunk: int = 512) -> Tuple[np.ndarray, np.ndarray]:
    """A_h of Eq. 4 by the definition of Eq. 1, in float64.  With an empty local segment (``k`` of 0 tokens) every
    anchor/passing key is visible to every query: a partial result in the sense of Eq. 5.

    ``rows`` (optional) restricts the computation to those local query positions; every computed row
    is still a full softmax over its complete masked key set.  ``chunk`` only bounds how many query
    rows are materialised at once.  Returns ``(O [n_rows, Hq, d] float64, lse [Hq, n_rows] float64)``
    with lse the natural-log sum of exponentials of the scaled visible logits."""
    qq = bf16_bits_to_f64(q)                                   # [L, Hq, d]
    L, hq, d = qq.shape
    k_cat = np.concatenate([bf16_bits_to_f64(k_anchor), bf16_bits_to_f64(k_pass), bf16_bits_to_f64(k)], axis=0)
    v_cat = np.concatenate([bf16_bits_to_f64(v_anchor), bf16_bits_to_f64(v_pass), bf16_bits_to_f64(v)], axis=0)
    l_a, n_pass = k_anchor.shape[0], k_pass.shape[0]
    hkv = k_cat.shape[1]
    l_k = k.shape[0]                  # local (causal) keys: L of them, or none (every key visible)
    if l_k not in (0, L) or hq % hkv or v_cat.shape != k_cat.shape or k_cat.shape[0] == 0:
        raise ValueError("inconsistent shapes")
    g = hq // hkv
    if rows is None:
        rows = np.arange(L, dtype=np.int64)
    rows = np.asarray(rows, dtype=np.int64)
    scale = float(scale)
    out = np.empty((rows.shape[0], hq, d), dtype=np.float64)
    lse = np.empty((hq, rows.shape[0]), dtype=np.float64)
    for lo in range(0, rows.shape[0], chunk):
        r = rows[lo: lo + chunk]
        mask = visibility_mask(r, l_a, n_pass, l_k)            # [r, S_kv]
        for h in range(hq):
            kv = h // g
            z = scale * (qq[r, h, :] @ k_cat[:, kv, :].T)      # [r, S_kv]
            z[~mask] = -np.inf
            m = z.max(axis=1, keepdims=True)
            e = np.exp(z - m)
            den = e.sum(axis=1, keepdims=True)
            out[lo: lo + r.shape[0], h, :] = (e @ v_cat[:, kv, :]) / den
            lse[h, lo: lo + r.shape[0]] = (m + np.log(den))[:, 0]
    return out, lse


# --------------------------------------------------------------------------- merge (Eq. 5)

def merge_lse(parts_out: Sequence[np.ndarray], parts_lse: Sequence[np.ndarray]) -> Tuple[np.ndarray, np.ndarray]:
    """Combine partial attention results over disjoint key sets (Eq. 5).

    ``parts_out[h]`` is ``[rows, Hq, d]`` (float64), ``parts_lse[h]`` is ``[Hq, rows]`` with the natural-log sum of
    exponentials of part h's scaled logits (``-inf`` for a part that saw no key).  Returns ``(A, lse)`` with
    ``A = sum_h e^{lse_h} A_h / sum_h e^{lse_h}`` and ``lse = log sum_h e^{lse_h}``, evaluated with the maximum
    factored out."""
    outs = np.stack([np.asarray(a, dtype=np.float64) for a in parts_out])        # [n, rows, Hq, d]
    lses = np.stack([np.asarray(a, dtype=np.float64) for a in parts_lse])        # [n, Hq, rows]
    m = lses.max(axis=0)                                                          # [Hq, rows]
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w = np.exp(lses - m_safe[None])                                               # exp(-inf) = 0
    den = w.sum(axis=0)                                                           # [Hq, rows]
    w_rhd = np.transpose(w, (0, 2, 1))[..., None]                                 # [n, rows, Hq, 1]
    with np.errstate(invalid="ignore", divide="ignore"):
        out = (w_rhd * outs).sum(axis=0) / np.transpose(den)[..., None]
        lse = m_safe + np.log(den)
    out = np.where(np.transpose(den)[..., None] > 0, out, 0.0)
    return out, lse
