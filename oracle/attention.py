"""Oracle for the reader of the paged K/V cache: causal softmax attention (Sec. 2.1).

TEST INFRASTRUCTURE ONLY, like the rest of this package: numpy fp64, one query row and one head at
a time, the definition written out; the GPU reader shares no code with it.

What the paper fixes (Sec. 2.1, in words): attention is causal softmax attention over the query,
key and value vectors of the tokens; a token's K and V never change once computed, so they are
cached and a later step reads all of them.  Sec. 2.3: K and V of tokens before the activation
point are the base model's, which is why a block written by one request can be read by another.
The paper gives no formula; the textbook definition is used:

    o[t, h, :] = sum_{j=0..p}  softmax_j( scale * <q[t, h, :], k_j[g(h), :]> ) * v_j[g(h), :]

for the row t at position p of its sequence, where k_j / v_j are the cached rows of position j of
that sequence, found through the sequence's block table:

    slot(j) = block_table[seq][j // block_size] * block_size + j % block_size

Readings where the paper is silent:
  - scale = 1 / sqrt(head_dim) unless given;
  - grouped-query attention: n_q_heads / n_kv_heads consecutive query heads share one K/V head,
    g(h) = h // (n_q_heads // n_kv_heads);
  - the row at position p attends to positions 0..p inclusive (its own K/V are in the cache by the
    time the reader runs: the projection of the same step wrote them);
  - no positional rotation is applied by the reader (none is applied by the projection either).
"""
from __future__ import annotations

from typing import Optional

import numpy as np


def context_slots(block_table_row: np.ndarray, n_ctx: int, block_size: int) -> np.ndarray:
    """Cache slots of positions 0..n_ctx-1 of one sequence."""
    j = np.arange(n_ctx, dtype=np.int64)
    return block_table_row[j // block_size].astype(np.int64) * block_size + j % block_size


def paged_attention(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, block_tables: np.ndarray,
                    token_seq_ids: np.ndarray, token_positions: np.ndarray, block_size: int,
                    n_q_heads: int, n_kv_heads: int, head_dim: int, scale: Optional[float] = None,
                    rows: Optional[np.ndarray] = None) -> np.ndarray:
    """q [T, n_q_heads*head_dim]; caches [n_slots, n_kv_heads*head_dim]; block_tables
    [n_seq, max_blocks]; returns o [len(rows), n_q_heads*head_dim] in fp64 (rows = all by default)."""
    q = np.asarray(q, dtype=np.float64)
    k_cache = np.asarray(k_cache, dtype=np.float64)
    v_cache = np.asarray(v_cache, dtype=np.float64)
    assert n_q_heads % n_kv_heads == 0
    group = n_q_heads // n_kv_heads
    if scale is None:
        scale = 1.0 / np.sqrt(float(head_dim))
    if rows is None:
        rows = np.arange(q.shape[0])
    out = np.zeros((len(rows), n_q_heads * head_dim), dtype=np.float64)
    for i, t in enumerate(rows):
        p = int(token_positions[t])
        slots = context_slots(block_tables[int(token_seq_ids[t])], p + 1, block_size)
        K = k_cache[slots].reshape(p + 1, n_kv_heads, head_dim)
        V = v_cache[slots].reshape(p + 1, n_kv_heads, head_dim)
        for h in range(n_q_heads):
            g = h // group
            qh = q[t, h * head_dim:(h + 1) * head_dim]
            score = scale * (K[:, g, :] @ qh)                 # [p+1]
            w = np.exp(score - score.max())
            w = w / w.sum()
            out[i, h * head_dim:(h + 1) * head_dim] = w @ V[:, g, :]
    return out
