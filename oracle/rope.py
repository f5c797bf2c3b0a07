"""CPU fp64 oracle of the rotary position embedding applied to the q and k parts of projected rows.

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py): imported by tests/ alone; the GPU library shares no code
with it.

The paper does not treat positions (Sec. 2.1 speaks of per-token query, key and value vectors only); a
served Llama-family layer rotates q and k between the projection and the cache write, which is why the
fusion is listed as the step next to the path.  What is computed is the textbook rotation (RoFormer, Su et
al. 2021, in the "rotate-half" pairing the Llama family uses): within every head of dimension D, feature i
and feature i + D/2 form a plane that is turned by the angle the caller's table gives for (position, i):

    out[i]       = y[i] * cos[p, i] - y[i + D/2] * sin[p, i]
    out[i + D/2] = y[i + D/2] * cos[p, i] + y[i] * sin[p, i]            0 <= i < D/2

q heads and k heads are rotated, v is not.  The table is an input (fp32 values widened to fp64 by the
caller), so the oracle holds no trigonometry of its own.  Pinned by tests/test_rope_pins.py.
"""
from __future__ import annotations

import numpy as np


def rope_rows(y, positions, cos, sin, n_q_heads: int, n_kv_heads: int, head_dim: int) -> np.ndarray:
    """y: [R, (n_q_heads + 2 * n_kv_heads) * head_dim] projected rows (q | k | v); positions: [R];
    cos, sin: [max_pos, head_dim / 2].  Returns the rows with q and k rotated."""
    y = np.array(y, dtype=np.float64)
    cos = np.asarray(cos, dtype=np.float64)
    sin = np.asarray(sin, dtype=np.float64)
    half = head_dim // 2
    out = y.copy()
    for r in range(y.shape[0]):
        p = int(positions[r])
        c, s = cos[p], sin[p]
        for h in range(n_q_heads + n_kv_heads):          # the q heads, then the k heads; v follows and stays
            lo = h * head_dim
            a = y[r, lo:lo + half]
            b = y[r, lo + half:lo + head_dim]
            out[r, lo:lo + half] = a * c - b * s
            out[r, lo + half:lo + head_dim] = b * c + a * s
    return out
