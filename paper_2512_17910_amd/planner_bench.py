#!/usr/bin/env python3
"""Host-side timing of the block cache / suffix planner on a long-context, multi-turn shape
(4 conversations of 16384 tokens, block size 16: a base turn fills the cache, an aLoRA turn reuses
it and plans only its suffix).
Prints one JSON line.   python -m paper_2512_17910_amd.planner_bench"""
from __future__ import annotations

import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def run(make, n_seq=4, n_tok=16384, bs=16, tail=96, seed=3):
    rng = np.random.default_rng(seed)
    convs = [rng.integers(0, 32000, n_tok).astype(np.int32) for _ in range(n_seq)]
    c = make(bs, 2 * n_seq * (n_tok // bs + 8))
    t0 = time.perf_counter()
    rows_base = sum(c.admit_commit_finish(i, convs[i][: n_tok - tail], -1, 1 << 30) for i in range(n_seq))
    t1 = time.perf_counter()
    rows_alora = sum(c.admit_commit_finish(100 + i, convs[i], i % 3, n_tok - tail) for i in range(n_seq))
    t2 = time.perf_counter()
    return {"base_turn_s": t1 - t0, "alora_turn_s": t2 - t1, "rows_base_turn": int(rows_base),
            "rows_alora_turn": int(rows_alora), "tokens_hashed_per_turn": n_seq * n_tok}


class Lib:
    def __init__(self, bs, n_blocks):
        from paper_2512_17910_amd import planner as pl
        self.pl, self.p = pl, pl.Planner(bs, n_blocks)

    def admit_commit_finish(self, rid, tokens, adapter, start):
        b = self.pl.Batch(len(tokens), 1)
        self.p.admit(rid, tokens, adapter, start, b)
        self.p.commit(rid)
        self.p.finish(rid)
        return b.n_rows


def main() -> int:
    lib = run(Lib)
    n = lib["tokens_hashed_per_turn"]
    print(json.dumps({"what": "block cache / suffix planner, host only", "library": lib,
                      "tokens_per_s_base_turn": n / lib["base_turn_s"],
                      "tokens_per_s_alora_turn": n / lib["alora_turn_s"]}))
    return 0


if __name__ == "__main__":
    sys.exit(main())
