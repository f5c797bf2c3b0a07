#!/usr/bin/env python3
"""What cache reuse saves per layer (Sec. 2.3 / Sec. 4 of the paper, in this library's kernels): one turn of
REQS requests that each append SUFFIX tokens (an adapter's invocation sequence and the tokens after it) to a
conversation of CONTEXT tokens whose K/V blocks the base model wrote earlier.

  aLoRA turn  the blocks before the activation point are the base model's and stay valid: only the SUFFIX rows
              are projected (adapter applied to all of them, rotary embedding fused) and attend over the cached
              context + themselves (row-block reader, contexts cut into parts).
  LoRA turn   a standard LoRA changes K/V from position 0: every one of the CONTEXT tokens is projected again
              with the adapter and the whole causal attention is recomputed (row-block reader, unsplit).

Both through the C ABI on synthetic data (8B shapes: hidden 4096, 32 query / 8 K/V heads of 128, rank-32
adapter, block size 16, bf16).  Prints one JSON line with the two times per layer and their ratio.

    python -m paper_2512_17910_amd.reuse_bench [--reqs 4] [--context 16384] [--suffix 64] [--steps 10]
"""
from __future__ import annotations

import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--reqs", type=int, default=4)
    ap.add_argument("--context", type=int, default=16384)
    ap.add_argument("--suffix", type=int, default=64)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    args = ap.parse_args()

    import torch
    from paper_2512_17910_amd import binding as ab
    from paper_2512_17910_amd import workloads as wl

    dev = "cuda"
    H, Hq, Hkv, D, bs, r, L = 4096, 32, 8, 128, 16, 32, 4
    Nq, Nkv = Hq * D, Hkv * D
    N = Nq + 2 * Nkv
    R, C, S = args.reqs, args.context, args.suffix
    assert C % bs == 0 and 0 < S <= C
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    rnd = lambda shape, std: (torch.randn(shape, device=dev, generator=g, dtype=torch.float32) * std).to(torch.bfloat16)
    W = rnd((H, N), H ** -0.5)
    A = [rnd((H, r), H ** -0.5) for _ in range(L)]
    B = [rnd((r, N), r ** -0.5) for _ in range(L)]
    nb = C // bs
    perm = np.random.default_rng(5).permutation(R * nb).astype(np.int32)
    bt = perm.reshape(R, nb)
    kc = rnd((R * C, Nkv), 1.0)          # the context's K/V as an earlier base-model turn left them
    vc = rnd((R * C, Nkv), 1.0)
    cos, sin = wl.rope_table(C, D)
    rope = (torch.from_numpy(cos).to(dev), torch.from_numpy(sin).to(dev))
    bt_d = torch.from_numpy(bt).to(dev)

    def turn(rows_per_req: int, activation: int):
        """Buffers and the two calls for a turn that projects the last rows_per_req positions of every request."""
        T = R * rows_per_req
        pos = np.tile(np.arange(C - rows_per_req, C, dtype=np.int32), R)
        seg = np.repeat(np.arange(R, dtype=np.int32), rows_per_req)
        slot = (bt[seg, pos // bs].astype(np.int64) * bs + pos % bs)
        d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        x = rnd((T, H), 1.0)
        aid = d((seg % L).astype(np.int32))
        start = d(np.full(R, activation, np.int32))
        seg_d, pos_d, slot_d = d(seg), d(pos), d(slot)
        dims = ab.make_dims(ab.ALORA_BF16, T, H, Hq, Hkv, D, L, r, R, R * C, seg_d, pos_d)
        ws = ab.alloc_workspace(dims)
        q = torch.empty((T, Nq), dtype=torch.bfloat16, device=dev)
        out = torch.empty_like(q)
        adims = ab.make_attn_dims(q, kc, bt_d, Hq, Hkv, D, bs)
        aws = torch.empty(max(ab.alora_paged_attention_suffix_workspace_bytes(adims), 16), dtype=torch.uint8, device=dev)

        def project():
            ab.alora_qkv_forward_ex(x, aid, start, W, A, B, q, kc, vc, slot_d, bs, dims, ws, rope=rope)

        def attend():
            ab.alora_paged_attention_suffix_split(q, kc, vc, bt_d, seg_d, pos_d, out, adims, aws)
        return T, project, attend

    def time_ms(fn):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.steps

    res = {}
    for name, rows, act in (("alora", S, C - S), ("lora", C, 0)):
        T, project, attend = turn(rows, act)
        res[name] = {"rows_projected": T, "projection_ms": time_ms(project), "attention_ms": time_ms(attend)}
        res[name]["layer_ms"] = res[name]["projection_ms"] + res[name]["attention_ms"]
        torch.cuda.empty_cache()
    out = {"metric": "per-layer time of one turn: aLoRA (cached prefix reused) vs LoRA (prefix recomputed), 1 MI355X",
           "value": res["lora"]["layer_ms"] / res["alora"]["layer_ms"], "unit": "x (LoRA layer time / aLoRA layer time)",
           "higher_is_better": True, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": f"turn-{R}x{C}-suffix{S}", "requests": R, "context": C, "suffix": S, "hidden": H,
                      "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "rank": r, "block_size": bs, "rotary_embedding_fused": True},
           "alora": res["alora"], "lora": res["lora"]}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
