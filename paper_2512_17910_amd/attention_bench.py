#!/usr/bin/env python3
"""Timing of the paged-cache reader (alora_paged_attention) on the decode batch of configuration 3:
256 sequences x 1 query row, 32 query / 8 K/V heads of 128, block size 16, contexts of 2..2048
positions (the positions of that configuration), bf16.  K/V caches of 2 x 1.07 GB live in HBM, the
rows' contexts cover about half of them, far more than the on-package caches hold.

Prints one JSON line with the roofline of the kernel (bound: HBM; algorithmic bytes = K and V rows
of every row's context; for the row-block kernel of --suffix the bf16 matrix unit, algorithmic flops =
4 x head_dim per (query head, context position)).  Parity is checked by tests/test_gpu_attention.py.

    python -m paper_2512_17910_amd.attention_bench [--steps K] [--warmup W] [--long | --few | --suffix ROWS]
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
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--long", action="store_true", help="contexts of 8k-16k positions on 64 sequences instead")
    ap.add_argument("--few", action="store_true",
                    help="8 sequences with contexts of 32k-64k positions (an adapter evaluated on a few long "
                         "conversations), through alora_paged_attention_split; --single-pass times the plain call on it")
    ap.add_argument("--single-pass", action="store_true")
    ap.add_argument("--suffix", type=int, default=0, metavar="ROWS",
                    help="4 sequences of 16384 positions whose last ROWS positions are query rows (a projected suffix over "
                         "a cached prefix), through alora_paged_attention_suffix; with --single-pass through the per-row call")
    ap.add_argument("--split", action="store_true", help="with --suffix: through alora_paged_attention_suffix_split")
    ap.add_argument("--decode-through-suffix", action="store_true", help="the default decode batch through the suffix call")
    args = ap.parse_args()

    import torch
    from paper_2512_17910_amd import binding as ab
    from paper_2512_17910_amd import workloads as wl

    dev = "cuda"
    Hq, Hkv, D, bs = 32, 8, 128, 16
    rows_per_seq = 1
    if args.suffix:
        lens = np.full(4, 16384)
        rows_per_seq = args.suffix
        name = f"suffix-4x16384-last{args.suffix}"
    elif args.few:
        rng = np.random.default_rng(13)
        lens = rng.integers(32768, 65537, 8)
        name = "decode-8x64k"
    elif args.long:
        rng = np.random.default_rng(12)
        lens = rng.integers(8192, 16385, 64)
        name = "decode-64x16k"
    else:
        w = wl.config3(with_values=False)
        lens = w.token_positions.astype(np.int64) + 1
        name = "cfg3-8b-decode"
    n_seq = len(lens)
    nb = (lens + bs - 1) // bs
    n_blocks = int(nb.sum()) + 8 if (args.long or args.few or args.suffix) else n_seq * (2048 // bs)
    perm = np.random.default_rng(5).permutation(n_blocks).astype(np.int32)
    bt = np.full((n_seq, int(nb.max())), -1, np.int32)
    o = 0
    for s in range(n_seq):
        bt[s, :nb[s]] = perm[o:o + nb[s]]
        o += int(nb[s])
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    kc = torch.randn((n_blocks * bs, Hkv * D), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    vc = torch.randn((n_blocks * bs, Hkv * D), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    seq_h = np.repeat(np.arange(n_seq, dtype=np.int32), rows_per_seq)
    pos_h = np.concatenate([np.arange(l - rows_per_seq, l, dtype=np.int32) for l in lens])
    q = torch.randn((len(seq_h), Hq * D), device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    bt_d = torch.from_numpy(bt).to(dev)
    seq_d = torch.from_numpy(seq_h).to(dev)
    pos_d = torch.from_numpy(pos_h).to(dev)
    dims = ab.make_attn_dims(q, kc, bt_d, Hq, Hkv, D, bs)
    assert ab.alora_paged_attention_validate(bt_d, seq_d, pos_d, dims) == ab.ALORA_OK

    call = lambda: ab.alora_paged_attention(q, kc, vc, bt_d, seq_d, pos_d, out, dims)
    if (args.suffix and not args.single_pass) or args.decode_through_suffix:
        call = lambda: ab.alora_paged_attention_suffix(q, kc, vc, bt_d, seq_d, pos_d, out, dims)
        name += "-rowblocks"
        if args.split:
            ws = torch.empty(max(ab.alora_paged_attention_suffix_workspace_bytes(dims), 16), dtype=torch.uint8, device=dev)
            call = lambda: ab.alora_paged_attention_suffix_split(q, kc, vc, bt_d, seq_d, pos_d, out, dims, ws)
            name += "-split"
    if args.few and not args.single_pass:
        ws = torch.empty(max(ab.alora_paged_attention_workspace_bytes(dims), 16), dtype=torch.uint8, device=dev)
        call = lambda: ab.alora_paged_attention_split(q, kc, vc, bt_d, seq_d, pos_d, out, dims, ws)
        name += "-split"
    for _ in range(args.warmup):
        call()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    ev[0].record()
    for i in range(args.steps):
        call()
        ev[i + 1].record()
    torch.cuda.synchronize()
    per = np.asarray([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)])   # ms, back-to-back launches
    ms = float(ev[0].elapsed_time(ev[-1]) / args.steps)

    ctx_positions = int((pos_h.astype(np.int64) + 1).sum())          # context positions over all rows
    ctx_bytes = int(lens.sum()) * 2 * Hkv * D * 2                      # every cached row once
    io_bytes = ctx_bytes + 2 * len(seq_h) * Hq * D * 2
    flops = 4.0 * ctx_positions * Hq * D
    res = {"metric": "paged-attention reader, context positions/s at 1 MI355X; % HBM GB/s", "value": float(ctx_positions) / (ms * 1e-3),
           "unit": "context positions/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms,
           "step_us_median": float(np.median(per) * 1e3), "higher_is_better": True, "dtype": "bf16", "data": "synthetic",
           "tflops": flops / (ms * 1e-3) / 1e12,
           "config": {"workload": name, "rows": int(len(seq_h)), "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": D, "block_size": bs,
                      "context_positions": ctx_positions, "max_context": int(lens.max())},
           "roofline": {"bound": "hbm", "achieved": io_bytes / (ms * 1e-3) / 1e9, "peak": 8000.0, "unit": "GB/s",
                        "frac": io_bytes / (ms * 1e-3) / 1e9 / 8000.0, "traffic": None, "kernel": "paged_attention_kernel<128, 4, true, true>",
                        "kernel_ms": ms, "algorithmic_bytes_per_launch": io_bytes}}

    if "rowblocks" in name:
        # the row-block kernel loads every cached row once per 128 / G query rows: its bound is the bf16 matrix unit
        res["roofline"] = {"bound": "mfma", "achieved": res["tflops"], "peak": 2500.0, "unit": "TFLOP/s",
                           "frac": res["tflops"] / 2500.0, "traffic": None, "kernel": "paged_attention_blocks_kernel<4, true>",
                           "kernel_ms": ms, "algorithmic_flops_per_launch": flops}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
