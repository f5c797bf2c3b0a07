#!/usr/bin/env python3
"""Benchmark of the masked multi-adapter aLoRA QKV projection + paged K/V write on one MI355X.

A "step" is one alora_qkv_forward call (classification/grouping, LoRA shrink, fused projection with
expand/select and the q_out + paged K/V stores) over one synthetic batch already resident in HBM.
Prints ONE JSON line: whole-job tokens/s, the roofline figures of the dominant kernel (the fused
projection GEMM, timed with HIP events recorded on the launch stream inside the timed region), and
the CPU fp64 oracle timed on the host cores over a bounded sample of the same batch.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
METRIC = "masked-aLoRA QKV tokens/s at 1 MI355X; % bf16 MFMA peak / % HBM GB/s"
BOUND = {2: "mfma", 3: "hbm", 4: "mfma", 5: "mfma", 6: "mfma"}
PROFILE_EVERY = 8            # the dominant kernel is timed with HIP events on every 8th step of the timed region


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=(2, 3, 4, 5, 6))
    ap.add_argument("--rotate", type=int, default=0,
                    help="distinct copies of W/A/B cycled through (0 = 8 for the decode config, else 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--operands", choices=("gaussian", "constant"), default="gaussian",
                    help="gaussian: the workload's recipe (default).  constant: x and W overwritten with 1.0, a probe of "
                         "how far the clock under load depends on operand toggling; not the workload, no parity check")
    ap.add_argument("--graph", action="store_true",
                    help="replay the call as a HIP graph (alora_qkv_graph_*), one graph per rotated weight copy; the "
                         "kernel-level roofline figures then come from rocprofv3, not from in-call events")
    ap.add_argument("--reuse-grouping", action="store_true",
                    help="not the headline step: time the per-layer call of a model whose layers share one token batch "
                         "(classification and grouping done once, before the timed region, and reused by every step)")
    ap.add_argument("--rope", action="store_true",
                    help="rotary embedding of q and k fused into the store (not the headline workload: the paper's path has none)")
    ap.add_argument("--library-gemm", action="store_true",
                    help="context, not part of the path: also time the vendor library's plain bf16 GEMM x @ W of the "
                         "same shape (torch.matmul: no adapters, no mask, no cache scatter) on the same box")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 256 MiB device copy (known size) so that a rocprofv3 --pmc run of this "
                         "command holds a reference dispatch for the FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import oracle
    from paper_2512_17910_amd import binding as ab
    from paper_2512_17910_amd import workloads as wl
    from gpu_util import DeviceBatch, host_operands, maxnorm_rel, to_dev, to_f64

    ab.lib()  # fail loudly if the HIP library is missing
    w = wl.CONFIGS[args.config]()
    db = DeviceBatch(w, cache_fill=False)
    if args.operands == "constant":
        db.x.fill_(1.0)
        db.W.fill_(1.0)
    rotate = args.rotate or (8 if args.config == 3 else 1)
    copies = [(db.W, db.A, db.B)]
    for _ in range(rotate - 1):
        copies.append((db.W.clone(), [a.clone() for a in db.A], [b.clone() for b in db.B]))

    graphs = []
    if args.graph:
        graphs = [ab.alora_qkv_graph_create(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot,
                                            w.block_size, db.dims, db.ws, bias=db.bias,
                                            adapter_ranks=w.adapter_ranks) for (W, A, B) in copies]

    rope = None
    if args.rope:
        cos, sin = wl.rope_table(int(w.token_positions.max()) + 1, w.head_dim)
        rope = (torch.from_numpy(cos).to("cuda"), torch.from_numpy(sin).to("cuda"))

    def step(i):
        if graphs:
            ab.alora_qkv_graph_launch(graphs[i % rotate])
            return
        W, A, B = copies[i % rotate]
        if rope is not None:
            ab.alora_qkv_forward_ex(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot, w.block_size, db.dims,
                                    db.ws, bias=db.bias, adapter_ranks=w.adapter_ranks, rope=rope)
            return
        if args.reuse_grouping:
            ab.alora_qkv_forward_ex(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot, w.block_size, db.dims,
                                    db.ws, bias=db.bias, adapter_ranks=w.adapter_ranks, reuse_grouping=True)
            return
        if db.bias is not None or w.adapter_ranks is not None:   # adapter-layout variants (config 6)
            ab.alora_qkv_forward_ex(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot,
                                    w.block_size, db.dims, db.ws, bias=db.bias, adapter_ranks=w.adapter_ranks)
            return
        ab.alora_qkv_forward(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot,
                             w.block_size, db.dims, db.ws)

    if args.calibrate_copy:
        src = torch.ones(256 * 1024 * 1024 // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)   # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst
    if args.reuse_grouping:   # the grouping every timed step reuses
        ab.alora_qkv_classify_group(db.aid, db.start, db.dims, db.ws)
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # HIP events around the projection kernel of every 8th step: an event pair costs a few microseconds of
    # stream time, which would otherwise be part of every decode-sized step
    ab.alora_qkv_profile_begin(args.steps, every=PROFILE_EVERY)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    gemm_ms, n_meas = ab.alora_qkv_profile_end()
    if n_meas == 0:   # graph replays carry no in-call events
        gemm_ms = float("nan")
    # spread of single steps: HIP events on the launch stream around each of 50 further steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(50)]
    for i, (e0, e1) in enumerate(evs):
        e0.record()
        step(i)
        e1.record()
    torch.cuda.synchronize()
    per_step_us = sorted(e0.elapsed_time(e1) * 1e3 for e0, e1 in evs)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = w.T * args.steps / (t1 - t0)

    # algorithmic work of the dominant kernel (fused projection): base GEMM + expand on active rows
    _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
    T_act = int(act.sum())
    used = len(set(int(a) for a in w.token_adapter_ids[act == 1]))
    T_w = int((w.slot_mapping >= 0).sum())
    e = w.elem_bytes
    rk = w.adapter_ranks or [w.rank] * w.n_adapters
    act_rank = float(sum(rk[int(a)] for a in w.token_adapter_ids[act == 1]))   # sum of the active rows' ranks
    flops = 2.0 * w.T * w.hidden * w.N + 2.0 * act_rank * w.N
    if args.config == 3:
        # small-batch path: the dominant kernel is the split projection, which streams x and W and, on
        # workgroups of its own, groups the batch and shrinks the adapted rows (their x rows again, the used
        # adapters' A, the fp32 shrink result out); B, rounding and the stores belong to the finishing kernel
        bytes_ = e * (w.T * w.hidden + w.hidden * w.N + T_act * w.hidden + used * w.hidden * w.rank) + T_act * w.rank * 4
    else:
        bytes_ = e * (w.T * w.hidden + w.hidden * w.N + used * w.rank * w.N + T_act * 2 * w.rank
                      + w.T * w.Nq + T_w * 2 * w.Nkv) + w.T * (1 + 8)
    bound = BOUND[args.config]
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(w.name, {}).get("hbm_bytes_per_launch")
    if gemm_ms != gemm_ms:
        roof = {"bound": bound, "achieved": None, "peak": PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBS,
                "unit": "TFLOP/s" if bound == "mfma" else "GB/s", "frac": None, "traffic": traffic}
    elif bound == "mfma":
        achieved = flops / (gemm_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic}
    else:
        achieved = bytes_ / (gemm_ms * 1e-3) / 1e9
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": traffic}
    roof.update({"kernel": "alora_gemm_bf16_kernel", "kernel_ms": None if gemm_ms != gemm_ms else gemm_ms,
                 "launches_timed": n_meas, "timed_every": PROFILE_EVERY,
                 "algorithmic_flops_per_launch": flops, "algorithmic_bytes_per_launch": bytes_})

    out = {"metric": METRIC, "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic" if args.operands == "gaussian" else "synthetic, x and W constant 1.0 (clock probe, not the workload)",
           "config": {"workload": w.name, "T": w.T, "hidden": w.hidden, "N": w.N, "n_adapters": w.n_adapters,
                      "rank": w.rank, "active_rows": T_act, "block_size": w.block_size,
                      "weight_copies_rotated": rotate, "hip_graph": bool(graphs),
                      "grouping_reused_from_an_earlier_call": bool(args.reuse_grouping),
                      "rotary_embedding_fused": bool(args.rope)},
           "host_enqueue_us_per_step": (t_enq - t0) * 1e6 / args.steps,
           "step_us_median": per_step_us[len(per_step_us) // 2], "step_us_min": per_step_us[0],
           "roofline": roof}

    if args.config == 5:
        # context, not the metric: the rate if the cached, skipped prefix tokens were counted as served
        served = sum(s.first_pos + s.n_tokens for s in w.segments
                     if s is max((u for u in w.segments if u.seq == s.seq), key=lambda u: u.first_pos))
        out["effective_tokens_per_s_counting_cached_prefix"] = served * args.steps / (t1 - t0)
    if not args.no_cpu_baseline and args.operands == "gaussian":
        x, W, A, B = host_operands(w)
        threads = oracle.num_threads()
        probe = wl.sample_rows(w, threads)          # about one row per thread
        tp = time.perf_counter()
        bias64 = wl.widen_f64(w.bias, w.dtype) if w.bias is not None else None
        oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, probe, bias64)
        row_time = (time.perf_counter() - tp) / max(1, -(-len(probe) // threads))
        n = int(max(threads, min(w.T, args.cpu_seconds * threads / max(row_time, 1e-9))))
        rows = wl.sample_rows(w, n)
        tc = time.perf_counter()
        y = oracle.alora_rows_var(x, W, A, B, w.token_adapter_ids, act, rows, bias64)
        secs = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": len(rows) / secs, "unit": "tokens/s", "cores": min(threads, len(rows)),
                               "kind": "oracle", "seconds": secs,
                               "sample": f"{len(rows)} of {w.T} token rows (activation boundaries +-2, segment "
                                         f"ends, evenly spaced rest), full projection + LoRA per row, fp64"}
        # parity of the timed GPU result on the same sample
        q = to_f64(db.q[torch.from_numpy(rows.astype(np.int64)).to("cuda")])
        out["parity_sample_max_rel_err_q"] = maxnorm_rel(q, y[:, : w.Nq])
    if args.library_gemm:
        o = torch.empty((w.T, w.N), dtype=db.x.dtype, device="cuda")
        for i in range(args.warmup):
            torch.matmul(db.x, copies[i % rotate][0], out=o)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(args.steps):
            torch.matmul(db.x, copies[i % rotate][0], out=o)
        e1.record()
        torch.cuda.synchronize()
        lib_ms = e0.elapsed_time(e1) / args.steps
        out["library_plain_gemm"] = {"what": "torch.matmul(x, W_qkv), bf16, same shape and box; no adapters, mask or scatter",
                                     "us": lib_ms * 1e3, "tflops": 2.0 * w.T * w.hidden * w.N / (lib_ms * 1e-3) / 1e12}
    for g in graphs:
        ab.alora_qkv_graph_destroy(g)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
