#!/usr/bin/env python3
"""Benchmark of the masked multi-adapter aLoRA QKV projection + paged K/V write on one MI355X.

A "step" is one alora_qkv_forward call (classification/grouping, LoRA shrink, projection with
expand/select and the q_out + paged K/V stores) over one synthetic batch already resident in HBM.

Default run: every benchmark workload in turn -- the 70B-shaped prefill (the largest single-GPU shape,
whose numbers are the headline fields), the 8B-shaped prefill chunk, the 8B-shaped decode batch and the
long-context suffix mix -- each with its own warm-up and timed steps.  Prints ONE JSON line: the headline
fields, a "configs" list with every workload's step time, tokens/s and roofline figures, and the CPU fp64
oracle timed on the host cores over a bounded sample of the headline batch.

Roofline figures.  Prefill-sized workloads are bound by the bf16 matrix pipe: algorithmic flops of the
dominant kernel (the fused projection: base product + low-rank expand) over that kernel's duration, timed
with HIP events the library records on the launch stream inside the timed region.  The decode-sized
workload is bound by HBM: algorithmic bytes of the WHOLE call (x, W, the used adapters' A and B, q_out, the
K/V rows, the index arrays) over the whole step's duration; the projection kernel's own figure is given
beside it.  HBM traffic counters come from rocprofv3 runs of this command (profiles/), not from this run.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2|3|4|5|6] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
METRIC = "masked-aLoRA QKV tokens/s at 1 MI355X; % bf16 MFMA peak / % HBM GB/s"
BOUND = {2: "mfma", 3: "hbm", 4: "mfma", 5: "mfma", 6: "mfma"}
PROFILE_EVERY = 8            # the dominant kernel is timed with HIP events on every 8th step of the timed region
HEADLINE = 4                 # the largest single-GPU workload
DEFAULT_ORDER = (4, 2, 3, 5)


def measure(cfg: int, args, cpu_baseline: bool) -> dict:
    """Warm up, time args.steps steps of workload `cfg`, and return its record."""
    import numpy as np
    import torch
    from paper_2512_17910_amd import binding as ab
    from paper_2512_17910_amd import workloads as wl
    from paper_2512_17910_amd.harness import DeviceBatch, host_operands, maxnorm_rel, to_f64

    w = wl.CONFIGS[cfg]()
    db = DeviceBatch(w, cache_fill=False)
    if args.operands == "constant":
        db.x.fill_(1.0)
        db.W.fill_(1.0)
    # the decode batch's 50 MB of weights would sit in the memory-side cache: rotate through copies (a stack of layers)
    rotate = args.rotate or (8 if cfg == 3 else 1)
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
        if rope is not None or args.reuse_grouping or db.bias is not None or w.adapter_ranks is not None:
            ab.alora_qkv_forward_ex(db.x, db.aid, db.start, W, A, B, db.q, db.kc, db.vc, db.slot, w.block_size, db.dims,
                                    db.ws, bias=db.bias, adapter_ranks=w.adapter_ranks, rope=rope,
                                    reuse_grouping=bool(args.reuse_grouping))
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

    # algorithmic work (what the method itself must do; rows that keep the base output cost no adapter flops,
    # adapters no active row uses cost no bytes)
    # (which rows are adapted: the library's own classification of this batch, read back from the workspace)
    act = ab.alora_qkv_classify_group(db.aid, db.start, db.dims, db.ws)[0].cpu().numpy()
    T_act = int(act.sum())
    used_ids = sorted(set(int(a) for a in w.token_adapter_ids[act == 1]))
    T_w = int((w.slot_mapping >= 0).sum())
    e = w.elem_bytes
    rk = w.adapter_ranks or [w.rank] * w.n_adapters
    act_rank = float(sum(rk[int(a)] for a in w.token_adapter_ids[act == 1]))   # sum of the active rows' ranks
    used_rank = float(sum(rk[a] for a in used_ids))
    # dominant kernel (fused projection): base product + expand on active rows
    k_flops = 2.0 * w.T * w.hidden * w.N + 2.0 * act_rank * w.N
    k_bytes = e * (w.T * w.hidden + w.hidden * w.N + used_rank * w.N + T_act * 2 * w.rank
                   + w.T * w.Nq + T_w * 2 * w.Nkv) + w.T * (1 + 8)
    # whole call: also the shrink (A) and the index arrays
    call_flops = k_flops + 2.0 * act_rank * w.hidden
    call_bytes = e * (w.T * w.hidden + w.hidden * w.N + used_rank * (w.hidden + w.N) + w.T * w.Nq + T_w * 2 * w.Nkv) \
        + w.T * (4 + 4 + 4 + 8) + 4 * w.n_segments
    bound = BOUND[cfg]
    kernel_ms = None if gemm_ms != gemm_ms else gemm_ms
    if bound == "mfma":
        achieved = None if kernel_ms is None else k_flops / (kernel_ms * 1e-3) / 1e12
        roof = {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                "frac": None if achieved is None else achieved / PEAK_BF16_TFLOPS, "traffic": None,
                "over": "dominant kernel (fused projection), HIP events on the launch stream",
                "kernel": "alora_gemm_bf16_kernel", "kernel_ms": kernel_ms,
                "algorithmic_flops_per_launch": k_flops, "algorithmic_bytes_per_launch": k_bytes}
    else:
        step_s = per_step_us[len(per_step_us) // 2] * 1e-6
        achieved = call_bytes / step_s / 1e9
        # the split projection kernel alone: it streams x and W and, on workgroups of its own, groups the batch
        # and shrinks the adapted rows; B, rounding and the stores belong to the finishing kernel
        pk_bytes = e * (w.T * w.hidden + w.hidden * w.N + T_act * w.hidden + used_rank * w.hidden) + T_act * w.rank * 4
        roof = {"bound": "hbm", "achieved": achieved, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": achieved / PEAK_HBM_GBS, "traffic": None,
                "over": "whole step (every kernel of one call): algorithmic bytes of the call / median step time",
                "kernel": "alora_gemm_bf16_kernel (split projection) + finish_bf16_kernel", "kernel_ms": kernel_ms,
                "algorithmic_bytes_per_step": call_bytes, "algorithmic_flops_per_step": call_flops,
                "projection_kernel_alone": None if kernel_ms is None else {
                    "algorithmic_bytes_per_launch": pk_bytes, "GB/s": pk_bytes / (kernel_ms * 1e-3) / 1e9,
                    "frac": pk_bytes / (kernel_ms * 1e-3) / 1e9 / PEAK_HBM_GBS}}
    roof.update({"launches_timed": n_meas, "timed_every": PROFILE_EVERY})

    rec = {"workload": w.name, "value": tokens_per_s, "ms_per_step": ms_per_step,
           "config": {"workload": w.name, "T": w.T, "hidden": w.hidden, "N": w.N, "n_adapters": w.n_adapters,
                      "rank": w.rank, "active_rows": T_act, "block_size": w.block_size,
                      "weight_copies_rotated": rotate, "hip_graph": bool(graphs),
                      "grouping_reused_from_an_earlier_call": bool(args.reuse_grouping),
                      "rotary_embedding_fused": bool(args.rope)},
           "host_enqueue_us_per_step": (t_enq - t0) * 1e6 / args.steps,
           "step_us_median": per_step_us[len(per_step_us) // 2], "step_us_min": per_step_us[0],
           "roofline": roof}
    if cfg == 5:
        # context, not the metric: the rate if the cached, skipped prefix tokens were counted as served
        served = sum(s.first_pos + s.n_tokens for s in w.segments
                     if s is max((u for u in w.segments if u.seq == s.seq), key=lambda u: u.first_pos))
        rec["effective_tokens_per_s_counting_cached_prefix"] = served * args.steps / (t1 - t0)
    if cpu_baseline and args.operands == "gaussian":
        import oracle   # test infrastructure: only this leg of the benchmark touches it
        _, act = oracle.classify(w.token_adapter_ids, w.token_seg_ids, w.token_positions, w.activation_start)
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
        del x, W, A, B
        rec["cpu_baseline"] = {"value": len(rows) / secs, "unit": "tokens/s", "cores": min(threads, len(rows)),
                               "kind": "oracle", "seconds": secs,
                               "sample": f"{len(rows)} of {w.T} token rows of {w.name} (activation boundaries +-2, segment "
                                         f"ends, evenly spaced rest), full projection + LoRA per row, fp64"}
        # parity of the timed GPU result on the same sample
        q = to_f64(db.q[torch.from_numpy(rows.astype(np.int64)).to("cuda")])
        rec["parity_sample_max_rel_err_q"] = maxnorm_rel(q, y[:, : w.Nq])
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
        rec["library_plain_gemm"] = {"what": "torch.matmul(x, W_qkv), bf16, same shape and box; no adapters, mask or scatter",
                                     "us": lib_ms * 1e3, "tflops": 2.0 * w.T * w.hidden * w.N / (lib_ms * 1e-3) / 1e12}
    for g in graphs:
        ab.alora_qkv_graph_destroy(g)
    del db, copies
    gc.collect()
    torch.cuda.empty_cache()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=0, choices=(0, 2, 3, 4, 5, 6),
                    help="0 (default): every benchmark workload in turn, headline = the 70B-shaped prefill; else that one workload")
    ap.add_argument("--rotate", type=int, default=0,
                    help="distinct copies of W/A/B cycled through (0 = 8 for the decode config, else 1)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
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

    from paper_2512_17910_amd import binding as ab
    ab.lib()  # fail loudly if the HIP library is missing

    order = (args.config,) if args.config else DEFAULT_ORDER
    head_cfg = args.config or HEADLINE
    recs = {c: measure(c, args, cpu_baseline=(c == head_cfg and not args.no_cpu_baseline)) for c in order}
    head = recs[head_cfg]
    out = {"metric": METRIC, "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "bf16",
           "data": "synthetic" if args.operands == "gaussian" else "synthetic, x and W constant 1.0 (clock probe, not the workload)",
           "config": head["config"]}
    for k, v in head.items():
        if k not in ("workload", "value", "ms_per_step", "config"):
            out[k] = v
    if not args.config:
        out["configs"] = [{"workload": r["workload"], "T": r["config"]["T"], "ms_per_step": r["ms_per_step"],
                           "tokens_per_s": r["value"], "step_us_median": r["step_us_median"],
                           "weight_copies_rotated": r["config"]["weight_copies_rotated"],
                           "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac", "kernel_ms", "over")}}
                          for r in (recs[c] for c in order)]
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
