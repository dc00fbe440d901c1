#!/usr/bin/env python3
"""Benchmark of the DraftAttention hot path on one MI355X.

A step is one da_forward over one batch of synthetic Q, K, V (pool -> draft logits ->
top-k -> reorder -> block-sparse attention -> restore), inputs resident in HBM.  The
workload is the headline configuration: 118 800 tokens (33 latent frames of 45x80), 24
heads of 128, 8x8 pooling, 90 % sparsity, bf16.  Prints ONE JSON line.

  value        effective TFLOP/s of the whole step: 4*N*N*d*H*(k/g) / step time
  ms_per_step  milliseconds per layer (the other half of the metric): the K timed steps / K;
               ms_per_step_median is the median of the same K steps (HIP events between them)
  roofline     the block-sparse attention kernel against the bf16 MFMA peak, three ways, all
               measured in this run with HIP events on the launch stream (medians over the steps):
                 frac           EFFECTIVE flop 4*N*N*d*H*(k/g) / launch time / peak, for the launch
                                da_forward makes (queries read, outputs written in the original
                                token order): the figure the build target names;
                 executed.frac  flop of the matrix instructions the kernel actually issued (it counts
                                its tiles: da_sparse_attn_ex) / the same time / peak.  Padding adds
                                work, the kernel's drop rule takes work away; on these peaked
                                synthetic inputs it takes away a lot;
                 no_drop.frac   the same launch, same block lists, with Q scaled by 2^-5 so that the
                                scores of a row lie close together and nothing is dropped: what the
                                kernel does on inputs whose attention is not peaked.
               The other stages are timed in a loop that issues the C-ABI calls one by one
               (da_forward fuses some of them: it reorders K inside the pooling pass and makes
               no reordered copies of Q and O, so ms_per_step is smaller than their sum)
  cpu_baseline the NumPy float64 oracle timed on this host on a bounded sample
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2505_14708_amd import workloads as W  # noqa: E402

METRIC = "sparse-attn ms/layer + effective MFMA TFLOP/s @118.8k tokens, 90% sparsity"
PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA, published
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E, published
# HBM-side bytes per launch of the attention kernel (read, written): NOT measured in this run (counters need
# rocprofv3) but copied from a counter run of this program: FETCH_SIZE and WRITE_SIZE, scaled by what the same
# counters read for the row-copy kernel of known size in the same run.  The file named holds the figures and the
# command; it is regenerated whenever the kernel changes.  Workloads without a counter run: null.
ATTN_TRAFFIC = {"720p_hunyuan": {"read": 56.38e9, "written": 0.744e9, "no_drop_read": 110.27e9, "no_drop_written": 0.731e9,
                                 "source": "profiles/pmc_attn_720p_hunyuan.txt"}}
FLOP_PER_MFMA = 2.0 * 32 * 32 * 16     # v_mfma_f32_32x32x16_bf16


def cpu_baseline(w, Q, K, V, budget_s=20.0, whole_map=False):
    """Time the oracle (as it stands) on head 0: pooling, draft logits, selection and the
    reordering in full, the attention on as many evenly spaced query blocks as fit the
    budget; extrapolate to one layer."""
    from oracle import draft_attention as oa
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    q, k, v = Q[0, 0], K[0, 0], V[0, 0]
    t0 = time.perf_counter()
    dims = oa.derive_dims(w.T, w.fh, w.fw, w.ph, w.pw, w.sparsity)
    perm, valid = oa.reorder_index(w.T, w.fh, w.fw, w.ph, w.pw)
    inv = oa.restore_index(perm, dims["n"])
    qp = oa.pool_canonical_f32(oa.widen_f32(q, w.dtype), perm, valid, dims["block"])
    kp = oa.pool_canonical_f32(oa.widen_f32(k, w.dtype), perm, valid, dims["block"])
    L = oa.draft_logits_canonical_f32(qp, kp)
    if whole_map:
        idx = oa.lists_of(*oa.select_blocks_global(L, oa.global_budget(dims["g"], w.sparsity))[:2])
    else:
        idx, _ = oa.select_blocks(L, dims["k"])
    Qp, Kp, Vp = (oa.permute(oa.widen_f64(x, w.dtype), perm) for x in (q, k, v))
    t_fixed = time.perf_counter() - t0
    g = dims["g"]
    done, t_attn = 0, 0.0
    Op = None
    order = np.argsort((np.arange(g) * 0.6180339887498949) % 1.0, kind="stable")   # every prefix is spread evenly over the blocks
    while done < len(order) and t_attn < max(2.0, budget_s - t_fixed):
        rows = order[done:done + 8]
        t1 = time.perf_counter()
        Op = oa.sparse_attention_blocks(Qp, Kp, Vp, idx, valid, dims["block"], rows=rows)
        t_attn += time.perf_counter() - t1
        done += len(rows)
    t1 = time.perf_counter()
    oa.restore(Op, inv)
    t_fixed += time.perf_counter() - t1
    per_head = t_fixed + t_attn * g / done
    layer_s = per_head * w.B * w.H
    eff_flop = 4.0 * w.N * w.N * w.d * w.B * w.H * dims["k"] / g
    return {"value": eff_flop / layer_s / 1e12, "unit": "TFLOP/s effective", "cores": int(threads),
            "kind": "oracle", "ms_per_layer_extrapolated": layer_s * 1e3,
            "sample": (f"head 0 of {w.H}: pool+draft+top-k+reorder+restore in full ({t_fixed:.1f} s), attention on "
                       f"{done} of {g} query blocks ({t_attn:.1f} s); extrapolated to {w.B * w.H} heads")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="720p_hunyuan", choices=list(W.CONFIGS) + list(W.EXTRA_CONFIGS))
    ap.add_argument("--selection", default="rows", choices=["rows", "whole_map"],
                    help="rows: k key blocks per query block (the headline); whole_map: the threshold over a head's "
                         "whole map (Section 3.2.2), lists of any length")
    ap.add_argument("--sparsity", type=float, default=None,
                    help="another sparsity for the chosen workload's shape (0: a dense layer, every block kept)")
    ap.add_argument("--heads", type=int, default=None, help="another number of heads for the chosen workload's shape")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probes", action="store_true", help="skip the machine's measuring sticks")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path is independent per head and would shard "
              "by heads with no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    w = W.CONFIGS[args.config] if args.config in W.CONFIGS else W.EXTRA_CONFIGS[args.config]
    if args.sparsity is not None or args.heads is not None:   # a variant of the workload: named so, not the headline
        s_new = w.sparsity if args.sparsity is None else args.sparsity
        h_new = w.H if args.heads is None else args.heads
        w = w.with_(name=f"{w.name}_H{h_new}_s{s_new:g}", sparsity=s_new, H=h_new)
    t0 = time.time()
    Q, K, V = W.make_qkv(w, threads=8)
    print(f"[bench] inputs for {w.name} generated in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    import torch
    from paper_2505_14708_amd import binding as da
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    bf16 = w.dtype == W.BF16
    tdt = torch.bfloat16 if bf16 else torch.float32

    def dev(x):
        if not bf16:
            return torch.from_numpy(x).cuda()
        return torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)

    def timed(fn, reps):
        """Durations in ms of `reps` calls of fn, one HIP event pair each, on the launch stream."""
        out = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            out.append(a.elapsed_time(b))
        return out

    p = da.problem_of(w)
    dims = da.da_derive(p)
    dQ, dK, dV = dev(Q), dev(K), dev(V)
    O = torch.empty((w.B, w.H, dims.n, w.d), dtype=tdt, device="cuda")
    whole_map = args.selection == "whole_map"
    gsz = da.da_global_sizes(p) if whole_map else None
    ws = torch.empty(gsz.forward_ws if whole_map else da.da_workspace_size(p), dtype=torch.uint8, device="cuda")
    g, k = dims.g, dims.k
    # kept fraction of the map: k/g per row, or the budget of the whole map over g^2 (rows the threshold
    # leaves empty keep one block more each; not counted)
    density = gsz.budget / (g * g) if whole_map else k / g
    eff_flop = 4.0 * w.N * w.N * w.d * w.B * w.H * density

    def step():
        if whole_map:
            da.da_forward_global(p, dQ, dK, dV, O, ws)
        else:
            da.da_forward(p, dQ, dK, dV, O, ws)

    # ---- the timed region: K steps of the whole path, events between the steps for the median
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record()
    for i in range(args.steps):
        step()
        marks[i + 1].record()
    torch.cuda.synchronize()
    ms_step = marks[0].elapsed_time(marks[-1]) / args.steps
    ms_step_median = float(np.median([marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps)]))

    # ---- the same launches stage by stage, HIP events (torch's current stream is the launch stream)
    Qp = torch.empty((w.B, w.H, dims.n_pad, w.d), dtype=tdt, device="cuda")
    Kp, Op = torch.empty_like(Qp), torch.empty_like(Qp)
    Vt = torch.empty((w.B, w.H, g, w.d, dims.block), dtype=tdt, device="cuda")
    q_pool = torch.empty((w.B, w.H, g, w.d), dtype=torch.float32, device="cuda")
    k_pool = torch.empty_like(q_pool)
    logits = torch.empty((w.B, w.H, g, g), dtype=torch.float32, device="cuda")
    idx = torch.empty((w.B, w.H, gsz.cap if whole_map else g * k), dtype=torch.int32, device="cuda")
    row_ptr = torch.empty((w.B, w.H, g + 1), dtype=torch.int32, device="cuda")
    sel_ws = torch.empty(gsz.select_ws if whole_map else 256, dtype=torch.uint8, device="cuda")
    if whole_map:
        select = lambda: da.da_select_blocks_global(p, logits, row_ptr, idx, sel_ws)
        attend = lambda: da.da_sparse_attn_lists(p, Qp, Kp, Vt, row_ptr, idx, gsz.cap, Op, None)
    else:
        select = lambda: da.da_select_blocks(p, logits, idx, None)
        attend = lambda: da.da_sparse_attn(p, Qp, Kp, Vt, idx, Op, None)
    stages = [
        ("pool+draft_logits", lambda: da.da_draft_map(p, dQ, dK, q_pool, k_pool, logits, None)),
        ("select", select),
        ("reorder_qkv", lambda: (da.da_permute(p, dQ, Qp, da.DA_REORDER_ROWS), da.da_permute(p, dK, Kp, da.DA_REORDER_ROWS),
                                 da.da_permute(p, dV, Vt, da.v_layout(p.dtype)))),
        ("sparse_attn_reordered_q", attend),
        ("restore", lambda: da.da_permute(p, Op, O, da.DA_RESTORE)),
    ]
    per = {name: [] for name, _ in stages}
    for it in range(args.warmup + args.steps):
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(len(stages) + 1)]
        evs[0].record()
        for i, (_, fn) in enumerate(stages):
            fn()
            evs[i + 1].record()
        torch.cuda.synchronize()
        if it >= args.warmup:
            for i, (name, _) in enumerate(stages):
                per[name].append(evs[i].elapsed_time(evs[i + 1]))
    stage_ms = {name: float(np.median(v)) for name, v in per.items()}
    esz = 2 if bf16 else 4
    reorder_bytes = 3.0 * (dims.n + dims.n_pad) * w.d * esz * w.B * w.H
    restore_bytes = 1.0 * (dims.n + dims.n_pad) * w.d * esz * w.B * w.H

    # ---- the attention launch da_forward makes (bf16, k per row: Q and O in the original token order), timed by
    # itself; the tiles it goes through and carries out; and the same launch with nothing dropped
    roof = {"kernel": "da::ring::attn_bf16_ring_kernel", "bound": "mfma", "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "flop_per_launch": eff_flop, "timing": f"median of {args.steps} launches, HIP events on the launch stream"}
    if bf16 and not whole_map:
        counts = torch.zeros(2, dtype=torch.int64, device="cuda")

        def tile_flop(q_in):
            counts.zero_()
            da.da_sparse_attn_ex(p, q_in, Kp, Vt, idx, O, None, 1, counts)
            torch.cuda.synchronize()
            seen, kept = (int(x) for x in counts.cpu().numpy())
            return seen, kept, 16.0 * (seen + kept) * FLOP_PER_MFMA

        direct = lambda: da.da_sparse_attn_ex(p, dQ, Kp, Vt, idx, O, None, 1, None)
        timed(direct, args.warmup)
        attn_ms = float(np.median(timed(direct, args.steps)))
        seen, kept, exe_flop = tile_flop(dQ)
        roof.update({"launch": "da_sparse_attn_ex, original_order=1: the launch da_forward makes",
                     "launch_ms": attn_ms, "achieved": eff_flop / (attn_ms * 1e-3) / 1e12,
                     "frac": eff_flop / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                     "executed": {"tiles": seen, "tiles_carried_out": kept, "flop_per_launch": exe_flop,
                                  "achieved": exe_flop / (attn_ms * 1e-3) / 1e12,
                                  "frac": exe_flop / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}})
        dQs = dQ * (2.0 ** -5)                         # exact in bf16
        flat = lambda: da.da_sparse_attn_ex(p, dQs, Kp, Vt, idx, O, None, 1, None)
        timed(flat, 1)
        flat_ms = float(np.median(timed(flat, max(5, args.steps // 2))))
        seen2, kept2, exe2 = tile_flop(dQs)
        roof["no_drop"] = {"what": "same launch and block lists, Q scaled by 2^-5: every tile is carried out",
                           "launch_ms": flat_ms, "tiles": seen2, "tiles_carried_out": kept2,
                           "achieved": eff_flop / (flat_ms * 1e-3) / 1e12,
                           "frac": eff_flop / (flat_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                           "executed_frac": exe2 / (flat_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}
        del dQs
    else:
        attn_ms = stage_ms["sparse_attn_reordered_q"]
        roof.update({"launch": "the attention stage of the staged loop", "launch_ms": attn_ms,
                     "achieved": eff_flop / (attn_ms * 1e-3) / 1e12,
                     "frac": eff_flop / (attn_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS})
    tr = ATTN_TRAFFIC.get(w.name) if not whole_map else None
    roof["traffic"] = tr["read"] + tr["written"] if tr else None
    roof["traffic_unit"] = "HBM-side bytes per launch (read + written)"
    roof["traffic_source"] = (tr["source"] + " (a counter run of this program; not measured in this run)") if tr else None
    roof["compulsory_bytes"] = 4.0 * dims.n_pad * w.d * esz * w.B * w.H
    if tr and "no_drop" in roof:
        roof["no_drop"]["traffic"] = tr["no_drop_read"] + tr["no_drop_written"]

    # ---- what this machine sustains: a pure matrix-instruction loop (~10 ms of it), a plain copy, a plain read
    hbm = {"reorder_qkv_GBs": reorder_bytes / (stage_ms["reorder_qkv"] * 1e-3) / 1e9,
           "restore_GBs": restore_bytes / (stage_ms["restore"] * 1e-3) / 1e9, "peak_GBs": PEAK_HBM_GBS}
    if not args.no_probes:
        from paper_2505_14708_amd import probe
        sink = torch.empty(1 << 20, dtype=torch.float32, device="cuda")
        probe.da_probe_mfma_bf16(2000, sink)               # warm-up
        torch.cuda.synchronize()
        flop = [0.0]
        ms = timed(lambda: flop.__setitem__(0, probe.da_probe_mfma_bf16(6000, sink)), 1)[0]
        roof["measured_mfma_loop"] = flop[0] / (ms * 1e-3) / 1e12
        roof["frac_of_measured"] = roof["achieved"] / roof["measured_mfma_loop"]
        csrc = dQ.view(torch.uint8).flatten()
        ksrc = dK.view(torch.uint8).flatten()
        cdst = torch.empty_like(csrc)
        copy = lambda: probe.da_probe_copy(csrc, cdst, csrc.numel())
        timed(copy, 1)
        hbm["measured_copy_GBs"] = 2.0 * csrc.numel() / (float(np.median(timed(copy, 5))) * 1e-3) / 1e9
        # a plain read of Q and K one after the other (more than the last-level cache holds)
        read = lambda: (probe.da_probe_read(csrc, csrc.numel(), sink), probe.da_probe_read(ksrc, ksrc.numel(), sink))
        timed(read, 1)
        hbm["measured_read_GBs"] = (csrc.numel() + ksrc.numel()) / (float(np.median(timed(read, 5))) * 1e-3) / 1e9
        del cdst, sink
    # the pooling pass by itself (Definition 3.2): Q and K read once, the pooled rows written
    # (four launches per event pair: a single launch of a quarter millisecond is too short for the pair's own cost)
    pool_only = lambda: [da.da_draft_map(p, dQ, dK, q_pool, k_pool, None, None) for _ in range(4)]
    timed(pool_only, 1)
    stage_ms["pool_only"] = float(np.median(timed(pool_only, max(5, args.steps // 2)))) / 4.0
    pool_bytes = 2.0 * dims.n * w.d * esz * w.B * w.H + 2.0 * g * w.d * 4 * w.B * w.H
    hbm["pool_GBs"] = pool_bytes / (stage_ms["pool_only"] * 1e-3) / 1e9

    out = {
        "metric": METRIC,
        "value": eff_flop / (ms_step * 1e-3) / 1e12,
        "unit": "TFLOP/s effective (whole step)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "ms_per_step_median": ms_step_median,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "H": w.H, "d": w.d, "T": w.T, "frame": [w.fh, w.fw], "N": w.N,
                   "pool": [w.ph, w.pw], "sparsity": w.sparsity, "g": g, "k": k, "n_pad": int(dims.n_pad),
                   "selection": args.selection},
        "roofline": roof,
        "stages_ms": stage_ms,
        "hbm_stages": hbm,
    }
    if whole_map:
        torch.cuda.synchronize()
        lens = (row_ptr[:, :, 1:] - row_ptr[:, :, :-1]).flatten().cpu().numpy()
        out["config"]["whole_map"] = {"budget_per_head": int(gsz.budget), "list_min": int(lens.min()),
                                      "list_mean": float(lens.mean()), "list_max": int(lens.max())}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, Q, K, V, whole_map=whole_map)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
