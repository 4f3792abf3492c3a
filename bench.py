#!/usr/bin/env python3
"""Benchmark of the MoC attention hot path on ONE MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload eight|single|tiny] [--window frame|shot]

A step is one pass of the hot path over one synthetic batch resident in HBM:
moc_route (mean pooling, scores, top-k) -> moc_attn_fwd -> moc_attn_bwd.
moc_chunk_meta depends on the layout only and is built once per layout; its
time is reported separately (meta_ms).

Prints ONE JSON line. `value` = algorithmic routed-attention FLOPs, forward +
backward (3.5 x 4 d sum_i |Omega(i)| per head, attended pairs only), divided by
the whole step time. `roofline` describes the kernel with the largest share of
the step, timed with HIP events on the launch stream during the timed steps.
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# vector instructions per matrix instruction in the score + top-k pass, from the counter run recorded in
# profiles/moc_kernels_eight_shot_frame_window_counters.txt (SQ_INSTS_VALU / SQ_INSTS_MFMA)
ROUTE_VALU_PER_MFMA = 22.0


def layout_counts(lay, sel, chunk_of_t, topk, causal=True):
    """Attended (query, key) pairs per head-sum, split into forced and routed, and
    the number of routing candidates - all from the layout and the selection."""
    import torch
    off = lay.offsets.astype(np.int64)
    C = lay.C
    lens = np.diff(off)
    is_text = np.zeros(C, bool)
    for s, e in lay.text_spans.reshape(-1, 2):
        is_text |= (off[:-1] >= s) & (off[1:] <= e)
    win = lay.window.astype(np.int64)
    text_total = int(lens[is_text].sum())
    # forced keys of a window: all text + the window's non-text tokens
    wids, winv = np.unique(win, return_inverse=True)
    win_nontext = np.bincount(winv, weights=lens * (~is_text), minlength=len(wids))
    forced_per_chunk = text_total + win_nontext[winv]            # per chunk of the query
    forced_pairs = float((forced_per_chunk * lens).sum())         # per head
    dev = sel.device
    lens_t = torch.from_numpy(lens).to(dev)
    routed_pairs = float((lens_t[sel.clamp(min=0).long()] * (sel >= 0)).sum().item())   # all heads
    # candidates: earlier chunks that are neither text nor in the own window
    nontext_before = np.concatenate([[0], np.cumsum(~is_text)])[:-1]
    first_of_win = np.zeros(len(wids), np.int64)
    for w in range(len(wids)):
        first_of_win[w] = np.nonzero(winv == w)[0][0]
    own_before = np.array([np.sum((~is_text)[first_of_win[winv[c]]:c]) for c in range(C)])
    elig_per_chunk = nontext_before - own_before
    if not causal:           # every non-text chunk outside the own window
        win_nt_chunks = np.bincount(winv, weights=(~is_text).astype(np.float64), minlength=len(wids))
        elig_per_chunk = (~is_text).sum() - win_nt_chunks[winv]
    eligible = float((elig_per_chunk * lens).sum())               # per head
    return forced_pairs, routed_pairs, eligible


def cpu_baseline(lay, cfg, q, k, v, d_o, topk, budget_queries, causal=True):
    """Oracle on one head: the queries that attend eight sampled video chunks plus
    random queries up to `budget_queries`: forward + dQ for those queries, dK/dV
    for the sampled chunks. Algorithmic FLOPs as for the GPU path."""
    from oracle import moc_oracle as mo
    L = mo.OracleLayout.from_layout(lay)
    N, d = lay.N, cfg["d"]
    f64 = lambda t: t[0:1, 0:1].float().cpu().numpy().astype(np.float64)
    qn, kn, vn, don = f64(q), f64(k), f64(v), f64(d_o)
    rng = np.random.default_rng(0)
    t0 = time.perf_counter()
    kbar = mo.pool(L, kn)
    sel_all, _ = mo.route(L, qn, kbar, topk, causal)
    t_route = time.perf_counter() - t0
    video = np.nonzero(L.kind == 0)[0]
    chunks = np.sort(rng.choice(video[len(video) // 4:], size=min(8, len(video)), replace=False)).astype(np.int32)
    att = np.zeros(N, bool)
    for j in chunks:
        att |= (L.win[L.chunk_of] == L.win[j]) | (sel_all[0, 0] == j).any(-1)
    extra = rng.choice(N, size=min(N, budget_queries), replace=False)
    att[extra[: max(0, budget_queries - int(att.sum()))]] = True
    qidx = np.nonzero(att)[0].astype(np.int32)
    sel_s = sel_all[:, :, qidx]
    t0 = time.perf_counter()
    o, lse, pairs_q = mo.attn_fwd(L, qn, kn, vn, sel_s, None, qidx)
    dq = mo.attn_bwd_dq(L, qn, kn, vn, sel_s, o, lse, don[:, :, qidx], None, qidx)
    o_full = np.zeros((1, 1, N, d)); o_full[0, 0, qidx] = o[0, 0]
    lse_full = np.zeros((1, 1, N)); lse_full[0, 0, qidx] = lse[0, 0]
    mo.attn_bwd_dkdv(L, qn, kn, vn, sel_all, o_full, lse_full, don, None, chunks)
    dt = time.perf_counter() - t0
    pairs_k = 0
    for j in chunks:
        n_att = int(((L.win[L.chunk_of] == L.win[j]) | (sel_all[0, 0] == j).any(-1)).sum())
        pairs_k += n_att * int(L.off[j + 1] - L.off[j])
    flops = 2.0 * d * (3 * pairs_q + 4 * pairs_k)
    return dict(value=flops / dt / 1e12, unit="TFLOP/s", cores=int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
                kind="oracle",
                sample=f"head 0 of the workload: fwd + dQ for {len(qidx)} queries, dK/dV for video chunks "
                       f"{chunks.tolist()} ({pairs_q} + {pairs_k} attended pairs, {dt:.1f} s; "
                       f"pool + route of all {N} queries took another {t_route:.1f} s, not counted)")


def bench_outer(args, lay, cfg, q, k, v, d_o, mi, mb, torch):
    """Outer-loop routing of the last shot against the earlier ones (captions mandatory), then the gather."""
    B, H, d, N = cfg["B"], cfg["H"], cfg["d"], lay.N
    seg, cap = mb.outer_segments(lay.offsets, lay.shot, lay.text_spans)
    g, M = len(seg) - 2, args.outer
    x = k[0].permute(1, 0, 2).reshape(N, H * d).contiguous()       # token features [N, H d]
    D = x.shape[1]

    def step():
        _, _, sel, kept = mb.outer_route(x, seg, cap, g, M, True)
        ranges = [(int(seg[j]), int(seg[j + 1] - seg[j])) for j in kept]
        return [mb.gather_rows(t, ranges) for t in (q, k, v, d_o)], kept

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    mb.prof_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        red, kept = step()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) * 1e3 / args.steps
    kern = {n: ms / max(c, 1) for n, (c, ms) in mb.prof_read().items()}
    mb.prof_enable(False)
    esz = x.element_size()
    n_red = red[0].shape[2]
    pool_bytes = N * D * esz + (N / 64 + len(seg)) * D * 4.0
    gather_bytes = 2.0 * B * H * n_red * d * esz                     # per tensor: read + write
    kernels = {"outer_partial": dict(ms=round(kern["outer_partial"], 4),
                                     gbs=round(pool_bytes / kern["outer_partial"] / 1e6, 1)),
               "outer_mean_score_select": dict(ms=round(kern["outer_mean_score_select"], 4)),
               "gather_rows": dict(ms=round(kern["gather_rows"], 4), gbs=round(gather_bytes / kern["gather_rows"] / 1e6, 1))}
    ach = kernels["outer_partial"]["gbs"]
    total_bytes = pool_bytes + 4 * gather_bytes
    print(json.dumps({
        "metric": "outer_route_and_gather_GBs", "value": round(total_bytes / ms_step / 1e6, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32 sums of bf16",
        "data": "synthetic",
        "config": {"workload": f"{args.workload} ({lay.name}): N={N} D={D} segments={len(seg) - 1} "
                               f"(captions mandatory) M={M} g={g}; reduced stream {n_red} tokens x 4 tensors"},
        "kernels": kernels,
        "roofline": dict(kernel="outer_partial", bound="hbm", achieved=ach, peak=PEAK_HBM_GBS, unit="GB/s",
                         frac=round(ach / PEAK_HBM_GBS, 4), traffic=None, avg_ms=kernels["outer_partial"]["ms"]),
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="eight", choices=["eight", "single", "tiny", "sweep", "short", "paper", "long"])
    ap.add_argument("--window", default=None, choices=[None, "frame", "shot", "chunk"])
    ap.add_argument("--chunk", type=int, default=None)
    ap.add_argument("--topk", type=int, default=None)
    ap.add_argument("--cpu-queries", type=int, default=1 << 30, help="oracle sample size, capped at N (0 = skip the CPU baseline)")
    ap.add_argument("--seed", type=int, default=1234)
    ap.add_argument("--perturb", default=None, metavar="P_MAX,LAMBDA,MAX_IN",
                    help="route with context drop-off / drop-in (training-time regularisers); rows widen by MAX_IN")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time its replays (launch gaps removed)")
    ap.add_argument("--outer", type=int, default=None, metavar="M",
                    help="time the outer-loop routing instead: segment means + top-M shots over [N, H d] features, "
                         "then the gather of q, k, v, dO into the reduced stream")
    ap.add_argument("--fused-route", action="store_true",
                    help="route with moc_route_fused (pooling, scoring and top-k in one launch) instead of moc_route")
    ap.add_argument("--no-secondary", dest="secondary", action="store_false",
                    help="skip the secondary rows (shot window, S2 inputs) that the default run of the benchmark workload adds")
    ap.add_argument("--inputs", default="S1", choices=["S1", "S2"],
                    help="S1: q, k, v, dO iid N(0,1) (graded); S2: chunk-coherent q and k (queries of a chunk select nearly the same chunks)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (heads are independent: shard heads across GPUs with no "
              "collective inside the layer); --gpus must be 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    import moc_inputs as mi
    from paper_2508_21058_amd import binding as mb

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    cfg = dict(mi.CONFIGS[args.workload])
    if args.topk is not None:
        cfg["topk"] = args.topk
    lay = mi.config_layout(args.workload, window=args.window, chunk=args.chunk)
    B, H, d, topk, N = cfg["B"], cfg["H"], cfg["d"], cfg["topk"], lay.N
    causal = bool(cfg.get("causal", True))
    tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
    q, k, v, d_o = (t.to(tdt).contiguous() for t in mi.qkv_do(B, H, N, d, args.seed, "cuda"))
    if args.inputs == "S2":
        del q, k
        qc, kc = mi.coherent_qk(lay, B, H, d, args.seed)
        q, k = qc.to(tdt).to("cuda").contiguous(), kc.to(tdt).to("cuda").contiguous()
        del qc, kc

    if args.outer is not None:
        return bench_outer(args, lay, cfg, q, k, v, d_o, mi, mb, torch)

    perturb = None
    if args.perturb:
        p_max, lam, max_in = args.perturb.split(",")
        perturb = (float(p_max), float(lam), int(max_in))
    tensors = (q, k, v, d_o)
    out = measure(args, lay, cfg, tensors, args.steps, args.warmup, perturb, args.graph, True, mi, mb, torch)

    # secondary rows of the same build, each a whole step on its own workload, fewer steps, no CPU leg:
    # the benchmark layout with the whole shot as the local window (the paper's multi-shot forced link), and the
    # primary workload on chunk-coherent inputs (S2)
    if args.secondary and args.workload == "eight" and not args.perturb and args.inputs == "S1":
        sec = {}
        lay2 = mi.config_layout("eight", window="shot" if lay.meta.get("window") != "shot" else "frame", chunk=args.chunk)
        r = measure(args, lay2, cfg, tensors, 4, 2, None, False, False, mi, mb, torch)
        sec[f"window_{lay2.meta.get('window')}"] = secondary_row(r)
        qc, kc = mi.coherent_qk(lay, B, H, d, args.seed, device="cuda")
        r = measure(args, lay, cfg, (qc.to(tdt).contiguous(), kc.to(tdt).contiguous(), v, d_o), 4, 2, None, False, False,
                    mi, mb, torch, inputs="S2")
        del qc, kc
        sec["inputs_S2_chunk_coherent"] = secondary_row(r)
        out["secondary"] = sec
    if args.cpu_queries > 0:
        out["cpu_baseline"] = cpu_baseline(lay, cfg, q, k, v, d_o, topk, args.cpu_queries, causal)
    print(json.dumps(out))


def secondary_row(r):
    return {"workload": r["config"]["workload"], "inputs": r["config"]["inputs"], "ms_per_step": r["ms_per_step"],
            "tflops": r["value"], "frac_of_bf16_mfma_peak": r["frac_of_bf16_mfma_peak"],
            "keys_per_query": r["keys_per_query"], "sparsity": r["sparsity"],
            "kernels_ms": {n: row["ms"] for n, row in r["kernels"].items()}}


def read_traffic(workload, window):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE + WRITE_SIZE, each scaled by what the
    counter reads for a copy of known size); the figures live in profiles/, written from a run of this script."""
    tfile = os.path.join(ROOT, "profiles", "moc_kernels_eight_shot_frame_window.txt")
    out = {}
    if os.path.exists(tfile):
        key = f"traffic {workload}:{window}:"
        for line in open(tfile):
            if line.startswith(key):
                name, val = line[len(key):].split("=")
                out[name.strip()] = float(val)
    return out, "profiles/" + os.path.basename(tfile)


def measure(args, lay, cfg, tensors, steps, warmup, perturb, use_graph, with_probes, mi, mb, torch, inputs=None):
    """Times `steps` whole steps (route -> forward -> backward) on one layout and returns the bench line."""
    q, k, v, d_o = tensors
    B, H, d, topk, N = cfg["B"], cfg["H"], cfg["d"], cfg["topk"], lay.N
    if args.topk is not None:
        topk = args.topk
    causal = bool(cfg.get("causal", True))
    tdt = q.dtype
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    meta = mb.chunk_meta(lay.offsets, lay.shot, lay.window, lay.text_spans)
    torch.cuda.synchronize()
    meta_ms = (time.perf_counter() - t0) * 1e3

    width = topk + (perturb[2] if perturb else 0)
    ws = mb.attn_workspace(meta, B, H, d, width, tdt, True)
    o = torch.empty_like(q); lse = torch.empty(B, H, N, dtype=torch.float32, device="cuda")
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)

    def step(ev=None):
        if ev: ev[0].record()
        if perturb:
            pooled, sel = mb.route_perturbed(meta, q, k, topk, causal, *perturb, args.seed)
        elif args.fused_route:
            pooled, sel = mb.route_fused(meta, q, k, topk, causal)
        else:
            pooled, sel = mb.route(meta, q, k, topk, causal)
        if ev: ev[1].record()
        mb.attn_fwd(meta, q, k, v, sel, None, ws, (o, lse))
        if ev: ev[2].record()
        # the backward of a training step follows its forward: the lists built there are used again
        mb.attn_bwd(meta, q, k, v, o, lse, d_o, sel, None, ws, (dq, dk, dv), after_fwd=True)
        if ev: ev[3].record()
        return sel

    for _ in range(warmup):
        sel = step()
    torch.cuda.synchronize()
    graph_ms = None
    if use_graph:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for s in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_ms = (time.perf_counter() - t0) * 1e3 / steps
    evs = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
    mb.prof_enable(True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(steps):
        sel = step(evs[s])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern = mb.prof_read()
    mb.prof_enable(False)
    ms_step = wall * 1e3 / steps
    stage_all = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(3)] for e in evs])
    stage = stage_all.mean(0)

    forced_pairs, routed_pairs, eligible = layout_counts(lay, sel, None, topk, causal)
    BH = B * H
    pairs_f, pairs_r = forced_pairs * BH, routed_pairs
    pairs = pairs_f + pairs_r
    fwd_flops = 4.0 * d * pairs
    total_flops = 3.5 * fwd_flops
    esz = 2 if tdt == torch.bfloat16 else 4
    row = N * d * esz * BH                    # one [B, H, N, d] tensor
    # algorithmic work per kernel launch: (kind, amount, algorithmic HBM bytes)
    alg = {
        "attn_fwd_forced": ("flop", 4.0 * d * pairs_f, None), "attn_fwd_routed": ("flop", 4.0 * d * pairs_r, None),
        "attn_fwd": ("flop", 4.0 * d * pairs, 4.0 * row),                        # q, k, v in; o out
        "attn_bwd_dkdv": ("flop", 8.0 * d * pairs, 6.0 * row),                   # q, k, v, dO in; dk, dv out
        "attn_bwd_dq_forced": ("flop", 2.0 * d * pairs_f, None), "attn_bwd_dq_routed": ("flop", 2.0 * d * pairs_r, None),
        "attn_bwd_dq": ("flop", 2.0 * d * pairs, 5.0 * row),                     # q, k, v, dO in; dq out
        "pool": ("byte", BH * (N * d * esz + lay.C * d * 4.0), None),
        "route_topk": ("byte", BH * (N * d * esz + lay.C * d * 4.0 + N * topk * 4.0), None),
        "route_perturb": ("byte", BH * N * (topk + width) * 4.0, None),
        "route_fused": ("byte", BH * (2 * N * d * esz + lay.C * d * 4.0 + N * topk * 4.0), None),
    }
    traffic, tsrc = read_traffic(args.workload, lay.meta.get("window"))
    kernels = {}
    for name, (cnt, ms) in kern.items():
        per = ms / max(cnt, 1)
        krow = dict(ms=round(per, 4))
        if name in alg:
            kind, amt, _ = alg[name]
            if kind == "flop":
                krow["tflops"] = round(amt / (per * 1e-3) / 1e12, 2)
            else:
                krow["gbs"] = round(amt / (per * 1e-3) / 1e9, 1)
        kernels[name] = krow
    # measured HBM bytes against algorithmic bytes, per pass (the routed and forced kernels of a pass share its tensors)
    traffic_ratio = {}
    for pas, parts in (("attn_fwd", ("attn_fwd_routed", "attn_fwd_forced")), ("attn_bwd_dkdv", ("attn_bwd_dkdv",)),
                       ("attn_bwd_dq", ("attn_bwd_dq_routed", "attn_bwd_dq_forced"))):
        if all(p_ in traffic for p_ in parts):
            meas = sum(traffic[p_] for p_ in parts)
            traffic_ratio[pas] = {"measured_GB": round(meas, 2), "algorithmic_GB": round(alg[pas][2] / 1e9, 2),
                                  "ratio": round(meas * 1e9 / alg[pas][2], 2)}
    dom = max((n for n in kernels if n in alg), key=lambda n: kernels[n]["ms"])
    if alg[dom][0] == "flop":
        ach = alg[dom][1] / (kernels[dom]["ms"] * 1e-3) / 1e12
        roof = dict(kernel=dom, bound="mfma", achieved=round(ach, 2), peak=PEAK_BF16_TFLOPS, unit="TFLOP/s",
                    frac=round(ach / PEAK_BF16_TFLOPS, 4), traffic=None, avg_ms=kernels[dom]["ms"])
    else:
        ach = alg[dom][1] / (kernels[dom]["ms"] * 1e-3) / 1e9
        roof = dict(kernel=dom, bound="hbm", achieved=round(ach, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                    frac=round(ach / PEAK_HBM_GBS, 4), traffic=None, avg_ms=kernels[dom]["ms"])
    if dom in traffic:
        # HBM bytes per launch of the dominant kernel (FETCH_SIZE + WRITE_SIZE counter runs, scaled; see the source file)
        roof["traffic"] = round(traffic[dom] * 1e9)
        roof["traffic_unit"] = "bytes per launch"
        roof["traffic_source"] = tsrc

    measured = None
    if with_probes:
        # what this GPU sustains on a plain streaming copy and on a bare MFMA loop (context for the fractions above)
        pbuf = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        c_ms, c_bytes = mb.probe("copy", pbuf, 20)
        m_ms, m_flops = mb.probe("mfma", pbuf, 100000)
        # matrix and vector work of different waves on one SIMD: alone and together (do they overlap?)
        it = 20000
        mix = {kind: mb.probe(kind, pbuf, it)[0] for kind in ("mfma4", "valu4", "mfma4+valu4", "mfma4+valu_same_wave")}
        # data paths inside a compute unit (bytes per clock and CU at the nominal 2.4 GHz): LDS operand reads, and
        # the global -> LDS tile copies from cache-resident data, asynchronous (as the kernels do) or via registers
        cu = {}
        for kind in ("lds_read", "lds_read_transposed", "copy_to_lds_async", "copy_via_registers"):
            p_ms, p_bytes = mb.probe(kind, pbuf, 2000)
            cu[kind + "_B_per_clk_cu"] = round(p_bytes / 256 / (p_ms * 1e-3 * 2.4e9), 1)
        del pbuf
        measured = {"hbm_copy_GBs": round(c_bytes / (c_ms * 1e-3) / 1e9, 1),
                    "bf16_mfma_TFLOPs": round(m_flops / (m_ms * 1e-3) / 1e12, 1),
                    "mfma_valu_coissue": {"mfma_waves_alone_ms": round(mix["mfma4"], 3),
                                          "valu_waves_alone_ms": round(mix["valu4"], 3),
                                          "both_ms": round(mix["mfma4+valu4"], 3),
                                          "both_in_one_wave_ms": round(mix["mfma4+valu_same_wave"], 3),
                                          "both_over_sum": round(mix["mfma4+valu4"] / (mix["mfma4"] + mix["valu4"]), 3)},
                    "cu_data_paths": cu}
        roof["frac_of_measured"] = round(roof["achieved"] / (measured["bf16_mfma_TFLOPs"] if roof["bound"] == "mfma"
                                                             else measured["hbm_copy_GBs"]), 4)

    # routing: bytes as asked, and the score contraction's rate on the unit it runs on (three bf16 matrix
    # products per fp32-accurate score). Which resource bounds the pass is read off the measured rates.
    routing = {}
    if "pool" in kernels:
        routing["pool_GBs"] = kernels["pool"]["gbs"]
        routing["pool_frac_of_hbm_peak"] = round(kernels["pool"]["gbs"] / PEAK_HBM_GBS, 4)
    if "route_topk" in kernels:
        r_ms = kernels["route_topk"]["ms"]
        routing["score_topk_GBs"] = kernels["route_topk"]["gbs"]
        routing["score_topk_frac_of_hbm_peak"] = round(kernels["route_topk"]["gbs"] / PEAK_HBM_GBS, 4)
        routing["score_TFLOPs_algorithmic"] = round(2.0 * d * eligible * BH / (r_ms * 1e-3) / 1e12, 2)
        # executed on the matrix cores: whole 32-chunk tiles up to the causal limit, three bf16 planes per score
        tiles = float(np.ceil(np.repeat(np.arange(lay.C), np.diff(lay.offsets)) / 32.0).sum()) if causal else \
            float(N) * np.ceil(lay.C / 32.0)
        exec_flops = 3.0 * 2.0 * d * 32.0 * tiles * BH
        routing["score_TFLOPs_executed_bf16"] = round(exec_flops / (r_ms * 1e-3) / 1e12, 1)
        routing["score_frac_of_bf16_mfma_peak"] = round(exec_flops / (r_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
        routing["candidates_per_query"] = round(eligible / N, 1)
        routing["valu_per_mfma_instruction"] = ROUTE_VALU_PER_MFMA
        hb, mf = routing["score_topk_frac_of_hbm_peak"], routing["score_frac_of_bf16_mfma_peak"]
        routing["bound"] = ("selection (vector instructions): neither HBM nor the matrix cores are near their peak"
                            if max(hb, mf) < 0.4 else ("hbm" if hb >= mf else "mfma"))
    # the same step priced as a dense causal attention of the same length (2 N^2 d per head forward, x3.5)
    dense_flops = 3.5 * 2.0 * float(N) * N * d * BH
    dense = {"flops": dense_flops, "equivalent_TFLOPs": round(dense_flops / (ms_step * 1e-3) / 1e12, 1),
             "flop_ratio_dense_over_routed": round(dense_flops / total_flops, 2)}

    out = {
        "metric": "routed_attn_tflops_fwd_bwd", "value": round(total_flops / (ms_step * 1e-3) / 1e12, 2),
        "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": round(ms_step, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if tdt == torch.bfloat16 else "f32(bf16 mfma)", "data": "synthetic",
        "config": {"workload": f"{args.workload} ({lay.name}): B={B} H={H} N={N} d={d} C={lay.C} "
                               f"chunk={lay.meta.get('chunk')} window={lay.meta.get('window')} topk={topk} {'causal' if causal else 'non-causal'}",
                   "inputs": ("S1 iid N(0,1) rounded to bf16, seeded" if (inputs or args.inputs) == "S1" else
                              "S2 chunk-coherent q and k (rho = 0.9, planted earlier target chunk), v and dO iid, seeded"),
                   "pass": "route + attn fwd + attn bwd",
                   **({"perturb": f"drop-off p_max={perturb[0]} drop-in lambda={perturb[1]} max_in={perturb[2]}"}
                      if perturb else {})},
        "frac_of_bf16_mfma_peak": round(total_flops / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "attn_only_tflops": round(total_flops / ((stage[1] + stage[2]) * 1e-3) / 1e12, 2),
        "stage_ms": {"route": round(float(stage[0]), 3), "attn_fwd": round(float(stage[1]), 3),
                     "attn_bwd": round(float(stage[2]), 3), "chunk_meta_once": round(meta_ms, 3)},
        "stage_ms_median": [round(float(x), 3) for x in np.median(stage_all, 0)],
        "stage_ms_min": [round(float(x), 3) for x in stage_all.min(0)],
        "routing": routing, "dense_equivalent": dense,
        "keys_per_query": round(pairs / (BH * N), 1), "sparsity": round(1 - pairs / (BH * float(N) * N), 4),
        "kernels": kernels, "traffic_ratio": traffic_ratio, "roofline": roof,
    }
    if measured:
        out["measured_peaks"] = measured
    if graph_ms is not None:
        out["graph_replay"] = {"ms_per_step": round(graph_ms, 3),
                               "tflops": round(total_flops / (graph_ms * 1e-3) / 1e12, 2)}
    meta.close()
    del ws, o, lse, dq, dk, dv
    return out


if __name__ == "__main__":
    main()
