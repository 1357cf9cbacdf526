#!/usr/bin/env python3
"""Benchmark of the Fier decode hot path on one MI355X.

A "step" is one whole per-layer decode step of Alg. 1 with the append of Sec. 3.1 -- append one key/value
row, score every cached token from the 1-bit keys, select the top-B tokens per kv head, attend over the
selected rows -- issued as ONE call of ``fier_decode_step`` on one layer's cache.  Successive steps rotate
over R distinct layer caches (R x touched bytes >= 1 GB) so that the 256 MB Infinity Cache cannot hold the
working set; all inputs are resident in HBM before the timed region.

Prints ONE JSON line.  Byte model: 16 + 512/g bytes of packed keys and (s, z) per cached token and unit, 512 bytes
per selected token and unit (its K and V rows), 768 bytes per query head (q in, fp32 output out).
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

HBM_PEAK_GBPS = 8000.0

WORKLOADS = {
    # LLaMA-7B-shaped decode layer (the configuration the headline metric is quoted on)
    "config2": dict(batch=1, n_q_heads=32, n_kv_heads=32, L=32768, budget=3604, dtype=0, chan="ones",
                    n_planted=64, rotate=12, label="llama7b_mha32_ctx32768_budget3604_fp16_append1"),
    # Llama-3-8B-shaped GQA layer, batch 4, 128k context
    "config3": dict(batch=4, n_q_heads=32, n_kv_heads=8, L=131072, budget=4096, dtype=1, chan="lognormal",
                    n_planted=64, rotate=5, label="llama3_8b_gqa32x8_b4_ctx131072_budget4096_bf16_append1"),
    "config1": dict(batch=1, n_q_heads=8, n_kv_heads=8, L=4096, budget=512, dtype=0, chan="ones",
                    n_planted=16, rotate=4, label="small_mha8_ctx4096_budget512_fp16_append1"),
    # budget sweep at 64k context: --budget picks the point (256, 1024, 4096, 7209, 16384)
    "config4": dict(batch=1, n_q_heads=32, n_kv_heads=32, L=65536, budget=7209, dtype=0, chan="ones",
                    n_planted=64, rotate=16, label="mha32_ctx65536_fp16_append1"),
    # batched ragged serving step: 16 sequences, lengths U{8192..65536}, budget 11 % of each, 32 layers per step
    "config5": dict(batch=16, n_q_heads=32, n_kv_heads=8, L="ragged", L_lo=8192, L_hi=65536, budget="11%",
                    dtype=1, chan="lognormal", n_planted=64, rotate=1, layers=32,
                    label="llama3_8b_gqa32x8_b16_ragged8k-64k_budget11pct_bf16_32layers_append1"),
}


def shape_of(w, seed):
    """Per-sequence context lengths and budgets of a workload (ragged ones are drawn from the seed)."""
    batch = w["batch"]
    if w["L"] == "ragged":
        rng = np.random.default_rng(seed)
        lens = rng.integers(w["L_lo"], w["L_hi"] + 1, size=batch).astype(np.int64)
    else:
        lens = np.full(batch, w["L"], np.int64)
    if w["budget"] == "11%":
        buds = np.array([int(round(0.11 * int(l))) for l in lens], np.int64)
    else:
        buds = np.full(batch, w["budget"], np.int64)
    return lens, buds


def algorithmic_bytes(w, lens, buds):
    """Bytes the method has to move per layer step: packed keys + (s, z) metadata (16 + 512/g B per cached token
    and unit: 32 B at g = 32), the selected K and V rows (512 B per selected token and unit), query in and fp32
    output out."""
    hkv = w["n_kv_heads"]
    heads = w["batch"] * w["n_q_heads"]
    n_tok = lens + 1
    packed = int(hkv * n_tok.sum() * (16 + 512 // w.get("group_size", 32)))
    kv = int(hkv * np.minimum(buds, n_tok).sum() * 512)
    qo = heads * (256 + 512)
    return dict(packed=packed, selected_kv=kv, q_out=qo, total=packed + kv + qo)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=600)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--workload", default="config2", choices=sorted(WORKLOADS))
    ap.add_argument("--budget", type=int, default=None, help="token budget (config4's sweep point)")
    ap.add_argument("--group-size", type=int, default=32, choices=[32, 64, 128, 256],
                    help="tokens per quantization group (32 is the paper's default; 128 / 256 are its ablation)")
    ap.add_argument("--selector", default="fier", choices=["fier", "quest", "quant-page"],
                    help="what picks the tokens: fier = the fused 1-bit token-level step (default); quest = page min/max "
                         "scores (Eq. 1-3, pages of 16 tokens), top pages, their tokens; quant-page = the same with the "
                         "averaged 1-bit score per page as the page metric (Sec. 4.4 ablation).  The page selectors run "
                         "as separate calls: append, page score, fier_topk over pages, expansion, fier_sparse_attn")
    ap.add_argument("--dense-first", type=int, default=0,
                    help="run full attention on the first N layers of every step (the paper's deployment leaves the "
                         "first two layers dense); only the step time changes")
    ap.add_argument("--loop-steps", type=int, default=0,
                    help="instead of the default measurement: this many consecutive token steps (append, growing "
                         "context) over all the workload's layer caches in one call per token, eager and as one graph")
    ap.add_argument("--block-tokens", type=int, default=0,
                    help="hold the K / V rows in a block pool of this block size behind a shuffled block table "
                         "(a paged serving cache); 0 = contiguous rows")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--stage-steps", type=int, default=240, help="launches per stage for the per-stage timing")
    ap.add_argument("--other-workloads", default="config3,config4:256,config4:16384",
                    help="comma-separated workloads (name or name:budget) measured after the headline one and reported, "
                         "in short form, under other_workloads of the same JSON line ('' = none; 'all' adds config5)")
    ap.add_argument("--pmc-calibration", action="store_true",
                    help="also run a plain element-wise copy of 256 MiB (read 256 MiB, write 256 MiB) three times, "
                         "so that a rocprofv3 --pmc run holds a kernel of known traffic to scale the counters by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    res = measure(args, args.workload, args.budget, detail=True)
    if res is None:
        return
    plain = (args.selector == "fier" and args.dense_first == 0 and args.group_size == 32 and not args.block_tokens
             and args.workload == "config2" and args.budget is None)
    others = args.other_workloads
    if others == "all":
        others = "config3,config4:256,config4:16384,config5"
    if plain and others:
        import gc

        import torch
        res["other_workloads"] = {}
        for item in others.split(","):
            name, _, b = item.partition(":")
            gc.collect()
            torch.cuda.empty_cache()
            short = measure(args, name, int(b) if b else None, detail=False)
            res["other_workloads"][short.pop("label")] = short
    print(json.dumps(res), flush=True)


def measure(args, workload, budget_arg, detail):
    """Measure one workload.  detail=True: everything the headline line carries; False: the short form (step time,
    roofline fraction, kernel times, dense attention at the same shape, algorithmic bytes)."""
    import torch

    from paper_2508_08256_amd import binding as B
    from paper_2508_08256_amd import synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    B.lib()  # fail loudly if the HIP library is missing
    w = dict(WORKLOADS[workload])
    if budget_arg is not None:
        w["budget"] = budget_arg
        w["label"] += f"_budget{budget_arg}"
    elif workload == "config4":
        w["label"] += f"_budget{w['budget']}"
    w["group_size"] = args.group_size
    if args.group_size != 32:
        w["label"] += f"_g{args.group_size}"
    if args.block_tokens:
        w["label"] += f"_paged{args.block_tokens}"
    R, NL = w["rotate"], w.get("layers", 1)
    batch, Hq, Hkv, dtype = w["batch"], w["n_q_heads"], w["n_kv_heads"], w["dtype"]
    lens, buds = shape_of(w, 5000)
    L, budget = int(lens.max()), int(buds.max())   # the largest context and budget (all of them when not ragged)
    gran = max(64, args.group_size) if args.selector == "fier" else 1024
    gran = max(gran, args.block_tokens)
    max_ctx = -(-(L + 1 + max(0, args.loop_steps)) // gran) * gran
    cfg = B.make_config(batch, Hq, Hkv, max_ctx, dtype, group_size=args.group_size)
    units, n_rep = cfg.units, cfg.n_rep
    steps, warmup, ns = args.steps, args.warmup, args.stage_steps
    if not detail:
        steps, warmup, ns = min(steps, 240), min(warmup, 24), min(ns, 120)
    if NL > 1 and steps >= 240:
        steps, warmup, ns = 40, 4, 16   # a step is NL layers

    # ---- resident inputs: R sets of NL layer caches, quantized once (prefill), fresh q / k_new / v_new each ---
    t0 = time.time()
    caches, qs, kns, vns, hosts = [], [], [], [], None
    seq_lens = torch.as_tensor(lens.astype(np.int32), device="cuda")
    budgets = torch.as_tensor(buds.astype(np.int32), device="cuda")
    for r in range(R):
        cl, ql, kl, vl = [], [], [], []
        for layer in range(NL):
            d = synth.make_workload_device(f"{workload}_cache{r}_{layer}", 1000 * 2 + r * NL + layer, batch, Hq,
                                           Hkv, lens, buds, dtype, max_ctx=max_ctx, chan=w["chan"],
                                           n_planted=w["n_planted"])
            if r == 0 and layer == 0:
                hosts = {k: (v[:min(units, 32)].clone() if k in ("K", "V", "q", "k_new", "v_new") else v)
                         for k, v in d.items()}
            if args.block_tokens:
                bt, per_seq = args.block_tokens, max_ctx // args.block_tokens
                gen = torch.Generator(device="cpu").manual_seed(7 + r * NL + layer)
                table = torch.randperm(batch * per_seq, generator=gen).to(torch.int32).cuda()
                pools = []
                for name in ("K", "V"):
                    blocks = d[name].view(batch, Hkv, per_seq, bt, 128).permute(0, 2, 1, 3, 4).reshape(-1, Hkv, bt, 128).contiguous()
                    pool = torch.empty_like(blocks)
                    pool[table.long()] = blocks
                    pools.append(pool)
                    d[name] = None
                c = B.DeviceCache(cfg, pools[0], pools[1], seq_lens, table.view(batch, per_seq).contiguous())
            else:
                c = B.DeviceCache(cfg, d["K"], d["V"], seq_lens)
            B.quantize_keys(cfg, c)
            cl.append(c)
            ql.append(d["q"].reshape(batch, Hq, 128))
            kl.append(d["k_new"].reshape(units, 128))
            vl.append(d["v_new"].reshape(units, 128))
            del d
        caches.append(cl)
        qs.append(torch.stack(ql).contiguous())
        kns.append(torch.stack(kl).contiguous())
        vns.append(torch.stack(vl).contiguous())
    torch.cuda.synchronize()
    t_setup = time.time() - t0

    if args.loop_steps > 0:
        decode_loop(args, w, cfg, caches, qs, kns, vns, seq_lens, budgets, lens, buds, budget, t_setup)
        return None

    # the timed steps share ONE workspace (as a model's layers would); the per-kernel timing below needs every
    # layer cache to keep its own intermediate state, hence one workspace per layer cache there
    wss = [[B.make_workspace(cfg, budget) for _ in range(NL)] for _ in range(R)]
    ws_dense = B.make_workspace(cfg, max_ctx)
    out = torch.zeros((NL, batch, Hq, 128), dtype=torch.float32, device="cuda")
    out1 = torch.zeros((1, batch, Hq, 128), dtype=torch.float32, device="cuda")
    idx = torch.zeros((NL, units, budget), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((NL, units), dtype=torch.int32, device="cuda")
    scores = torch.zeros((units, max_ctx), dtype=torch.float32, device="cuda")

    if args.dense_first > 0:
        w["label"] += f"_dense{args.dense_first}"
        ws_mixed = B.make_workspace(cfg, max_ctx)
        dense_flags = [l < args.dense_first for l in range(NL)]

    if args.selector != "fier":
        assert NL == 1 and w["L"] != "ragged", "the page selectors are benchmarked on single-layer, fixed-length workloads"
        PG = 16
        w["label"] += f"_{args.selector}_p{PG}"
        n_pages = max_ctx // PG
        assert n_pages % 64 == 0, "context capacity must be a multiple of 1024 for the page-level top-k"
        pcfg = B.make_config(batch, Hq, Hkv, n_pages, dtype)
        metas = []
        for r in range(R):
            m = torch.zeros(B.page_meta_bytes(cfg, PG) // 4, dtype=torch.int32, device="cuda")
            B.page_minmax(cfg, caches[r][0], PG, m)
            metas.append(m)
        max_pages = max(1, budget // PG)
        page_budgets = torch.full((batch,), max_pages, dtype=torch.int32, device="cuda")
        page_lens = torch.full((batch,), -(-(L + 1) // PG), dtype=torch.int32, device="cuda")
        pscores = torch.zeros((units, n_pages), dtype=torch.float32, device="cuda")
        pidx = torch.zeros((units, max_pages), dtype=torch.int32, device="cuda")
        pcnt = torch.zeros((units,), dtype=torch.int32, device="cuda")
        tidx = torch.zeros((units, budget), dtype=torch.int32, device="cuda")
        tcnt = torch.zeros((units,), dtype=torch.int32, device="cuda")

    def page_step(i):
        r = i % R
        c = caches[r][0]
        B.append_key(cfg, c, kns[r][0], vns[r][0])                  # K/V rows + 1-bit cache (quant-page needs it)
        if args.selector == "quest":
            B.page_append(cfg, seq_lens, PG, kns[r][0], metas[r])
            B.page_score(cfg, metas[r], PG, seq_lens, 1, qs[r][0], 0, pscores)
        else:
            B.score(cfg, c, qs[r][0], 1, scores)
            B.page_mean_score(cfg, scores, seq_lens, 1, PG, pscores)
        B.topk(pcfg, pscores, page_lens, 0, page_budgets, max_pages, pidx, pcnt)
        B.expand_pages(cfg, pidx, pcnt, max_pages, seq_lens, 1, PG, tidx, tcnt, budget)
        B.sparse_attn(cfg, c, qs[r][0], tidx, tcnt, budget, out1, wss[0][0])

    def step(i):
        r = i % R
        if args.selector != "fier":
            page_step(i)
        elif args.dense_first > 0:
            B.decode_step_mixed(cfg, caches[r], dense_flags, qs[r], kns[r], vns[r], budgets, budget, out, idx, cnt,
                                ws_mixed)
        else:
            B.decode_step(cfg, caches[r], qs[r], kns[r], vns[r], budgets, budget, out, None, None, wss[0][0])

    def step_with_index_list(i):
        r = i % R
        B.decode_step(cfg, caches[r], qs[r], kns[r], vns[r], budgets, budget, out, idx, cnt, wss[0][0])

    def timed(fn, n, warm):
        for i in range(warm):
            fn(i)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t_wall = time.perf_counter()
        e0.record()
        for i in range(n):
            fn(warm + i)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / n * 1e3, (time.perf_counter() - t_wall) / n * 1e6   # us (events), us (wall)

    # ---- the timed region: K whole steps ----------------------------------------------------------------
    us_step, us_wall = timed(step, steps, warmup)
    n_kernels = B.decode_step_kernels(cfg, budget)

    single, us_graph, us_step_idx = None, None, None
    if detail:
        us_step_idx, _ = timed(step_with_index_list, min(steps, 240), 8) if args.selector == "fier" and not args.dense_first else (None, None)
        # ---- spread of single steps: an event between consecutive steps --------------------------------------
        n_dist = min(steps, 200)
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_dist + 1)]
        evs[0].record()
        for i in range(n_dist):
            step(i)
            evs[i + 1].record()
        torch.cuda.synchronize()
        single = np.array([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(n_dist)])

        # ---- the same steps replayed from one HIP graph --------------------------------------------------------
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for r in range(R):
                    step(r)
            torch.cuda.current_stream().wait_stream(side)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                for r in range(R):
                    step(r)
            torch.cuda.synchronize()
            n_rep_g = max(3, min(steps, 240) // R)
            us_graph, _ = timed(lambda i: graph.replay(), n_rep_g, 2)
            us_graph /= R
            del graph
        except Exception as e:  # a capture problem must not lose the measurement above
            sys.stderr.write(f"bench.py: graph replay skipped: {e}\n")

    # ---- each kernel of the fused step alone (HIP events on the launch stream, rotating caches) ----------
    # argument tuples per layer cache, prepared once (slicing tensors inside the timed loop would make it CPU-bound)
    # (the kernels of the form the timed step takes: without the index list; the list kernel of the two-kernel form
    # is timed with the list given, where a call with the list takes that form too)
    largs = [[(cfg, caches[r][l:l + 1], qs[r][l:l + 1], kns[r][l:l + 1], vns[r][l:l + 1], budgets, budget,
               out[l:l + 1], None, None, wss[r][l]) for l in range(NL)] for r in range(R)]
    largs_list = [[a[:8] + (idx[l:l + 1], cnt[l:l + 1]) + a[10:] for l, a in enumerate(la)] for la in largs]
    list_kernel = n_kernels == 2 and B.decode_step_kernels(cfg, budget, True) == 2

    def phase(*ps, with_list=False):
        def run(i):
            for a in (largs_list if with_list else largs)[i % R]:
                for p in ps:
                    B.decode_step_phase(*a, p)
        return run

    for r in range(R):                    # a whole step per layer cache on its own workspace
        phase(1, 2, 3)(r)
    torch.cuda.synchronize()

    # The first kernel adds into the unit histograms that the second consumes and clears, so the second cannot be
    # repeated alone: it is timed as (first + second) - (first).  In the three-kernel form the third kernel only
    # reads what the second left and is timed alone; in the two-kernel form the third is the optional index-list
    # kernel, also timed alone (null where a call that asks for the list takes the three-kernel form instead).
    nw = 12 if NL == 1 else 2
    us_k1, _ = timed(phase(1), ns, nw)
    for r in range(R):
        phase(2)(r)                       # clears the accumulated histograms
    us_k12, _ = timed(phase(1, 2), ns, nw)
    us_k2 = us_k12 - us_k1
    us_k3 = None
    if n_kernels == 3:
        us_k3, _ = timed(phase(3), ns, nw)
    elif list_kernel:
        us_k3, _ = timed(phase(3, with_list=True), ns, nw)

    # layer (r, l) of the flattened cache list, for the per-layer calls
    flat = [(r, l) for r in range(R) for l in range(NL)]

    def st_dense(i):
        r, l = flat[i % len(flat)]
        B.dense_attn(cfg, caches[r][l], qs[r][l:l + 1], 1, out1, ws_dense)

    us_dense, _ = timed(st_dense, max(24, ns // 10), 4)

    ab = algorithmic_bytes(w, lens, buds)          # per layer
    us_layer = us_step / NL
    achieved = ab["total"] / (us_layer * 1e-6) / 1e9
    # The dominant kernel by algorithmic bytes is the one that gathers the selected K / V rows (+ q in, output out):
    # the second kernel of the two-kernel form (threshold + attention + merge in one launch, timed as first + second
    # minus first), the third of the three-kernel form (selection + attention + merge, timed alone).
    gather_bytes = ab["selected_kv"] + ab["q_out"]
    if n_kernels == 2:
        dom_name, us_dom = "step_attend_kernel (exact threshold, gather attention, merge)", us_k2
        kernels_us = {"append_score_hist": round(us_k1 / NL, 3), "threshold_attend_merge": round(us_k2 / NL, 3),
                      "sum": round((us_k1 + us_k2) / NL, 3),
                      "index_list_optional": round(us_k3 / NL, 3) if us_k3 is not None else None}
    else:
        dom_name, us_dom = "select_attend_kernel (selection, gather attention, merge)", us_k3
        kernels_us = {"append_score_hist": round(us_k1 / NL, 3), "threshold": round(us_k2 / NL, 3),
                      "select_attend_merge": round(us_k3 / NL, 3), "sum": round((us_k1 + us_k2 + us_k3) / NL, 3)}
    dom_gbps = gather_bytes / (us_dom / NL * 1e-6) / 1e9
    k1_gbps = ab["packed"] / (us_k1 / NL * 1e-6) / 1e9
    dense_bytes = int(Hkv * (lens + 1).sum() * 512) + ab["q_out"]
    config = {"workload": w["label"], "batch": batch, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": 128,
              "context": L if w["L"] != "ragged" else [int(x) for x in lens],
              "budget": budget if w["budget"] != "11%" else [int(x) for x in buds],
              "group_size": args.group_size, "layers_per_step": NL, "rotating_caches": R * NL,
              "kernels_per_layer_step": n_kernels,
              "kernels_per_layer_step_with_index_list": B.decode_step_kernels(cfg, budget, True),
              "algorithmic_bytes_per_layer": ab["total"]}
    if not detail:
        return {"label": w["label"], "us_per_layer": round(us_layer, 3), "achieved_GBps": round(achieved, 1),
                "hbm_frac": round(achieved / HBM_PEAK_GBPS, 4), "kernels_us": kernels_us,
                "dominant_kernel": {"kernel": dom_name, "GBps": round(dom_gbps, 1),
                                    "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "bytes_per_launch": gather_bytes},
                "dense_attn_us": round(us_dense, 3), "speedup_vs_dense_attn": round(us_dense / us_layer, 3),
                "steps": steps, "config": config}

    # what this machine's memory system gives a plain streaming copy (torch's own, 1 GiB operands, far beyond the
    # 256 MB Infinity Cache): context for the roofline figures, which are quoted against the nominal 8 TB/s
    big_a = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
    big_b = torch.empty_like(big_a)
    us_copy, _ = timed(lambda i: big_b.copy_(big_a), 10, 2)
    ceiling = {"copy_GBps": round(2 * big_a.numel() * 4 / (us_copy * 1e-6) / 1e9, 1),
               "how": "torch copy_ of 1 GiB of float32, bytes read + bytes written; the read-only counterpart is "
                      "dense_attn_GBps (this build's whole-cache attention)"}
    del big_a, big_b

    # ---- stand-alone entry points (separate kernels, index list through memory) --------------------------
    def st_score(i):
        r, l = flat[i % len(flat)]
        B.score(cfg, caches[r][l], qs[r][l:l + 1], 1, scores)

    def st_topk(i):
        B.topk(cfg, scores, seq_lens, 1, budgets, budget, idx[0:1], cnt[0:1])

    def st_topk_ws(i):
        B.topk_ws(cfg, scores, seq_lens, 1, budgets, budget, idx[0:1], cnt[0:1], wss[0][0])

    def st_attn(i):
        r, l = flat[i % len(flat)]
        B.sparse_attn(cfg, caches[r][l], qs[r][l:l + 1], idx[0:1], cnt[0:1], budget, out1, wss[0][0])

    us_score, _ = timed(st_score, max(24, ns // 4), 4)
    us_topk, _ = timed(st_topk, max(24, ns // 4), 4)
    us_topk_ws, _ = timed(st_topk_ws, max(24, ns // 4), 4)
    us_attn, _ = timed(st_attn, max(24, ns // 4), 4)

    # ---- the bulk quantizer (once per sequence, after prefill) and the stand-alone append ------------------
    # (after everything else: fier_append_key rewrites row L of the caches with the same k_new the steps used)
    def st_quant(i):
        r, l = flat[i % len(flat)]
        B.quantize_keys(cfg, caches[r][l])

    def st_append(i):
        r, l = flat[i % len(flat)]
        B.append_key(cfg, caches[r][l], kns[r][l], vns[r][l])

    us_quant, _ = timed(st_quant, max(6, min(24, len(flat))), 2)
    us_append, _ = timed(st_append, max(24, ns // 4), 4)
    quant_bytes = int(Hkv * lens.sum() * (256 + 16 + 512 // args.group_size))   # K rows in, codes and (s, z) out

    stages = None
    if args.selector != "fier":
        def st_est(i):
            r = i % R
            if args.selector == "quest":
                B.page_append(cfg, seq_lens, PG, kns[r][0], metas[r])
                B.page_score(cfg, metas[r], PG, seq_lens, 1, qs[r][0], 0, pscores)
            else:
                B.score(cfg, caches[r][0], qs[r][0], 1, scores)
                B.page_mean_score(cfg, scores, seq_lens, 1, PG, pscores)

        def st_recall(i):
            B.topk(pcfg, pscores, page_lens, 0, page_budgets, max_pages, pidx, pcnt)
            B.expand_pages(cfg, pidx, pcnt, max_pages, seq_lens, 1, PG, tidx, tcnt, budget)

        def st_pattn(i):
            r = i % R
            B.sparse_attn(cfg, caches[r][0], qs[r][0], tidx, tcnt, budget, out1, wss[0][0])

        stages = {"importance_estimation": round(timed(st_est, ns, 4)[0], 3),
                  "topk_recall": round(timed(st_recall, ns, 4)[0], 3),
                  "topk_self_attention": round(timed(st_pattn, ns, 4)[0], 3)}

    if args.pmc_calibration:
        a = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device="cuda")
        bq = torch.empty_like(a)
        for _ in range(3):
            torch.mul(a, 1.0, out=bq)
        torch.cuda.synchronize()
        del a, bq

    # HBM traffic of the dominant kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE / WRITE_SIZE runs,
    # scaled by what the same counters read for a plain copy of known size): a constant read from that file, not a
    # counter read in this run; None for workloads without a committed summary
    traffic, traffic_source = None, None
    tpath = os.path.join(ROOT, "profiles", f"decode_step_{workload}_traffic.json")
    if os.path.exists(tpath) and budget_arg is None and args.group_size == 32 and not args.block_tokens:
        with open(tpath) as f:
            tj = json.load(f)
        if tj.get("kernel", "").split("(")[0].strip() == dom_name.split("(")[0].strip():
            traffic = tj.get("traffic_bytes_per_launch")
            traffic_source = f"profiles/decode_step_{workload}_traffic.json (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"

    res = {
        "metric": "per-layer decode-step latency (us) + achieved HBM GB/s vs peak",
        "value": round(us_layer, 3),
        "unit": "us",
        "n_gpus": 1,
        "steps": steps,
        "warmup": warmup,
        "ms_per_step": round(us_step / 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16" if dtype == 0 else "bf16",
        "data": "synthetic",
        "config": config,
        "achieved_GBps": round(achieved, 1),
        "hbm_frac": round(achieved / HBM_PEAK_GBPS, 4),
        "us_per_step_wall": round(us_wall, 3),
        "timed_step_outputs": "attention output and kept-up-to-date caches (idx_out / count_out NULL: the ascending "
                              "index list is an optional output; the same loop with it: us_per_layer_with_index_list)",
        "us_per_layer_with_index_list": None if us_step_idx is None else round(us_step_idx / NL, 3),
        "single_step_us": {"min": round(float(single.min()), 3), "median": round(float(np.median(single)), 3),
                           "p95": round(float(np.percentile(single, 95)), 3), "n": int(len(single))},
        "graph_replay_us_per_step": None if us_graph is None else round(us_graph, 3),
        "kernels_us": kernels_us,
        "kernel_GBps": {"append_score_hist": round(k1_gbps, 1), "gather_attention": round(dom_gbps, 1)},
        "standalone_calls_us": {"fier_score": round(us_score, 3), "fier_topk": round(us_topk, 3),
                                "fier_topk_ws": round(us_topk_ws, 3),
                                "fier_sparse_attn": round(us_attn, 3), "fier_append_key": round(us_append, 3),
                                "fier_quantize_keys": round(us_quant, 3)},
        "quantize_GBps": round(quant_bytes / (us_quant * 1e-6) / 1e9, 1),
        "dense_attn_us": round(us_dense, 3),
        "dense_attn_GBps": round(dense_bytes / (us_dense * 1e-6) / 1e9, 1),
        "speedup_vs_dense_attn": round(us_dense / us_layer, 3),
        "measured_ceiling": ceiling,
        "roofline": {"bound": "hbm", "kernel": dom_name,
                     "achieved": round(dom_gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(dom_gbps / HBM_PEAK_GBPS, 4), "traffic": traffic, "traffic_source": traffic_source,
                     "bytes_per_launch": gather_bytes, "us_per_launch": round(us_dom / NL, 3)},
        "setup_s": round(t_setup, 1),
    }
    if stages is not None:
        res["selector"] = args.selector
        res["selector_stages_us"] = stages      # the unfused page-level pipeline, stage by stage (cf. Tab. 6)
        for k in ("kernels_us", "kernel_GBps", "roofline"):
            res[k] = None                       # those describe the fused token-level step, not this pipeline

    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(hosts, w, lens, buds)
    return res


def decode_loop(args, w, cfg, caches, qs, kns, vns, seq_lens, budgets, lens, buds, budget, t_setup):
    """The decode loop of Sec. 3.1 on this workload: N token steps, each ONE fier_decode_step call over all the
    layer caches (append one row per layer, score, select, attend) followed by the caller's seq_lens += 1."""
    import torch

    from paper_2508_08256_amd import binding as B

    N = args.loop_steps
    layers = [c for cl in caches for c in cl]
    NLt = len(layers)
    q = torch.cat(qs).contiguous()
    kn = torch.cat(kns).contiguous()
    vn = torch.cat(vns).contiguous()
    batch, Hq = w["batch"], w["n_q_heads"]
    ws = B.make_workspace(cfg, budget)
    out = torch.zeros((NLt, batch, Hq, 128), dtype=torch.float32, device="cuda")
    idx = torch.zeros((NLt, cfg.units, budget), dtype=torch.int32, device="cuda")
    cnt = torch.zeros((NLt, cfg.units), dtype=torch.int32, device="cuda")
    lens0 = seq_lens.clone()

    def tokens(n, with_list=False):
        # the attention output is the step's result; the ascending index list is an optional output
        for _ in range(n):
            B.decode_step(cfg, layers, q, kn, vn, budgets, budget, out, idx if with_list else None,
                          cnt if with_list else None, ws)
            seq_lens.add_(1)

    def timed_tokens(fn):
        seq_lens.copy_(lens0)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / N

    tokens(4)                                   # warm-up
    us_eager = timed_tokens(lambda: tokens(N))
    us_eager_list = timed_tokens(lambda: tokens(N, True))
    us_graph = None
    try:
        seq_lens.copy_(lens0)
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            tokens(2)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        seq_lens.copy_(lens0)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            tokens(N)
        torch.cuda.synchronize()
        timed_tokens(graph.replay)
        us_graph = timed_tokens(graph.replay)
    except Exception as e:
        sys.stderr.write(f"bench.py: graph replay skipped: {e}\n")
    # bytes of the middle token step
    ab = algorithmic_bytes(w, lens + N // 2, buds)
    us_layer = us_eager / NLt
    res = {
        "metric": "per-layer decode-step latency (us) + achieved HBM GB/s vs peak",
        "value": round(us_layer, 3), "unit": "us", "n_gpus": 1, "steps": N, "warmup": 4,
        "ms_per_step": round(us_eager / 1e3, 6), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if w["dtype"] == 0 else "bf16", "data": "synthetic",
        "config": {"workload": w["label"] + f"_decode_loop{N}", "batch": batch, "n_q_heads": Hq,
                   "n_kv_heads": w["n_kv_heads"], "head_dim": 128, "context_start": [int(x) for x in lens],
                   "tokens_appended": N, "layers_per_token": NLt, "group_size": args.group_size,
                   "algorithmic_bytes_per_layer": ab["total"]},
        "achieved_GBps": round(ab["total"] / (us_layer * 1e-6) / 1e9, 1),
        "hbm_frac": round(ab["total"] / (us_layer * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
        "us_per_token_eager": round(us_eager, 3),
        "us_per_layer_with_index_list": round(us_eager_list / NLt, 3),
        "us_per_token_graph": None if us_graph is None else round(us_graph, 3),
        "us_per_layer_graph": None if us_graph is None else round(us_graph / NLt, 3),
        "setup_s": round(t_setup, 1),
    }
    print(json.dumps(res), flush=True)


def cpu_baseline(d, w, lens, buds):
    """The CPU oracle, as it stands, timed on this machine's host cores on the same kind of layer step."""
    import oracle
    from paper_2508_08256_amd import synth

    oracle.build()
    threads = oracle.max_threads()
    hkv = w["n_kv_heads"]
    units = w["batch"] * hkv
    n_rep = w["n_q_heads"] // hkv
    # bounded sample: at most 32 units of the first layer cache (all of config 2; the first 32 units of larger ones)
    su = min(units, 32)
    K = synth.words_of(d["K"][:su])
    V = synth.words_of(d["V"][:su])
    q = synth.words_of(d["q"][:su]).reshape(su, n_rep, 128)
    kn = synth.words_of(d["k_new"][:su])
    vn = synth.words_of(d["v_new"][:su])
    L = np.repeat(lens, hkv)[:su].astype(np.int32)
    bud = np.repeat(buds, hkv)[:su].astype(np.int32)
    max_budget = int(buds.max())
    g = w.get("group_size", 32)
    bits, s, z = oracle.quantize(K, L, g, w["dtype"], threads)         # prefill, not timed

    def layer_step(nthreads):
        t0 = time.perf_counter()
        oracle.append(K, V, L, kn, vn, bits, s, z, g, w["dtype"])
        L1 = (L + 1).astype(np.int32)
        sc = oracle.score(bits, s, z, q, L1, g, w["dtype"], nthreads)
        idx, cnt = oracle.topk(sc, L1, bud, max_budget)
        oracle.attention(K, V, q, L1, 1.0 / np.sqrt(128.0), w["dtype"], idx, cnt, nthreads)
        return time.perf_counter() - t0

    reps, t_total = 0, 0.0
    while reps < 3 or (t_total < 10.0 and reps < 20):
        t_total += layer_step(threads)
        reps += 1
    t_single = layer_step(1)
    frac = float((np.repeat(lens, hkv) + 1).sum()) / float((L + 1).sum())   # whole layer / sample, by tokens
    us = t_total / reps * 1e6 * frac
    return {"value": round(us, 1), "unit": "us per layer step", "cores": threads, "kind": "oracle",
            "single_thread_value": round(t_single * 1e6 * frac, 1),
            "sample": f"{reps} repetitions of the layer step on {su} of {units} units of the first layer cache"
                      f"{' (scaled to all units by token count)' if su != units else ''}, OpenMP over units; "
                      f"single_thread_value: one repetition with 1 thread"}


if __name__ == "__main__":
    main()
