#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

A "step" is one verify step of the target model over a draft token tree: L layers of
tree-masked attention, then per-node vocab argmax, the greedy acceptance walk and KV
compaction of the accepted path -- all four C-ABI calls of libspecvlm, inputs resident in HBM.
Default workload: the LLaVA-1.6-7B anyres-shaped configuration (2880 visual + 128 text + 256
generated prefix tokens, 60-node tree, 32 layers x 32 heads x 128, bf16), synthetic data.

Prints ONE JSON line: whole-step KV-cache streaming rate (algorithmic K+V bytes of all layers
divided by the step time), verify steps/s, the roofline of the attention kernel and the fp64
CPU oracle timed on this host on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak



def source_sha256(*source_names: str) -> str:
    """SHA-256 over the named kernel source files under csrc/, in the order given."""
    import hashlib
    h = hashlib.sha256()
    for name in source_names:
        with open(os.path.join(ROOT, "paper_2509_11815_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()


def measured_traffic(profile_name: str, *source_names: str):
    """HBM bytes per launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in
    profiles/<profile_name>: the summary ends with a `traffic_json:` line that names the commit
    it was taken at and the SHA-256 of the kernel's source files at that commit.  Returns None when
    there is no such line or when the kernel source has changed since (the counters then describe
    another kernel)."""
    try:
        with open(os.path.join(ROOT, "profiles", profile_name)) as f:
            lines = [l for l in f if l.startswith("traffic_json:")]
        rec = json.loads(lines[-1][len("traffic_json:"):])
        sha = source_sha256(*source_names)
    except (OSError, IndexError, ValueError):
        return None
    if rec.get("source_sha256") != sha:
        return None
    return {"read_bytes": rec["read_bytes"], "write_bytes": rec["write_bytes"],
            "bytes": rec["read_bytes"] + rec["write_bytes"], "taken_at_commit": rec.get("commit"),
            "from": "profiles/" + profile_name}



def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "C4", "C5"])
    ap.add_argument("--splits", type=int, default=0, help="key-range splits per (request, head); 0 = library default")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--skip-cpu", action="store_true", help="skip the CPU oracle baseline leg")
    ap.add_argument("--evidence", action="store_true",
                    help="also time all layers folded into one batched attention call, and one layer through the "
                         "vector-ALU kernel (evidence only; off by default so that a kernel trace of the default run "
                         "holds per-layer matrix-core calls only)")
    ap.add_argument("--skip-configs", action="store_true",
                    help="skip the attention-only timings of the other bf16 configurations (C2, C4, C5)")
    ap.add_argument("--vector-alu", action="store_true",
                    help="profile helper: with --attn-only, run the layers through specvlm_tree_verify_attn_vector_alu")
    ap.add_argument("--skip-ceilings", action="store_true", help="skip the library copy / read-only bandwidth legs")
    ap.add_argument("--attn-only", action="store_true", help="profile helper: run only the attention launches")
    ap.add_argument("--pool-only", action="store_true",
                    help="profile helper: run only the visual-token pooling launches (8 requests of 2880 x 4096, ratio 20)")
    ap.add_argument("--head-only", action="store_true", help="profile helper: run only the fused output-head launches")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="profile helper: run plain device copies of a known size (scale for the HBM byte counters)")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import paper_2509_11815_amd as sv
    import workloads as W

    sv.load_library()                       # fails loudly when the HIP library is missing
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        # 1 GiB read + 1 GiB written per copy kernel: the reference for FETCH_SIZE / WRITE_SIZE
        src = torch.randint(0, 255, (1 << 30,), dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": 1 << 30, "copy_bytes_written": 1 << 30, "copies": 5}))
        return
    cfg = W.CONFIGS[args.workload]
    L, B, H, D, N = cfg.L, cfg.B, cfg.H, cfg.D, cfg.N
    P = W.prefix_lengths(cfg)
    S = P.astype(np.int64) + N
    path_cap = cfg.depth + 1
    torch.manual_seed(W.config_seed(cfg))

    # ---- synthetic inputs, resident in HBM; every layer has its own K/V memory -------------
    q = torch.randn((L, B, N, H, D), dtype=torch.bfloat16, device=dev)
    if cfg.paged:
        bs = cfg.block_size
        bpr = W.round_up(int(S.max()), bs) // bs
        table_np, nb = W.block_table(np.random.default_rng(W.config_seed(cfg, 0, 3)), B, bpr)
        kshape = (L, nb, H, bs, D)
        table = torch.from_numpy(table_np).to(dev)
    else:
        kshape = (L, B, H, W.round_up(int(S.max()), 16), D)
        table = None
    k = torch.empty(kshape, dtype=torch.bfloat16, device=dev)
    v = torch.empty(kshape, dtype=torch.bfloat16, device=dev)
    for l in range(L):                      # N(0,1) like the parity inputs
        k[l].normal_()
        v[l].normal_()
    tb = W.make_trees(cfg)
    parent = torch.from_numpy(tb.parent).to(dev)
    draft_tok = torch.from_numpy(tb.draft_tok).to(dev)
    logits = torch.from_numpy(tb.logits.view(np.int16)).to(dev).view(torch.bfloat16)
    prefix_len = torch.from_numpy(P).to(dev)

    out = torch.empty_like(q)
    err = torch.zeros(1, dtype=torch.int32, device=dev)
    desc = sv.binding.make_attn_desc(q[0], k[0], out[0], block_table=table, num_splits=args.splits)
    wbytes = sv.specvlm_tree_verify_attn_workspace_bytes(desc)
    workspace = torch.zeros(max(wbytes, 256), dtype=torch.uint8, device=dev)
    amax = torch.empty((B, N), dtype=torch.int32, device=dev)
    acc_out = (torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, path_cap), dtype=torch.int32, device=dev),
               torch.empty(B, dtype=torch.int32, device=dev), torch.empty((B, path_cap), dtype=torch.int32, device=dev))
    new_prefix = torch.empty(B, dtype=torch.int32, device=dev)

    def attn_layers():
        for l in range(L):
            sv.specvlm_tree_verify_attn(q[l], k[l], v[l], prefix_len, parent, block_table=table, out=out[l],
                                        workspace=workspace, err_flag=err, desc=desc)

    counters = torch.zeros(B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device=dev)

    def sample_and_compact():
        # per-node argmax and the greedy acceptance walk as one launch, compaction as one more
        sv.specvlm_node_argmax_accept(logits, parent, draft_tok, counters=counters, amax=amax, err_flag=err, out=acc_out)
        # the prefix length is NOT advanced between steps, so every step sees the same workload
        sv.specvlm_kv_compact(k, v, prefix_len, acc_out[1], acc_out[0], block_table=table, new_prefix_len=new_prefix, err_flag=err)

    def step():
        attn_layers()
        sample_and_compact()

    def make_runner(fn):
        if args.no_graph:
            return fn
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    def timed(run, iters, warmup, stats=None):
        """ms per iteration: `iters` iterations timed as up to 5 equal back-to-back batches between HIP
        events recorded on the stream the library calls are launched on (torch's current stream, which
        the binding passes to every call); the median batch is returned, the mean goes to `stats`."""
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        nb = min(5, iters)
        sizes = [iters // nb + (1 if i < iters % nb else 0) for i in range(nb)]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(nb + 1)]
        ev[0].record()
        for i, n in enumerate(sizes):
            for _ in range(n):
                run()
            ev[i + 1].record()
        torch.cuda.synchronize()
        per = sorted(ev[i].elapsed_time(ev[i + 1]) / sizes[i] for i in range(nb))
        if stats is not None:
            stats["mean"] = ev[0].elapsed_time(ev[nb]) / iters
            stats["min"], stats["max"] = per[0], per[-1]
        return per[nb // 2]

    if args.head_only:
        E_h = 128 * H
        hid = torch.randn((B, N, E_h), device=dev).to(torch.bfloat16)
        heads = [torch.empty((cfg.V, E_h), dtype=torch.bfloat16, device=dev).normal_(0.0, 2.0 / E_h ** 0.5) for _ in range(8)]
        h_ws = torch.zeros(sv.specvlm_head_argmax_workspace_bytes(B, N, cfg.V), dtype=torch.uint8, device=dev)
        h_out = torch.empty((B, N), dtype=torch.int32, device=dev)

        def head_calls():
            for w in heads:
                sv.specvlm_head_argmax(hid, w, out=h_out, workspace=h_ws)

        ms = timed(make_runner(head_calls), args.steps, args.warmup) / len(heads)
        print(json.dumps({"head_argmax_ms_per_call": ms}))
        return
    if args.pool_only:
        # eight requests' visual features (2880 tokens x 4096, the 7B-shaped projector output) pooled 20x;
        # eight input copies are cycled so that none is served from the 256 MB cache
        Bp, Tp, Ep, rp = 8, 2880, 4096, 20
        xs = [torch.randn((Bp, Tp, Ep), device=dev).to(torch.bfloat16) for _ in range(8)]
        yp = torch.zeros((Bp, (Tp + rp - 1) // rp, Ep), dtype=torch.bfloat16, device=dev)
        ntok = torch.empty(Bp, dtype=torch.int32, device=dev)

        def pool_calls():
            for xp in xs:
                sv.specvlm_visual_pool(xp, rp, out=yp, out_tokens=ntok)

        ms = timed(make_runner(pool_calls), args.steps, args.warmup) / len(xs)
        nbytes = xs[0].numel() * 2 + yp.numel() * 2
        print(json.dumps({"visual_pool_ms_per_call": ms, "bytes_per_call": nbytes,
                          "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_of_8TBps": round(nbytes / (ms * 1e-3) / 8e12, 4)}))
        return
    if args.attn_only and args.vector_alu:
        # measurement aid: the same layers through the vector-ALU kernel (no matrix cores); slow, so few layers
        def valu_layers():
            for l in range(min(L, 4)):
                sv.specvlm_tree_verify_attn_vector_alu(q[l], k[l], v[l], prefix_len, parent, block_table=table,
                                                       out=out[l], err_flag=err, desc=desc)
        ms = timed(make_runner(valu_layers), args.steps, args.warmup)
        print(json.dumps({"vector_alu_ms_per_layer_call": ms / min(L, 4)}))
        return
    if args.attn_only:
        run_attn = make_runner(attn_layers)
        ms = timed(run_attn, args.steps, args.warmup)
        print(json.dumps({"attn_only_ms_per_step": ms, "ms_per_layer_call": ms / L}))
        return

    # the attention-only leg runs first: the step leg below then starts on a chip that has been busy for
    # some 60 ms (5 warm-up steps are 3 ms, not enough for the clocks to settle after the input set-up)
    run_attn = make_runner(attn_layers)
    ms_attn = timed(run_attn, max(args.steps, 100), max(args.warmup, 10))
    run_step = make_runner(step)
    step_stats = {}
    ms_step = timed(run_step, args.steps, args.warmup, step_stats)
    # Evidence only, never the headline: the same L x B layer problems handed over as ONE call (layers
    # folded into the batch dimension).  A model cannot do this -- a layer's queries depend on the layer
    # before -- but it shows what the kernel streams once the per-call fixed costs (launch, first-tile
    # latency, the merge of the splits) are paid once instead of L times.
    ms_folded = None
    if not cfg.paged and args.evidence:
        qf, kf, vf, of = (t.view(L * B, *t.shape[2:]) for t in (q, k, v, out))
        pf, parf = prefix_len.repeat(L), parent.repeat(L, 1)
        dfold = sv.binding.make_attn_desc(qf, kf, of)
        wsf = torch.zeros(max(sv.specvlm_tree_verify_attn_workspace_bytes(dfold), 256), dtype=torch.uint8, device=dev)
        run_fold = make_runner(lambda: sv.specvlm_tree_verify_attn(qf, kf, vf, pf, parf, out=of, workspace=wsf,
                                                                   err_flag=err, desc=dfold))
        ms_folded = timed(run_fold, max(args.steps // 4, 5), 3)
    # Evidence as well: one layer through the vector-ALU kernel (the measurement aid of the header), i.e. what
    # the step costs without the matrix cores.
    ms_valu = None
    if args.evidence:
        ms_valu = timed(make_runner(lambda: sv.specvlm_tree_verify_attn_vector_alu(
            q[0], k[0], v[0], prefix_len, parent, block_table=table, out=out[0], err_flag=err, desc=desc)), 5, 2)

    # ---- the other bf16 configurations, attention only, same method (HIP-graph replay of per-layer calls,
    # every layer its own K/V memory; at most 8 layers are built -- 1.1 to 3.2 GB, far beyond the 256 MB cache)
    def attention_only(name, capacity=None, tail=False):
        """One attention call per layer of configuration `name` (up to 8 layers resident), graph replay.
        `capacity` (contiguous caches): a cache preallocated for that many slots instead of one that
        just fits the lengths.  `tail`: also time the configuration's argmax + accept launch."""
        c = W.CONFIGS[name]
        Lc = min(c.L, 8)
        Pc = W.prefix_lengths(c)
        Sc = Pc.astype(np.int64) + c.N
        qc = torch.randn((Lc, c.B, c.N, c.H, c.D), dtype=torch.bfloat16, device=dev)
        if c.paged:
            bpr = W.round_up(int(Sc.max()), c.block_size) // c.block_size
            t_np, nbc = W.block_table(np.random.default_rng(W.config_seed(c, 0, 3)), c.B, bpr)
            shape, tbl = (Lc, nbc, c.H, c.block_size, c.D), torch.from_numpy(t_np).to(dev)
        else:
            shape, tbl = (Lc, c.B, c.H, capacity or W.round_up(int(Sc.max()), 16), c.D), None
        kc = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        vc = torch.empty(shape, dtype=torch.bfloat16, device=dev)
        for l in range(Lc):
            kc[l].normal_()
            vc[l].normal_()
        par_c = torch.from_numpy(W.make_trees(c).parent).to(dev)
        P_dev = torch.from_numpy(Pc).to(dev)
        oc = torch.empty_like(qc)
        dc = sv.binding.make_attn_desc(qc[0], kc[0], oc[0], block_table=tbl)
        wsc = torch.zeros(max(sv.specvlm_tree_verify_attn_workspace_bytes(dc), 256), dtype=torch.uint8, device=dev)

        def layers():
            for l in range(Lc):
                sv.specvlm_tree_verify_attn(qc[l], kc[l], vc[l], P_dev, par_c, block_table=tbl, out=oc[l],
                                            workspace=wsc, err_flag=err, desc=dc)

        us = timed(make_runner(layers), 40, 10) * 1e3 / Lc
        nbytes = W.kv_bytes_per_layer(c)
        rec = {"attn_us_per_launch": round(us, 3), "algorithmic_bytes_per_launch": nbytes,
               "GBps": round(nbytes / (us * 1e-6) / 1e9, 1), "frac": round(nbytes / (us * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
               "num_splits": sv.specvlm_tree_verify_attn_num_splits(dc), "layers_timed": Lc,
               "shape": f"B={c.B}, H={c.H}, D={c.D}, prefix={Pc.tolist()}, paged={c.paged}"
                        + (f", cache capacity {capacity}" if capacity else "")}
        if tail:
            # the per-node argmax over the vocabulary + the greedy walk, one launch: B*N*V logits read once
            tbc = W.make_trees(c)
            lg = torch.from_numpy(tbc.logits.view(np.int16)).to(dev).view(torch.bfloat16)
            tok = torch.from_numpy(tbc.draft_tok).to(dev)
            cnt = torch.zeros(c.B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device=dev)
            am = torch.empty((c.B, c.N), dtype=torch.int32, device=dev)
            oo = (torch.empty(c.B, dtype=torch.int32, device=dev), torch.empty((c.B, c.depth + 1), dtype=torch.int32, device=dev),
                  torch.empty(c.B, dtype=torch.int32, device=dev), torch.empty((c.B, c.depth + 1), dtype=torch.int32, device=dev))
            us_t = timed(make_runner(lambda: sv.specvlm_node_argmax_accept(lg, par_c, tok, counters=cnt, amax=am,
                                                                           err_flag=err, out=oo)), 100, 10) * 1e3
            lbytes = lg.numel() * lg.element_size()
            rec["node_argmax_accept"] = {"us_per_launch": round(us_t, 3), "algorithmic_bytes_per_launch": lbytes, "bound": "hbm",
                                         "GBps": round(lbytes / (us_t * 1e-6) / 1e9, 1),
                                         "frac": round(lbytes / (us_t * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4)}
        return rec

    other_configs = {}
    if not args.skip_configs:
        for name in ("C2", "C4", "C5"):
            if name != cfg.name:
                other_configs[name] = attention_only(name, tail=(name == "C4"))
                torch.cuda.empty_cache()
        # a short request in a cache preallocated for a long one: the split count follows the capacity
        c3 = W.CONFIGS["C3"]
        other_configs["C2_lengths_in_a_cache_of_C3_capacity"] = attention_only(
            "C2", capacity=W.round_up(int(W.prefix_lengths(c3).max()) + c3.N, 16))
        torch.cuda.empty_cache()
    run_tail = make_runner(sample_and_compact)
    ms_tail = timed(run_tail, args.steps, args.warmup)
    # not part of the step (the headline metric is greedy): the temperature-1 acceptance walk on the same trees
    gen = torch.Generator(device=dev)
    gen.manual_seed(W.config_seed(cfg, 0, 9))
    u_accept = torch.rand((B, N), device=dev, generator=gen)
    u_bonus = torch.rand(B, device=dev, generator=gen)
    smp_out = tuple(torch.empty_like(t) for t in acc_out)
    run_smp = make_runner(lambda: sv.specvlm_tree_accept_sample(parent, draft_tok, logits, u_accept, u_bonus,
                                                                temperature=1.0, err_flag=err, out=smp_out))
    ms_smp = timed(run_smp, args.steps, args.warmup)
    # also outside the step: the draft side's tree growth (Top-K 10, ten nodes expanded per level, `depth`
    # levels, 60 nodes; the draft model's own forward passes are not part of it) ...
    K = 10
    lvl_logits = [torch.randn((B, 1 if d == 0 else K, cfg.V), device=dev, generator=gen).mul_(2).to(torch.bfloat16)
                  for d in range(cfg.depth)]
    C = K + (cfg.depth - 1) * K * K
    c_score = torch.zeros((B, C), dtype=torch.float32, device=dev)
    c_tok = torch.zeros((B, C), dtype=torch.int32, device=dev)
    c_par = torch.full((B, C), -1, dtype=torch.int32, device=dev)
    sel = [(torch.empty((B, K), dtype=torch.int32, device=dev), torch.empty((B, K), dtype=torch.float32, device=dev),
            torch.empty(B, dtype=torch.int32, device=dev)) for _ in range(cfg.depth)]
    fin = (torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty((B, N), dtype=torch.int32, device=dev),
           torch.empty((B, N), dtype=torch.int32, device=dev), torch.empty(B, dtype=torch.int32, device=dev))
    root_tok = torch.zeros(B, dtype=torch.int32, device=dev)

    grow_counters = torch.zeros(B * sv.binding.COUNTER_STRIDE, dtype=torch.int32, device=dev)

    def grow():
        # a level = Top-K of the expanded nodes' rows + the choice of the nodes the next level expands, one launch
        base, count = 0, 0
        for d in range(cfg.depth):
            rows = 1 if d == 0 else K
            nb = base + count
            out = dict(score_out=c_score[:, nb:nb + rows * K], token_out=c_tok[:, nb:nb + rows * K],
                       parent_out=c_par[:, nb:nb + rows * K])
            prev = dict(cum=sel[d][1], parent_idx=sel[d][0]) if d else {}
            if d + 1 < cfg.depth:
                sv.specvlm_draft_topk_select(lvl_logits[d], K, K, index_base=nb, sel_out=sel[d + 1][0],
                                             sel_score_out=sel[d + 1][1], count_out=sel[d + 1][2],
                                             counters=grow_counters, **prev, **out)
            else:
                sv.specvlm_draft_topk(lvl_logits[d], K, **prev, **out)
            base, count = nb, rows * K
        sv.specvlm_draft_finalize(c_score, c_par, c_tok, root_tok, N, err_flag=err, out=fin)

    ms_grow = timed(make_runner(grow), args.steps, args.warmup)
    # ... and the output head fused with the greedy choice (it would replace "logits + argmax" of the step when
    # the caller hands over hidden states instead of logits): hidden 4096 (5120 for the 40-head model), vocab V.
    # Eight copies of the head matrix are cycled so that none is served from the 256 MB cache.
    E_h = 128 * H
    hid = torch.randn((B, N, E_h), device=dev, generator=gen).to(torch.bfloat16)
    # (drawn in bf16 directly: fp32 temporaries twice the size would fragment the allocator's memory)
    heads = [torch.empty((cfg.V, E_h), dtype=torch.bfloat16, device=dev).normal_(0.0, 2.0 / E_h ** 0.5, generator=gen)
             for _ in range(8)]
    h_ws = torch.zeros(sv.specvlm_head_argmax_workspace_bytes(B, N, cfg.V), dtype=torch.uint8, device=dev)
    h_out = torch.empty((B, N), dtype=torch.int32, device=dev)

    def head_calls():
        for w in heads:
            sv.specvlm_head_argmax(hid, w, out=h_out, workspace=h_ws)

    ms_head = timed(make_runner(head_calls), max(args.steps // 4, 5), 3) / len(heads)
    head_bytes = cfg.V * E_h * 2          # the head matrix once, however many blocks of 64 node rows share the pass
    assert int(err.item()) == 0, "device error flag set"

    kv_bytes_layer = W.kv_bytes_per_layer(cfg)
    kv_bytes_step = kv_bytes_layer * L
    value = kv_bytes_step / (ms_step * 1e-3) / 1e9
    attn_launch_us = ms_attn * 1e3 / L
    achieved = kv_bytes_layer / (attn_launch_us * 1e-6) / 1e9

    result = {
        "metric": "tree-verify attn KV GB/s (% HBM peak); verify steps/s at 2880-token prefix",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5),
        "ms_per_step_note": "median of up to 5 equal batches of the timed steps; mean %.5f, fastest batch %.5f, slowest %.5f"
                            % (step_stats["mean"], step_stats["min"], step_stats["max"]),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {cfg.note}; B={B}, L={L}, H={H}, D={D}, prefix={P.tolist()}, "
                               f"tree nodes={N}, depth={cfg.depth}, vocab={cfg.V}, paged={cfg.paged}",
                   "launch": "HIP graph replay of one whole step" if not args.no_graph else "eager launches",
                   "timing": "HIP events on the stream the calls are launched on",
                   "num_splits": sv.specvlm_tree_verify_attn_num_splits(desc),
                   "accept_len": acc_out[0].tolist()},
        "verify_steps_per_s": round(1e3 / ms_step, 1),
        "pct_hbm_peak": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "breakdown_ms": {"attention_all_layers": round(ms_attn, 5), "argmax_accept_compact": round(ms_tail, 5)},
        "evidence_layers_folded_into_one_call": None if ms_folded is None else {
            "ms": round(ms_folded, 5), "GBps": round(kv_bytes_step / (ms_folded * 1e-3) / 1e9, 1),
            "frac_of_peak": round(kv_bytes_step / (ms_folded * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "note": "all layers' attention as one call with batch L*B: not possible in a model (layers depend on "
                    "each other), shows the streaming rate without L-fold per-call costs"},
        "evidence_vector_alu_kernel": None if ms_valu is None else {
            "us_per_layer_call": round(ms_valu * 1e3, 1), "GBps": round(W.kv_bytes_per_layer(cfg) / (ms_valu * 1e-3) / 1e9, 1),
            "note": "one layer through specvlm_tree_verify_attn_vector_alu (no matrix cores): what the matrix-core kernel is measured against"},
        "outside_the_step_ms": {"tree_accept_sample_T1": round(ms_smp, 5), "draft_tree_growth": round(ms_grow, 5),
                                "head_argmax_fused": round(ms_head, 5)},
        "roofline_head_argmax": {"kernel": "specvlm::head_argmax_kernel<%d>" % (1 if B * N <= 64 else 2 if B * N <= 128 else 4 if B * N <= 256 else 8), "bound": "hbm",
                                 "achieved": round(head_bytes / (ms_head * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                                 "unit": "GB/s", "frac": round(head_bytes / (ms_head * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                                 "algorithmic_bytes_per_launch": head_bytes, "avg_launch_us": round(ms_head * 1e3, 3),
                                 "traffic": measured_traffic("head_argmax_kernel_C3.txt", "head_argmax.hip") if cfg.name == "C3" else None},
        "roofline": {"kernel": "specvlm::attn_mfma_kernel<128, 4, 2> (the whole specvlm_tree_verify_attn call of one layer)",
                     "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": kv_bytes_layer,
                     "avg_launch_us": round(attn_launch_us, 3),
                     "traffic": measured_traffic("attn_mfma_kernel_C3.txt", "attn_mfma.hip", "attn_mfma_body.inc") if cfg.name == "C3" else None},
        "configs": dict({cfg.name: {"attn_us_per_launch": round(attn_launch_us, 3), "algorithmic_bytes_per_launch": kv_bytes_layer,
                                    "GBps": round(achieved, 1), "frac": round(achieved / HBM_PEAK_GBPS, 4),
                                    "num_splits": sv.specvlm_tree_verify_attn_num_splits(desc), "layers_timed": L}},
                        **other_configs),
    }

    # ---- what plain library kernels reach on this machine: device copy (read + write) and a read-only pass ----
    if not args.skip_ceilings:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        ms_copy = timed(lambda: dst.copy_(src), 10, 3)
        ms_sum = timed(lambda: src.sum(), 10, 3)
        nbytes = src.numel() * 4
        result["measured_ceilings"] = {
            "device_copy_GBps": round(2 * nbytes / (ms_copy * 1e-3) / 1e9, 1),
            "read_only_sum_GBps": round(nbytes / (ms_sum * 1e-3) / 1e9, 1),
            "note": "torch copy_ / sum over 1 GiB of fp32, bytes read + written per second"}
        del src, dst

    # ---- CPU baseline: the fp64 oracle as it stands, on this host, on a bounded sample ------
    if not args.skip_cpu:
        import oracle
        oracle.build()
        q0 = q[0].view(torch.int16).cpu().numpy().view(np.uint16)
        k0 = k[0].view(torch.int16).cpu().numpy().view(np.uint16)
        v0 = v[0].view(torch.int16).cpu().numpy().view(np.uint16)
        t0 = time.perf_counter()
        oracle.tree_attn(q0, k0, v0, P, tb.parent, block_table=None if table is None else table_np)
        t_layer = time.perf_counter() - t0
        n_layers = int(min(L, max(1, round(15.0 / max(t_layer, 1e-3)))))
        t0 = time.perf_counter()
        for _ in range(n_layers):
            oracle.tree_attn(q0, k0, v0, P, tb.parent, block_table=None if table is None else table_np)
        r_amax = oracle.node_argmax(tb.logits)
        r_m, r_path, _, _ = oracle.tree_accept(tb.parent, tb.draft_tok, r_amax, path_cap=path_cap)
        kk, vv = k0[None].copy(), v0[None].copy()
        for _ in range(n_layers):
            oracle.kv_compact(kk, vv, P, r_path, r_m, block_table=None if table is None else table_np)
        t_cpu = time.perf_counter() - t0
        result["cpu_baseline"] = {
            "value": round(kv_bytes_layer * n_layers / t_cpu / 1e9, 4), "unit": "GB/s",
            "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n_layers} of {L} layers of attention and compaction (one layer's tensors reused) + "
                      f"argmax + accept, {t_cpu:.2f} s; a full step would take about {t_cpu * L / n_layers:.1f} s",
            "host_cpus": os.cpu_count()}
    print(json.dumps(result))


if __name__ == "__main__":
    main()
