#!/usr/bin/env python3
"""Benchmark of REST's draft-and-verify hot path on one MI355X.

One step = rest_retrieve (1 context) -> rest_tree_attention (all layers x heads, one launch, mask straight
from the retrieve output in HBM) -> rest_accept, on the Llama-2-7B-shaped synthetic workload:
100M-token Zipf(1.1) datastore with planted motifs, contexts of 512 tokens, K=5000, m=16, c=64,
32 layers x 32 heads x 128, KV length 2048, bf16.  All inputs are resident in HBM before timing starts.

Prints ONE JSON line (metric, value, roofline, cpu_baseline, extra side measurements).  The CPU oracle is used only for the
`cpu_baseline` leg and a sampled parity check, never inside the timed region.
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

HBM_PEAK_GBS = 8000.0


def note(msg: str) -> None:
    """progress lines go to stderr; stdout carries the one JSON line"""
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


SETTLE_STEPS = 100      # untimed steps before the caller's warm-up steps (see where they are taken)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama7b", choices=["llama7b", "llama13b", "batched2b", "tiny"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-layer and batched-retrieval side measurements")
    ap.add_argument("--sweep", action="store_true",
                    help="also time tree attention over the tree-size / KV-length sweep (random tries, 32 x 32 heads)")
    ap.add_argument("--ablation", action="store_true",
                    help="only run the paper's ablation sweeps (draft strategy, n_max, c) with a toy model on the tiny "
                         "synthetic datastore and print the mean generated length per step")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy five times (reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--attention-only", metavar="NbxHxTxP[:kv8|:f32][:gqaG][:layers]", default=None,
                    help="only run rest_tree_attention at that shape 3 + 10 times (for rocprofv3 runs of one kernel): Nb batch "
                         "entries x H K/V heads, T draft tokens, P cached keys; kv8 = 8-bit (E4M3) cache; gqaG = G query heads "
                         "per K/V head stacked along the row axis; layers = one launch per batch entry")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    import synth
    import paper_2311_08252_amd as rest

    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")
    if args.copy_calibration:
        a = torch.zeros(1 << 28, dtype=torch.int32, device=dev)     # 1 GiB read + 1 GiB written per copy
        b = torch.ones(1 << 28, dtype=torch.int32, device=dev)
        for _ in range(5):
            a.copy_(b)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes_read": 1 << 30, "copy_calibration_bytes_written": 1 << 30}))
        return 0
    if args.ablation:
        print(json.dumps({"ablation": ablation(rest, torch, synth, np, dev)}))
        return 0
    if args.attention_only:
        print(json.dumps(attention_only(rest, torch, synth, np, dev, args.attention_only)))
        return 0
    w = synth.WORKLOADS[args.workload]
    B = w.batch         # contexts per step: 1, or 32 for the batched workload (one layer, per-context masks)
    n_ctx = 16 if B == 1 else 2     # the timed steps rotate over this many context sets (half copied, half i.i.d.)

    # ---------------- inputs, resident in HBM
    t0 = time.time()
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs, dtype=w.token_dtype,
                             workers=16 if w.n_tokens > 600_000_000 else 8)
    ctx_np, len_np = synth.make_contexts(corp, n_ctx * B, w.ctx_len, w.query_seed)
    t_gen = time.time() - t0
    note(f"datastore generated in {t_gen:.1f} s")
    d_corpus = torch.from_numpy(corp.tokens).to(dev)
    d_ctx = torch.from_numpy(ctx_np).to(dev)
    d_len = torch.from_numpy(len_np).to(dev)
    torch.cuda.synchronize()
    t0 = time.time()
    index = rest.rest_build_index(d_corpus, w.sa_bytes)
    torch.cuda.synchronize()
    t_build = time.time() - t0
    note(f"index built in {t_build:.2f} s")
    t_build32 = None
    if not args.no_extras:      # the depth-limited build of the same stream (enough for n_max + cont_len <= 32)
        t0 = time.time()
        lim = rest.rest_build_index_prefix(d_corpus, w.sa_bytes, 32)
        torch.cuda.synchronize()
        t_build32 = time.time() - t0
        note(f"depth-32 index built in {t_build32:.2f} s (ordered by {lim.sort_depth or 'all'} tokens)")
        del lim

    Nb, H, D, P, c = (w.layers if B == 1 else B), w.heads, w.head_dim, w.kv_len, w.max_nodes
    Lk = P + c
    gen = torch.Generator(device=dev)
    gen.manual_seed(w.qkv_seed)
    q = torch.randn((Nb, H, c, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    k = torch.randn((Nb, H, Lk, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    v = torch.randn((Nb, H, Lk, D), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
    out = torch.empty_like(q)
    scale = 1.0 / float(np.sqrt(D))
    prm = dict(n_max=w.n_max, n_min=w.n_min, max_matches=w.max_matches, cont_len=w.cont_len, max_nodes=c)

    trees = [rest.Tree.empty(B, c, dev) for _ in range(n_ctx)]
    ids = []
    for i in range(n_ctx):      # model token ids per position (inputs of rest_accept), derived once from the trees
        rest.rest_retrieve(index, d_ctx[i * B:(i + 1) * B], d_len[i * B:(i + 1) * B], out=trees[i], **prm)
        torch.cuda.synchronize()
        ids_np = np.stack([synth.sampled_ids(w.qkv_seed + 100 + i * B + b, trees[i].draft_tokens[b].cpu().numpy(),
                                             trees[i].parent_idx[b].cpu().numpy(), int(trees[i].n_nodes[b]))
                           for b in range(B)])
        ids.append(torch.from_numpy(ids_np).to(dev))
    alen = torch.empty(B, dtype=torch.int32, device=dev)
    apath = torch.empty((B, w.cont_len), dtype=torch.int32, device=dev)
    nxt = torch.empty(B, dtype=torch.int32, device=dev)
    desc = rest.make_attn_desc(q, k, v, out, P, scale, B > 1)
    ws_bytes = rest.rest_tree_attention_workspace_bytes(desc)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    ctx_rows = [d_ctx[i * B:(i + 1) * B] for i in range(n_ctx)]
    len_rows = [d_len[i * B:(i + 1) * B] for i in range(n_ctx)]
    # [c, words] views: one mask shared by all layers; batched: [B, c, words], one mask per context
    masks = [t.tree_mask[0] if B == 1 else t.tree_mask for t in trees]

    def step(i, ev=None):
        j = i % n_ctx
        tree = trees[j]
        rest.rest_retrieve(index, ctx_rows[j], len_rows[j], out=tree, **prm)
        if ev is not None:
            ev[0].record()
        rest.rest_tree_attention(q, k, v, masks[j], P, scale, out=out, workspace=ws)
        if ev is not None:
            ev[1].record()
        rest.rest_accept(ids[j], tree, w.cont_len, alen, apath, nxt)

    note("inputs resident, timing")
    # The chip takes a few milliseconds of sustained load to settle: steps 20 .. 40 of a process run 6 % slower than
    # the steps before and after them (attention 187 us instead of 175 us), whatever --warmup says.  So the run first
    # takes a fixed number of untimed steps of its own, then the caller's warm-up steps, then the timed ones.
    for i in range(SETTLE_STEPS):
        step(i)
    torch.cuda.synchronize()
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    # HIP events (on the stream the kernels are launched on) bracket the attention launch of every 4th timed step (of
    # about twenty steps in a longer run): an event pair costs about 7 us of stream time, which would otherwise be 3 %
    # of every step
    ev_every = max(4, args.steps // 20)
    events = {i: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for i in range(0, args.steps, ev_every)}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i, events.get(i))
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    in_step = sorted(a.elapsed_time(b) for a, b in events.values())

    # The roofline figure comes from a loop of its own, so that it does not depend on --steps: 20 warm launches of
    # the attention call of the step, then 100 timed ones between two HIP events on the launch stream.
    slabs = Nb * H
    alg_bytes = slabs * (2 * Lk * D * 2 + 2 * c * D * 2) + B * c * ((c + 63) // 64) * 8
    n_roof = 100

    def attn_once(i=0):
        rest.rest_tree_attention(q, k, v, masks[i % n_ctx], P, scale, out=out, workspace=ws)

    for i in range(20):
        attn_once(i)
    torch.cuda.synchronize()
    batches = []
    for rep in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(n_roof):
            attn_once(i)
        e1.record()
        torch.cuda.synchronize()
        batches.append(e0.elapsed_time(e1) / n_roof)
    attn_ms = sorted(batches)[1]                # median of three batches of 100
    achieved = alg_bytes / (attn_ms * 1e-3) / 1e9
    kernel_name = attention_kernel_name(Nb * H, c, False)
    traffic, traffic_from = profiled_traffic(args.workload)

    result = {
        "metric": {"llama7b": "draft-verify steps/s (retrieve+tree-attn+accept) at 7B shape",
                   "batched2b": "draft-verify steps/s (retrieve+tree-attn+accept), 32 contexts per step, 2B-token datastore",
                   "llama13b": "draft-verify steps/s (retrieve+tree-attn+accept) at 13B shape",
                   "tiny": "draft-verify steps/s (retrieve+tree-attn+accept), tiny config"}[args.workload],
        "value": round(1e3 / ms_per_step, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "settle_steps": SETTLE_STEPS, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_tokens}-token Zipf(1.1)+motif datastore, {B} context(s) x {w.ctx_len} per step "
                               f"(rotating over {n_ctx} sets), K={w.max_matches}, m={w.cont_len}, c={c}, tree attention "
                               + (f"{Nb} layers x {H} heads x {D}, KV length {P}+{c}, one launch over all layers" if B == 1 else
                                  f"{B} contexts x {H} heads x {D} (one layer, per-context masks), KV length {P}+{c}"),
                   "global_batch": B, "kv_len": P, "tree_nodes": c},
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": traffic, "traffic_from": traffic_from, "algorithmic_bytes_per_launch": alg_bytes,
                     "avg_launch_us": round(attn_ms * 1e3, 2), "launches_timed": 3 * n_roof,
                     "batches_of_100_us": [round(x * 1e3, 2) for x in batches]},
        "extra": {"attn_inside_step_us_p10_p50_p90": [round(in_step[int(len(in_step) * f)] * 1e3, 1) for f in (0.1, 0.5, 0.9)]
                  if in_step else None,
                  "index_build_s": round(t_build, 3),
                  "index_build_depth32_s": None if t_build32 is None else round(t_build32, 3), "corpus_gen_s": round(t_gen, 2),
                  "contexts_per_s": round(B * 1e3 / ms_per_step, 1),
                  "tree_nodes_per_context": [int(x) for t in trees for x in t.n_nodes.tolist()][:32],
                  "matched_len_per_context": [int(x) for t in trees for x in t.matched_len.tolist()][:32]},
    }

    if B == 1 and Nb > 1:
        # The same step as a model has to take it: layer l + 1 needs layer l's output, so the attention of the 32 layers is
        # 32 launches in a row, one layer of H heads each.  Timed as the whole step (retrieve, the launches, accept),
        # and the launches alone both from the host and replayed as one HIP graph (no host time between them).
        views = [(q[nb:nb + 1], k[nb:nb + 1], v[nb:nb + 1], out[nb:nb + 1]) for nb in range(Nb)]
        d1 = rest.make_attn_desc(*views[0], P, scale, False)
        ws1 = torch.empty(max(rest.rest_tree_attention_workspace_bytes(d1), 16), dtype=torch.uint8, device=dev)

        def layers(mask):
            for qq, kk, vv, oo in views:
                rest.rest_tree_attention(qq, kk, vv, mask, P, scale, out=oo, workspace=ws1)

        def step_layers(i):
            j = i % n_ctx
            rest.rest_retrieve(index, ctx_rows[j], len_rows[j], out=trees[j], **prm)
            layers(masks[j])
            rest.rest_accept(ids[j], trees[j], w.cont_len, alen, apath, nxt)

        for i in range(5):
            step_layers(i)
        torch.cuda.synchronize()
        n_lay = 50
        t0 = time.perf_counter()
        for i in range(n_lay):
            step_layers(i)
        torch.cuda.synchronize()
        ms_step_layers = (time.perf_counter() - t0) * 1e3 / n_lay
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            layers(masks[0])
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                layers(masks[0])
        torch.cuda.synchronize()
        lay = {}
        for name, fn in (("host_launches", lambda: layers(masks[0])), ("hip_graph_replay", graph.replay)):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(20):
                fn()
            e1.record()
            torch.cuda.synchronize()
            lay[name] = e0.elapsed_time(e1) / 20
        del graph
        per_launch_ms = min(lay.values()) / Nb
        bytes_layer = H * (2 * Lk * D * 2 + 2 * c * D * 2) + c * ((c + 63) // 64) * 8
        result["value_layer_by_layer"] = round(1e3 / ms_step_layers, 2)
        result["roofline_layer_by_layer"] = {
            "bound": "hbm", "kernel": attention_kernel_name(H, c, False), "launches_per_step": Nb,
            "achieved": round(bytes_layer / (per_launch_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(bytes_layer / (per_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
            "algorithmic_bytes_per_launch": bytes_layer, "avg_launch_us": round(per_launch_ms * 1e3, 2),
            "all_layers_us": {kk: round(vv * 1e3, 1) for kk, vv in lay.items()},
            "note": "launch-to-launch period of back-to-back launches on one stream (start-up and the gap between "
                    "kernels included); `value` and `roofline` above are the one-launch form of the same work"}
        result["extra"]["ms_per_step_layer_by_layer"] = round(ms_step_layers, 5)
        result["extra"]["attn_per_layer_launches_us_total"] = round(lay["host_launches"] * 1e3, 1)
    if not args.no_extras and B == 1:
        result["extra"].update(side_measurements(rest, torch, synth, corp, index, w, q, k, v, out, trees[0], P, scale, prm))
    if args.sweep:
        result["extra"]["attention_sweep"] = attention_sweep(rest, torch, synth, np, dev)
    if not args.no_cpu_baseline:
        note("timing the CPU oracle on a sample")
        result["cpu_baseline"], result["extra"]["parity_sample_max_abs_err"] = cpu_baseline(
            np, torch, corp, ctx_np, w, q, k, v, out, trees, ids, P, scale, step, B)
    print(json.dumps(result))
    return 0


def attention_only(rest, torch, synth, np, dev, spec):
    """rest_tree_attention alone at one shape: 3 warm launches, then 10 between two HIP events."""
    parts = spec.split(":")
    Nb, H, T, P = (int(x) for x in parts[0].split("x"))
    kv8 = "kv8" in parts[1:]
    f32 = "f32" in parts[1:]
    by_layer = "layers" in parts[1:]
    g_heads = max([int(x[3:]) for x in parts[1:] if x.startswith("gqa")] + [1])
    Tq = T * g_heads
    g = torch.Generator(device=dev)
    g.manual_seed(T * 100000 + P + g_heads)
    q = torch.randn((Nb, H, Tq, 128), generator=g, device=dev)
    if not f32:
        q = q.to(torch.bfloat16)
    k, v = (torch.randn((Nb, H, P + T, 128), generator=g, device=dev) for _ in range(2))
    sc = None
    if f32:
        pass
    elif kv8:
        k, v = (x.to(torch.float8_e4m3fn).view(torch.uint8) for x in (k, v))
        sc = torch.full((Nb * H,), 1.0, dtype=torch.float32, device=dev)
    else:
        k, v = (x.to(torch.bfloat16) for x in (k, v))
    mask = torch.from_numpy(synth.random_tree(T, 14 + T)[3].view(np.int64)).to(dev)
    out = torch.empty_like(q)
    scale = 1.0 / float(np.sqrt(128.0))
    mr = T if g_heads > 1 else 0
    if by_layer:
        views = [(q[i:i + 1], k[i:i + 1], v[i:i + 1], out[i:i + 1], None if sc is None else sc[i * H:(i + 1) * H]) for i in range(Nb)]
    else:
        views = [(q, k, v, out, sc)]
    desc = rest.make_attn_desc(*views[0][:4], P, scale, False, 0, mr, views[0][4], views[0][4])
    ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc), 16), dtype=torch.uint8, device=dev)

    def run():
        for qq, kk, vv, oo, ss in views:
            rest.rest_tree_attention(qq, kk, vv, mask, P, scale, out=oo, workspace=ws, mask_rows=mr, k_scale=ss, v_scale=ss)

    for _ in range(3):
        run()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(10):
        run()
    b.record()
    torch.cuda.synchronize()
    us = a.elapsed_time(b) / 10 * 1e3
    esz = 4 if f32 else 2
    alg = Nb * H * (2 * (P + T) * 128 * (1 if kv8 else esz) + 2 * Tq * 128 * esz) + T * ((T + 63) // 64) * 8
    flops = Nb * H * 4.0 * Tq * (P + T) * 128
    if f32:
        nw = 1 if Tq <= 32 else 2 if Tq <= 64 else 4 if Tq <= 128 else 8
        return {"attention_only": spec, "kernel": f"tree_attn_f32_tiled_kernel<{nw}>", "launches_per_run": len(views),
                "us_per_run": round(us, 1), "algorithmic_bytes_per_run": alg, "GB/s": round(alg / us / 1e3, 1),
                "frac_of_8TB/s": round(alg / us / 1e3 / HBM_PEAK_GBS, 3), "TFLOP/s": round(flops / us / 1e6, 1),
                "frac_of_157.3_TFLOP/s_fp32_matrix_peak": round(flops / us / 1e6 / 157.3, 3)}
    return {"attention_only": spec, "kernel": attention_kernel_name((H if by_layer else Nb * H) * ((Tq + 255) // 256), min(Tq, 256), kv8),
            "launches_per_run": len(views), "us_per_run": round(us, 1), "algorithmic_bytes_per_run": alg,
            "GB/s": round(alg / us / 1e3, 1), "frac_of_8TB/s": round(alg / us / 1e3 / HBM_PEAK_GBS, 3),
            "TFLOP/s": round(flops / us / 1e6, 1)}


def attention_kernel_name(units, Tq, kv8):
    """The kernel rest_tree_attention launches for `units` (batch, head) slabs of Tq <= 256 query rows (the
    library's plan: streams of 2, 4 or 8 wavefronts by the number of query rows; few units of at most 64 rows
    take the split plan)."""
    kv = "true" if kv8 else "false"
    if Tq <= 64 and units <= 128:
        return f"tree_attn_split_kernel<{kv}>"
    return f"tree_attn_bf16_kernel<{2 if Tq <= 64 else 4 if Tq <= 128 else 8}, {kv}>"


def profiled_traffic(workload):
    """HBM bytes per attention launch of this workload as counted by rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE) and
    kept under profiles/: a figure from a file, not from this run.  It is reported only while the kernel source it
    was counted on is the one being benchmarked (the file records the source's SHA-256)."""
    import hashlib
    path = os.path.join(ROOT, "profiles", f"tree_attn_bf16_{workload}_traffic.json")
    src = os.path.join(ROOT, "paper_2311_08252_amd", "csrc", "attention.hip")
    try:
        rec = json.load(open(path))
        if rec.get("attention_hip_sha256") != hashlib.sha256(open(src, "rb").read()).hexdigest():
            return None, f"profiles/{os.path.basename(path)} is for an older kernel source: not reported"
        return rec.get("hbm_bytes_per_launch"), f"profiles/{os.path.basename(path)} (rocprofv3 --pmc, counted {rec.get('captured', '?')})"
    except Exception:
        return None, None


def side_measurements(rest, torch, synth, corp, index, w, q, k, v, out, tree, P, scale, prm):
    """Untimed-in-`value` extras: retrieval alone (batch 1 and a 4096-context batch), attention launched layer
    by layer, acceptance alone."""
    dev = q.device
    res = {}

    def timed(fn, iters):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters

    ctx_b, len_b = synth.make_contexts(corp, 4096, w.ctx_len, w.query_seed + 1)
    d_ctx, d_len = torch.from_numpy(ctx_b).to(dev), torch.from_numpy(len_b).to(dev)
    big = rest.Tree.empty(4096, w.max_nodes, dev)
    ms = timed(lambda: rest.rest_retrieve(index, d_ctx, d_len, out=big, **prm), 10)
    res["retrieve_batch4096_contexts_per_s"] = round(4096 / (ms * 1e-3), 1)
    one = rest.Tree.empty(1, w.max_nodes, dev)
    lat = []
    for j in range(8):
        lat.append(timed(lambda: rest.rest_retrieve(index, d_ctx[j:j + 1], d_len[j:j + 1], out=one, **prm), 20))
    # launched from Python one call at a time, the binding's host time per call (about 20 us) hides the kernel ...
    res["retrieve_batch1_host_launched_us"] = [round(x * 1e3, 1) for x in lat]
    # ... so the same 20 calls are also captured once into a HIP graph and replayed: the kernel plus the gap between
    # two dependent launches, with no host time in between (the call is one kernel launch and nothing else)
    side = torch.cuda.Stream()
    lat = []
    for j in range(8):
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            rest.rest_retrieve(index, d_ctx[j:j + 1], d_len[j:j + 1], out=one, **prm)
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                for _ in range(20):
                    rest.rest_retrieve(index, d_ctx[j:j + 1], d_len[j:j + 1], out=one, **prm)
        torch.cuda.synchronize()
        lat.append(timed(graph.replay, 10) / 20)
        del graph
    res["retrieve_batch1_us"] = [round(x * 1e3, 1) for x in lat]
    # inside a step the attention launch has swept the caches before every retrieval: two graphs, 16 x (attention,
    # retrieval of context j) and 16 x attention alone; their difference per pair is what a retrieval adds to a step
    both, alone = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
    per_batch = tree.tree_mask.shape[0] > 1
    amask = tree.tree_mask if per_batch else tree.tree_mask[0]
    aws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(rest.make_attn_desc(q, k, v, out, P, scale, per_batch)), 16),
                      dtype=torch.uint8, device=dev)
    with torch.cuda.stream(side):
        rest.rest_tree_attention(q, k, v, amask, P, scale, out=out, workspace=aws)
        torch.cuda.synchronize()
        with torch.cuda.graph(both, stream=side):
            for j in range(16):
                rest.rest_tree_attention(q, k, v, amask, P, scale, out=out, workspace=aws)
                rest.rest_retrieve(index, d_ctx[j:j + 1], d_len[j:j + 1], out=one, **prm)
        with torch.cuda.graph(alone, stream=side):
            for j in range(16):
                rest.rest_tree_attention(q, k, v, amask, P, scale, out=out, workspace=aws)
    torch.cuda.synchronize()
    t_both = min(timed(both.replay, 5) for _ in range(3))
    t_alone = min(timed(alone.replay, 5) for _ in range(3))
    res["retrieve_inside_step_us"] = round((t_both - t_alone) * 1e3 / 16, 1)
    del both, alone

    # the same datastore left in pinned host memory (what one larger than the GPU's memory would need): the kernels
    # read it in place over the host link
    if corp.tokens.size <= 200_000_000:
        h_corpus = torch.empty(corp.tokens.shape, dtype=torch.from_numpy(corp.tokens[:1]).dtype, pin_memory=True)
        h_corpus.copy_(torch.from_numpy(corp.tokens))
        sa_dev = index.suffix_array()
        h_sa = torch.empty(sa_dev.shape, dtype=sa_dev.dtype, pin_memory=True)
        h_sa.copy_(sa_dev)
        del sa_dev
        torch.cuda.synchronize()
        hidx = rest.rest_index_from_sa(h_corpus, h_sa)
        lat = [timed(lambda: rest.rest_retrieve(hidx, d_ctx[j:j + 1], d_len[j:j + 1], out=one, **prm), 20) for j in range(8)]
        res["retrieve_batch1_host_resident_datastore_us"] = [round(x * 1e3, 1) for x in lat]
        del hidx, h_corpus, h_sa

    # the index as a file: suffix array through a pinned staging buffer to a temporary file and back (fingerprint of the
    # stream computed on the GPU both ways)
    if corp.tokens.size <= 200_000_000:
        import tempfile
        with tempfile.TemporaryDirectory() as td:
            path = os.path.join(td, "bench.restsa")
            t0 = time.time()
            rest.rest_index_save(index, path)
            res["index_save_s"] = round(time.time() - t0, 3)
            t0 = time.time()
            again = rest.rest_index_load(path, index._corpus)
            torch.cuda.synchronize()
            res["index_load_s"] = round(time.time() - t0, 3)
            res["index_file_MB"] = round(os.path.getsize(path) / 1e6, 1)
            del again

    Nb = q.shape[0]
    mask = tree.tree_mask[0]

    ms = timed(lambda: rest.rest_tree_attention(q, k, v, mask, P, scale, out=out), 20)
    res["attn_single_launch_us"] = round(ms * 1e3, 1)

    # the cache steps either side of verification, all layers in one call each: rotary embedding of the draft
    # tokens + append of their keys/values (reads q, k, v of the T tokens, writes q and two cache rows per token),
    # and the move of the accepted path's rows (here: a path of 8)
    T, H = q.shape[2], q.shape[1]
    q2, kn, vn = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    for t in (q2, kn, vn):
        t.copy_(q)
    pos = tree.pos_ids[0]
    ms = timed(lambda: rest.rest_rope_append(q2, kn, vn, k, v, pos, P), 20)
    by = 6 * Nb * H * T * 128 * 2
    res["rope_append_us"] = round(ms * 1e3, 1)
    res["rope_append_GBps"] = round(by / (ms * 1e-3) / 1e9, 1)
    apath = torch.tensor([[0, 2, 5, 9, 14, 20, 27, 35] + [-1] * (w.cont_len - 8)], dtype=torch.int32, device=dev)
    alen = torch.tensor([8], dtype=torch.int32, device=dev)
    ms = timed(lambda: rest.rest_kv_compact(k, v, apath, alen, T, P), 20)
    res["kv_compact_path8_us"] = round(ms * 1e3, 1)
    res["kv_compact_GBps"] = round(4 * Nb * H * 8 * 128 * 2 / (ms * 1e-3) / 1e9, 1)

    # nucleus sampling of the model's token at the root and the T draft positions (vocabulary 32000, temperature 0.8,
    # top-p 0.95: the paper's code-generation setting), the input of rest_accept when decoding is not greedy
    g = torch.Generator(device=dev)
    g.manual_seed(77)
    logits = torch.randn((1 + T, 32000), generator=g, device=dev) * 2.0
    logits[:, :8] += 9.0
    u = torch.rand(1 + T, generator=g, device=dev)
    sid = torch.empty(1 + T, dtype=torch.int32, device=dev)
    ws_s = torch.empty(rest.rest_sample_ids_workspace_bytes(1 + T, 128256), dtype=torch.uint8, device=dev)
    ms = timed(lambda: rest.rest_sample_ids(logits, u, 0.8, 0.95, out=sid, workspace=ws_s), 20)
    res["sample_ids_65x32000_us"] = round(ms * 1e3, 1)
    res["sample_ids_65x32000_GBps"] = round((1 + T) * 32000 * 4 / (ms * 1e-3) / 1e9, 1)
    big_logits = torch.randn((1 + T, 128256), generator=g, device=dev) * 2.0
    big_logits[:, :8] += 9.0
    ms = timed(lambda: rest.rest_sample_ids(big_logits, u, 0.8, 0.95, out=sid, workspace=ws_s), 20)
    res["sample_ids_65x128256_us"] = round(ms * 1e3, 1)
    del big_logits

    # the step with its cache steps: retrieve -> embed + append -> attention -> accept -> compact (greedy ids)
    ctx1, len1 = d_ctx[:1], d_len[:1]
    ids = torch.zeros((1, 1 + T), dtype=torch.int32, device=dev)
    al = torch.empty(1, dtype=torch.int32, device=dev)
    ap = torch.empty((1, w.cont_len), dtype=torch.int32, device=dev)
    nx = torch.empty(1, dtype=torch.int32, device=dev)
    desc = rest.make_attn_desc(q2, k, v, out, P, scale, False)
    ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc), 16), dtype=torch.uint8, device=dev)

    def full_step():
        rest.rest_retrieve(index, ctx1, len1, out=one, **prm)
        rest.rest_rope_append(q2, kn, vn, k, v, one.pos_ids[0], P)
        rest.rest_tree_attention(q2, k, v, one.tree_mask[0], P, scale, out=out, workspace=ws)
        rest.rest_accept(ids, one, w.cont_len, al, ap, nx)
        rest.rest_kv_compact(k, v, ap, al, T, P)

    ms = timed(full_step, 50)
    res["step_with_cache_steps_us"] = round(ms * 1e3, 1)

    # the same on an 8-bit (E4M3) cache with per-(layer, head) scales: half the cache bytes per step
    sc_k = torch.full((Nb * H,), 0.5, dtype=torch.float32, device=dev)
    sc_v = torch.full((Nb * H,), 0.5, dtype=torch.float32, device=dev)
    k8 = (k.float() / 0.5).to(torch.float8_e4m3fn).view(torch.uint8)
    v8 = (v.float() / 0.5).to(torch.float8_e4m3fn).view(torch.uint8)
    ms = timed(lambda: rest.rest_tree_attention(q, k8, v8, mask, P, scale, out=out, k_scale=sc_k, v_scale=sc_v), 20)
    res["attn_8bit_cache_single_launch_us"] = round(ms * 1e3, 1)
    res["attn_8bit_cache_GBps"] = round(Nb * H * (2 * (P + T) * 128 + 2 * T * 128 * 2) / (ms * 1e-3) / 1e9, 1)
    desc8 = rest.make_attn_desc(q2, k8, v8, out, P, scale, False, k_scale=sc_k, v_scale=sc_v)
    ws8 = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc8), 16), dtype=torch.uint8, device=dev)

    def full_step_8bit():
        rest.rest_retrieve(index, ctx1, len1, out=one, **prm)
        rest.rest_rope_append(q2, kn, vn, k8, v8, one.pos_ids[0], P, k_scale=sc_k, v_scale=sc_v)
        rest.rest_tree_attention(q2, k8, v8, one.tree_mask[0], P, scale, out=out, workspace=ws8, k_scale=sc_k, v_scale=sc_v)
        rest.rest_accept(ids, one, w.cont_len, al, ap, nx)
        rest.rest_kv_compact(k8, v8, ap, al, T, P)

    ms = timed(full_step_8bit, 50)
    res["step_with_cache_steps_8bit_cache_us"] = round(ms * 1e3, 1)
    return res


def attention_sweep(rest, torch, synth, np, dev):
    """Tree attention alone over draft-tree sizes and KV lengths at the 7B head shape (32 layers x 32 heads x 128,
    one launch), random tries with branching <= 8 and depth <= 16."""
    rows = []
    for T in (16, 64, 128, 256):
        mask = torch.from_numpy(synth.random_tree(T, 14 + T)[3].view(np.int64)).to(dev)
        for P in (1024, 4096, 8192):
            g = torch.Generator(device=dev)
            g.manual_seed(T * 100000 + P)
            q = torch.randn((32, 32, T, 128), generator=g, device=dev).to(torch.bfloat16)
            k = torch.randn((32, 32, P + T, 128), generator=g, device=dev).to(torch.bfloat16)
            v = torch.randn((32, 32, P + T, 128), generator=g, device=dev).to(torch.bfloat16)
            out = torch.empty_like(q)
            scale = 1.0 / float(np.sqrt(128.0))
            desc = rest.make_attn_desc(q, k, v, out, P, scale, False)
            ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc), 16), dtype=torch.uint8, device=dev)
            for _ in range(3):
                rest.rest_tree_attention(q, k, v, mask, P, scale, out=out, workspace=ws)
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(10):
                rest.rest_tree_attention(q, k, v, mask, P, scale, out=out, workspace=ws)
            b.record()
            torch.cuda.synchronize()
            us = a.elapsed_time(b) / 10 * 1e3
            alg = 1024 * (2 * (P + T) * 128 * 2 + 2 * T * 128 * 2) + T * ((T + 63) // 64) * 8
            rows.append({"T": T, "P": P, "us": round(us, 1), "GB/s": round(alg / us / 1e3, 1),
                         "frac_of_8TB/s": round(alg / us / 1e3 / HBM_PEAK_GBS, 3)})
            del q, k, v, out, ws
    # grouped-query attention as a view: 32 layers x 8 K/V heads, g query heads of 64 draft tokens stacked along the
    # row axis of each (Tq = 64 g rows, mask_rows = 64); 8-bit cache as a second variant
    mask = torch.from_numpy(synth.random_tree(64, 78)[3].view(np.int64)).to(dev)
    for g_heads in (4, 8):
        for P in (2048, 8192):
            for kv8 in (False, True):
                g = torch.Generator(device=dev)
                g.manual_seed(7000 + g_heads * 100 + P)
                Tq = 64 * g_heads
                q = torch.randn((32, 8, Tq, 128), generator=g, device=dev).to(torch.bfloat16)
                k, v = (torch.randn((32, 8, P + 64, 128), generator=g, device=dev) for _ in range(2))
                if kv8:
                    k, v = (x.to(torch.float8_e4m3fn).view(torch.uint8) for x in (k, v))
                else:
                    k, v = (x.to(torch.bfloat16) for x in (k, v))
                out = torch.empty_like(q)
                scale = 1.0 / float(np.sqrt(128.0))
                desc = rest.make_attn_desc(q, k, v, out, P, scale, False, 0, 64)
                ws = torch.empty(max(rest.rest_tree_attention_workspace_bytes(desc), 16), dtype=torch.uint8, device=dev)
                for _ in range(3):
                    rest.rest_tree_attention(q, k, v, mask, P, scale, out=out, workspace=ws, mask_rows=64)
                torch.cuda.synchronize()
                a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(10):
                    rest.rest_tree_attention(q, k, v, mask, P, scale, out=out, workspace=ws, mask_rows=64)
                b.record()
                torch.cuda.synchronize()
                us = a.elapsed_time(b) / 10 * 1e3
                alg = 256 * (2 * (P + 64) * 128 * (1 if kv8 else 2) + 2 * Tq * 128 * 2)
                rows.append({"grouped_query_heads": g_heads, "kv_heads": 8, "T": 64, "P": P, "cache": "e4m3" if kv8 else "bf16",
                             "us": round(us, 1), "GB/s": round(alg / us / 1e3, 1),
                             "TFLOP/s": round(256 * 4.0 * Tq * (P + 64) * 128 / us / 1e6, 1)})
                del q, k, v, out, ws
    return rows


def ablation(rest, torch, synth, np, dev):
    """The paper's ablations as sweeps on synthetic data: draft strategy (Trie top-c vs at most eight random candidates
    of eight tokens), n_max and c, each reported as M = mean number of tokens generated per verification step
    (accepted draft tokens + 1).  The "model" is a deterministic toy, a 4-gram model of the datastore with back-off
    (most frequent continuation), so drafts hit often but not always, and suffixes longer than its order cannot
    help.  Retrieval and acceptance run on the GPU through the library, the toy model on the host."""
    w = synth.WORKLOADS["tiny"]
    corp = synth.make_corpus(w.n_tokens, w.corpus_seed, w.n_motifs)
    tok = corp.tokens.astype(np.int64)
    V = 32000
    tables = {}
    for order in (4, 3, 2):                          # most frequent next token after each `order`-gram of the datastore
        key = np.zeros(tok.size - order, dtype=np.int64)
        for j in range(order):
            key = key * V + tok[j:tok.size - order + j]
        nxt = tok[order:]
        idx = np.lexsort((nxt, key))
        key, nxt = key[idx], nxt[idx]
        run_start = np.flatnonzero(np.r_[True, (key[1:] != key[:-1]) | (nxt[1:] != nxt[:-1])])
        run_len = np.diff(np.r_[run_start, key.size])
        rk, rn = key[run_start], nxt[run_start]
        best = np.lexsort((rn, -run_len, rk))         # per key: longest run first, smaller token on ties
        first = np.r_[True, rk[best][1:] != rk[best][:-1]]
        tables[order] = dict(zip(rk[best][first].tolist(), rn[best][first].tolist()))

    def model(last4):
        """next token given the last four tokens: the datastore's most frequent continuation of the longest of its
        4-, 3-, 2-gram suffixes that occurs there, else a hash"""
        for order in (4, 3, 2):
            kk = 0
            for t in last4[4 - order:]:
                kk = kk * V + t
            hit = tables[order].get(kk)
            if hit is not None:
                return hit
        return (last4[-2] * 31 + last4[-1] * 17 + 7) % V

    index = rest.rest_build_index(torch.from_numpy(corp.tokens).to(dev), 4)
    prompts = [corp.tokens[s:s + 48].astype(np.int32) for s in (1000, 250_000, 500_000, 750_000)]

    def run(n_max, c, random_seqs, cont_len, n_new=160, max_matches=None, strided=False):
        gen, steps = 0, 0
        for pi, prompt in enumerate(prompts):
            seq = [int(x) for x in prompt]
            made = 0
            while made < n_new:
                ctx = torch.tensor([seq[-64:]], dtype=torch.int32, device=dev)
                ln = torch.tensor([ctx.shape[1]], dtype=torch.int32, device=dev)
                tree = rest.rest_retrieve(index, ctx, ln, n_max=n_max, n_min=min(2, n_max),
                                          max_matches=max_matches or w.max_matches, cont_len=cont_len, max_nodes=c,
                                          random_seqs=random_seqs, seed=1000 * pi + steps, strided=strided)
                n = int(tree.n_nodes[0])
                t_tok = tree.draft_tokens[0, :n].cpu().tolist()
                t_par = tree.parent_idx[0, :n].cpu().tolist()
                ids = np.zeros((1, 1 + c), dtype=np.int32)
                ids[0, 0] = model(seq[-4:])
                paths = []
                for i in range(n):           # the model's token after node i: a function of the last four tokens there
                    path = (paths[t_par[i]] if t_par[i] >= 0 else seq[-4:]) + [t_tok[i]]
                    paths.append(path[-4:])
                    ids[0, 1 + i] = model(paths[i])
                alen, apath, nxt = rest.rest_accept(torch.from_numpy(ids).to(dev), tree, cont_len)
                a = int(alen[0])
                seq += [t_tok[j] for j in apath[0, :a].cpu().tolist()] + [int(nxt[0])]
                made += a + 1
                gen += a + 1
                steps += 1
        return round(gen / steps, 3)

    res = {"datastore_tokens": w.n_tokens, "prompts": len(prompts), "tokens_per_prompt": 160,
           "M_trie_c64_nmax16": run(16, 64, 0, 10), "M_random_8x8_nmax16": run(16, 64, 8, 8),
           "M_by_n_max_trie_c64": {n: run(n, 64, 0, 10) for n in (2, 4, 8, 16)},
           "M_by_c_trie_nmax16": {c: run(16, c, 0, 10) for c in (4, 16, 64, 256)},
           # which occurrences a small cap keeps (short suffixes, so that match sets are large)
           "M_nmax2_by_max_matches_head_vs_evenly_spaced": {
               K: [run(2, 64, 0, 10, max_matches=K), run(2, 64, 0, 10, max_matches=K, strided=True)] for K in (8, 32, 128)}}
    return res


def cpu_baseline(np, torch, corp, ctx_np, w, q, k, v, out, trees, ids, P, scale, step, B=1):
    """The plain CPU oracle on a bounded sample of the same workload, on this machine's host cores."""
    import oracle
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    n_ret = 3
    t0 = time.perf_counter()
    cpu_trees = [oracle.draft_tree(corp.tokens, ctx_np[i], w.n_max, w.n_min, w.max_matches, w.cont_len, w.max_nodes,
                                   one_pass=corp.tokens.size > 600_000_000)
                 for i in range(n_ret)]
    t_ret = (time.perf_counter() - t0) / n_ret * B
    # attention: a seeded sample of (layer, head) slabs incl. the first and the last
    step(0)
    torch.cuda.synchronize()
    Nb, H = q.shape[0], q.shape[1]
    rng = np.random.default_rng(1234)
    picks = {(0, 0), (Nb - 1, H - 1)}
    while len(picks) < 48:
        picks.add((int(rng.integers(Nb)), int(rng.integers(H))))
    picks = sorted(picks)
    all_masks = trees[0].tree_mask.cpu().numpy().view(np.uint64)          # [B, c, words]
    slab_mask = [all_masks[a if B > 1 else 0] for a, _ in picks]
    slabs = [(q[a, b].float().cpu().numpy(), k[a, b].float().cpu().numpy(), v[a, b].float().cpu().numpy()) for a, b in picks]
    t0 = time.perf_counter()
    refs = [oracle.tree_attention(qq, kk, vv, mm, P, scale) for (qq, kk, vv), mm in zip(slabs, slab_mask)]
    t_attn = (time.perf_counter() - t0) * (Nb * H) / len(picks)
    err = max(float(np.abs(out[a, b].float().cpu().numpy() - r).max()) for (a, b), r in zip(picks, refs))
    t0 = time.perf_counter()
    for i in range(n_ret):
        oracle.accept(ids[0][i].cpu().numpy() if B > 1 else ids[i][0].cpu().numpy(), cpu_trees[i].draft_tokens,
                      cpu_trees[i].parent_idx, cpu_trees[i].n_nodes, w.cont_len)
    t_acc = (time.perf_counter() - t0) / n_ret * B
    total = t_ret + t_attn + t_acc
    base = {"value": round(1.0 / total, 4), "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"retrieval+Trie: {n_ret} of the contexts, scaled to the {B} of a step: {t_ret:.3f} s; attention: {len(picks)} of "
                      f"{Nb * H} (layer, head) slabs in float64, scaled to all: {t_attn:.3f} s; accept {t_acc * 1e6:.0f} us"}
    return base, err


if __name__ == "__main__":
    sys.exit(main())
