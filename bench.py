#!/usr/bin/env python3
"""Benchmark of the tree-verification step on one MI355X.

A step = one whole verification cycle on device-resident inputs: ancestor mask, embedding,
all decoder layers (tree attention + projections), LM head + argmax, greedy walk, KV
compaction (goose_verify_step).  Default workload: the 7B shape, B=64 spine tree, KV prefix
1024, consecutive steps with the accepted path committed between steps.

Prints ONE JSON line.  `value` = steps/s; `roofline` prices the dominant kernel (gate/up
projection GEMM) against the 8 TB/s HBM peak from live HIP-event timings; `cpu_baseline` is the
fp64 NumPy oracle timed on this machine's host cores on a bounded sample.
"""
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
    # name: (shape, B, P0, tree generator(seed), default steps)
    "7b_B64_P1024": ("7b", 64, 1024, "spine_7b", 100),
    "13b_B80_P2048": ("13b", 80, 2048, "spine_13b", 100),
    "33b_B80_P4096": ("33b", 80, 4096, "spine_33b", 50),
    "7b_stress_B128_P16384": ("7b", 128, 16384, "spine_stress", 50),
    "7b_balanced_B128_P16384": ("7b", 128, 16384, "balanced", 50),
    "small_B64_P200": ("small_bf16", 64, 200, "spine_7b", 20),
    "llama3_8b_B64_P1024": ("llama3_8b", 64, 1024, "spine_7b", 100),
    "qwen3_8b_B64_P1024": ("qwen3_8b", 64, 1024, "spine_7b", 100),
    "7b_f16_B64_P1024": ("7b_f16", 64, 1024, "spine_7b", 100),
}


COPY_PROBE_BYTES = 256 << 20


def recorded_traffic(workload):
    """What the committed profiler summary of this workload says (rocprofv3 FETCH_SIZE + WRITE_SIZE runs,
    scaled by the copy probe): HBM bytes per launch of the gate/up kernel, HBM bytes of a whole step,
    when it was recorded and for which sources.  Counters cannot be read from inside this process; the
    summary names the commands that produced it.  The figures are reported only when the summary was
    recorded for the sources of this very build (hash over csrc/ and goose.h), else as null."""
    from paper_2604_02047_amd.profiling import source_hash
    rel = f"profiles/traffic_{workload}.txt"
    out = {"gate_up_bytes": None, "step_bytes": None, "source": None}
    try:
        with open(os.path.join(ROOT, rel)) as f:
            lines = f.read().splitlines()
    except OSError:
        return out
    date = sha = None
    for line in lines:
        m = line.split()
        try:
            if line.startswith("recorded "):
                date, sha = m[1], m[-1]
            elif line.startswith("last step of the run:"):
                out["step_bytes"] = int(round((float(m[m.index("fetch") + 1]) + float(m[m.index("write") + 1])) * 1e6))
            # the SwiGLU epilogue is template argument 4 == 1 of k_gemm_bf16<MT, NW, TERMS, EPI, ..>
            elif line.startswith("k_gemm_bf16<") and line.split(">")[0].split(",")[3].strip() == "1" \
                    and out["gate_up_bytes"] is None:
                out["gate_up_bytes"] = int(round((float(m[-2]) + float(m[-1])) * 1e6))
        except (ValueError, IndexError):
            pass
    same = sha is not None and sha == source_hash()
    out["source"] = f"{rel}, recorded {date} for sources {sha}" + ("" if same else " (NOT this build: figures withheld)")
    if not same:
        out["gate_up_bytes"] = out["step_bytes"] = None
    return out


def cap_for(P0, B, total_steps):
    """Slots per head of the KV cache for a run of `total_steps` steps from a prefix of P0 (a step commits
    at most about 20 slots); the launches of a step are sized for cache lengths up to cap - B."""
    return (P0 + total_steps * 20 + 2 * B + 63) // 64 * 64


def make_tree(kind, seed):
    import goose_inputs as gi
    return {"spine_7b": lambda: gi.tree_spine_7b(seed), "spine_13b": gi.tree_spine_13b,
            "spine_33b": gi.tree_spine_33b, "spine_stress": gi.tree_spine_stress,
            "balanced": gi.tree_balanced}[kind]()


def step_bytes(shape, B, P):
    """Algorithmic HBM bytes of one step: every weight once, the KV prefix once, the tail rows written and read."""
    es = 4 if shape.dtype == "f32" else 2
    w = shape.n_layers * shape.layer_param_count() * es
    head = shape.vocab * shape.hidden * es
    kv_prefix = 2 * P * shape.kv_dim * es * shape.n_layers
    kv_tail = 2 * 2 * B * shape.kv_dim * es * shape.n_layers
    return w + head + kv_prefix + kv_tail


def greedy_lookahead(gm, root, n):
    """The model's next n greedy tokens after `root`, by n single-node steps; the cache length is restored."""
    import goose_inputs as gi
    P_keep = gm.P
    tree = gi.tree_single()
    out, tok = [], root
    for _ in range(n):
        r = gm.verify_step_calls([tok], tree.parent, tree.is_spine, commit=True)
        tok = r["bonus"]
        out.append(tok)
    gm.set_P(P_keep)
    return np.asarray(out, dtype=np.int32)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="7b_B64_P1024", choices=sorted(WORKLOADS))
    ap.add_argument("--drafts", default="planted", choices=["planted", "random"])
    ap.add_argument("--graph", type=int, default=1, help="replay each step as a captured HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--harvest", type=int, default=0, metavar="K",
                    help="also harvest every cycle's logits into [vocab][K] successor tables (not part of the headline step)")
    ap.add_argument("--requests", type=int, default=1, metavar="N",
                    help="N requests with trees of --request-budget nodes verified per step in one pass "
                         "(goose_verify_step_batched), timed beside the same requests verified one after the other")
    ap.add_argument("--request-budget", type=int, default=32)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also launch the library's 256 MiB copy kernel (calibrates profiler traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the verification pass of one request does not shard); "
              f"--gpus {args.gpus} is not supported.", file=sys.stderr)
        sys.exit(2)

    import torch
    import goose_inputs as gi
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    shape_name, B, P0, tree_kind, dflt_steps = WORKLOADS[args.workload]
    shape = gi.SHAPES[shape_name]
    K = args.steps if args.steps is not None else dflt_steps
    W = args.warmup
    total = K + W
    cap = cap_for(P0, B, total)
    P_max = cap - B

    def log(msg):
        print(f"[bench] {msg}", file=sys.stderr, flush=True)

    if args.requests > 1:
        return bench_batched(args, shape, P0, K, W, log)

    t0 = time.time()
    gm = GooseModel(ModelDesc.from_shape(shape), B, cap,
                    lambda l: gi.layer_weights(shape, args.seed, l, dev),
                    gi.embedding(shape, args.seed, dev), gi.lm_head(shape, args.seed, dev),
                    gi.final_norm(shape, args.seed, dev))
    torch.cuda.synchronize()
    log(f"model {shape.name} resident ({gm.packed_layers.numel() / 1e9:.2f} GB packed) in {time.time() - t0:.1f}s")

    # ---- prefill P0 random tokens through the verification path itself (chain trees, all rows kept)
    prefix = gi.prefix_tokens(args.seed, P0, shape.vocab)
    done = 0
    while done < P0:
        n = min(B, P0 - done)
        ch = gi.tree_chain(n)
        r = gm.verify_step_calls(prefix[done:done + n], ch.parent, ch.is_spine, commit=False)
        done += n
        gm.set_P(done)
    root0 = int(r["argmax"][n - 1].item())
    log(f"prefill done, P={gm.P}")

    # ---- staging buffers of a step (device resident)
    # tokens | parents | spine tags of the current step in one record: staged with one small copy
    cur_rec = torch.zeros(9 * B, dtype=torch.uint8, device=dev)
    cur_tok = cur_rec[0:4 * B].view(torch.int32)
    cur_par = cur_rec[4 * B:8 * B].view(torch.int32)
    cur_spn = cur_rec[8 * B:9 * B]
    next_root = torch.zeros(1, dtype=torch.int32, device=dev)

    bound = {"P_max": P_max}  # upper bound of the device-resident P that sizes the launches

    succ_ids = succ_sc = None
    if args.harvest:
        succ_ids = torch.full((shape.vocab, args.harvest), -1, dtype=torch.int32, device=dev)
        succ_sc = torch.zeros((shape.vocab, args.harvest), dtype=torch.float32, device=dev)

    def one_step():
        gm.verify_step_fused(cur_tok, cur_par, cur_spn, B, bound["P_max"], next_root=next_root, succ_ids=succ_ids,
                             succ_scores=succ_sc)

    # ---- rehearsal (untimed): fixes the inputs of every step.  Planted drafts follow the model's own
    # continuation, so they depend on what earlier steps accepted; this pass runs the same entry point
    # as the timed pass, reads the outcome back each step and records the trees.
    # The launches are sized from an upper bound of the device-resident P (it picks the number of
    # key splits, hence the order of the attention sums): a serving loop knows how far a request
    # can grow; here the bound is a guess of 3 slots per step, checked by the rehearsal itself and
    # widened if the walk outgrew it.  Rehearsal and timed run use the same bound.
    bound["P_max"] = min(P_max, P0 + 3 * total)
    while True:
        trees, toks, P_hist, acc_hist = [], [], [], []
        root = root0
        gm.set_P(P0)
        for t in range(total):
            tree = make_tree(tree_kind, t)
            tk = gi.draft_tokens_uniform(args.seed * 7919 + t, tree.parent, shape.vocab, root)
            if args.drafts == "planted":
                cont = greedy_lookahead(gm, root, 6)
                tk = gi.plant_drafts(args.seed * 104729 + t, tree.parent, tree.is_spine, tk, cont, shape.vocab,
                                     p_spine=0.6, p_branch=0.5, p_grand=0.3)
            P_hist.append(gm.P)
            cur_tok.copy_(torch.as_tensor(tk.astype(np.int32)))
            cur_par.copy_(torch.as_tensor(tree.parent.astype(np.int32)))
            cur_spn.copy_(torch.as_tensor(tree.is_spine.astype(np.uint8)))
            one_step()
            torch.cuda.synchronize()
            gm.P = int(gm.d_P.item())
            trees.append(tree)
            toks.append(tk)
            acc_hist.append(int(gm.accept_len.item()))
            root = int(gm.bonus.item())
        P_final = gm.P
        assert P_final + B <= cap
        if max(P_hist) <= bound["P_max"] or bound["P_max"] == P_max:
            break
        log(f"P reached {max(P_hist)} > bound {bound['P_max']}: rehearsing again with a wider bound")
        bound["P_max"] = min(P_max, bound["P_max"] + 3 * total)
    log(f"rehearsal done: mean accepted drafts/step {np.mean(acc_hist):.2f}, P {P0} -> {P_final} "
        f"(launch bound {bound['P_max']})")

    # ---- device-resident inputs of the timed run
    rec_all = torch.as_tensor(np.stack([np.concatenate([tk.astype(np.int32).view(np.uint8),
                                                        tr.parent.astype(np.int32).view(np.uint8),
                                                        tr.is_spine.astype(np.uint8)])
                                        for tk, tr in zip(toks, trees)]), device=dev)

    def stage(t):  # tiny device-to-device copies; the root is the previous step's bonus token
        cur_rec.copy_(rec_all[t])
        if t > 0:
            cur_tok[0:1].copy_(next_root)

    graph = None
    if args.graph:
        try:
            gm.set_P(P0)
            stage(0)
            s = torch.cuda.Stream()
            s.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(s):
                one_step()  # warm the stream before capture
            torch.cuda.current_stream().wait_stream(s)
            torch.cuda.synchronize()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=s):
                one_step()
            torch.cuda.synchronize()
        except Exception as e:  # capture unavailable: plain launches (still the HIP path)
            log(f"graph capture failed ({e}); timing plain launches")
            graph = None

    def run(n_from, n_to):
        for t in range(n_from, n_to):
            stage(t)
            if graph is not None:
                graph.replay()
            else:
                one_step()

    # ---- timed region
    gm.set_P(P0)
    run(0, W)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    run(W, total)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    elapsed = t2 - t1
    P_end = int(gm.d_P.item())
    if P_end != P_final:
        log(f"ERROR: replay ended at P={P_end}, rehearsal at P={P_final}")
        sys.exit(4)
    ms_per_step = elapsed / K * 1e3
    bytes_timed = sum(step_bytes(shape, B, P_hist[t]) for t in range(W, total))
    achieved = bytes_timed / elapsed / 1e9

    if args.copy_probe:
        from paper_2604_02047_amd.binding import goose_copy_probe
        src = torch.ones(COPY_PROBE_BYTES, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            goose_copy_probe(src, dst, COPY_PROBE_BYTES)
        torch.cuda.synchronize()
        del src, dst

    # ---- per-kernel timing with HIP events on the launch stream, over the same steps
    roofline, kernels = None, None
    rec = recorded_traffic(args.workload)
    if not args.no_kernel_timing:
        gm.set_P(P0)
        for t in range(W):
            stage(t)
            one_step()
        torch.cuda.synchronize()
        gm.ctx.goose_profile_enable(True)
        prof = {}
        for t in range(W, total):
            stage(t)
            one_step()
            if (t - W) % 32 == 31 or t == total - 1:   # (the library times a bounded number of launches per read)
                for k, (ms, n) in gm.ctx.goose_profile_read().items():
                    prof[k] = (prof.get(k, (0.0, 0))[0] + ms, prof.get(k, (0.0, 0))[1] + n)
        gm.ctx.goose_profile_enable(False)
        kernels = {k: {"avg_us": ms / max(n, 1) * 1e3, "launches": n} for k, (ms, n) in prof.items() if n}
        # what a pair of events reads with nothing between them (part of every figure above)
        pairs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(200)]
        for a, b in pairs:
            a.record()
            b.record()
        torch.cuda.synchronize()
        floor_us = float(np.median([a.elapsed_time(b) for a, b in pairs])) * 1e3
        es = 2
        gu_bytes = 2 * shape.ffn * shape.hidden * es + B * shape.hidden * es + B * shape.ffn * es
        gu = kernels["gemm_gate_up_swiglu"]
        ach = gu_bytes / (gu["avg_us"] * 1e-6) / 1e9
        roofline = {"kernel": "k_gemm_bf16<MT,NW,EPI_SWIGLU> (gate/up projection + SwiGLU)", "bound": "hbm",
                    "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(ach / HBM_PEAK_GBPS, 4), "traffic": rec["gate_up_bytes"],
                    "traffic_source": rec["source"],
                    "bytes_per_launch": gu_bytes, "avg_us": round(gu["avg_us"], 2),
                    "timing": "HIP events around each launch on the launch stream, averaged over the timed steps",
                    "empty_event_pair_us": round(floor_us, 2)}

    # ---- CPU baseline: the oracle on a bounded sample (two layers + LM head of the same step)
    cpu = None
    if not args.no_cpu_baseline:
        n_cpu = max(2, min(8, int(round(8 * 6.7e9 / (shape.n_layers * shape.layer_param_count())))))
        cpu = cpu_baseline(shape, gm, args.seed, [(trees[t], toks[t], P_hist[t]) for t in range(W, min(total, W + n_cpu))], log)

    out = {
        "metric": "tree-verify steps/s + achieved HBM GB/s, 7B-shape, B=64 spine tree, KV 1024"
                  if args.workload == "7b_B64_P1024" else f"tree-verify steps/s, {args.workload}",
        "value": round(K / elapsed, 2), "unit": "steps/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": shape.dtype, "data": "synthetic",
        "config": {"workload": args.workload, "shape": shape.name, "B": B, "P0": P0, "P_end": P_end,
                   "tree": tree_kind, "drafts": args.drafts, "launch": "hipGraph per step" if graph else "plain",
                   "mean_accepted_drafts_per_step": round(float(np.mean(acc_hist[W:])), 3),
                   "harvest_top_k": args.harvest},
        "draft_tokens_verified_per_s": round(B * K / elapsed, 1),
        "tokens_emitted_per_s": round(float(np.sum(np.asarray(acc_hist[W:]) + 1)) / elapsed, 1),
        "achieved_GBps": round(achieved, 1), "hbm_frac": round(achieved / HBM_PEAK_GBPS, 4),
        "algorithmic_GB_per_step": round(bytes_timed / K / 1e9, 3),
        # HBM bytes of one step by the hardware counters (profiles/traffic_<workload>.txt, same build only)
        "counter_GB_per_step": None if rec["step_bytes"] is None else round(rec["step_bytes"] / 1e9, 3),
        # evidence that the matrix cores keep up with the stream (not the bound): 2 flops per weight per node
        # for the projections and the LM head, 4 * B * (P + B) * hidden per layer for the attention
        "achieved_TFLOPs": round(sum(2.0 * B * (shape.n_layers * shape.layer_param_count() + shape.vocab * shape.hidden)
                                     + 4.0 * B * (P_hist[t] + B) * shape.n_heads * shape.head_dim * shape.n_layers
                                     for t in range(W, total)) / elapsed / 1e12, 1),
        "roofline": roofline, "cpu_baseline": cpu, "kernels_avg_us": kernels,
    }
    print(json.dumps(out), flush=True)


def bench_batched(args, shape, P0, K, W, log):
    """Cross-request batched verification (the batch sweep of App. D): N requests, each with its own KV
    cache (prefix P0) and a tree of `request_budget` nodes with random draft tokens, share one pass
    over the weights per step.  Timed as one HIP graph per step, beside the same requests verified one
    after the other through goose_verify_step.  Prints one JSON line; value = request-steps/s."""
    import torch
    import goose_inputs as gi
    from paper_2604_02047_amd import ModelDesc
    from paper_2604_02047_amd.runner import GooseModel

    dev = torch.device("cuda:0")
    n, Br = args.requests, args.request_budget
    rows = n * ((Br + 31) // 32 * 32)
    total = K + W
    cap = (P0 + 2 * total * 2 + 2 * Br + 63) // 64 * 64   # random drafts: a request grows by about one slot per step
    P_max = cap - Br
    gm = GooseModel(ModelDesc.from_shape(shape), min(128, rows), cap,
                    lambda l: gi.layer_weights(shape, args.seed, l, dev), gi.embedding(shape, args.seed, dev),
                    gi.lm_head(shape, args.seed, dev), gi.final_norm(shape, args.seed, dev), max_rows=rows)
    i32 = dict(dtype=torch.int32, device=dev)
    reqs = []
    for r in range(n):
        kc, vc = torch.zeros_like(gm.kcache), torch.zeros_like(gm.vcache)
        gm.kcache, gm.vcache = kc, vc
        gm.set_P(0)
        prefix = gi.prefix_tokens(args.seed + 31 * r, P0, shape.vocab)
        done = 0
        while done < P0:
            m = min(128, rows, P0 - done)
            ch = gi.tree_chain(m)
            out = gm.verify_step_calls(prefix[done:done + m], ch.parent, ch.is_spine, commit=False)
            done += m
            gm.set_P(done)
        log(f"request {r} prefilled")
        tree = gi.tree_random(Br, seed=r, spine_len=min(8, Br - 1))
        tokens = gi.draft_tokens_uniform(args.seed + r, tree.parent, shape.vocab, int(out["argmax"][m - 1].item()))
        t, p, s = gm.stage_tree(tokens, tree.parent, tree.is_spine)
        reqs.append({"tokens": t.clone(), "parent": p.clone(), "is_spine": s.clone(), "B": Br, "P_max": P_max,
                     "kcache": kc, "vcache": vc, "P": torch.full((1,), P0, **i32), "accept_len": torch.zeros(1, **i32),
                     "path": torch.zeros(rows, **i32), "bonus": torch.zeros(1, **i32),
                     "next_root": torch.zeros(1, **i32)})
    log(f"{n} requests prefilled to P={P0}, {Br} nodes each ({rows} rows per pass)")
    argmax_all = torch.zeros(rows, **i32)

    def batched():
        gm.ctx.goose_verify_step_batched(gm.model_ptrs(), reqs, argmax_all)
        for q in reqs:
            q["tokens"][0:1].copy_(q["next_root"])

    def one_by_one():
        for q in reqs:
            gm.kcache, gm.vcache = q["kcache"], q["vcache"]
            gm.ctx.goose_verify_step(gm.model_ptrs(), {
                "tokens": q["tokens"], "parent": q["parent"], "is_spine": q["is_spine"], "P": q["P"],
                "argmax": argmax_all, "accept_len": q["accept_len"], "path": q["path"], "bonus": q["bonus"],
                "next_root": q["next_root"], "logits": None, "margin": None, "succ_ids": None, "succ_scores": None,
                "harvest_k": 0}, Br, P_max)
            q["tokens"][0:1].copy_(q["next_root"])

    def timed(fn):
        for q in reqs:
            q["P"].fill_(P0)
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            fn()
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        if args.graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=s):
                fn()
            torch.cuda.synchronize()
            step = g.replay
        else:   # plain launches (what the profiler's counter passes use)
            step = fn
        for q in reqs:
            q["P"].fill_(P0)
        for _ in range(W):
            step()
        torch.cuda.synchronize()
        log(f"{fn.__name__}: timing {K} steps")
        t1 = time.perf_counter()
        for _ in range(K):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        P_end = [int(q["P"].item()) for q in reqs]
        assert max(P_end) <= P_max, (P_end, P_max)
        return dt, P_end

    dt_b, P_b = timed(batched)
    dt_s, P_s = timed(one_by_one)
    if P_b != P_s:
        log(f"ERROR: batched run ended at P={P_b}, one-by-one at P={P_s}")
        sys.exit(4)
    es = 2
    w_bytes = (shape.n_layers * shape.layer_param_count() + shape.vocab * shape.hidden) * es
    kv_bytes = n * shape.n_layers * 2 * shape.kv_dim * es * (P0 + (sum(P_b) / n - P0) / 2 + 2 * Br)
    out = {"metric": f"batched tree-verify request-steps/s, {args.workload}, {n} requests x {Br} nodes",
           "value": round(n * K / dt_b, 2), "unit": "request-steps/s", "n_gpus": 1, "steps": K, "warmup": W,
           "ms_per_step": round(dt_b / K * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": shape.dtype, "data": "synthetic",
           "config": {"workload": args.workload, "shape": shape.name, "requests": n, "B_per_request": Br,
                      "rows_per_pass": rows, "P0": P0, "P_end": P_b, "drafts": "random",
                      "launch": "hipGraph per step" if args.graph else "plain"},
           "one_by_one_ms_per_step": round(dt_s / K * 1e3, 4), "speedup_over_one_by_one": round(dt_s / dt_b, 3),
           "draft_tokens_verified_per_s": round(n * Br * K / dt_b, 1),
           "achieved_GBps": round((w_bytes + kv_bytes) / (dt_b / K) / 1e9, 1),
           "hbm_frac": round((w_bytes + kv_bytes) / (dt_b / K) / 1e9 / HBM_PEAK_GBPS, 4),
           # projections + LM head only (2 flops per weight per row); dense bf16 MFMA peak 2500 TFLOP/s
           "projection_TFLOPs": round(2.0 * n * Br * (w_bytes / es) / (dt_b / K) / 1e12, 1)}
    out["mfma_frac"] = round(out["projection_TFLOPs"] / 2500.0, 4)
    # beyond 128 stacked rows the projections meet the matrix cores: priced against the dense MFMA peak of
    # the operand type, as a whole-step rate (matrix flops of all projections / step time; the kernels' own
    # durations and matrix-core counters are in profiles/*_batched_*.txt).  No oracle timing in this mode.
    out["roofline"] = {"kernel": "projections of the step (k_gemm_rows beyond 128 rows, k_gemm_bf16 up to 128)",
                       "bound": "mfma" if rows > 128 else "hbm",
                       "achieved": out["projection_TFLOPs"] if rows > 128 else out.get("achieved_GBps"),
                       "peak": 2500.0 if rows > 128 else HBM_PEAK_GBPS, "unit": "TFLOP/s" if rows > 128 else "GB/s",
                       "frac": out["mfma_frac"] if rows > 128 else out.get("hbm_frac"), "traffic": None}
    out["cpu_baseline"] = None
    print(json.dumps(out), flush=True)


def cpu_baseline(shape, gm, seed, steps_in, log):
    """Times the NumPy fp64 oracle on the first timed steps of this very run: the same trees and draft
    tokens, each step's own committed KV prefix (read back from the device: the prefix is an input of the
    step on both sides), the same weights, through ALL decoder layers, the LM head, the argmax and the
    walk.  One layer's weights are converted to fp64 at a time, outside the timed region (the GPU side
    is timed with its weights resident too); only the oracle's arithmetic is timed."""
    import torch
    import goose_inputs as gi
    from oracle import goose_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1

    def f64(t):
        return t.detach().to("cpu").to(torch.float64).numpy()

    n_steps, L = len(steps_in), shape.n_layers
    log(f"cpu baseline: {n_steps} whole steps through the {L}-layer oracle")
    om = orc.OracleModel(shape.n_heads, shape.head_dim, shape.rope_base, shape.rms_eps, [None] * L,
                         f64(gm.embed), f64(gi.lm_head(shape, seed, gm.device)),
                         f64(gi.final_norm(shape, seed, gm.device)), n_kv_heads=shape.kv_heads, qk_norm=shape.qk_norm)
    P_top = max(P for _, _, P in steps_in)
    kr, vr = gm.k_rows(0, P_top), gm.v_rows(0, P_top)   # slots below a step's P still hold that step's prefix
    steps = []
    t_total = 0.0
    for tree, toks, P in steps_in:
        ta = time.perf_counter()
        anc, depth = orc.ancestor_mask(tree.parent)
        steps.append({"tree": tree, "toks": toks, "P": P, "pos": P + depth,
                      "allow": np.concatenate([np.ones((tree.B, P), dtype=bool), anc], axis=1),
                      "x": om.embed[np.asarray(toks).astype(np.int64)]})
        t_total += time.perf_counter() - ta
    for l in range(L):
        w = {k: f64(v) for k, v in gi.layer_weights(shape, seed, l, gm.device).items()}
        Kc, Vc = f64(kr[l]), f64(vr[l])
        ta = time.perf_counter()
        for st in steps:
            st["x"], _, _ = orc.decoder_layer(om, w, st["x"], Kc[:, :st["P"]], Vc[:, :st["P"]], st["pos"], st["allow"])
        t_total += time.perf_counter() - ta
        del w, Kc, Vc
    ta = time.perf_counter()
    for st in steps:
        logits = orc.final_logits(om, st["x"])
        x_hat = orc.argmax_lowest(logits)
        orc.greedy_walk(st["tree"].parent, st["toks"], st["tree"].is_spine, x_hat)
    t_total += time.perf_counter() - ta
    t_step = t_total / n_steps
    log(f"cpu baseline: {n_steps} steps x {L} layers + heads {t_total:.2f}s -> {t_step:.2f}s/step on {threads} threads")
    return {"value": round(1.0 / t_step, 5), "unit": "steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"the first {n_steps} timed steps of this run (same trees, draft tokens and KV prefixes), "
                      f"all {L} decoder layers + LM head + argmax + walk",
            "extrapolated": False, "blas_threads": int(threads), "nproc": int(os.cpu_count() or 1),
            "seconds_measured": round(t_total, 2)}


if __name__ == "__main__":
    main()
