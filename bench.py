#!/usr/bin/env python3
"""Benchmark of the tree-verification step on one MI355X.

A "step" is one pass of the whole hot path: ghd_verify_stack_argmax (32 decoder
layers + LM head over a 64-node tree against a 2048-token KV cache, 7B-shaped;
the row argmaxes are reduced in the LM-head finish) followed by ghd_accept_path
(greedy acceptance of the longest matching root path).  Inputs are synthetic (random fp16 weights, random cache),
already resident in HBM when the timed region starts.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload stack7b]
"""
import argparse
import ctypes as C
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0     # MI355X published HBM3E peak


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_gpu_model(wl, B, model, w, device, capacity=None):
    s = w.shape
    capacity = capacity or w.capacity
    layers, caches = [], []
    for l in range(s.L):
        layers.append(model.upload_layer(wl.layer_weights(s, w.seed, l, device=device), s.d, device))
        caches.append(model.upload_cache(*wl.kv_cache(s, capacity, w.kv_len, w.seed, l, device=device),
                                         device=device))
        if l % 8 == 7:
            log("  built layer %d/%d" % (l + 1, s.L))
    head = model.upload_head(wl.head_weights(s, w.seed, device=device), device)
    return model.build_stack(s, capacity, layers, caches, head)


def decode_loop(torch, B, wl, stack, w, stream, steps, K=5, R=10):
    """Whole predict-then-verify steps back to back (ghd_spec_step: embed, verify, accept,
    commit, draft), with the one host read per step that tells the caller how far the
    context grew.  The drafting heads are untrained synthetic matrices, so acceptance stays
    near one token per step: the figure shows what a full step costs, not what trained heads
    would accept."""
    dev = "cuda"
    s = w.shape
    acc = wl.head_accuracies(K, R)
    parent, rank, expect = B.ghd_tree_build(acc.tolist(), w.M)
    M = len(parent)
    embed = wl.embedding_table(s, w.seed, device=dev)
    heads = B.ghd_pack_weight(wl.drafting_heads(s, K, w.seed, device=dev))
    spec = B.SpecState(stack, embed, heads, K, R)
    pd = torch.tensor(parent, dtype=torch.int32, device=dev)
    rd = torch.tensor(rank, dtype=torch.int32, device=dev)
    tokens = torch.from_numpy(wl.draft_tokens(M, s.V, w.seed)).to(dev)
    res = torch.zeros(2 + M, dtype=torch.int32, device=dev)
    cap = stack.cfg.kv_capacity
    ws = B.workspace(spec.workspace_bytes(M, cap - M))
    res_host = torch.zeros(2 + M, dtype=torch.int32).pin_memory()
    kv, produced, done = w.kv_len, 0, 0
    with torch.cuda.stream(stream):
        for _ in range(3):                       # warm-up on the same cache rows
            B.ghd_spec_step(spec, pd, rd, w.kv_len, tokens, res, ws)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        while done < steps and kv + M <= cap:
            B.ghd_spec_step(spec, pd, rd, kv, tokens, res, ws)
            res_host.copy_(res, non_blocking=True)
            stream.synchronize()
            n = int(res_host[0])
            kv += n
            produced += n
            done += 1
        dt = time.perf_counter() - t0
    head_bytes = 2 * K * s.V * s.H
    out = {"steps": done, "tokens": produced, "tokens_per_s": round(produced / dt, 1),
           "us_per_step": round(dt / done * 1e6, 1), "mean_accepted": round(produced / done, 3),
           "tree_nodes": M, "heads": K, "candidates_per_head": R,
           "expected_accepted_at_synthetic_accuracies": round(expect, 3),
           "drafting_head_bytes": head_bytes,
           "note": "untrained synthetic heads; one 4-byte host read per step included"}
    out["drafts_right_at_synthetic_accuracies"] = planted_loop(
        torch, B, wl, spec, stack, embed, heads, w, stream, steps, K, R, acc, parent, rank, pd, rd, ws)
    return out


def planted_loop(torch, B, wl, spec, stack, embed, heads, w, stream, steps, K, R, acc, parent, rank,
                 pd, rd, ws):
    """The same loop with drafts that are right as often as the synthetic accuracy table
    says: the model's own continuation is first produced one token at a time (same
    library, one-node tree); in every tree step candidate r of head k then carries the true
    token of its slot with probability acc[k][r] (at most one candidate per head), a wrong
    one otherwise.  The drafting heads still run (their cost is in the time); their output
    is replaced by these drafts.  Shows the loop accepting several tokens per step, as
    trained heads would make it, and reports whether the produced tokens are those of
    one-at-a-time decoding."""
    import numpy as np
    dev = "cuda"
    s = w.shape
    M = len(parent)
    cap = stack.cfg.kv_capacity
    need = min(steps * (K + 1) + K + 1, cap - w.kv_len - M)
    # one token at a time
    one_p = torch.tensor([-1], dtype=torch.int32, device=dev)
    one_r = torch.zeros(1, dtype=torch.int32, device=dev)
    tok1 = torch.tensor([int(wl.draft_tokens(M, s.V, w.seed)[0])], dtype=torch.int32, device=dev)
    res1 = torch.zeros(3, dtype=torch.int32, device=dev)
    ws1 = B.workspace(spec.workspace_bytes(1, cap - 1))
    first = int(tok1[0])
    with torch.cuda.stream(stream):
        seq = torch.zeros(need, dtype=torch.int32, device=dev)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(need):
            B.ghd_spec_step(spec, one_p, one_r, w.kv_len + i, tok1, res1, ws1)
            seq[i:i + 1].copy_(res1[1:2])          # tok1 already holds it for the next step
        torch.cuda.synchronize()
        seq_dt = time.perf_counter() - t0
    want = seq.cpu().numpy().tolist()
    # the tree loop
    depth = [0] * M
    for i in range(1, M):
        depth[i] = depth[parent[i]] + 1
    rng = np.random.default_rng([w.seed, 4242])
    cum = np.cumsum(acc, axis=1)
    tokens_host = torch.zeros(M, dtype=torch.int32).pin_memory()
    tokens = torch.zeros(M, dtype=torch.int32, device=dev)
    res = torch.zeros(2 + M, dtype=torch.int32, device=dev)
    res_host = torch.zeros(2 + M, dtype=torch.int32).pin_memory()
    kv, got, done, last = w.kv_len, [], 0, first
    with torch.cuda.stream(stream):
        t0 = time.perf_counter()
        while done < steps and len(got) + K + 1 <= need:
            future = want[len(got):len(got) + K]
            u = rng.random(K)
            right = [int(np.searchsorted(cum[k], u[k], side="right")) for k in range(K)]   # == R: none
            th = tokens_host.numpy()
            th[0] = last
            for i in range(1, M):
                k = depth[i] - 1
                th[i] = future[k] if rank[i] == right[k] else (future[k] + 1 + rank[i]) % s.V
            tokens.copy_(tokens_host, non_blocking=True)
            B.ghd_spec_step(spec, pd, rd, kv, tokens, res, ws)
            res_host.copy_(res, non_blocking=True)
            stream.synchronize()
            n = int(res_host[0])
            path = res_host[2:2 + n].tolist()
            got += [int(th[i]) for i in path[1:]] + [int(res_host[1])]
            last = int(res_host[1])
            kv += n
            done += 1
        dt = time.perf_counter() - t0
    return {"steps": done, "tokens": len(got), "tokens_per_s": round(len(got) / dt, 1),
            "us_per_step": round(dt / done * 1e6, 1), "mean_accepted": round(len(got) / done, 3),
            "equals_one_at_a_time_decoding": got == want[:len(got)],
            "one_at_a_time_tokens_per_s": round(need / seq_dt, 1),
            "speedup_over_one_at_a_time": round(len(got) / dt / (need / seq_dt), 2),
            "note": "drafts planted from the model's own continuation with the synthetic "
                    "accuracies; host builds and uploads the 64 draft tokens every step"}


def time_steps(torch, B, stack, x_in, parent, tokens, kv_len, ws, aws, logits, res, amax, stream,
               steps, warmup):
    # the row argmaxes come out of the LM-head finish; no logits are written
    def step():
        B.ghd_verify_stack_argmax(stack, x_in, parent, kv_len, ws=ws, amax=amax)
        B.ghd_accept_path(amax, tokens, parent, res=res)

    with torch.cuda.stream(stream):
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        e0 = torch.cuda.Event(enable_timing=True)
        e1 = torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
    return e0.elapsed_time(e1) / steps, wall_ms / steps


def step_spread(torch, B, stack, x_in, parent, tokens, kv_len, ws, aws, logits, res, amax, stream, steps):
    """Per-step durations (an event between every two steps, no host synchronisation inside):
    median, 10th and 90th percentile in microseconds."""
    with torch.cuda.stream(stream):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        ev[0].record(stream)
        for i in range(steps):
            B.ghd_verify_stack_argmax(stack, x_in, parent, kv_len, ws=ws, amax=amax)
            B.ghd_accept_path(amax, tokens, parent, res=res)
            ev[i + 1].record(stream)
        torch.cuda.synchronize()
    us = sorted(ev[i].elapsed_time(ev[i + 1]) * 1e3 for i in range(steps))
    pick = lambda q: us[min(steps - 1, int(round(q * (steps - 1))))]
    return {"median_us": round(pick(0.5), 1), "p10_us": round(pick(0.1), 1), "p90_us": round(pick(0.9), 1)}


def recorded_traffic(workload):
    """HBM bytes per launch of the linear-layer kernel from the committed counter
    summary (FETCH_SIZE and WRITE_SIZE runs, each scaled by a copy kernel of known
    size); None when the kernel sources have changed since, or for a workload the
    counters were not taken on."""
    path = os.path.join(ROOT, "profiles", "k_linear_%s_hbm_traffic.md" % workload)
    if not os.path.exists(path):
        return None
    from paper_2505_23219_amd.profile_summary import source_digest
    vals = {}
    for line in open(path):
        if line.startswith(("traffic_bytes_per_launch:", "source_sha256:")):
            k, v = line.split(":", 1)
            vals[k] = v.strip()
    if vals.get("source_sha256") != source_digest():
        return None
    try:
        return int(vals["traffic_bytes_per_launch"])
    except (KeyError, ValueError):
        return None


def timed_launches(torch, B, stack, x_in, parent, kv_len, ws, logits, stream, what, steps):
    lib = B.lib()
    lib.ghd_debug_profile_read.argtypes = [C.POINTER(C.c_float)]
    tot_ms, launches = 0.0, 0
    with torch.cuda.stream(stream):
        for _ in range(steps):
            lib.ghd_debug_profile(what)
            B.ghd_verify_stack(stack, x_in, parent, kv_len, logits=logits, ws=ws)
            lib.ghd_debug_profile(0)
            torch.cuda.synchronize()
            ms = C.c_float(0)
            launches += lib.ghd_debug_profile_read(C.byref(ms))
            tot_ms += ms.value
    return tot_ms, launches


def linear_roofline(torch, B, stack, x_in, parent, kv_len, ws, logits, stream, w, steps):
    """Dominant kernel: the persistent skinny-GEMM kernel (it streams every weight byte of
    the step).  Its launches are bracketed by HIP events inside the library, on the launch
    stream.  Where the QKV layer shares its launch with the attention, that launch is timed
    and reported on its own ("qkv_attention": QKV weights + the layer's cache), and the
    linear figure covers the launches that are linear layers only (output, gate|up and down
    projections and the LM head): achieved = their weight bytes / launches / average
    duration (every launch reads its matrix exactly once)."""
    s = w.shape
    qkv_bytes = 2 * s.L * 3 * s.H * s.H
    weight_bytes = 2 * (s.L * (3 * s.H * s.H + s.H * s.H + 2 * s.F * s.H + s.H * s.F) + s.V * s.H)
    kv_bytes = 2 * 2 * s.L * s.nh * s.d * (kv_len + w.M)
    tot_ms, launches = timed_launches(torch, B, stack, x_in, parent, kv_len, ws, logits, stream, 1, steps)
    per_step = launches // steps
    fused_ms, fused_n = timed_launches(torch, B, stack, x_in, parent, kv_len, ws, logits, stream, 3, steps)
    fused = fused_n > 0
    lin_bytes = weight_bytes - (qkv_bytes if fused else 0)
    per_launch_bytes = lin_bytes / per_step
    avg_ms = tot_ms / launches
    achieved = per_launch_bytes / (avg_ms * 1e-3) / 1e9
    out = {"bound": "hbm", "kernel": "k_linear<MT, R, RB>", "achieved": round(achieved, 1),
           "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
           "traffic": recorded_traffic(w.name), "launches_per_step": per_step,
           "avg_launch_us": round(avg_ms * 1e3, 2),
           "algorithmic_bytes_per_launch": int(per_launch_bytes)}
    if fused:
        b = (qkv_bytes + kv_bytes) / (fused_n // steps)
        out["qkv_attention"] = {"kernel": "k_qkv_attn<MT, R, D>", "launches_per_step": fused_n // steps,
                                "avg_launch_us": round(fused_ms / fused_n * 1e3, 2),
                                "algorithmic_bytes_per_launch": int(b),
                                "achieved": round(b / (fused_ms / fused_n * 1e-3) / 1e9, 1)}
    else:
        att_ms, att_n = timed_launches(torch, B, stack, x_in, parent, kv_len, ws, logits, stream, 2, steps)
        out["attention"] = {"kernel": "k_attention<MT, D>", "launches_per_step": att_n // steps,
                            "avg_launch_us": round(att_ms / att_n * 1e3, 2),
                            "algorithmic_bytes_per_launch": int(kv_bytes / (att_n // steps)),
                            "achieved": round(kv_bytes / (att_n // steps) / (att_ms / att_n * 1e-3) / 1e9, 1)}
    return out


def sweep(torch, B, model, wl, stream, sets=4, iters=40):
    """Tree-size sweep: one 7B-shaped layer, 2048 cached tokens, M in 1..128, chain and
    bushy trees.  `sets` distinct weight + cache sets (1.8 GB) are used round-robin so that
    every timed call streams from HBM, not from the memory-side cache."""
    dev = "cuda"
    rows = []
    shape = wl.sweep_workload(1, "chain").shape
    cap = wl.sweep_workload(128, "chain").capacity
    layers = [model.upload_layer(wl.layer_weights(shape, 3, l, device=dev), shape.d, dev) for l in range(sets)]
    caches = [model.upload_cache(*wl.kv_cache(shape, cap, 2048, 3, l, device=dev), device=dev) for l in range(sets)]
    cfg = B.make_cfg(shape, cap)
    for M in (1, 4, 8, 16, 32, 64, 128):
        for kind in (("chain",) if M == 1 else ("chain", "bushy")):
            w = wl.sweep_workload(M, kind)
            parent = torch.from_numpy(w.parent).to(dev)
            x = wl.activations(M, shape.H, 3).float().to(dev)
            ws = B.workspace(B.ghd_workspace_bytes(cfg, M, 2048))
            with torch.cuda.stream(stream):
                for i in range(sets):
                    B.ghd_verify_layer(cfg, layers[i], *caches[i], x, parent, 2048, ws=ws)
                torch.cuda.synchronize()
                e0 = torch.cuda.Event(enable_timing=True)
                e1 = torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for i in range(iters):
                    B.ghd_verify_layer(cfg, layers[i % sets], *caches[i % sets], x, parent, 2048, ws=ws)
                e1.record(stream)
                torch.cuda.synchronize()
            require_clean_status(B, ws, "the sweep at M=%d (%s)" % (M, kind))
            us = e0.elapsed_time(e1) / iters * 1e3
            nbytes = 2 * (4 * shape.H * shape.H + 3 * shape.H * shape.F) + 4 * shape.H * (2048 + M)
            rows.append({"M": M, "tree": kind, "layer_us": round(us, 1),
                         "gbps": round(nbytes / us / 1e3, 1)})
            log("  sweep M=%3d %-5s %7.1f us  %6.1f GB/s" % (M, kind, us, nbytes / us / 1e3))
    return rows


def tree_part_comparison(torch, B, model, wl, stream, iters=200):
    """The drafted tokens' own attention block two ways (the paper's Figure 8b on this chip):
    from the nonzeros of the tree mask (one dot product per (token, ancestor) pair,
    ghd_tree_part_attention_coo) and as the masked MFMA tile of the attention kernel
    (ghd_tree_attention on a cache that holds the tree rows only), 32 heads x 128, for a
    chain, a bushy tree (depth <= 5) and a wide depth-2 tree at 64 and 128 nodes.  Each
    figure is the time of one call (set-up launch + kernel) by events on the stream."""
    dev = "cuda"
    nh, d = 32, 128
    shape = wl.ModelShape("tp", H=nh * d, nh=nh, d=d, F=8, V=8, L=1)
    rows = []
    for M in (64, 128):
        kc, vc = wl.kv_cache(shape, 128, 128, 5, 0, device=dev)
        kd, vd = model.upload_cache(kc, vc, device=dev)
        q = wl.activations(M, nh * d, 5, tag="q").reshape(M, nh, d).to(dev)
        ws = B.workspace(B.lib().ghd_attention_workspace_bytes(M, 0, nh, d))
        out = torch.empty_like(q)
        for kind, parent in (("chain", wl.tree_chain(M)), ("bushy", wl.tree_random(M, 5, 3)),
                             ("depth2", wl.tree_wide_shallow(M, 32, 4))):
            pd = torch.from_numpy(parent).to(dev)
            depth = [0] * M
            for i in range(1, M):
                depth[i] = depth[parent[i]] + 1
            res = {"M": M, "tree": kind, "mask_nonzeros": int(sum(depth) + M)}
            for name, call in (("coo_us", lambda: B.ghd_tree_part_attention_coo(q, kd, vd, pd, 0, ws=ws, out=out)),
                               ("masked_mfma_us", lambda: B.ghd_tree_attention(q, kd, vd, pd, 0, ws=ws))):
                with torch.cuda.stream(stream):
                    for _ in range(10):
                        call()
                    torch.cuda.synchronize()
                    e0 = torch.cuda.Event(enable_timing=True)
                    e1 = torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    for _ in range(iters):
                        call()
                    e1.record(stream)
                    torch.cuda.synchronize()
                res[name] = round(e0.elapsed_time(e1) / iters * 1e3, 2)
            rows.append(res)
            log("  tree part M=%3d %-6s nnz %4d: coo %6.2f us, masked MFMA tile %6.2f us"
                % (M, kind, res["mask_nonzeros"], res["coo_us"], res["masked_mfma_us"]))
    return rows


def cpu_model_name():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(wl, w, sample_layers):
    """The CPU oracle, as it stands, timed on the host cores on the same workload:
    `sample_layers` decoder layers (all of them by default), one after the other as the
    oracle's stack routine runs them, then the LM head and the acceptance.  Weights and
    cache of a layer are drawn right before its call and dropped after it (not timed), so
    the host never holds more than one layer.  If fewer layers than the model has are
    timed, the figure is scaled and says so."""
    import numpy as np
    from oracle import Oracle
    orc = Oracle("f32")
    s = w.shape
    n = min(sample_layers, s.L) if sample_layers > 0 else s.L
    x = wl.activations(w.M, s.H, w.seed).numpy().astype(np.float32)
    t_layers = 0.0
    for l in range(n):
        lw = {k: v.numpy() for k, v in wl.layer_weights(s, w.seed, l).items()}
        kc, vc = wl.kv_cache(s, w.capacity, w.kv_len, w.seed, l)
        kc, vc = kc.numpy(), vc.numpy()
        t0 = time.perf_counter()
        x = orc.verify_layer(s, lw, kc, vc, x, w.parent, w.kv_len, True)
        t_layers += time.perf_counter() - t0
        del lw, kc, vc
    head = {k: v.numpy() for k, v in wl.head_weights(s, w.seed).items()}
    t0 = time.perf_counter()
    logits = orc.lm_head(s, head["g_final"], head["Wlm"], x, True)
    orc.accept_greedy(logits, wl.draft_tokens(w.M, s.V, w.seed), w.parent)
    t_head = time.perf_counter() - t0
    full = t_layers * (s.L / n) + t_head
    threads = int(os.environ.get("OMP_NUM_THREADS", "0")) or len(os.sched_getaffinity(0))
    sample = "%d of %d layers + LM head + acceptance, M=%d, kv_len=%d; %.2f s of oracle time" % (
        n, s.L, w.M, w.kv_len, t_layers + t_head)
    if n != s.L:
        sample += ", layers scaled x%g" % (s.L / n)
    return {"value": round(full * 1e6, 1), "unit": "us", "cores": threads, "kind": "oracle",
            "sample": sample, "cpu_model": cpu_model_name(),
            "omp_num_threads": os.environ.get("OMP_NUM_THREADS"),
            "host_logical_cpus": os.cpu_count()}


def require_clean_status(B, ws, what):
    """A bounded wait that gave up inside the timed region leaves its code in the step's
    status word: such a region is not a measurement."""
    st = B.ghd_step_status(ws)
    if st != 0:
        sys.exit("bench.py: %s ended with step status %d (a workgroup wait gave up); no figure printed"
                 % (what, st))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="stack7b")
    ap.add_argument("--cpu-sample-layers", type=int, default=0,
                    help="decoder layers the CPU oracle is timed on (0 = all of them)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false",
                    help="skip the tree-size sweep (one 7B-shaped layer at tree sizes 1..128, the \"sweep\" list)")
    ap.add_argument("--loop", type=int, default=0,
                    help="also run this many whole predict-then-verify steps (adds \"decode_loop\")")
    ap.add_argument("--tree-part", action="store_true",
                    help="also time the drafted tokens' own attention block from the mask nonzeros and as a "
                         "masked MFMA tile (adds \"tree_part\")")
    ap.add_argument("--stream-probe", action="store_true",
                    help="only run the stream probe (the bare weight stream with matrix-core, dot-product and "
                         "no multiply; a program of its own built next to the library) and print its table")
    ap.add_argument("--pmc-calibrate", action="store_true",
                    help="also launch one plain 1 GiB copy kernel (for scaling profiler byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the verification step runs on a single MI355X and "
                 "there is no multi-GPU path (--gpus %d refused)" % args.gpus)

    if args.stream_probe:
        import subprocess
        probe = os.path.join(ROOT, "paper_2505_23219_amd", "ghd_stream_probe")
        if not os.path.exists(probe):
            sys.exit("%s is not built: run python -m paper_2505_23219_amd.build" % probe)
        sys.exit(subprocess.run([probe]).returncode)

    import torch
    from paper_2505_23219_amd import binding as B, model, workloads as wl
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    B.lib()
    dev = "cuda"
    w = wl.workload(args.workload)
    s = w.shape
    log("building %s: L=%d H=%d F=%d V=%d M=%d kv_len=%d" % (w.name, s.L, s.H, s.F, s.V, w.M, w.kv_len))
    # a decode loop needs cache rows for the tokens it will produce
    capacity = w.capacity + (64 * ((args.loop * 8 + 63) // 64) if args.loop else 0)
    stack = build_gpu_model(wl, B, model, w, dev, capacity)
    cfg = stack.cfg
    stream = torch.cuda.Stream()

    def inputs(M, parent_np):
        return dict(
            x_in=wl.activations(M, s.H, w.seed).to(dev),
            parent=torch.from_numpy(parent_np).to(dev),
            tokens=torch.from_numpy(wl.draft_tokens(M, s.V, w.seed)).to(dev),
            ws=B.workspace(B.ghd_workspace_bytes(cfg, M, w.kv_len)),
            aws=B.workspace(B.lib().ghd_accept_workspace_bytes(M)),
            logits=torch.empty((M, s.V), dtype=torch.float32, device=dev),
            res=torch.zeros(2 + M, dtype=torch.int32, device=dev),
            amax=torch.empty(M, dtype=torch.int32, device=dev))

    if args.pmc_calibrate:
        src = torch.zeros(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        rc = B.lib().ghd_debug_copy(C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                    C.c_size_t(src.numel() * 4), C.c_void_p(0))
        torch.cuda.synchronize()
        log("calibration copy of %d bytes: rc=%d" % (src.numel() * 4, rc))
        del src, dst
    tree = inputs(w.M, w.parent)
    ms, wall_ms = time_steps(torch, B, stack, tree["x_in"], tree["parent"], tree["tokens"], w.kv_len,
                             tree["ws"], tree["aws"], tree["logits"], tree["res"], tree["amax"],
                             stream, args.steps, args.warmup)
    require_clean_status(B, tree["ws"], "the timed tree steps")
    log("tree step: %.1f us (wall %.1f us)" % (ms * 1e3, wall_ms * 1e3))
    spread = step_spread(torch, B, stack, tree["x_in"], tree["parent"], tree["tokens"], w.kv_len,
                         tree["ws"], tree["aws"], tree["logits"], tree["res"], tree["amax"], stream,
                         max(args.steps, 20))
    require_clean_status(B, tree["ws"], "the per-step spread run")
    log("per-step spread:", spread)
    # the same model as a plain 1-token decode step: denominator of the "within 1.3x" target
    dec = inputs(1, wl.tree_chain(1))
    dec_ms, _ = time_steps(torch, B, stack, dec["x_in"], dec["parent"], dec["tokens"], w.kv_len,
                           dec["ws"], dec["aws"], dec["logits"], dec["res"], dec["amax"], stream,
                           args.steps, args.warmup)
    require_clean_status(B, dec["ws"], "the timed decode steps")
    log("decode step: %.1f us" % (dec_ms * 1e3))
    roof = linear_roofline(torch, B, stack, tree["x_in"], tree["parent"], w.kv_len, tree["ws"],
                           tree["logits"], stream, w, max(2, min(args.steps, 5)))
    require_clean_status(B, tree["ws"], "the per-launch timing run")
    log("roofline:", roof)

    step_bytes = w.algorithmic_bytes()
    gbps = step_bytes / (ms * 1e-3) / 1e9
    out = {
        "metric": "tree_verify_step_latency", "value": round(ms * 1e3, 1), "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "%s: %d-layer 7B-shaped stack + LM head, %d-node tree (depth<=5), "
                               "kv_len %d, greedy acceptance" % (w.name, s.L, w.M, w.kv_len)
                   if w.name == "stack7b" else w.name,
                   "M": w.M, "kv_len": w.kv_len, "L": s.L, "H": s.H, "F": s.F, "V": s.V},
        "step_spread": spread,
        "step_algorithmic_bytes": step_bytes,
        "step_hbm_gbps": round(gbps, 1),
        "step_hbm_frac_of_peak": round(gbps / HBM_PEAK_GBPS, 4),
        "decode_step_us": round(dec_ms * 1e3, 1),
        "tree_over_decode": round(ms / dec_ms, 3),
        "roofline": roof,
    }
    if args.loop:
        out["decode_loop"] = decode_loop(torch, B, wl, stack, w, stream, args.loop)
        log("decode loop:", out["decode_loop"])
    if args.sweep:
        del stack
        torch.cuda.empty_cache()
        out["sweep"] = sweep(torch, B, model, wl, stream)
        # the width with the most expected accepted tokens per layer-time, for the synthetic
        # head accuracies (5 heads, 10 candidates) and the latencies just measured
        rows = [r for r in out["sweep"] if r["tree"] == ("chain" if r["M"] == 1 else "bushy")]
        widths = [r["M"] for r in rows]
        i, rate = B.ghd_choose_width(wl.head_accuracies(5, 10).tolist(), widths, [r["layer_us"] for r in rows])
        out["width_choice"] = {"widths": widths, "chosen": widths[i],
                               "expected_tokens_per_layer_ms": [round(x * 1e3, 3) for x in rate]}
        log("width choice:", out["width_choice"])
    if args.tree_part:
        out["tree_part"] = tree_part_comparison(torch, B, model, wl, stream)
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on %s layers ..." % (args.cpu_sample_layers or "all"))
        out["cpu_baseline"] = cpu_baseline(wl, w, args.cpu_sample_layers)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
