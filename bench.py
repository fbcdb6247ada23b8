#!/usr/bin/env python3
"""Benchmark of the HyLRA decode-attention hot path on one MI355X.

A "step" is one hylra_decode_step: every layer of the workload, Full layers (streaming
attention + top-k) and Reuse layers (gather attention) in policy order, for one decode token
per sequence.  Inputs are synthetic, drawn on the GPU, and resident in HBM before timing.

Prints ONE JSON line: tokens/s over all layers, the roofline position of the dominant kernel
(measured live with HIP events on the launch stream), and the CPU oracle timed on the host
cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E, published peak

DTYPE = ("f32 (bf16 q/K/V in; scores, softmax and accumulation in fp32; the matrix-core kernels feed the "
         "softmax weights to P.V as a hi+lo bf16 pair = 16 mantissa bits)")


def measured_traffic(workload, kernel):
    """HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this bench,
    scaled by the copy-kernel calibration: profiles/traffic.json, written by
    `python -m paper_2602_00777_amd.profile_summary`.  None if that workload was not profiled."""
    try:
        with open(os.path.join(ROOT, "profiles", "traffic.json")) as f:
            return json.load(f).get(workload, {}).get(kernel)
    except (OSError, ValueError):
        return None


def log(msg):
    print(msg, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b_32k")
    ap.add_argument("--policy", default="hylra", choices=["hylra", "full", "jump3", "search"],
                    help="hylra = the workload's policy; full = every layer Full; jump3 = Full every 3rd layer; "
                         "search = profile an all-Full pass on the synthetic data and run the policy search")
    ap.add_argument("--theta", type=float, default=-1.0,
                    help="--policy search: similarity threshold; negative = the median similarity of adjacent layers")
    ap.add_argument("--block", type=int, default=0,
                    help="block-level variant: rows per block (TopK keeps top_k / block blocks); 0 = token level")
    ap.add_argument("--paged", type=int, default=0,
                    help="paged KV cache: rows per page (pages scattered over a pool by a random block table); 0 = contiguous")
    ap.add_argument("--ragged", action="store_true",
                    help="sequence lengths uniform in [N/4, N] instead of all N (with or without --paged)")
    ap.add_argument("--offload", type=int, default=0,
                    help="index-guided prefetch: keep the Reuse layers' caches in pinned host memory and fetch only "
                         "the selected rows over PCIe into this many staging slots (0 = everything resident)")
    ap.add_argument("--append", action="store_true",
                    help="hylra_decode_step_append: every layer first writes the current token's key / value row into "
                         "its cache (the last row; with --ragged, the row behind each sequence's length minus one)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one decode step in a HIP graph (through torch) and time its replays")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-probe", action="store_true",
                    help="skip the untimed ceilings (plain copy / streaming read of 4 GiB, bare gather of the Reuse rows)")
    ap.add_argument("--no-parity", action="store_true",
                    help="skip the untimed post-run comparison of the step's outputs with the CPU oracle")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value")
    args = ap.parse_args()

    world = int(os.environ.get("WORLD_SIZE", "1"))
    if args.gpus != 1 or world != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "--gpus %d / WORLD_SIZE %d is not supported" % (args.gpus, world), file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2602_00777_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = "cuda:0"
    w = synth.WORKLOADS[args.workload]
    policy = w.policy()
    if args.policy == "full":
        policy[:] = synth.FULL
    elif args.policy == "jump3":
        policy[:] = synth.REUSE
        policy[::3] = synth.FULL
    n_full = int((policy == synth.FULL).sum())
    n_reuse = int((policy == synth.REUSE).sum())

    t0 = time.time()
    planted = synth.planted_positions(w)
    data = []
    for l in range(w.n_layers):
        data.append(synth.make_layer(w, l, planted[l], dev))
    torch.cuda.synchronize()
    log("generated %s: %d layers, %.1f GiB of KV in %.1f s" %
        (w.name, w.n_layers, w.n_layers * w.kv_bytes_per_layer() / 2**30, time.time() - t0))
    qs, Ks, Vs = [x[0] for x in data], [x[1] for x in data], [x[2] for x in data]
    paged, lens = None, None
    if args.paged:
        table = synth.page_table(w.batch, w.ctx_len, args.paged, w.seed)
        n_pages = int(table.max()) + 1
        for l in range(w.n_layers):             # layer by layer, so that only one extra copy is alive
            Ks[l] = synth.to_pool(Ks[l], table, args.paged, n_pages)
            Vs[l] = synth.to_pool(Vs[l], table, args.paged, n_pages)
            data[l] = None
        lens = synth.ragged_lengths(w.batch, w.ctx_len, w.seed) if args.ragged else None
        paged = binding.PagedCache(torch.from_numpy(table).to(dev), args.paged, w.ctx_len,
                                   torch.from_numpy(lens).to(dev) if lens is not None else None)
        torch.cuda.synchronize()
        log("paged: %d pages of %d rows%s" % (n_pages, args.paged, ", ragged lengths %s" % lens.tolist() if lens is not None else ""))
    elif args.ragged:
        lens = synth.ragged_lengths(w.batch, w.ctx_len, w.seed)
        paged = binding.PagedCache(None, 0, w.ctx_len, torch.from_numpy(lens).to(dev))
        log("contiguous cache, ragged lengths %s" % lens.tolist())

    ctx = binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k)
    for o in args.opt:
        name, val = o.split("=")
        ctx.set_option(name, int(val))
    if args.block < 0 or (args.block and w.top_k % args.block):
        print("bench.py: --block must divide the workload's top_k (%d)" % w.top_k, file=sys.stderr)
        sys.exit(2)
    k_sel = w.top_k // args.block if args.block else w.top_k
    searched = None
    if args.policy == "search":
        if args.block or args.paged or args.ragged:
            print("bench.py: --policy search runs on the contiguous token-level layout", file=sys.stderr)
            sys.exit(2)
        # offline profiling as in the paper: full attention at every layer, top-k sets, pairwise
        # overlap, path search (on synthetic data, so the policy says nothing about a real model)
        t0 = time.time()
        sets = [ctx.full_attn_topk(qs[l], Ks[l], Vs[l], w.top_k)[1] for l in range(w.n_layers)]
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        counts = ctx.overlap_counts(sets, w.ctx_len)
        e1.record()
        torch.cuda.synchronize()
        M = binding.similarity_matrix(counts.cpu().numpy())
        theta = args.theta if args.theta >= 0 else float(np.median(np.diag(M, 1)))
        policy, n_full_found, sim = binding.policy_search(M, theta)
        searched = {"theta": round(theta, 4), "adjacent_similarity_median": round(float(np.median(np.diag(M, 1))), 4),
                    "overlap_counts_us": round(1e3 * e0.elapsed_time(e1), 1), "sum_similarity": round(sim, 3),
                    "policy": "".join("F" if a == synth.FULL else "r" for a in policy)}
        log("policy search: theta %.4f -> %s (%d Full), profiling %.1f s" % (theta, searched["policy"], n_full_found, time.time() - t0))
        n_full = int((policy == synth.FULL).sum())
        n_reuse = int((policy == synth.REUSE).sum())
        del sets
    if args.offload:
        if args.graph or args.append:
            print("bench.py: --offload is launched eagerly and without --append", file=sys.stderr)
            sys.exit(2)
        t0 = time.time()
        for l in range(w.n_layers):
            if policy[l] == synth.REUSE:
                Ks[l] = Ks[l].cpu().pin_memory()
                Vs[l] = Vs[l].cpu().pin_memory()
                data[l] = None
        log("offloaded %d Reuse layers (%.1f GiB) to pinned host memory in %.1f s" %
            (n_reuse, n_reuse * w.kv_bytes_per_layer() / 2**30, time.time() - t0))
        run, outs, idx_buf, _copy_stream = ctx.prepare_step_offloaded(policy, qs, Ks, Vs, k_sel, n_slots=args.offload,
                                                                      block=args.block, paged=paged)
    elif args.append:
        if args.block:
            print("bench.py: --append runs at token level", file=sys.stderr)
            sys.exit(2)
        gen = torch.Generator(device=dev).manual_seed(12345)
        k_new = [torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen, device=dev).to(torch.bfloat16) for _ in range(w.n_layers)]
        v_new = [torch.randn((w.batch, w.n_kv_heads, w.head_dim), generator=gen, device=dev).to(torch.bfloat16) for _ in range(w.n_layers)]
        if lens is not None:        # lengths before the append: one row fewer, so that the step attends to `lens` rows
            paged = binding.PagedCache(paged.block_table, paged.page_size, w.ctx_len, torch.from_numpy(lens - 1).to(dev))
        run, outs, idx_buf = ctx.prepare_step_append(policy, qs, k_new, v_new, Ks, Vs, k_sel, paged=paged)
    else:
        run, outs, idx_buf = ctx.prepare_step(policy, qs, Ks, Vs, k_sel, block=args.block, paged=paged)

    step = run
    if args.graph:
        # the step is kernel launches on the current stream and nothing else (no allocation, no
        # host synchronisation, no memset), so it can be captured as it is
        run()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            run()
        step = graph.replay
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps
    tokens_per_s = w.batch / (elapsed / args.steps)

    # Algorithm 2 as written runs TopK at every Full layer; the step above skips it where the set
    # would be overwritten unread (a Full layer directly followed by another).  Same outputs;
    # the step with every TopK is timed beside it.
    ms_every = None
    plain = not (args.offload or args.graph or args.append)
    if plain:
        ctx_every = binding.Context(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k,
                                    topk_every_full_layer=True)
        for o in args.opt:
            name, val = o.split("=")
            ctx_every.set_option(name, int(val))
        run_every, _, _ = ctx_every.prepare_step(policy, qs, Ks, Vs, k_sel, block=args.block, paged=paged)
        for _ in range(args.warmup):
            run_every()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            run_every()
        torch.cuda.synchronize()
        ms_every = 1e3 * (time.perf_counter() - t0) / args.steps
        ctx_every.close()

    # per-kernel durations: the same steps again, every launch bracketed by HIP events on
    # the launch stream
    ctx.profile_enable(True)
    ctx.profile_reset()
    prof_steps = max(1, min(args.steps, 4096 // (2 * w.n_layers)))
    for _ in range(prof_steps):
        run()
    torch.cuda.synchronize()
    prof = ctx.profile_read()
    ctx.profile_enable(False)
    kernels = {name: {"launches": n, "avg_us": (1e3 * ms / n if n else None)}
               for name, (n, ms) in prof.items() if n}

    B, Hq, Hkv, d, N, k = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, w.ctx_len, w.top_k
    small = B * Hq * d * 2 + B * Hq * d * 4 + B * Hkv * k_sel * 4     # q + out + idx
    rows_total = int(lens.sum()) if lens is not None else B * N        # rows a Full layer attends to
    sel_total = int(np.minimum(lens, k).sum()) if lens is not None else B * k
    full_bytes = 4 * Hkv * rows_total * d + small
    reuse_bytes = 4 * Hkv * sel_total * d + small

    def roof(label, kernel, nbytes, avg_us):
        if not avg_us:
            return None
        gbs = nbytes / (avg_us * 1e-6) / 1e9
        return {"bound": "hbm", "kernel": label, "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(gbs / HBM_PEAK_GBS, 4),
                "algorithmic_bytes": nbytes, "avg_us": round(avg_us, 2),
                "traffic": None if args.paged or args.block or args.ragged else measured_traffic(w.name, kernel)}

    def total_us(name):
        kk = kernels.get(name)
        return kk["avg_us"] * kk["launches"] / prof_steps if kk else 0.0

    # A Full layer is its streaming pass plus its second kernel (merge of the partials, TopK):
    # the headline fraction charges both to the layer's bytes; the streaming pass alone (the
    # one kernel a rocprofv3 trace shows under that name) is given beside it.
    full_layer_us = (total_us("full_attn") + total_us("full_finalize")) / n_full if n_full else 0.0
    reuse_us = (kernels.get("reuse_attn") or {}).get("avg_us") or 0.0
    full_layer = roof("full layer = streaming pass (full_attn) + merge and top-k (full_finalize), mean over the step's Full layers",
                      "full_attn", full_bytes, full_layer_us)
    full_pass = roof("full_attn (streaming pass alone)", "full_attn", full_bytes, (kernels.get("full_attn") or {}).get("avg_us"))
    reuse = roof("reuse_attn", "reuse_attn", reuse_bytes, reuse_us)
    if full_layer_us * n_full >= reuse_us * n_reuse:
        roofline, other = full_layer, reuse
    else:
        roofline, other = reuse, full_layer

    # Untimed ceilings on this machine: plain copy and streaming read of 4 GiB, and the bare gather
    # of the rows the Reuse layers read (same index sets, no arithmetic).
    probe = None
    if not args.no_probe and not (args.paged or args.block or args.offload):
        nbytes = 4 << 30
        src = torch.empty(nbytes, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        sink = torch.empty(16384, dtype=torch.uint8, device=dev)
        ctx.profile_enable(True)
        probe = {}
        for name, fn in (("copy", lambda: ctx.probe_copy(dst, src)), ("read", lambda: ctx.probe_read(src, sink))):
            fn()
            torch.cuda.synchronize()
            ctx.profile_reset()
            for _ in range(10):
                fn()
            torch.cuda.synchronize()
            n, ms = ctx.profile_read()["probe"]
            moved = nbytes * (2 if name == "copy" else 1)
            probe[name + "_GBps"] = round(moved / (ms / n * 1e-3) / 1e9, 1)
        del src, dst
        reuse_layers = [l for l in range(w.n_layers) if policy[l] == synth.REUSE]
        if reuse_layers:
            for l in reuse_layers:
                ctx.probe_gather(Ks[l], Vs[l], idx_buf, sink)
            torch.cuda.synchronize()
            ctx.profile_reset()
            for _ in range(5):
                for l in reuse_layers:          # a different layer's cache every launch: nothing stays cached
                    ctx.probe_gather(Ks[l], Vs[l], idx_buf, sink)
            torch.cuda.synchronize()
            n, ms = ctx.profile_read()["probe"]
            probe["gather_us"] = round(1e3 * ms / n, 2)
            probe["gather_GBps"] = round(4 * Hkv * sel_total * d / (ms / n * 1e-3) / 1e9, 1)
        ctx.profile_enable(False)

    # Untimed: the step's outputs against the CPU oracle on every (batch, KV head) pair of
    # sampled layers (the first Full layer that hands its set on, the first and the last Reuse
    # layer, the last Full layer); tests/test_gpu_full_size.py does all layers.
    parity = None
    if not args.no_parity and plain and not (args.paged or args.block or args.ragged):
        from tests.step_check import check_step

        fulls = [l for l in range(w.n_layers) if policy[l] == synth.FULL]
        reuses = [l for l in range(w.n_layers) if policy[l] == synth.REUSE]
        sample = {fulls[-1]}
        sample |= set([l for l in fulls if l + 1 < w.n_layers and policy[l + 1] == synth.REUSE][:1])
        if reuses:
            sample |= {reuses[0], reuses[-1]}
        run()
        torch.cuda.synchronize()
        t0 = time.time()
        res = check_step(ctx, policy, qs, Ks, Vs, w.top_k, outs, idx_buf, layers=sorted(sample))
        parity = {"layers": sorted(sample), "pairs_per_layer": B * Hkv, "out_tolerance": 2e-3,
                  "max_err_full": float("%.3g" % res["max_err_full"]), "max_err_reuse": float("%.3g" % res["max_err_reuse"]),
                  "idx_rule": "exact outside a 1e-4 score band around the k-th score",
                  "sets_differing_inside_band": res["sets_differing_in_band"], "seconds": round(time.time() - t0, 1)}
        log("parity: %s" % parity)

    cpu = None
    if not args.no_cpu_baseline and not args.paged and not args.ragged:
        cpu = cpu_baseline(w, policy, qs, Ks, Vs, n_full, n_reuse, args.block)

    line = {
        "metric": "decode-attention tokens/sec (all layers) at 32K ctx; achieved HBM GB/s vs peak" if w.ctx_len == 32768
                  else "decode-attention tokens/sec (all layers)",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": DTYPE, "data": "synthetic",
        "config": {"workload": w.name, "description": w.description, "policy": args.policy,
                   "n_layers": w.n_layers, "full_layers": n_full, "reuse_layers": n_reuse,
                   "batch": B, "n_q_heads": Hq, "n_kv_heads": Hkv, "head_dim": d, "ctx_len": N,
                   "top_k": k, "block": args.block or 1, "page_size": args.paged or None,
                   "seq_lens": lens.tolist() if lens is not None else None, "hip_graph": bool(args.graph),
                   "append": bool(args.append),
                   "kv_dtype": "bf16", "accumulate": "f32",
                   # what the library chose for the Reuse layers (hylra_get_info)
                   "reuse_launch": {"partials_per_pair": ctx.get_info("last_reuse_splits"),
                                    "wave_rows": ctx.get_info("last_reuse_wave_rows"),
                                    "merge": ("second kernel", "arrival counter", "packets", "one workgroup per pair")[
                                        ctx.get_info("last_reuse_merge")]} if n_reuse else None},
        "ms_per_step_topk_at_every_full_layer": round(ms_every, 4) if ms_every else None,
        "parity_checked": parity is not None,
        "parity": parity,
        "roofline": roofline,
        "roofline_other": other,
        "roofline_streaming_pass": full_pass,
        "kernels_us": {n: round(v["avg_us"], 2) for n, v in kernels.items()},
        "cpu_baseline": cpu,
    }
    if probe:
        line["probe"] = probe
    if searched:
        line["config"]["policy_search"] = searched
    if args.offload:
        g = kernels.get("reuse_combine")        # class 3 = the gather launches in this mode
        moved = 4 * B * Hkv * k * d
        line["config"]["offload"] = {
            "slots": args.offload, "host_resident_GiB": round(n_reuse * w.kv_bytes_per_layer() / 2**30, 1),
            "gather_us": round(g["avg_us"], 1) if g else None,
            "gather_GBps": round(moved / (g["avg_us"] * 1e-6) / 1e9, 1) if g else None,
            "pcie_peak_GBps": 64.0,
            "full_cache_transfer_ms_at_peak": round(w.kv_bytes_per_layer() / 64e9 * 1e3, 1)}
    ctx.close()
    print(json.dumps(line), flush=True)


def cpu_baseline(w, policy, qs, Ks, Vs, n_full, n_reuse, block=0, budget_s=12.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload:
    the first Full layers and the first Reuse layers of the step (up to 3 each, up to 8
    sequences of the batch), in policy order with the oracle's own index sets, repeated in
    rounds until about budget_s seconds of oracle time have been spent; the step time is
    n_full * mean(t_full) + n_reuse * mean(t_reuse), scaled to the whole batch."""
    import oracle

    threads = oracle.threads()
    nb = min(w.batch, 8)
    sample, have_full, have_reuse = [], 0, 0
    for l in range(w.n_layers):
        is_full = policy[l] == 0
        if (is_full and have_full >= 3) or (not is_full and (have_reuse >= 3 or have_full == 0)):
            continue
        sample.append((is_full, qs[l][:nb].cpu(), Ks[l][:nb].cpu(), Vs[l][:nb].cpu()))
        have_full += is_full
        have_reuse += not is_full
        if have_full >= 3 and (have_reuse >= 3 or n_reuse == 0):
            break
    t_full, t_reuse, spent, rounds = [], [], 0.0, 0
    while spent < budget_s and rounds < 100:
        idx = None
        for is_full, q, K, V in sample:
            t0 = time.perf_counter()
            if is_full:
                if block:
                    _, idx, _ = oracle.full_attn_topk_blocks(q, K, V, block, w.top_k // block)
                else:
                    _, idx, _ = oracle.full_attn_topk(q, K, V, w.top_k)
            elif block:
                oracle.reuse_block_attn(q, K, V, idx, block)
            else:
                oracle.reuse_sparse_attn(q, K, V, idx)
            dt = time.perf_counter() - t0
            (t_full if is_full else t_reuse).append(dt)
            spent += dt
        rounds += 1
    mf = sum(t_full) / len(t_full)
    mr = sum(t_reuse) / len(t_reuse) if t_reuse else 0.0
    scale = w.batch / nb
    step_s = (n_full * mf + n_reuse * mr) * scale
    return {"value": round(w.batch / step_s, 4), "unit": "tokens/s", "cores": threads, "kind": "oracle",
            "sample": "%d Full layers (mean %.3f s) and %d Reuse layers (mean %.4f s) on %d of %d sequences, "
                      "%d rounds, %.1f s of oracle time; step extrapolated as (%d*t_full + %d*t_reuse) * %g"
                      % (have_full, mf, have_reuse, mr, nb, w.batch, rounds, spent, n_full, n_reuse, scale)}


if __name__ == "__main__":
    main()
