#!/usr/bin/env python3
"""Decode throughput of the early-exit decode step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A "step" is one decode iteration of the whole batch (Algorithm 1: layer loop with exit checks, KV filling,
token selection).  The workload is the Llama-7B-shaped batch-32 configuration: random-init bf16 weights,
32 prompts of 512 uniform-random tokens prefilled through the decode step itself (full layers), then W + K
greedy decode iterations.  Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

value      = early-exit decode tokens/s (threshold 0.9, exit head after every layer), batch * K / wall time
also       = the same K iterations on the full-layer path (no exit heads) and with a threshold that never
             fires (checks paid, nothing skipped), per-kernel-class times from HIP events, roofline of the
             dominant kernel, exit-layer histogram, and the CPU oracle timed on one iteration.
"""
import argparse
import collections
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(cfg, cls):
    """Bytes one launch of a projection class must move: its weights, once."""
    d, f, V = cfg.d_model, cfg.d_ffn, cfg.vocab
    return {"qkv": 3 * d * d * 2, "o_proj": d * d * 2, "gate_up": 2 * f * d * 2, "down": d * f * 2, "head": V * d * 2}.get(cls)


def kv_bytes_per_position(cfg):
    """K and V of one cached position of one layer (what attention must read for it)."""
    return 2 * cfg.d_model * 2


def layers_with_head(cfg, upto):
    return sum(1 for i in range(1, upto + 1) if i < cfg.n_layers and i % cfg.exit_every == 0)


def iteration_bytes(cfg, kind, L, attended_layer_positions):
    """Algorithmic HBM bytes of ONE decode iteration that left at batch exit layer L.
    attended_layer_positions: sum over sequences of (layers the sequence attended in) x (positions it attends, this
    one included): L x (context + 1) under Algorithm 1, its own exit layer x (context + 1) when sequences leave on
    their own (a sequence that has left attends nothing).
    kind: "full" (no heads), "head" (an LM-head pass per checked layer), "dot" (head-less measures)."""
    n, d = cfg.n_layers, cfg.d_model
    total = L * sum(algorithmic_bytes(cfg, c) for c in ("qkv", "o_proj", "gate_up", "down"))
    total += attended_layer_positions * kv_bytes_per_position(cfg)
    if kind == "head":
        total += layers_with_head(cfg, L) * algorithmic_bytes(cfg, "head")
        if L == n:
            total += algorithmic_bytes(cfg, "head")               # the final LM-head pass
    else:
        total += algorithmic_bytes(cfg, "head")                   # one LM-head pass for the tokens
    total += (n - L) * 2 * d * d * 2                              # KV filling: K and V rows of every skipped layer
    return total


# Thresholds of the two measures that need no LM head.  The weights are random, so no value is "right": these are
# set where the batch leaves around the middle of the model (see the exit-layer histograms in the output).
SIM_THRESHOLD = {1: 0.967}
CLS_THRESHOLD = {1: 0.5}
SR_THRESHOLD = {1: 0.6}     # softmax response as the paper writes it: top-1 minus top-2 probability


def profile_figures(name, key):
    """Lines `<key> <label...> <value>` of a committed rocprofv3 summary under profiles/ (the machine-readable part)."""
    out = {}
    try:
        with open(os.path.join(ROOT, "profiles", name)) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 3 and parts[0] == key:
                    out[" ".join(parts[1:-1])] = float(parts[-1])
    except OSError:
        pass
    return out


def traffic_ratios():
    """Measured HBM bytes per algorithmic byte of each kernel class (FETCH_SIZE + WRITE_SIZE, calibrated against a
    plain copy of known size)."""
    return profile_figures("hbm_traffic_llama7b_b32_pmc.md", "traffic_ratio")


def measure_peaks(torch, B):
    """Attainable rates of this chip, measured with the library's calibration kernels (HIP events on the stream they
    run on): a plain device copy, a plain streaming read, and a register-only loop of bf16 matrix instructions."""
    st = torch.cuda.current_stream()

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for i in range(reps):
            fn(i)
        e1.record(st)
        e1.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    out = {}
    bufs = [torch.full((100 << 20,), 1.0 + i, dtype=torch.float32, device="cuda") for i in range(4)]   # 4 x 400 MiB, rotating
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(bufs[0])
    t = timed(lambda i=0: B.ee_calibration_copy(bufs[i % 3], dst), 12)
    out["copy_GBps_read_plus_write"] = 2 * bufs[0].numel() * 4 / t / 1e9
    best = 0.0
    for wgs in (256, 512, 1024, 2048):
        t = timed(lambda i=0: B.ee_calibration_read(bufs[i % 4], sink, wgs), 16)
        best = max(best, bufs[0].numel() * 4 / t / 1e9)
    out["read_GBps"] = best
    # one workgroup per compute unit, half of the loads from a weight-like stream (HBM), half from 4 MiB that everybody
    # walks (L2): what a compute unit takes in, by the loads it keeps in flight.  "own": every workgroup has its stream to
    # itself; "pairs": two workgroups of one XCD share a stream (every byte leaves HBM once and L2 twice), as the two
    # row blocks of a column block of the ring projection kernel do
    common = torch.full((1 << 20,), 3.0, dtype=torch.float32, device="cuda")
    for pairs in (False, True):
        for depth in (8, 16, 32, 48):
            t = timed(lambda i=0: B.ee_calibration_intake(bufs[i % 4], common, 256, depth, pairs, sink), 8)
            per_wg = (2 if pairs else 1) * bufs[0].numel() * 4 / 256      # bytes of the stream one workgroup reads
            out[f"intake_GBps_per_cu_{'pairs' if pairs else 'own'}_{depth * 4}_KiB_in_flight"] = 2 * per_wg / t / 1e9
    iters = 20000
    for per_simd in (1, 2):
        wgs = 256 * per_simd
        t = timed(lambda i=0: B.ee_calibration_mfma(wgs, iters, sink), 3)
        out[f"mfma_bf16_TFLOPs_{per_simd}_wavefront_per_simd"] = wgs * 4 * iters * 4 * 2.0 * 32 * 32 * 16 / t / 1e12
    steps = 8000
    for reads in (0, 8):   # the inner loop of a 128 x 128 wavefront tile alone, one workgroup per compute unit
        t = timed(lambda i=0: B.ee_calibration_mfma_tile(256, steps, reads, sink), 3)
        out[f"mfma_bf16_TFLOPs_4x4_tile_loop_{reads}_lds_fragment_reads_per_step"] = 256 * 4 * steps * 16 * 2.0 * 32 * 32 * 16 / t / 1e12
    out["note"] = "library calibration kernels, HIP events; published peaks: HBM 8000 GB/s, bf16 MFMA 2500 TFLOP/s"
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark configs (default 1: 7B shape, batch 32)")
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (debugging only; invalidates the result)")
    ap.add_argument("--profile-steps", type=int, default=8)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--peaks", action="store_true",
                    help="also measure this chip's attainable copy / read / MFMA rates with the library's calibration kernels")
    ap.add_argument("--modes", default="ee,full,never,ee+ps,sim,sr",
                    help="ee: the config's softmax-response heads; full: no heads; never: heads that never fire; "
                         "sr: softmax response as the paper writes it (top-1 minus top-2 probability); "
                         "sim / cls: hidden-state-similarity / dedicated-classifier checks (no LM head in the loop); "
                         "a +ps suffix lets each sequence leave at its own layer (extension of Algorithm 1).  "
                         "The headline value is always mode ee")
    ap.add_argument("--per-sequence", action="store_true",
                    help="modes ee, sim and cls let each sequence leave at its own layer (extension of Algorithm 1) "
                         "instead of the whole batch leaving together")
    ap.add_argument("--sim-threshold", type=float, default=0.0, help="threshold of mode sim (0: a built-in per-config value)")
    ap.add_argument("--cls-threshold", type=float, default=0.0, help="threshold of mode cls (0: a built-in per-config value)")
    ap.add_argument("--sr-threshold", type=float, default=0.0, help="threshold of mode sr (0: a built-in per-config value)")
    ap.add_argument("--synthetic-kv", action="store_true",
                    help="fill the cache with seeded random K/V instead of prefilling through the decode step "
                         "(always used when prompt lengths are ragged)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch size (exit-rate sweep members)")
    ap.add_argument("--context", type=int, default=0, help="override the context length (exit-rate sweep members)")
    ap.add_argument("--forced-layer", type=int, default=0,
                    help="force every sequence to leave at this layer (measures KV filling over the layers above it)")
    ap.add_argument("--forced-mean", type=float, default=0.0,
                    help="exit-rate sweep: force per-sequence exit layers from the truncated geometric distribution on "
                         "[8, n] with this mean instead of using the confidence")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 256 MiB device copies (copy_f32_kernel) so that byte counters can be calibrated")
    ap.add_argument("--no-graph", action="store_true", help="enqueue every iteration eagerly instead of replaying a HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2407_20272_amd import binding as B
    from paper_2407_20272_amd import workloads as W

    B.lib()                                   # no fallback: raises if the HIP library is missing
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.config]
    if args.layers:
        cfg = cfg.with_(n_layers=args.layers, name=cfg.name + f"_{args.layers}layers_DEBUG")
    if args.batch:
        cfg = cfg.with_(batch=args.batch, name=cfg.name + f"_b{args.batch}")
    if args.context:
        cfg = cfg.with_(prompt_len=args.context, min_prompt_len=args.context, name=cfg.name + f"_ctx{args.context}")
    K, Wm, P = args.steps, args.warmup, args.profile_steps
    Bsz, n = cfg.batch, cfg.n_layers
    t0 = time.time()
    w = W.make_weights(cfg, seed=0, device="cuda")
    w_cpu = None if args.no_cpu_baseline else W.weights_to(w, "cpu")
    model = B.DeviceModel(cfg, w)
    del w
    torch.cuda.empty_cache()
    lens = W.make_context_lens(cfg, seed=0)
    prompts = W.make_prompts(cfg.with_(prompt_len=min(cfg.prompt_len, 8)) if (args.synthetic_kv or cfg.min_prompt_len != cfg.prompt_len)
                             else cfg, seed=0, device="cuda")
    extra = Wm + K + P + 1
    bt, nb = W.make_block_tables(lens, extra, cfg.block_size, cfg.shuffled_blocks, 0)
    cache = B.PagedKV(cfg, nb)
    bt_dev = bt.cuda()
    max_ctx = int(lens.max()) + extra
    ws = B.Workspace(model.desc, Bsz, max_ctx)
    out_tok = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
    out_exit = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
    out_L = torch.zeros(1, dtype=torch.int32, device="cuda")
    tokens = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
    ctx = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
    batch = B.make_batch(tokens, ctx, bt_dev, max_ctx)

    # ---- prefill: teacher-forced through the decode step, no exit heads (positions 0 .. len-1) ----------
    lens_dev = lens.cuda()
    first = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
    synthetic_kv = args.synthetic_kv or int(lens.min()) != int(lens.max())
    if synthetic_kv:
        g = torch.Generator(device="cuda").manual_seed(1234)
        for i in range(n):
            cache.k[i].normal_(0.0, 0.5, generator=g)
            cache.v[i].normal_(0.0, 0.5, generator=g)
        first.copy_(prompts[:, 0])
    else:
        for t in range(int(lens.max())):
            tokens.copy_(prompts[:, t])
            ctx.fill_(t)
            B.ee_decode_iteration(model, cache, batch, 2.0, None, False, out_tok, out_exit, out_L, None, None, ws)
        first.copy_(out_tok)
    torch.cuda.synchronize()
    forced_all = None
    if args.forced_layer > 0:   # everybody leaves at this layer: the batch exit layer is known, KV filling covers n - it
        forced_all = torch.full((Wm + K + P + 4, Bsz), min(args.forced_layer, n), dtype=torch.int32, device="cuda")
    elif args.forced_mean > 0:
        forced_all = W.make_forced_exit_layers(Bsz, Wm + K + P + 4, args.forced_mean, 8, n, seed=0).cuda()
    if forced_all is not None:
        forced_cur = torch.zeros(Bsz, dtype=torch.int32, device="cuda")
        step_no = torch.zeros(1, dtype=torch.int64, device="cuda")
    setup_s = time.time() - t0

    # Per-iteration bookkeeping stays on the device so that one iteration (decode step + token feedback + position
    # advance + histograms) is a fixed sequence of kernels: it is captured once per mode into a HIP graph and
    # replayed, which removes the per-launch host cost of the ~300-400 kernels of an iteration.
    if args.calibrate_copy:
        ca = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
        cb = torch.empty_like(ca)
        for _ in range(3):
            B.ee_calibration_copy(ca, cb)
        torch.cuda.synchronize()
        del ca, cb
    L_hist = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
    E_hist = torch.zeros(n + 1, dtype=torch.int32, device="cuda")
    one1 = torch.ones(1, dtype=torch.int32, device="cuda")
    oneB = torch.ones(Bsz, dtype=torch.int32, device="cuda")
    L_last = torch.zeros(P + 1, dtype=torch.int32, device="cuda")

    variants = {"sim": model.with_conf_mode(2), "cls": model.with_conf_mode(3), "sr": model.with_conf_mode(1)}
    thr_of = {"ee": cfg.threshold, "full": 2.0, "never": 2.0, "sr": args.sr_threshold or SR_THRESHOLD.get(args.config, 0.5),
              "sim": args.sim_threshold or SIM_THRESHOLD.get(args.config, 0.99),
              "cls": args.cls_threshold or CLS_THRESHOLD.get(args.config, 0.9)}

    # Confidences of the instrumented pass only (None while the timed steps run): counts the decisions that sit
    # within NEAR_TOL of their threshold, i.e. the ones float rounding could flip against another implementation.
    NEAR_TOL = 1e-3
    conf_all = torch.empty(n, Bsz, dtype=torch.float32, device="cuda")
    conf_buf = None

    def iteration(mode):
        per_seq = args.per_sequence or mode.endswith("+ps")
        mode = mode.split("+")[0]
        thr = thr_of[mode]
        f = None
        if forced_all is not None and mode != "full" and mode != "never":
            torch.index_select(forced_all, 0, step_no % forced_all.shape[0], out=forced_cur.view(1, -1))
            step_no.add_(1)
            f = forced_cur
        how = B.EE_EXIT_NONE if mode == "full" else (
            B.EE_EXIT_PER_SEQUENCE if per_seq and mode != "never" else B.EE_EXIT_BATCH)
        B.ee_decode_iteration(variants.get(mode, model), cache, batch, thr, f, how, out_tok, out_exit, out_L, conf_buf, None, ws)
        L_hist.index_add_(0, out_L, one1)          # histograms of the timed steps (int32 indices: no cast launches)
        E_hist.index_add_(0, out_exit, oneB)
        torch.add(out_tok, 0, out=tokens)          # next iteration consumes the tokens just produced
        ctx.add_(1)

    results = {}
    prof = {}
    side = torch.cuda.Stream()
    for mode in args.modes.split(","):
        tokens.copy_(first)
        ctx.copy_(lens_dev)
        graph = None
        if not args.no_graph:
            with torch.cuda.stream(side):
                iteration(mode)                     # warm every lazy initialisation outside the capture
                torch.cuda.synchronize()
                tokens.copy_(first)
                ctx.copy_(lens_dev)
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph, stream=side):
                    iteration(mode)
            torch.cuda.synchronize()
            tokens.copy_(first)
            ctx.copy_(lens_dev)
        step = graph.replay if graph is not None else (lambda: iteration(mode))
        for _ in range(Wm):
            step()
        L_hist.zero_()
        E_hist.zero_()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(K):
            step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t1
        Lh, Eh = L_hist.cpu().tolist(), E_hist.cpu().tolist()
        base_mode = mode.split("+")[0]
        per_seq_mode = (args.per_sequence or mode.endswith("+ps")) and base_mode not in ("full", "never")
        kind = "full" if base_mode == "full" else ("dot" if base_mode in ("sim", "cls") else "head")
        mean_L = sum(i * c for i, c in enumerate(Lh)) / K
        mean_E = sum(i * c for i, c in enumerate(Eh)) / (K * Bsz)
        # positions attended per layer, summed over the batch, averaged over the timed steps (the context grows by one per step)
        positions = float(lens.sum()) + Bsz * (Wm + (K - 1) / 2.0 + 1)
        att = (mean_E if per_seq_mode else mean_L) * positions      # exit layer and context length taken as independent
        it_bytes = sum(c / K * iteration_bytes(cfg, kind, L_, 0.0) for L_, c in enumerate(Lh) if c) + att * kv_bytes_per_position(cfg)
        results[mode] = {"tokens_per_s": Bsz * K / dt, "ms_per_step": dt / K * 1e3,
                         "mean_batch_exit_layer": mean_L,
                         "batch_exit_layer_hist": {i: c for i, c in enumerate(Lh) if c},
                         "mean_seq_exit_layer": mean_E,
                         # the whole iteration against the HBM roofline: algorithmic bytes of the layers that ran
                         # (weights once per executed layer, cached K/V once per attending sequence and layer, LM head
                         # per check, K/V rows of the filled layers) over the measured time per step
                         "iteration": {"algorithmic_GB": it_bytes / 1e9, "GBps": it_bytes / (dt / K) / 1e9,
                                       "frac_hbm_peak": it_bytes / (dt / K) / 1e9 / HBM_PEAK_GBS}}
        # instrumented pass (eager): HIP events around every kernel, on the stream the kernels run on
        if P > 0:
            ctx_before = ctx.clone()
            B.ee_profile_enable(True)
            Lp = []
            near = torch.zeros(2, dtype=torch.int64, device="cuda")
            conf_buf = conf_all if (mode.split("+")[0] not in ("full",) and forced_all is None) else None
            E_steps = torch.zeros(P, Bsz, dtype=torch.int32, device="cuda")
            C_steps = torch.zeros(P, Bsz, dtype=torch.int32, device="cuda")
            for s_ in range(P):
                C_steps[s_].copy_(ctx)
                iteration(mode)
                L_last[s_].copy_(out_L[0])
                E_steps[s_].copy_(out_exit)
                if conf_buf is not None:
                    near[0] += ((conf_all - thr_of[mode.split("+")[0]]).abs() < NEAR_TOL).sum()
                    near[1] += (~torch.isnan(conf_all)).sum()
            conf_buf = None
            torch.cuda.synchronize()
            B.ee_profile_enable(False)
            results[mode]["near_threshold"] = {"tol": NEAR_TOL, "count": int(near[0]), "decisions": int(near[1]), "steps": P}
            recs = B.ee_profile_read()
            Lp = L_last[:P].cpu().tolist()
            E_cpu, C_cpu = E_steps.cpu(), C_steps.cpu()
            per_iter = len(recs) // P
            agg = collections.defaultdict(lambda: [0, 0.0, 0.0])     # launches, milliseconds, algorithmic bytes
            for it in range(P):
                for cls, layer, ms in recs[it * per_iter:(it + 1) * per_iter]:
                    # kernels of layers above the batch exit layer return at once; KV filling only runs after an
                    # early exit; the final LM pass (recorded at layer n) only when the loop reached layer n
                    executed = (Lp[it] < n) if cls == "kv_fill" else (layer == 0 or layer <= Lp[it])
                    # measures without an exit head: the one LM-head pass for the tokens (recorded at layer n) always runs
                    if base_mode in ("sim", "cls") and layer == n and cls in ("head", "norm", "combine"):
                        executed = True
                    if not executed:
                        continue
                    if cls == "kv_fill":      # K and V weight rows of every skipped layer
                        ab = (n - Lp[it]) * 2.0 * cfg.d_model * cfg.d_model * 2
                    elif cls == "attention":  # cached K/V of the sequences that still attend in this layer
                        attends = (E_cpu[it] >= layer) if per_seq_mode else torch.ones(Bsz, dtype=torch.bool)
                        ab = float((C_cpu[it][attends] + 1).sum()) * kv_bytes_per_position(cfg)
                    else:
                        ab = algorithmic_bytes(cfg, cls) or 0.0
                    a_ = agg[cls]
                    a_[0] += 1
                    a_[1] += ms
                    a_[2] += ab
            prof[mode] = {"mean_ctx_plus1": float(C_cpu.float().mean()) + 1}
            for cls, (cnt, ms, ab) in agg.items():
                # HIP-event time of a kernel = its duration in a rocprofv3 kernel trace + about 2 us (compared on the
                # same kernels, see profiles/); it is reported as measured, so the rates below are slightly low
                avg_us = ms / cnt * 1e3
                entry = {"launches_per_step": cnt / P, "avg_us": avg_us, "share_of_event_time": None}
                if ab:
                    entry["algorithmic_MB"] = ab / cnt / 1e6
                    entry["GBps"] = ab / (ms * 1e-3) / 1e9
                    entry["frac_hbm_peak"] = entry["GBps"] / HBM_PEAK_GBS
                prof[mode][cls] = entry
            tot = sum(v[1] for v in agg.values())
            for cls, (cnt, ms, ab) in agg.items():
                prof[mode][cls]["share_of_event_time"] = ms / tot

    head_mode = "ee" if "ee" in results else next(iter(results))
    r = results[head_mode]
    # dominant kernel = largest share of the instrumented time among the bandwidth-priced classes
    roof = None
    if prof.get(head_mode):
        cands = [(v["share_of_event_time"], k) for k, v in prof[head_mode].items() if isinstance(v, dict) and "GBps" in v]
        if cands:
            _, dom = max(cands)
            e = prof[head_mode][dom]
            ratio = traffic_ratios().get(dom) if args.config == 1 and not args.layers else None
            roof = {"bound": "hbm", "kernel": dom, "achieved": e["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": e["frac_hbm_peak"],
                    "traffic": (ratio * e["algorithmic_MB"] * 1e6) if ratio else None,
                    "traffic_source": "profiles/hbm_traffic_llama7b_b32_pmc.md (measured bytes per algorithmic byte x "
                                      "this launch's algorithmic bytes)" if ratio else None,
                    "avg_us": e["avg_us"],
                    "algorithmic_bytes_per_launch": e["algorithmic_MB"] * 1e6}

    # ---- CPU oracle on a bounded sample: decode iterations of the same workload (all sequences), about 10 s ---
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ee_oracle as O
        m = O.model_from_config(cfg, w_cpu)
        c0 = int(lens.max())
        cap = min(cfg.decode_steps, extra - 1)   # iterations until about 10 s of CPU work, at most the workload's steps
        Ks = [W.paged_to_dense(cache.k[i], bt, c0 + cap).cpu() for i in range(n)]
        Vs = [W.paged_to_dense(cache.v[i], bt, c0 + cap).cpu() for i in range(n)]
        oc = O.DenseKV.from_tensors(Ks, Vs, lens, cfg.dtype)
        del Ks, Vs
        tok_cpu, pos_cpu = first.cpu(), lens.long().clone()
        n_it = 0
        t1 = time.perf_counter()
        while n_it < cap and time.perf_counter() - t1 < 10.0:
            tok_cpu, _, _ = O.decode_iteration(m, oc, tok_cpu, pos_cpu, cfg.threshold)
            pos_cpu += 1
            n_it += 1
        dt = time.perf_counter() - t1
        cpu = {"value": n_it * Bsz / dt, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
               "sample": f"{n_it} early-exit decode iterations of the same workload (batch {Bsz}, context {c0}.., "
                         f"{n} layers), {dt:.1f} s; tokens/s = {n_it} x batch / that time"}

    # MFMA utilisation of the projection kernels is a counter measurement (rocprofv3 --pmc), not something this run can
    # take: the committed summary's figures, each with the batch (rows) it was taken at.  At batch 32 a projection has
    # 32 flop per weight byte, so 10 % of the MFMA peak is its ceiling at the HBM roofline.
    mfma = {"source": "profiles/mfma_utilisation_projections_pmc.md (SQ_VALU_MFMA_BUSY_CYCLES / GRBM_GUI_ACTIVE)",
            "percent_of_bf16_mfma_peak": profile_figures("mfma_utilisation_projections_pmc.md", "mfma_util")}
    peaks = measure_peaks(torch, B) if args.peaks else None

    line = {
        "metric": "decode tokens/sec/GPU early-exit vs full-layer; HBM GB/s + MFMA util %",
        "value": r["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": r["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "batch": Bsz, "prompt_len": int(lens.max()), "layers": n, "d_model": cfg.d_model,
                   "vocab": cfg.vocab, "threshold": cfg.threshold, "logit_scale": cfg.logit_scale,
                   "exit_every": cfg.exit_every, "kv_block": cfg.block_size, "mode": head_mode,
                   "context_lens": [int(lens.min()), int(lens.max())], "kv": "synthetic" if synthetic_kv else "prefilled",
                   "forced_exit_mean": args.forced_mean or None, "forced_exit_layer": args.forced_layer or None,
                   "launch": "eager" if args.no_graph else "hip_graph",
                   "exit_rule": "per_sequence" if args.per_sequence else "batch (Algorithm 1)"},
        "modes": results,
        "speedup_ee_vs_full": (results["ee"]["tokens_per_s"] / results["full"]["tokens_per_s"])
        if "ee" in results and "full" in results else None,
        "roofline": roof, "iteration_roofline": r.get("iteration"), "mfma_util": mfma, "measured_peaks": peaks,
        "kernels": prof, "cpu_baseline": cpu, "setup_s": setup_s,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
