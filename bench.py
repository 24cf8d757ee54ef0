#!/usr/bin/env python3
"""Throughput of the routed training step (mm_train_step + mm_apply_update) on one MI355X.

A step = one pass of the whole hot path over one synthetic batch of the chosen set-up: route,
embedding + positions, encoder and decoder forward, generator, label-smoothed cross-entropy,
full backward into the per-module buckets, and the Adam update of the touched modules.  Token
ids are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 2] [--accumulate A] [--no-cpu-baseline]

--accumulate A > 1: A routed passes (A sampled tasks, which may share modules) feed one update, the
single-GPU form of several tasks per device (paper section 3.2, algorithm 1: a module's gradient is
divided by the number of passes that used it).  A "step" is then A passes plus one update.
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

PEAK_BF16_FLOPS = 2.5e15   # MI355X dense bf16 MFMA
PEAK_F32_FLOPS = 157.3e12  # fp32 vector
PEAK_HBM = 8.0e12


def cpu_baseline(setup, batch, target_tokens=4096, reps=3):
    """The CPU oracle (fp64 numpy, as it stands): reps steps and updates on one batch (about 5 s
    each on the box's 16 cores)."""
    import numpy as np
    from threadpoolctl import threadpool_info

    import mm_synth
    from oracle.mammoth_oracle import build_from_setup

    n, tok = 0, 0
    while n < len(batch.lengths) and tok < target_tokens:
        tok += int(batch.lengths[n, 1]) - 1
        n += 1
    lengths = batch.lengths[:n]
    src = batch.src_ids[:n, :int(lengths[:, 0].max())]
    tgt = batch.tgt_ids[:n, :int(lengths[:, 1].max())]
    orc = build_from_setup(setup, dtype=np.float64, fill_params=mm_synth.fill_params)
    t0 = time.perf_counter()
    for _ in range(reps):
        orc.train_step(0, src, tgt, lengths)
        orc.apply_update(None, setup.shape.lr)
    dt = time.perf_counter() - t0
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    return {"value": reps * tok / dt, "unit": "target tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{reps} x (fwd+bwd+Adam) of the fp64 numpy oracle on the first {n} sentence pairs "
                      f"({tok} target tokens) of one batch, {dt:.1f} s"}


def bench_translate(args, setup, ctx, batches):
    """One step = one call of mm_translate_greedy on the source sentences of one (or several) batches."""
    import numpy as np
    import torch
    sh = setup.shape
    max_new = args.translate
    tasks = list(range(min(len(setup.tasks), 4)))
    for gen in sorted({j for t in tasks for j in ctx.mm_get_route(t) if setup.modules[j].kind == "gen"}):
        layout, _ = ctx.mm_get_layout(gen)               # generator bucket: matrix [d, V], then bias [V]
        w = ctx.mm_get_params(gen)
        w[layout[1][1] + 2] = -1e3                       # no EOS: every sentence runs every step
        ctx.mm_set_params(gen, w)
    s_len = np.concatenate([b.lengths[:, 0] for b in batches]).astype(np.int32)
    src_host = np.zeros((len(s_len), max(b.src_ids.shape[1] for b in batches)), dtype=np.int32)
    row = 0
    for b in batches:
        src_host[row:row + len(b.lengths), :b.src_ids.shape[1]] = b.src_ids
        row += len(b.lengths)
    src = torch.tensor(src_host, dtype=torch.int32, device="cuda")
    B = len(s_len)
    directions = [tasks[k % len(tasks)] for k in range(args.warmup + args.steps)]
    beam = max(0, args.beam)

    def translate(task):
        if beam:
            return ctx.mm_translate_beam(task, src, s_len, max_new, beam)[:2]
        return ctx.mm_translate_greedy(task, src, s_len, max_new)

    for k in range(args.warmup):
        translate(directions[k])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.warmup, args.warmup + args.steps):
        ids, n = translate(directions[k])
    elapsed = time.perf_counter() - t0
    assert (n == max_new).all()
    ctx.mm_profile(True)
    translate(directions[0])
    prof = ctx.mm_profile_read()
    ctx.mm_profile(False)
    classes = {name: {"ms_per_call": r["ms"], "launches_per_call": r["launches"]}
               for name, r in prof.items() if r["launches"]}
    # HBM bytes a decoding step has to read: the decoder stack's and the generator's working weights
    # once, plus every layer's keys/values of the encoder output
    route = ctx.mm_get_route(tasks[0])
    esz = 2 if sh.dtype == "bf16" else 4
    n_dec = sum(setup.modules[j].n_layers for j in route if setup.modules[j].kind == "dec")
    w_params = sum(ctx.mm_get_layout(j)[1] for j in route if setup.modules[j].kind in ("dec", "gen"))
    w_params -= 2 * sh.d_model * sh.d_model * n_dec      # the encoder-side key/value projections ran once
    step_bytes = w_params * esz + int(s_len.sum()) * 2 * sh.d_model * esz * n_dec
    step_s = elapsed / args.steps / max_new
    roofline = {"bound": "hbm", "kernel": f"one decoding step ({73 if beam else 71} launches at set-up 2; no single kernel dominates)",
                "achieved": step_bytes / step_s / 1e9, "peak": PEAK_HBM / 1e9, "unit": "GB/s",
                "frac": step_bytes / step_s / PEAK_HBM, "traffic": None, "bytes_per_step": step_bytes}
    cpu = None
    if not args.no_cpu_baseline:
        # the oracle's greedy translation (whole model recomputed per token, fp64 numpy) on a few sentences
        from oracle.mammoth_oracle import build_from_setup
        import mm_synth
        needed = set(ctx.mm_get_route(tasks[0]))
        orc = build_from_setup(setup, dtype=np.float64, fill_params=mm_synth.fill_params, needed=needed)
        gen = [j for j in needed if setup.modules[j].kind == "gen"][0]
        orc.modules[gen].p("bg")[2] = -1e3
        nb, steps_cpu = min(32, B), min(20, max_new)   # about 10 s
        t1 = time.perf_counter()
        if beam:
            nb, steps_cpu = min(4, B), min(8, max_new)
            _, n_cpu, _ = orc.beam_decode(tasks[0], src_host[:nb], s_len[:nb], steps_cpu, beam)
        else:
            _, n_cpu = orc.greedy_decode(tasks[0], src_host[:nb], s_len[:nb], steps_cpu)
        dt = time.perf_counter() - t1
        from threadpoolctl import threadpool_info
        threads = max([q.get("num_threads", 1) for q in threadpool_info()] or [1])
        cpu = {"value": float(n_cpu.sum()) / dt, "unit": "generated tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": f"{nb} sentences x {steps_cpu} tokens of the same batch, {dt:.1f} s"}
    print(json.dumps({
        "metric": (f"beam-{beam} translation" if beam else "greedy translation") + " tokens/s per MI355X (routed inference)",
        "value": B * max_new * args.steps / elapsed,
        "unit": "generated tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": 1e3 * elapsed / args.steps, "ms_per_decoding_step": 1e3 * elapsed / args.steps / max_new,
        "higher_is_better": True, "vs_baseline": None, "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}]: {setup.title}; {B} sentences, {int(s_len.sum())} source "
                               f"tokens, {max_new} tokens written per sentence"
                               + (f", {beam} hypotheses per sentence ({B * beam} decoder rows)" if beam else "")},
        "roofline": roofline, "cpu_baseline": cpu, "kernel_classes": classes}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3,
                    help="synthetic set-up 1-8; default 3 = the fully modular Transformer-base set-up the metric names "
                         "(4+4 language-specific stacks resident, 12 directions drawn per step)")
    ap.add_argument("--accumulate", type=int, default=1, help="routed passes per update")
    ap.add_argument("--translate-batches", type=int, default=1,
                    help="with --translate: merge the source sentences of this many batches into one call")
    ap.add_argument("--task-temperature", type=float, default=None,
                    help="draw each pass's task with probability proportional to (corpus size)^(1/T), "
                         "corpus sizes falling off as 1/rank, instead of uniformly")
    ap.add_argument("--sharing", default=None, metavar="ENC/DEC",
                    help="replace the set-up's modules and tasks by a layerwise sharing definition, one "
                         "PATTERN:LAYERS per module position, e.g. 'LANGUAGE:4,FULL:4/LANGUAGE:4' "
                         "(patterns: FULL, SRC_GROUP, TGT_GROUP, GROUP, SRC_LANGUAGE, TGT_LANGUAGE, LANGUAGE); "
                         "model shape, data and seeds stay those of --config")
    ap.add_argument("--languages", type=int, default=4, help="with --sharing: number of languages (all ordered pairs are tasks)")
    ap.add_argument("--groups", type=int, default=2, help="with --sharing: language l belongs to cluster l %% GROUPS")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--translate", type=int, default=0, metavar="MAX_NEW",
                    help="time routed greedy translation instead of training: every sentence of one batch "
                         "writes MAX_NEW tokens (EOS is suppressed so the work is fixed)")
    ap.add_argument("--beam", type=int, default=0, metavar="K",
                    help="with --translate: beam search with K hypotheses per sentence instead of greedy search")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, used to "
                         "scale rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on exactly one GPU (the path's cross-GPU gradient exchange is "
              "design only); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import mm_synth
    from paper_2403_07544_amd import context_from_setup

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    setup = mm_synth.build_setup(args.config)
    if args.sharing:
        enc_text, _, dec_text = args.sharing.partition("/")
        setup = mm_synth.pattern_setup(setup, args.languages, mm_synth.parse_stack(enc_text), mm_synth.parse_stack(dec_text),
                                       {l: l % max(1, args.groups) for l in range(args.languages)})
    sh = setup.shape
    A = max(1, args.accumulate)
    n_steps = (args.warmup + args.steps) * A      # routed passes; A of them per update
    batches = mm_synth.make_batches(setup)
    directions = mm_synth.sample_directions(setup, n_steps, temperature=args.task_temperature)
    ctx = context_from_setup(setup, fill_params=mm_synth.fill_params,
                             max_batch_tokens=16384 if args.translate else None)

    if args.translate:
        return bench_translate(args, setup, ctx, batches[:max(1, args.translate_batches)])

    # inputs resident in HBM before timing
    dev = []
    for k in range(n_steps):
        b = batches[k % len(batches)]
        dev.append((torch.tensor(b.src_ids, dtype=torch.int32, device="cuda"),
                    torch.tensor(b.tgt_ids, dtype=torch.int32, device="cuda"), b.lengths, b))
    torch.cuda.synchronize()

    def run(lo, hi, marks=None):
        """updates lo..hi-1; marks: one event per update boundary, on the library's (default) stream"""
        toks = 0
        for u in range(lo, hi):
            for k in range(u * A, (u + 1) * A):
                src, tgt, lengths, b = dev[k]
                # asynchronous: the host enqueues the next pass while this one runs (the loss is read
                # back once, after the last step)
                ctx.mm_train_step(int(directions[k]), src, tgt, lengths, sync=False)
                toks += b.n_tgt_tokens
            ctx.mm_apply_update(None, sh.lr)
            if marks is not None:
                marks[u - lo + 1].record()
        torch.cuda.synchronize()
        return toks, ctx.mm_last_loss()

    n_upd = args.warmup + args.steps
    run(0, args.warmup)
    torch.cuda.synchronize()
    if args.calibrate_copy:
        a = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        b = torch.empty_like(a)
        b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    marks[0].record()
    tokens, last_loss = run(args.warmup, n_upd, marks)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    per_step = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
    pct = lambda q: per_step[min(len(per_step) - 1, int(q * len(per_step)))]
    src_tokens = sum(dev[k][3].n_src_tokens for k in range(args.warmup * A, n_steps))

    # per-kernel-class timing with HIP events on the library's stream, same steps again
    ctx.mm_profile(True)
    run(args.warmup, n_upd)
    prof = ctx.mm_profile_read()
    ctx.mm_profile(False)
    g = prof["gemm"]
    peak = PEAK_BF16_FLOPS if sh.dtype == "bf16" else PEAK_F32_FLOPS
    achieved = g["work"] / (g["ms"] * 1e-3) if g["ms"] > 0 else 0.0
    roofline = {"bound": "mfma" if sh.dtype == "bf16" else "alu", "kernel": "gemm (all projection, FFN, "
                "generator, input- and weight-gradient products)", "achieved": achieved / 1e12,
                "peak": peak / 1e12, "unit": "TFLOP/s", "frac": achieved / peak, "traffic": None,
                "avg_launch_us": 1e3 * g["ms"] / max(1, g["launches"]), "launches_per_step": g["launches"] / args.steps}
    # HBM bytes per GEMM launch from the committed rocprofv3 FETCH_SIZE / WRITE_SIZE summary (same workload)
    tpath = os.path.join(ROOT, "profiles", f"bench_config{args.config}_gemm_traffic.json")
    if os.path.exists(tpath) and not args.sharing:
        t = json.load(open(tpath))
        roofline["traffic"] = t["read_bytes_per_launch"] + t["written_bytes_per_launch"]
        roofline["traffic_unit"] = "bytes per launch (rocprofv3 FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel)"
    classes = {}
    for name, r in prof.items():
        if r["launches"] == 0:
            continue
        rate = r["work"] / (r["ms"] * 1e-3) if r["ms"] > 0 else 0.0
        flop_bound = name in ("gemm", "attn_fwd", "attn_bwd")
        classes[name] = {"ms_per_step": r["ms"] / args.steps, "launches_per_step": r["launches"] / args.steps,
                         ("tflops" if flop_bound else "gbps"): rate / (1e12 if flop_bound else 1e9),
                         "frac_of_peak": rate / (peak if flop_bound else PEAK_HBM)}
        # LayerNorm is tallied with the bytes the operation needs (4 B/element forward: bf16 in and out;
        # 6 B/element backward); this design keeps the residual stream and its gradient in fp32 and
        # moves 6 and (with the residual gradient and the bf16 copy) 18 B/element
        if name in ("layernorm_fwd", "layernorm_bwd") and sh.dtype == "bf16":
            classes[name]["frac_of_peak_with_design_bytes"] = classes[name]["frac_of_peak"] * (1.5 if name == "layernorm_fwd" else 3.0)

    out = {
        "metric": "training tokens/s per MI355X (fwd+bwd+update), modular Transformer-base",
        "value": tokens / elapsed, "unit": "target tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": 1e3 * elapsed / args.steps,
        "ms_per_step_gpu": {"p10": pct(0.10), "p50": pct(0.50), "p90": pct(0.90)}, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": sh.dtype, "data": "synthetic",
        "config": {"workload": f"configs[{args.config - 1}]{' shape and data with' if args.sharing else ':'} {setup.title}; d={sh.d_model} heads={sh.n_heads} "
                               f"ffn={sh.d_ff} vocab={sh.vocab}, {len(setup.modules)} modules resident, "
                               f"{len(setup.tasks)} task(s), ~{sh.batch_tokens}-token length-bucketed batches"
                               + (f", {A} routed passes per update" if A > 1 else "")
                               + (f", tasks drawn with temperature {args.task_temperature}" if args.task_temperature else ""),
                   "target_tokens_per_step": tokens / args.steps, "source_tokens_per_step": src_tokens / args.steps,
                   "src_plus_tgt_tokens_per_s": (tokens + src_tokens) / elapsed, "last_loss": last_loss},
        "roofline": roofline,
        "kernel_classes": classes,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(setup, dev[args.warmup * A][3])
    print(json.dumps(out))


if __name__ == "__main__":
    main()
