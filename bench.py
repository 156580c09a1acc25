"""Benchmark: batch-1 decode through a 12-block BLOOM-176B-shaped span on one MI355X.

One step = one token through all 12 blocks (LayerNorm, int8 QKV / dense / MLP linears with
fp16 outlier columns, ALiBi attention against the session's KV cache).  Weights, KV prefix and
hidden states are seeded synthetic tensors of the real shapes, resident in HBM before timing.
Prints ONE JSON line.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def gemv_bytes(N, K):
    """Algorithmic HBM bytes of one one-row linear: int8 weights, fp32 row scales, fp16 biases."""
    return N * K + 4 * N + 2 * N


def step_bytes(cfg, L):
    """Algorithmic bytes of one decode step: per block the int8 weights (12 H^2), the row scales (36 H),
    biases (18 H) and LayerNorm parameters (8 H); per session the cached keys/values read (4 (L+1) H), the
    new ones written (4 H) and the hidden state in/out (4 H)."""
    H = cfg.hidden
    per_block = 12 * H * H + 36 * H + 18 * H + 8 * H + 4 * (L + 1) * H + 4 * H
    return cfg.n_blocks * per_block + 4 * H


def _block_params(args, cfg, block, dev):
    """The recipe's block parameters, drawn on the device; --weight-std other than the recipe's 0.02 rescales the
    four weight matrices (a context measurement: how the figures move with the number of outlier columns)."""
    from paper_2209_01188_amd import synth
    p = synth.block_params_device(cfg, block, dev)
    if args.weight_std != 0.02:
        for name in ("w_qkv", "w_dense", "w_up", "w_down"):
            p[name].mul_(args.weight_std / 0.02)
    return p


def _emit(args, line):
    if args.weight_std != 0.02:      # not the recipe: say so in the line
        line["config"]["weight_std"] = args.weight_std
        line["data"] = "synthetic (weights N(0, %g^2) instead of the recipe's N(0, 0.02^2))" % args.weight_std
    print(json.dumps(line))


def traffic_from_profile():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if present."""
    path = os.path.join(ROOT, "profiles", "k_gemv_row_c4_decode_pmc.txt")
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=64)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--prefix", type=int, default=2048, help="KV-cache prefix length of the headline figure")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile-events", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="decode mode: leave out the prefill call and the batched configuration (config.prefill, config.batched)")
    ap.add_argument("--mode", choices=["decode", "prefill", "batched", "generate", "backward", "mfma-peak"], default="decode",
                    help="decode: the headline batch-1 decode benchmark (its line also carries a prefill call and a batched "
                         "decode configuration as config.prefill / config.batched); mfma-peak: register-only loop of the "
                         "int8 matrix instruction; prefill: secondary, int8 MFMA GEMM regime; "
                         "batched: secondary, several sessions per decode step; generate: secondary, greedy "
                         "generation loop with the client-side embedding and LM head on the same GPU; backward: secondary, "
                         "forward + backward (gradients w.r.t. activations) of a fine-tuning batch")
    ap.add_argument("--vocab", type=int, default=250880, help="generate mode: rows of the embedding matrix (BLOOM: 250880)")
    ap.add_argument("--batched-config", choices=["C3", "C5span", "C5"], default="C3",
                    help="batched mode: C3 = 30 BLOOM-7B1-shaped blocks, 8 sessions; C5span = one 12-block span of the "
                         "70-block BLOOM-176B-shaped stack, 32 sessions; C5 = the whole 70-block stack (six chained "
                         "spans, about 250 GB of HBM), 32 sessions")
    ap.add_argument("--prefill-batch", type=int, default=8, help="sessions in the prefill call (512 tokens each)")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="generate mode: 0 = greedy (the LM head's own choice); > 0 = sample the next token")
    ap.add_argument("--top-k", type=int, default=0, help="generate mode with --temperature > 0: tokens in play (0 = all)")
    ap.add_argument("--weight-std", type=float, default=0.02,
                    help="standard deviation of the synthetic weights (0.02 is the recipe; smaller weights give "
                         "smaller activations and so fewer outlier columns in calls of many rows)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy, the known-size kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (with more, each GPU would hold a span of consecutive blocks); "
              "--gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2209_01188_amd import binding, synth

    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.mode == "prefill":
        return prefill_main(args, dev)
    if args.mode == "batched":
        return batched_main(args, dev)
    if args.mode == "generate":
        return generate_main(args, dev)
    if args.mode == "backward":
        return backward_main(args, dev)
    if args.mode == "mfma-peak":
        return mfma_peak_main(args, dev)
    cfg = synth.CONFIGS["C4"]
    H, F, nh, NB = cfg.hidden, cfg.F, cfg.n_heads, cfg.n_blocks
    K, W = args.steps, args.warmup
    prefixes = sorted(set(cfg.prefixes) | {args.prefix})

    t_setup = time.time()
    # sized for the 8 x 512 prefill call of the secondary figure too (the decode steps use one row of it)
    PRE_B, PRE_T = 8, 512
    span = binding.Span(NB, H, nh, F, 1 if args.no_secondary else PRE_B * PRE_T, 1e-5, 6.0, dev)
    block0_host = None
    for b in range(NB):
        p = _block_params(args, cfg, b, dev)
        span.load_block(b, p)
        if b == 0 and not args.no_cpu_baseline:
            block0_host = {k: v.cpu().numpy() for k, v in p.items()}
        del p
    torch.cuda.synchronize()
    print("[bench] %d blocks loaded (%.1f GB int8) in %.1f s" % (NB, span.weight_mem.numel() / 1e9, time.time() - t_setup),
          file=sys.stderr, flush=True)

    # hidden-state inputs of all steps, resident on the device
    n_calls = W + K
    xs = torch.from_numpy(np.concatenate([synth.hidden_states(cfg, 1 + i, 1, 1)[0] for i in range(n_calls)])).to(dev)
    out = torch.empty((1, H), dtype=torch.float16, device=dev)
    stream = torch.cuda.current_stream()

    def timed_decode(L, profile):
        se = span.open_session(L + n_calls + 1)
        for b in range(NB):
            se.import_kv(b, synth.kv_prefix_device(cfg, b, 0, L, 2.4, dev))
        for i in range(W):
            span.decode_step([se], xs[i:i + 1], out)
        torch.cuda.synchronize()
        if profile:
            binding.petals_span_profile_begin(span.handle, K * NB * 8)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for i in range(W, W + K):
            span.decode_step([se], xs[i:i + 1], out)
        e1.record(stream)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3
        ms = max(e0.elapsed_time(e1), 0.0)
        prof = binding.petals_span_profile_end(span.handle) if profile else None
        se.close()
        return max(ms, 0.0), wall_ms, prof

    if args.calibration_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    timed_decode(prefixes[0], profile=False)   # throwaway pass: the first timed configuration after the load is noisy
    results = {}
    for L in prefixes:
        # the throughput figure is timed with no instrumentation in the stream; a second pass over the same
        # steps brackets every heavy launch with HIP events (they cost a few microseconds each) to get the
        # dominant kernel's own duration
        ms, wall_ms, _ = timed_decode(L, profile=False)
        prof = None
        if L == args.prefix and not args.no_profile_events:
            _, _, prof = timed_decode(L, profile=True)
        total = max(ms, wall_ms) if abs(ms - wall_ms) > 0.2 * wall_ms else ms
        results[L] = dict(ms_per_step=total / K, tok_s=K / (total / 1e3), gbs=step_bytes(cfg, L) / (total / K / 1e3) / 1e9,
                          prof=prof)
        print("[bench] prefix %d: %.3f ms/step, %.1f tok/s, %.0f GB/s algorithmic" %
              (L, results[L]["ms_per_step"], results[L]["tok_s"], results[L]["gbs"]), file=sys.stderr, flush=True)

    main_r = results[args.prefix]
    # dominant kernel: the one-row int8 linear (4 launches per block), from the events of the headline run
    roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                "traffic": traffic_from_profile(),
                "traffic_source": "committed rocprofv3 counter summary profiles/k_gemv_row_c4_decode_pmc.txt, not this run",
                "kernel": "k_gemv_row"}
    if main_r["prof"] is not None:
        ms_cls, n_cls = main_r["prof"]
        n_gemv = n_cls[binding.PROFILE_GEMV]
        if n_gemv:
            per_block = sum(gemv_bytes(*span.shapes(i)) for i in range(4))
            total_bytes = per_block * (n_gemv / 4.0)
            achieved = total_bytes / (ms_cls[binding.PROFILE_GEMV] / 1e3) / 1e9
            roofline.update(achieved=round(achieved, 1), frac=round(achieved / HBM_PEAK_GBS, 4),
                            avg_launch_us=round(ms_cls[binding.PROFILE_GEMV] * 1e3 / n_gemv, 2), launches=n_gemv,
                            bytes_per_launch=round(per_block / 4.0),
                            attention_ms_per_step=round(ms_cls[binding.PROFILE_ATTENTION] / K, 4))

    # secondary figures, timed after the headline: one prefill call of 8 x 512 tokens through the same span
    # (int8 MFMA GEMM regime) and batched decode steps of the 30-block BLOOM-7B1-shaped configuration
    secondary = {}
    if not args.no_secondary:
        r = measure_prefill(args, span, dev, PRE_B, PRE_T, steps=2, warmup=1)
        secondary["prefill"] = {"workload": "%d sessions x %d tokens through the same 12-block span (%d rows per linear)"
                                            % (PRE_B, PRE_T, r["rows"]),
                                "ms_per_call": round(r["ms_per_call"], 3), "tokens_per_s": round(r["tokens_per_s"], 1),
                                "int8_top_s": round(r["int8_top_s"], 1), "mfma_frac": round(r["int8_top_s"] / 5000.0, 4),
                                "mfma_kernel": "k_gemm_lds on the QKV and up linears, against the 5000 TOP/s dense int8 peak",
                                "executed_int8_top_s_all_linears": round(r["executed_int8_top_s"], 1),
                                "mfma_frac_executed_all_linears": round(r["executed_int8_top_s"] / 5000.0, 4),
                                "per_block_ms": r["per_block_ms"], "per_linear_top_s": r["per_linear_top_s"],
                                "outlier_columns_mean_over_blocks": r["outlier_columns"]}
        print("[bench] prefill %d x %d: %.1f ms per call, int8 GEMM %.0f TOP/s" %
              (PRE_B, PRE_T, r["ms_per_call"], r["int8_top_s"]), file=sys.stderr, flush=True)
    span.close()
    del span
    torch.cuda.empty_cache()
    if not args.no_secondary:
        r = measure_batched(args, dev, "C3", 32, 4)
        secondary["batched"] = {"workload": r["name"] + ", 512-token prompts, one token per session per step, 8-bit codec "
                                            "at the span boundary",
                                "ms_per_step": round(r["ms_per_step"], 4), "tokens_per_s": round(r["tokens_per_s"], 1),
                                "hbm_frac": round(r["hbm_frac"], 4), "linears_ms_per_step": round(r["linears_ms_per_step"], 4),
                                "attention_ms_per_step": round(r["attention_ms_per_step"], 4)}
        print("[bench] batched C3: %.3f ms per step" % r["ms_per_step"], file=sys.stderr, flush=True)

    cpu_baseline = None
    if block0_host is not None:
        cpu_baseline = run_cpu_baseline(cfg, block0_host, dev, prefix=args.prefix)

    line = {
        "metric": "decode tokens/s per 12-block BLOOM-176B span (batch 1); achieved HBM GB/s",
        "value": round(main_r["tok_s"], 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(main_r["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "C4: 12-block BLOOM-176B-shaped span (H=14336, 112 heads, F=57344), int8 weights + fp16 "
                               "outlier columns, batch-1 decode, KV prefix %d" % args.prefix,
                   "prefix": args.prefix, "achieved_hbm_gbs": round(main_r["gbs"], 1),
                   "hbm_frac_whole_step": round(main_r["gbs"] / HBM_PEAK_GBS, 4),
                   "by_prefix": {str(L): {"tokens_per_s": round(r["tok_s"], 2), "ms_per_step": round(r["ms_per_step"], 4),
                                          "achieved_hbm_gbs": round(r["gbs"], 1)} for L, r in results.items()}},
        "roofline": roofline, "cpu_baseline": cpu_baseline,
    }
    line["config"].update(secondary)
    _emit(args, line)


def measure_prefill(args, span, dev, B, T=512, steps=2, warmup=1):
    """One prefill call (B sessions x T new tokens on fresh sessions) through `span`, timed over `steps` calls;
    a further call brackets every linear and the attention with HIP events.  Returns per-call and per-linear
    figures; int8_top_s is the int8 MFMA rate of the QKV and up linears (whose inputs carry few outlier columns,
    so their time is the int8 kernel's)."""
    import torch
    from paper_2209_01188_amd import binding, synth

    cfg = synth.CONFIGS["C4"]
    NB, M = span.n_blocks, B * T
    X = torch.from_numpy(synth.hidden_states(cfg, 0, B, T)).to(dev)
    out = torch.empty_like(X)
    kv = [torch.zeros(binding.petals_span_kv_bytes(span.cfg, T), dtype=torch.uint8, device=dev) for _ in range(B)]
    stream = torch.cuda.current_stream()

    def one_call():
        ses = [binding.petals_session_open(span.handle, kv[i], T) for i in range(B)]
        binding.petals_span_prefill(span.handle, ses, T, X, out)
        return ses

    def close(ses):
        torch.cuda.synchronize()
        for s in ses:
            binding.petals_session_close(s)

    for _ in range(warmup):
        close(one_call())
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    opened = [one_call() for _ in range(steps)]
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    for ses in opened:
        close(ses)
    binding.petals_span_profile_begin(span.handle, NB * 8)
    ses = one_call()
    torch.cuda.synchronize()
    pm, pn = binding.petals_span_profile_end(span.handle)
    close(ses)
    ops = [2.0 * M * n * k for n, k in (span.shapes(i) for i in range(4))]
    lin_ms = [pm[binding.PROFILE_LINEAR0 + i] / NB for i in range(4)]
    int8_ops, int8_ms = ops[0] + ops[2], lin_ms[0] + lin_ms[2]
    names = ("qkv", "dense", "up", "down")
    per_block = span.outlier_counts().cpu()                             # of the call just run, [block][linear]
    counts = per_block.float().mean(0).tolist()
    # int8 operations the matrix cores really execute per block: the four products, plus - where a linear has more
    # than 64 outlier columns - the 8 digit products (2 weight digits x 4 activation digit planes) over those columns
    digit_ops = [0.0] * 4
    for b in range(per_block.shape[0]):
        for i in range(4):
            c = int(per_block[b, i])
            if c > 64:
                digit_ops[i] += 2.0 * M * span.shapes(i)[0] * (64 * ((c + 63) // 64)) * 8 / per_block.shape[0]
    executed = (sum(ops) + sum(digit_ops)) / (sum(lin_ms) * 1e-3) / 1e12
    return {"outlier_columns": {n: round(counts[i], 1) for i, n in enumerate(names)},"ms_per_call": ms, "tokens_per_s": M / (ms * 1e-3), "rows": M, "sessions": B, "tokens_per_session": T,
            "int8_top_s": int8_ops / (int8_ms * 1e-3) / 1e12, "executed_int8_top_s": executed,
            "per_block_ms": dict({n: round(lin_ms[i], 3) for i, n in enumerate(names)},
                                 attention=round(pm[binding.PROFILE_ATTENTION] / NB, 3)),
            "per_linear_top_s": {n: round(ops[i] / (lin_ms[i] * 1e-3) / 1e12, 1) for i, n in enumerate(names)}}


def prefill_main(args, dev):
    """Secondary benchmark: a prefill call (sessions x 512 new tokens) through a 12-block BLOOM-176B-shaped span.
    One step = one prefill call on fresh sessions.  Reports tokens/s and, for the dominant kernel (the LDS-staged
    int8 MFMA GEMM, here on the QKV and up linears whose inputs carry few outlier columns), int8 TOP/s against
    the 5 POP/s dense int8 peak.  With the synthetic N(0, 0.02) weights the inputs of the dense and down linears
    have Gaussian tails beyond the threshold in thousands of columns at this row count, so those two also run the
    exact int8 digit products of their outlier columns; their time is reported separately."""
    from paper_2209_01188_amd import binding, synth

    cfg = synth.CONFIGS["C4"]
    H, F, nh, NB = cfg.hidden, cfg.F, cfg.n_heads, cfg.n_blocks
    B, T = args.prefill_batch, 512
    M = B * T
    K_steps, W = max(1, min(args.steps, 4)), max(1, min(args.warmup, 1))
    span = binding.Span(NB, H, nh, F, M, 1e-5, 6.0, dev)
    for b in range(NB):
        span.load_block(b, _block_params(args, cfg, b, dev))
    r = measure_prefill(args, span, dev, B, T, K_steps, W)
    achieved = r["int8_top_s"]
    line = {
        "metric": "prefill tokens/s per 12-block BLOOM-176B span; int8 MFMA TOP/s", "value": round(r["tokens_per_s"], 1),
        "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W, "ms_per_step": round(r["ms_per_call"], 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "12-block BLOOM-176B-shaped span (H=14336, F=57344), prefill of %d sessions x 512 tokens "
                               "(%d rows per linear)" % (B, M),
                   "per_block_ms": r["per_block_ms"], "per_linear_top_s": r["per_linear_top_s"],
                   "outlier_columns_mean_over_blocks": r["outlier_columns"],
                   "executed_int8_top_s_all_linears": round(r["executed_int8_top_s"], 1),
                   "mfma_frac_executed_all_linears": round(r["executed_int8_top_s"] / 5000.0, 4)},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": 5000.0, "unit": "TOP/s",
                     "frac": round(achieved / 5000.0, 4), "traffic": None, "kernel": "k_gemm_lds (qkv and up linears)"},
        "cpu_baseline": None,
    }
    span.close()
    _emit(args, line)


def mfma_peak_main(args, dev):
    """What the int8 matrix pipes sustain with no memory traffic: a register-only loop of the matrix instruction
    the prefill linear uses (and of its 32x32x32 sibling), with operands of one constant byte and of pseudo-random
    bytes.  One step = one launch of the loop on 512 workgroups of 4 waves (two per compute unit)."""
    import torch
    from paper_2209_01188_amd import binding

    wgs, iters = 512, 20000
    out = torch.empty(wgs * 256, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream()
    res = {}
    for kind, kname in ((0, "v_mfma_i32_16x16x64_i8"), (1, "v_mfma_i32_32x32x32_i8")):
        for rnd, rname in ((0, "constant"), (1, "random")):
            for _ in range(max(1, args.warmup)):
                binding.petals_bench_mfma(kind, rnd, iters, wgs, out)
            torch.cuda.synchronize()
            best = None
            for _ in range(max(1, min(args.steps, 8))):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                ops = binding.petals_bench_mfma(kind, rnd, iters, wgs, out)
                e1.record(stream)
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            tops = ops / (best * 1e-3) / 1e12
            # 256 compute units x 4 SIMDs x 2048 int8 operations per clock at the data-sheet rate
            res["%s, %s operands" % (kname, rname)] = {"top_s": round(tops, 1), "frac_of_5000": round(tops / 5000.0, 4),
                                                       "ms": round(best, 3),
                                                       "implied_clock_ghz": round(tops * 1e12 / (256 * 4 * 2048) / 1e9, 3)}
            print("[bench] %s, %s operands: %.0f TOP/s" % (kname, rname, tops), file=sys.stderr, flush=True)
    # One compute unit's share of the prefill linear's main loop (a 256 x 256 block's k-tile stage: 32 KiB of
    # asynchronous copies into LDS, 12 fragment reads and 32 matrix instructions per wave, 8 waves), piece by
    # piece and together, on random and on constant operand bytes: nanoseconds per stage, and the int8 rate the
    # stage's 2 * 256 * 256 * 64 operations would then have on 256 compute units.
    stages, regions, rounds = 224, 4, 4
    stage = {}
    for rname in ("random", "constant"):
        if rname == "random":
            src = torch.randint(0, 256, (regions * stages * 32 * 1024,), dtype=torch.uint8, device=dev)
        else:
            src = torch.full((regions * stages * 32 * 1024,), 1, dtype=torch.uint8, device=dev)
        sout = torch.empty(256 * rounds * 512, dtype=torch.int32, device=dev)
        for parts, pname in ((4, "products"), (6, "products + fragment reads"), (5, "products + copies"),
                             (7, "products + fragment reads + copies"), (1, "copies"), (2, "fragment reads")):
            binding.petals_bench_stage(parts, stages, regions, 256 * rounds, src, sout)
            torch.cuda.synchronize()
            best = None
            for _ in range(max(1, min(args.steps, 8))):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                binding.petals_bench_stage(parts, stages, regions, 256 * rounds, src, sout)
                e1.record(stream)
                torch.cuda.synchronize()
                ms = e0.elapsed_time(e1)
                best = ms if best is None else min(best, ms)
            ns = best * 1e6 / (stages * rounds)
            ent = {"ns_per_stage": round(ns, 1)}
            if parts & 4:
                ent["top_s"] = round(256 * 2.0 * 256 * 256 * 64 / (ns * 1e-9) / 1e12, 1)
            stage["%s, %s operands" % (pname, rname)] = ent
            print("[bench] stage loop, %s, %s operands: %.0f ns per stage" % (pname, rname, ns), file=sys.stderr, flush=True)
    key = "v_mfma_i32_16x16x64_i8, random operands"
    line = {"metric": "sustained int8 MFMA TOP/s, register-only loop", "value": res[key]["top_s"], "unit": "TOP/s",
            "n_gpus": 1, "steps": max(1, min(args.steps, 8)), "warmup": max(1, args.warmup), "ms_per_step": res[key]["ms"],
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
            "config": {"workload": "register-only loop of the int8 matrix instruction, 512 workgroups x 4 waves x %d "
                                   "iterations, no memory traffic" % iters, "variants": res, "stage_loop": stage},
            "roofline": {"bound": "mfma", "achieved": res[key]["top_s"], "peak": 5000.0, "unit": "TOP/s",
                         "frac": res[key]["frac_of_5000"], "traffic": None, "kernel": "k_mfma_loop"},
            "cpu_baseline": None}
    print(json.dumps(line))


def backward_main(args, dev):
    """Secondary benchmark: one fine-tuning call (forward + backward w.r.t. activations) of sessions x 512 tokens
    through a 12-block BLOOM-176B-shaped span.  One step = one petals_span_backward call.  Reports tokens/s and,
    for the dominant kernel of the backward half (the fp16 MFMA product dY Wd of the four linears), TFLOP/s
    against the 2.5 PFLOP/s dense fp16 peak."""
    import torch
    from paper_2209_01188_amd import binding, synth

    cfg = synth.CONFIGS["C4"]
    H, F, nh, NB = cfg.hidden, cfg.F, cfg.n_heads, cfg.n_blocks
    B, T = args.prefill_batch, 512
    M = B * T
    K_steps, W = max(1, min(args.steps, 3)), max(1, min(args.warmup, 1))
    span = binding.Span(NB, H, nh, F, M, 1e-5, 6.0, dev)
    for b in range(NB):
        span.load_block(b, _block_params(args, cfg, b, dev))
    X = torch.from_numpy(synth.hidden_states(cfg, 0, B, T)).to(dev)
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    dY = torch.empty(X.shape, dtype=torch.float32, device=dev).normal_(0.0, 1.0, generator=g).to(torch.float16)
    store = torch.empty(binding.petals_span_backward_bytes(span.cfg, B, T), dtype=torch.uint8, device=dev)
    gin = torch.empty_like(X)      # the forward output is not asked for: the client has it when it sends the gradient
    stream = torch.cuda.current_stream()
    for _ in range(W):
        binding.petals_span_backward(span.handle, store, X, dY, None, gin)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed():
        e0.record(stream)
        for _ in range(K_steps):
            binding.petals_span_backward(span.handle, store, X, dY, None, gin)
        e1.record(stream)
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / K_steps

    ms_rebuild = timed()            # the transposed fp16 weights are rebuilt from int8 in every call
    span.attach_backward_cache()    # ... or kept between calls (2 bytes per weight): the configuration reported
    binding.petals_span_backward(span.handle, store, X, dY, None, gin)
    torch.cuda.synchronize()
    ms = timed()
    binding.petals_span_profile_begin(span.handle, NB * 16)
    binding.petals_span_backward(span.handle, store, X, dY, None, gin)
    torch.cuda.synchronize()
    pm, pn = binding.petals_span_profile_end(span.handle)
    flops = sum(2.0 * M * n * k for n, k in (span.shapes(i) for i in range(4))) * NB
    bwd_gemm_ms = pm[binding.PROFILE_BWD_GEMM]
    achieved = flops / (bwd_gemm_ms * 1e-3) / 1e12
    fwd_ms = pm[binding.PROFILE_GEMM] + pm[binding.PROFILE_ATTENTION]
    line = {
        "metric": "fine-tuning tokens/s (forward + backward w.r.t. activations) per 12-block BLOOM-176B span",
        "value": round(M / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W,
        "ms_per_step": round(ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
        "data": "synthetic",
        "config": {"workload": "12-block BLOOM-176B-shaped span (H=14336, F=57344), %d sequences x 512 tokens "
                               "(%d rows per linear), forward then backward" % (B, M),
                   "store_gb": round(store.numel() / 1e9, 2),
                   "transposed_weight_cache_gb": round(span.backward_cache.numel() / 1e9, 2),
                   "ms_per_step_without_the_cache": round(ms_rebuild, 3),
                   "per_call_ms": {"forward_linears_and_attention": round(fwd_ms, 2),
                                   "backward_products": round(bwd_gemm_ms, 2),
                                   "backward_attention": round(pm[binding.PROFILE_BWD_ATTENTION], 2)}},
        "roofline": {"bound": "mfma", "achieved": round(achieved, 1), "peak": 2500.0, "unit": "TFLOP/s",
                     "frac": round(achieved / 2500.0, 4), "traffic": None,
                     "kernel": "k_gemm_lds<fp16> (backward products of the four linears)",
                     "avg_launch_us": round(bwd_gemm_ms * 1e3 / max(pn[binding.PROFILE_BWD_GEMM], 1), 1),
                     "launches": pn[binding.PROFILE_BWD_GEMM]},
        "cpu_baseline": None,
    }
    span.close()
    _emit(args, line)


def measure_batched(args, dev, which, K, W):
    """ decode steps with several sessions in one call (one new token per session), hidden
    states crossing the span boundary as blockwise 8-bit codes.  The prompts (512 tokens per session) go through
    the library's own prefill first.  One step = dequantize the incoming codes, one decode step for all sessions,
    quantize the result.  Reports aggregate tokens/s and, for the dominant kernel (the batched-decode int8
    linear), weight bytes streamed per second against the HBM peak."""
    import numpy as np
    import torch
    from paper_2209_01188_amd import binding, synth

    if which == "C3":
        cfg, NB, B = synth.CONFIGS["C3"], synth.CONFIGS["C3"].n_blocks, synth.CONFIGS["C3"].batch
        name = "C3: 30-block BLOOM-7B1-shaped span (H=4096, 32 heads, F=16384), %d sessions" % B
    else:
        cfg, NB, B = synth.CONFIGS["C4"], 12, 32
        name = "one 12-block span of C5 (H=14336, 112 heads, F=57344), %d sessions" % B
    H, F, nh, T = cfg.hidden, cfg.F, cfg.n_heads, 512
    chunk = max(1, min(B, 4096 // T))                      # sessions per prefill call
    span = binding.Span(NB, H, nh, F, max(B, chunk * T), 1e-5, 6.0, dev)
    for b in range(NB):
        span.load_block(b, _block_params(args, cfg, b, dev))
    ses = [span.open_session(T + W + K + 1) for _ in range(B)]
    Xp = synth.hidden_states(cfg, 0, B, T)
    for s0 in range(0, B, chunk):
        span.prefill(ses[s0:s0 + chunk], torch.from_numpy(Xp[s0:s0 + chunk]).to(dev))
    torch.cuda.synchronize()
    print("[bench] %d blocks loaded, %d x %d prompt tokens prefilled" % (NB, B, T), file=sys.stderr, flush=True)

    CB = 4096                                              # codec block
    nblk = (B * H + CB - 1) // CB
    codes, absmax = [], []
    for i in range(W + K):                                 # the incoming codes of every step, resident on the device
        x = torch.from_numpy(synth.hidden_states(cfg, 1 + i, B, 1)[:, 0]).to(dev)
        q = torch.empty(B * H, dtype=torch.uint8, device=dev)
        a = torch.empty(nblk, dtype=torch.float32, device=dev)
        binding.petals_hidden_quantize(x, CB, q, a)
        codes.append(q); absmax.append(a)
    xin = torch.empty((B, H), dtype=torch.float16, device=dev)
    out = torch.empty((B, H), dtype=torch.float16, device=dev)
    qo = torch.empty(B * H, dtype=torch.uint8, device=dev)
    ao = torch.empty(nblk, dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    handles = [s.handle for s in ses]

    def step(i):                                            # codes in (decoded inside the first LayerNorm), codes out
        binding.petals_span_prefill_q8(span.handle, handles, 1, codes[i], absmax[i], CB, out)
        binding.petals_hidden_quantize(out, CB, qo, ao)

    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(W, W + K):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / K
    # a second pass over one step with the heavy launches bracketed by events (sessions are one token longer)
    for s in ses:
        s.close()
    ses = [span.open_session(T + 2) for _ in range(B)]
    for s0 in range(0, B, chunk):
        span.prefill(ses[s0:s0 + chunk], torch.from_numpy(Xp[s0:s0 + chunk]).to(dev))
    torch.cuda.synchronize()
    handles = [s.handle for s in ses]
    binding.petals_span_profile_begin(span.handle, NB * 8)
    step(W)
    torch.cuda.synchronize()
    pm, pn = binding.petals_span_profile_end(span.handle)
    L = T + W + K // 2                                     # mean cached length over the timed steps
    wbytes = NB * sum(gemv_bytes(*span.shapes(i)) for i in range(4))
    total_bytes = NB * (12 * H * H + 62 * H) + B * NB * (4 * (L + 1) * H + 4 * H) + 2 * B * H * 3
    gemm_ms, n_gemm = pm[binding.PROFILE_GEMM], pn[binding.PROFILE_GEMM]
    achieved = wbytes / (gemm_ms * 1e-3) / 1e9 if n_gemm else None
    span.close()
    return {"name": name, "sessions": B, "ms_per_step": ms, "tokens_per_s": B / (ms * 1e-3),
            "hbm_gbs_whole_step": total_bytes / (ms * 1e-3) / 1e9,
            "hbm_frac": total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "linears_ms_per_step": gemm_ms, "attention_ms_per_step": pm[binding.PROFILE_ATTENTION],
            "gemm_launches": n_gemm, "gemm_gbs": achieved,
            "per_linear_gbs": {n: round(NB * gemv_bytes(*span.shapes(i)) / (pm[binding.PROFILE_LINEAR0 + i] * 1e-3) / 1e9, 1)
                               for i, n in enumerate(("qkv", "dense", "up", "down")) if pm[binding.PROFILE_LINEAR0 + i] > 0}}


def batched_main(args, dev):
    """Secondary benchmark: decode steps with several sessions in one call (see measure_batched)."""
    if args.batched_config == "C5":
        return c5_main(args, dev)
    r = measure_batched(args, dev, args.batched_config, args.steps, args.warmup)
    achieved = r["gemm_gbs"]
    line = {
        "metric": "decode tokens/s per span, all sessions of the call together; achieved HBM GB/s",
        "value": round(r["tokens_per_s"], 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(r["ms_per_step"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": r["name"] + ", 512-token prompts, one token per session per step, 8-bit codec at the span "
                               "boundary", "sessions": r["sessions"],
                   "achieved_hbm_gbs": round(r["hbm_gbs_whole_step"], 1),
                   "hbm_frac_whole_step": round(r["hbm_frac"], 4),
                   "linears_ms_per_step": round(r["linears_ms_per_step"], 4),
                   "attention_ms_per_step": round(r["attention_ms_per_step"], 4),
                   "per_linear_gbs": r["per_linear_gbs"]},
        "roofline": {"bound": "hbm", "achieved": round(achieved, 1) if achieved else None, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4) if achieved else None, "traffic": None,
                     "kernel": "k_gemm (batched-decode int8 linear)", "launches": r["gemm_launches"]},
        "cpu_baseline": None,
    }
    _emit(args, line)


def c5_main(args, dev):
    """The whole 70-block BLOOM-176B-shaped stack on one GPU: six chained spans (12+12+12+12+12+10 blocks,
    172.6 GB of int8 weights), 32 sessions, 512-token prompts (prefilled 8 sessions at a time), then decode steps;
    the hidden states cross every span boundary, and the stack's input and output, as blockwise 8-bit codes."""
    import numpy as np
    import torch
    from paper_2209_01188_amd import binding, synth

    cfg = synth.CONFIGS["C5"]
    H, F, nh, B, T = cfg.hidden, cfg.F, cfg.n_heads, cfg.batch, cfg.prompt
    K, W = min(args.steps, cfg.decode), min(args.warmup, 4)
    sizes = [12, 12, 12, 12, 12, 10]
    chunk = 4096 // T
    CB = 4096
    t0 = time.time()
    ws_cfg = binding.make_config(12, H, nh, F, chunk * T)
    shared_ws = torch.empty(binding.petals_span_workspace_bytes(ws_cfg), dtype=torch.uint8, device=dev)
    spans, blk = [], 0
    for n in sizes:
        sp = binding.Span(n, H, nh, F, chunk * T, 1e-5, 6.0, dev, workspace=shared_ws)
        for b in range(n):
            p = _block_params(args, cfg, blk, dev)
            sp.load_block(b, p)
            del p
            blk += 1
        torch.cuda.empty_cache()
        spans.append(sp)
        print("[bench] span %d: %d blocks loaded (%d so far, %.0f s, %.1f GB allocated)" %
              (len(spans), n, blk, time.time() - t0, torch.cuda.memory_allocated() / 1e9), file=sys.stderr, flush=True)
    cap = T + W + K + 2
    ses = [[sp.open_session(cap) for _ in range(B)] for sp in spans]
    print("[bench] KV caches for %d sessions x %d tokens: %.1f GB allocated" % (B, cap, torch.cuda.memory_allocated() / 1e9),
          file=sys.stderr, flush=True)

    def codec_buffers(rows):
        n = rows * H
        return (torch.empty(n, dtype=torch.uint8, device=dev), torch.empty((n + CB - 1) // CB, dtype=torch.float32, device=dev))

    def through_stack(x_codes, x_absmax, rows_shape, sess_lists, scratch):
        """codes in -> every span (dequantize, run, quantize) -> codes out"""
        q, a = x_codes, x_absmax
        hin, hout, qo, ao = scratch
        for sp, ss in zip(spans, sess_lists):
            binding.petals_hidden_dequantize(q, a, CB, hin)
            if len(rows_shape) == 3:
                binding.petals_span_prefill(sp.handle, [s.handle for s in ss], rows_shape[1], hin, hout)
            else:
                sp.decode_step(ss, hin, hout)
            binding.petals_hidden_quantize(hout, CB, qo, ao)
            q, a = qo, ao
        return qo, ao

    stream = torch.cuda.current_stream()
    # prefill, 8 sessions per call
    pre_scratch = (torch.empty((chunk, T, H), dtype=torch.float16, device=dev), torch.empty((chunk, T, H), dtype=torch.float16, device=dev),
                   *codec_buffers(chunk * T))
    qin, ain = codec_buffers(chunk * T)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    pre_ms = 0.0
    Xall = synth.hidden_states(cfg, 0, B, T)
    for s0 in range(0, B, chunk):
        X = torch.from_numpy(Xall[s0:s0 + chunk]).to(dev)
        binding.petals_hidden_quantize(X, CB, qin, ain)
        torch.cuda.synchronize()
        e0.record(stream)
        through_stack(qin, ain, (chunk, T, H), [ss[s0:s0 + chunk] for ss in ses], pre_scratch)
        e1.record(stream)
        torch.cuda.synchronize()
        pre_ms += e0.elapsed_time(e1)
    del pre_scratch, X, Xall
    print("[bench] prefill of %d x %d tokens through 70 blocks: %.2f s" % (B, T, pre_ms / 1e3), file=sys.stderr, flush=True)
    # decode
    dec_scratch = (torch.empty((B, H), dtype=torch.float16, device=dev), torch.empty((B, H), dtype=torch.float16, device=dev),
                   *codec_buffers(B))
    codes = []
    for i in range(W + K):
        x = torch.from_numpy(synth.hidden_states(cfg, 1 + i, B, 1)[:, 0]).to(dev)
        q, a = codec_buffers(B)
        binding.petals_hidden_quantize(x, CB, q, a)
        codes.append((q, a))
    for i in range(W):
        through_stack(codes[i][0], codes[i][1], (B, H), ses, dec_scratch)
    torch.cuda.synchronize()
    e0.record(stream)
    for i in range(W, W + K):
        through_stack(codes[i][0], codes[i][1], (B, H), ses, dec_scratch)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / K
    L = T + W + K // 2
    total_bytes = 70 * (12 * H * H + 62 * H) + B * 70 * (4 * (L + 1) * H + 4 * H) + 6 * 2 * B * H * 3
    line = {
        "metric": "decode tokens/s of the whole 70-block stack, all sessions together; achieved HBM GB/s",
        "value": round(B / (ms * 1e-3), 1), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "C5: 70 BLOOM-176B-shaped blocks as six chained spans (12+12+12+12+12+10) on one GPU, %d sessions, "
                               "512-token prompts, one token per session per step, 8-bit codec at every span boundary" % B,
                   "sessions": B, "hbm_gb_allocated": round(torch.cuda.max_memory_allocated() / 1e9, 1),
                   "prefill_s": round(pre_ms / 1e3, 3), "prefill_tokens_per_s": round(B * T / (pre_ms / 1e3), 1),
                   "achieved_hbm_gbs": round(total_bytes / (ms * 1e-3) / 1e9, 1),
                   "hbm_frac_whole_step": round(total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)},
        "roofline": {"bound": "hbm", "achieved": round(total_bytes / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(total_bytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "whole decode step (weights + KV + codec bytes over its duration)"},
        "cpu_baseline": None,
    }
    for sp in spans:
        sp.close()
    _emit(args, line)


def generate_main(args, dev):
    """Secondary benchmark: the greedy generation loop of the paper's Figure 2 on one GPU - embedding lookup,
    one decode step through the 12-block BLOOM-176B-shaped span (KV prefix args.prefix), LM head over the tied
    250880 x 14336 fp16 embedding matrix, and the chosen token fed back without leaving the device.  Reports
    tokens/s of the whole loop and, for the LM-head kernel, streamed bytes per second against the HBM peak."""
    import numpy as np
    import torch
    from paper_2209_01188_amd import binding, synth

    cfg = synth.CONFIGS["C4"]
    H, F, nh, NB, V = cfg.hidden, cfg.F, cfg.n_heads, cfg.n_blocks, args.vocab
    K, W, L = args.steps, args.warmup, args.prefix
    span = binding.Span(NB, H, nh, F, 1, 1e-5, 6.0, dev)
    for b in range(NB):
        span.load_block(b, _block_params(args, cfg, b, dev))
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    E = torch.empty((V, H), dtype=torch.float16, device=dev)
    for v0 in range(0, V, 16384):                         # unit-scale rows so the embedded vectors look like hidden states
        E[v0:v0 + 16384] = torch.randn((min(16384, V - v0), H), generator=g, device=dev, dtype=torch.float32).to(torch.float16)
    ln = [(1.0 + 0.02 * torch.randn(H, generator=g, device=dev)).to(torch.float16) if i % 2 == 0 else
          (0.02 * torch.randn(H, generator=g, device=dev)).to(torch.float16) for i in range(4)]
    cl = binding.Client(E, ln[0], ln[1], ln[2], ln[3], max_rows=1)
    se = span.open_session(L + W + K + 2)
    for b in range(NB):
        se.import_kv(b, synth.kv_prefix_device(cfg, b, 0, L, 2.4, dev))
    tok = torch.zeros(W + K + 1, dtype=torch.int32, device=dev)
    tok[0] = 12345 % V
    hid = torch.empty((1, H), dtype=torch.float16, device=dev)
    out = torch.empty((1, H), dtype=torch.float16, device=dev)
    stream = torch.cuda.current_stream()

    sampling = args.temperature > 0.0
    if sampling:     # the uniform numbers of all steps are drawn beforehand: nothing random inside the timed loop
        uniforms = torch.rand(W + K + 1, generator=g, device=dev, dtype=torch.float32).clamp_(max=0.99999994)
        logits = torch.empty((1, V), dtype=torch.float32, device=dev)

    def step(i):
        cl.embed(tok[i:i + 1], out=hid)
        span.decode_step([se], hid, out)
        if sampling:
            binding.petals_client_lm_head(cl.handle, out, logits, None)
            cl.sample(logits, args.temperature, args.top_k, uniforms[i:i + 1], next_out=tok[i + 1:i + 2])
        else:
            cl.lm_head(out, next_out=tok[i + 1:i + 2])

    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for i in range(W, W + K):
        step(i)
    e1.record(stream)
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / K
    # the LM head alone, bracketed by events on the same stream
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(8)]
    nxt = torch.empty(1, dtype=torch.int32, device=dev)
    for a, b_ in ev:
        a.record(stream)
        cl.lm_head(out, next_out=nxt)
        b_.record(stream)
    torch.cuda.synchronize()
    lm_ms = sorted(a.elapsed_time(b_) for a, b_ in ev)[len(ev) // 2]
    lm_bytes = V * H * 2
    distinct = len(set(tok[W + 1:].cpu().tolist()))

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        sample = min(V, 32768)
        Eh = E[:sample].cpu().numpy()
        xh = out.cpu().numpy()
        t0 = time.perf_counter()
        ref = oracle.lm_head(xh, Eh, ln[2].cpu().numpy(), ln[3].cpu().numpy())
        dt = time.perf_counter() - t0
        sub = binding.Client(E[:sample], ln[0], ln[1], ln[2], ln[3], max_rows=1)
        same = int(sub.lm_head(out).cpu()[0]) == int(ref[0])
        sub.close()
        cpu = {"value": round(1.0 / (dt * V / sample), 3), "unit": "LM-head evaluations/s", "cores": oracle.num_threads(),
               "kind": "oracle", "sample": "LM head over the first %d of %d embedding rows (%.2f s), extrapolated; "
               "GPU choice on the same rows %s the oracle's" % (sample, V, dt, "equals" if same else "DIFFERS FROM")}
    line = {
        "metric": "%s generation tokens/s, client ends + 12-block BLOOM-176B span on one GPU (batch 1)"
                  % ("sampled" if sampling else "greedy"),
        "value": round(1e3 / ms, 2), "unit": "tokens/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8 span, fp16 embeddings", "data": "synthetic",
        "config": {"workload": "embedding lookup + LayerNorm, 12-block BLOOM-176B-shaped span decode step at KV prefix %d, "
                               "final LayerNorm + tied LM head (%d x %d fp16) + %s, token fed back on the device"
                               % (L, V, H, ("sampling at temperature %g, top_k %d" % (args.temperature, args.top_k))
                                  if sampling else "greedy choice"),
                   "lm_head_ms": round(lm_ms, 4), "distinct_tokens_generated": distinct},
        "roofline": {"bound": "hbm", "achieved": round(lm_bytes / (lm_ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(lm_bytes / (lm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "kernel": "k_lm_head (LayerNorm and the final pick included in the timed call)"},
        "cpu_baseline": cpu,
    }
    cl.close()
    span.close()
    _emit(args, line)


def run_cpu_baseline(cfg, block0_host, dev, prefix=2048, budget_s=12.0):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: ONE of the 12 blocks, decode steps
    at the headline KV prefix for about `budget_s` seconds of CPU work on this machine's host cores; tokens/s
    extrapolated to 12 blocks.  The same block runs the first step on the GPU and the two outputs are compared."""
    import numpy as np
    import torch
    import oracle
    from paper_2209_01188_amd import binding, synth

    H, F, nh = cfg.hidden, cfg.F, cfg.n_heads
    L, max_steps = prefix, 256
    t0 = time.time()
    osp = oracle.Span(1, H, nh, F, 1e-5, 6.0)
    osp.load_block(0, block0_host)
    ose = osp.open_session(L + max_steps + 2)
    kv = synth.kv_prefix_device(cfg, 0, 0, L, 2.4, dev)
    ose.import_kv(0, kv.cpu().numpy())
    x = synth.hidden_states(cfg, 1, 1, 1)
    print("[bench] oracle block loaded in %.1f s" % (time.time() - t0), file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    y_ref = osp.step([ose], x)
    dt = time.perf_counter() - t0
    n_steps = int(min(max_steps, max(4, round(budget_s / max(dt, 1e-3)))))
    t0 = time.perf_counter()
    for i in range(1, n_steps):
        osp.step([ose], synth.hidden_states(cfg, 1 + i, 1, 1))
    total = dt + (time.perf_counter() - t0)
    # same block, same first step on the GPU
    gsp = binding.Span(1, H, nh, F, 1, 1e-5, 6.0, dev)
    gsp.load_block(0, block0_host)
    gse = gsp.open_session(L + 2)
    gse.import_kv(0, kv)
    y_gpu = gsp.decode_step([gse], torch.from_numpy(x[:, 0]).to(dev)).cpu().numpy()[:, None]
    gsp.close()
    osp.destroy()
    g, r = y_gpu.astype(np.float64), y_ref.astype(np.float64)
    rel = float(np.linalg.norm(g - r) / np.linalg.norm(r))
    exact = float((y_gpu.view(np.uint16) == y_ref.view(np.uint16)).mean())
    print("[bench] oracle: %d block-steps in %.1f s on %d threads; GPU vs oracle rel-L2 %.2e, bit-identical %.4f" %
          (n_steps, total, oracle.num_threads(), rel, exact), file=sys.stderr, flush=True)
    return {"value": round(n_steps / (total * cfg.n_blocks), 4), "unit": "tokens/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "1 of 12 blocks, %d decode steps at KV prefix %d (%.1f s of CPU work), extrapolated "
            "x12; GPU output of the same block's first step: rel-L2 %.1e vs oracle" % (n_steps, L, total, rel)}


if __name__ == "__main__":
    main()
