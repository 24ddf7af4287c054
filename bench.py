#!/usr/bin/env python3
"""Benchmark of the DISCO speculative-decoding hot path on one MI355X.

Workload (full-loop configuration: 13B-class target, 68M-class draft, bf16, batch 1): 16 random prompts
of 512 tokens, 256 new tokens each; every prompt goes through the dense prompt pass of both models,
then speculative iterations run with DISCO halting (cap 10) and 60 % seed-forced draft/target
agreement.  One "step" is one whole iteration: draft steps with the fused feature/classifier kernel,
the target's verification forward, greedy acceptance, KV rollback.  The clock runs inside iterations
only.  `value` counts the tokens emitted per second (accepted draft tokens plus the target's own
token of every iteration), inputs resident in HBM.

Prints ONE JSON line: metric, value, unit, steps, ms_per_step, config (the workload in words), a
`roofline` object for the dominant kernel and a `cpu_baseline` object (the CPU oracle timed on a
bounded sample).  Other modes (--sweep, --micro, --prefill) print one JSON line of their own.
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
TRAFFIC_FILES = {"cfg4": "gemm_gateup_13b_hbm_traffic.txt", "cfg3": "gemm_w1_15b_mqa_hbm_traffic.txt"}


def gateup_traffic_bytes(panels: int, config: str = "cfg4"):
    """HBM bytes per launch of the dominant kernel (the target's MLP-input GEMM) from the rocprofv3 FETCH_SIZE +
    WRITE_SIZE counter summary of that configuration under profiles/ (counters cannot be read from inside this
    process): the line 'traffic_bytes_per_launch panels=<1|2> <bytes>'.  None if the summary is missing or has
    no such line."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", TRAFFIC_FILES[config])
    try:
        for ln in open(path):
            w = ln.split()
            if len(w) == 3 and w[0] == "traffic_bytes_per_launch" and w[1] == f"panels={panels}":
                return int(w[2])
    except OSError:
        pass
    return None


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def cpu_baseline(target_shape, draft_shape, tw_host, dw_host, clf, gamma, tokens_per_iter, ctx, layers_sampled):
    """The oracle as it stands, timed on this host: gamma draft steps (full 68M-class draft) and one
    verification block of gamma + 1 tokens through `layers_sampled` of the target's layers plus
    embedding and LM head; the per-layer time is extrapolated to the full depth."""
    from oracle import disco_oracle as O
    from workloads import synth as W
    t_all0 = time.time()
    od = O.Model(draft_shape, dw_host, kv_bf16=True)
    kv_d = od.new_cache(ctx + 32)
    kv_d.fill(W.make_kv_fill(draft_shape, ctx, 2))
    tok = 17
    t0 = time.time()
    for j in range(gamma):
        logits = od.forward([tok], kv_d)[0]
        f = O.features(logits, j + 1)
        O.classifier(f["feats"], clf)
        tok = f["token"]
    t_draft = time.time() - t0
    blk = W.make_tokens(3, gamma + 1, target_shape.vocab).tolist()
    times = {}
    for nl in (0, layers_sampled):
        sh = W.scaled_shape(target_shape, n_layers=nl)
        om = O.Model(sh, tw_host, kv_bf16=True, cache_upcast=False)
        kv = om.new_cache(ctx + 32)
        if nl:
            kv.fill(W.make_kv_fill(sh, ctx, 2))
        else:
            kv.len = ctx
        t0 = time.time()
        lg = om.forward(blk, kv)
        a = [O.argmax_lowest(lg[r]) for r in range(gamma + 1)]
        O.accept(blk, a)
        times[nl] = time.time() - t0
    per_layer = (times[layers_sampled] - times[0]) / layers_sampled
    t_verify = times[0] + per_layer * target_shape.n_layers      # equals times[layers_sampled] when all layers are sampled
    t_iter = t_draft + t_verify
    return {
        "value": tokens_per_iter / t_iter, "unit": "tokens/s", "cores": torch.get_num_threads(), "kind": "oracle",
        "sample": (f"one iteration at static lookahead {gamma}: {gamma} oracle draft steps (full draft, ctx {ctx}) "
                   f"+ one oracle verification block of {gamma + 1} tokens through {layers_sampled} of "
                   f"{target_shape.n_layers} target layers, embedding and LM head (per-layer time extrapolated "
                   f"to {target_shape.n_layers}); tokens/iteration taken from the GPU run; "
                   f"{time.time() - t_all0:.0f} s of CPU work"),
        "draft_step_ms": 1e3 * t_draft / gamma, "verify_block_ms_extrapolated": 1e3 * t_verify,
    }


def micro(B, W, dev, reps):
    """Draft-step and verification-block micro-benchmarks: wall time per call (host enqueue to device
    idle, `reps` calls back to back) and algorithmic bytes per call / time."""
    def weight_bytes(s):
        return sum(int(torch.tensor(sh).prod()) for n_, sh, kind in W.weight_specs(s)
                   if kind == "matrix" and n_ not in ("tok_emb", "pos_emb")) * 2

    def timed(fn, warm=10, before=None):
        """(wall time per call over `reps` calls enqueued back to back, median of the per-call times between
        two events on the launch stream).  `before`, if given, runs ahead of every call, outside the events."""
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / reps
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in ev:
            if before is not None:
                before()
            e0.record()
            fn()
            e1.record()
        torch.cuda.synchronize()
        per = sorted(e0.elapsed_time(e1) * 1e-3 for e0, e1 in ev)
        return wall, per[len(per) // 2]

    out = {"micro": True, "reps": reps, "n_gpus": 1, "dtype": "bf16", "data": "synthetic", "hbm_peak_gbs": HBM_PEAK_GBS,
           "draft_step": [], "verify_block": []}
    ds = W.CFG1_DRAFT
    gd = B.DiscoModel(ds, W.make_weights(ds, 0, "bf16"), dev)
    clf = B.DiscoClf(W.make_classifier(100), dev)
    steps_rec = B.struct_tensor(B.ClfOut, B.MAX_BLOCK, dev)
    lo_d, lo_h = B.struct_tensor(B.LoopOut, 1, dev), B.struct_tensor(B.LoopOut, 1, pinned=True)
    logits = torch.empty(ds.vocab, dtype=torch.float32, device=dev)
    tok = W.make_tokens(3, 2, ds.vocab).to(dev)
    scratch = B.classify_scratch(dev)
    evict = torch.zeros(1 << 28, dtype=torch.float32, device=dev)          # 1 GiB read and written per eviction
    for ctx in (512, 1024, 2048):
        kv = B.DiscoKV(gd, ctx + 64, 16)
        kv.fill(W.make_kv_fill(ds, ctx, 2).to(dev))
        ws = gd.workspace(B.MAX_BLOCK, ctx + 64)

        def loop10():
            # ten draft steps, each followed by the feature / classifier kernel, no host round trip
            B.disco_draft_loop(gd, kv, clf, tok, 1, 10, 10, 1.0, 0.5, None, logits, steps_rec, lo_d, lo_h, ws)
            B.disco_kv_rollback(kv, ctx)

        out_one = B.struct_tensor(B.ClfOut, 1, dev)

        def step1():
            # one step through the two calls of the boundary (draft forward, then features + classifier)
            B.disco_draft_step(gd, kv, tok, 1, logits, ws)
            B.disco_classify(clf, logits, ds.vocab, 1.0, 0.5, 0, out_one, scratch=scratch)
            B.disco_kv_rollback(kv, ctx)

        t, t_med = timed(loop10)
        t, t_med = t / 10, t_med / 10
        # cold: the memory-side cache (256 MB, larger than the draft's 87 MB of weights) is overwritten before
        # every step, as the target's 26 GB verification forward does before the first draft step of an iteration
        _, t_warm1 = timed(step1)
        _, t_cold1 = timed(step1, warm=2, before=lambda: evict.add_(1))
        nbytes = weight_bytes(ds) + ds.n_layers * 2 * ctx * ds.d_kv * 2 + ds.vocab * 4
        out["draft_step"].append({"ctx": ctx, "us_per_step": 1e6 * t, "us_per_step_median_events": 1e6 * t_med,
                                  "us_single_step_warm_cache": 1e6 * t_warm1, "us_single_step_cold_cache": 1e6 * t_cold1,
                                  "bytes": nbytes, "gbs": nbytes / t / 1e9, "frac": nbytes / t / 1e9 / HBM_PEAK_GBS,
                                  "gbs_cold_cache": nbytes / t_cold1 / 1e9,
                                  "frac_cold_cache": nbytes / t_cold1 / 1e9 / HBM_PEAK_GBS})
        log(f"[bench] draft step ctx {ctx}: {1e6 * t:.1f} us ({1e6 * t_med:.1f} median by events; single step warm "
            f"{1e6 * t_warm1:.1f}, cold {1e6 * t_cold1:.1f}), {nbytes / t / 1e9:.0f} GB/s")
    del gd, evict
    ts = W.CFG2_TARGET
    gt = B.DiscoModel(ts, W.make_weights(ts, 0, "bf16", device=dev), dev)
    torch.cuda.empty_cache()
    ctx = 1024
    kv = B.DiscoKV(gt, ctx + 64, 16)
    kv.fill(W.make_kv_fill(ts, ctx, 2, device=dev))
    ws = gt.workspace(B.MAX_BLOCK, ctx + 64)
    blk = W.make_tokens(3, B.MAX_BLOCK, ts.vocab).to(dev)
    am = torch.zeros(B.MAX_BLOCK, dtype=torch.int32, device=dev)
    acc = B.struct_tensor(B.AcceptOut, 1, dev)
    for m in (1, 2, 4, 8, 11):
        def verify():
            B.disco_verify(gt, kv, blk, m, am, None, ws)
            B.disco_accept(blk, am, m, acc)
            B.disco_kv_rollback(kv, ctx)

        t, t_med = timed(verify)
        nbytes = weight_bytes(ts) + ts.n_layers * 2 * ctx * ts.d_kv * 2 + m * ts.n_layers * 2 * ts.d_kv * 2 + m * ts.vocab * 4
        out["verify_block"].append({"m": m, "ctx": ctx, "ms": 1e3 * t, "ms_median_events": 1e3 * t_med, "bytes": nbytes,
                                    "gbs": nbytes / t / 1e9, "frac": nbytes / t / 1e9 / HBM_PEAK_GBS})
        log(f"[bench] verify block of {m} at ctx {ctx}: {1e3 * t:.3f} ms ({1e3 * t_med:.3f} median by events), {nbytes / t / 1e9:.0f} GB/s")
    return out


def dense_kernel_args(epi, n_tiles, n_groups, bf16_act):
    """Template arguments the library's launch rule picks for a dense GEMM of n_tiles 16-row tiles over n_groups
    token groups: <epilogue, k-tiles in flight, row tiles per wavefront, bf16 activations>."""
    ncb = -(-n_groups // (8 if bf16_act else 4))
    if bf16_act and n_tiles % 8 == 0 and -(-n_tiles // 32) * ncb >= 256:
        return "%d, 3, 8, true" % epi
    rt = 4 if -(-n_tiles // 16) * ncb >= 256 else 2
    return "%d, %d, %d, %s" % (epi, 4 if bf16_act else 5, rt, "true" if bf16_act else "false")


def prefill_bench(B, W, dev, reps, models=("68m_draft", "13b_target"), lengths=(512, 1024, 2048), bf16_act=False):
    """Prompt pass of both models at 512 / 1024 / 2048 tokens: the dense pass against the same prompt fed
    in blocks of 16 through the verification forward.  Rates are ALGORITHMIC flops (2 per weight and
    token in the projections and the LM head of the last token, 4 n ctx d_q / 2 causal attention flops
    per layer; the bf16 hi + lo split of the activations is an implementation cost and not counted)
    over wall time, against the dense bf16 matrix peak."""
    MFMA_PEAK_TFLOPS = 2500.0

    def flops(s, n):
        mats = sum(int(torch.tensor(sh).prod()) for n_, sh, kind in W.weight_specs(s)
                   if kind == "matrix" and n_ not in ("tok_emb", "pos_emb", "wlm"))
        attn = s.n_layers * 4 * (n * (n + 1) // 2) * s.n_heads * s.d_head
        return 2 * mats * n + attn + 2 * s.vocab * s.d_model

    flags = B.PREFILL_BF16_ACTIVATIONS if bf16_act else 0
    out = {"prefill": True, "reps": reps, "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
           "activations": "bf16 (hi panel only)" if bf16_act else "fp32 grade (bf16 hi + lo panels)",
           "mfma_peak_tflops": MFMA_PEAK_TFLOPS, "rows": []}
    for name, shape, on_dev in (("68m_draft", W.CFG1_DRAFT, False), ("13b_target", W.CFG2_TARGET, True),
                                ("mqa_draft", W.CFG3_DRAFT, False), ("15b_mqa_target", W.CFG3_TARGET, True)):
        if name not in models:
            continue
        gm = B.DiscoModel(shape, W.make_weights(shape, 0, "bf16", device=dev if on_dev else "cpu"), dev)
        torch.cuda.empty_cache()
        am = torch.zeros(B.MAX_BLOCK, dtype=torch.int32, device=dev)
        for n in lengths:
            toks = W.make_prompt(1, n, shape.vocab).to(torch.int32).to(dev)
            kv = B.DiscoKV(gm, n + 32, 16)
            pws = gm.prefill_workspace(n, n + 32)
            ws = gm.workspace(B.MAX_BLOCK, n + 32)

            def dense():
                B.disco_kv_rollback(kv, 0)
                B.disco_prefill(gm, kv, toks, n, None, pws, flags=flags)

            def blocks():
                B.disco_kv_rollback(kv, 0)
                for i in range(0, n, B.MAX_BLOCK):
                    B.disco_verify(gm, kv, toks.data_ptr() + 4 * i, B.MAX_BLOCK, am, None, ws)

            res = {}
            for label, fn, r in (("dense", dense, reps), ("blocks", blocks, max(1, reps // 4))):
                fn()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(r):
                    fn()
                torch.cuda.synchronize()
                res[label] = (time.perf_counter() - t0) / r
            # the dominant kernel, the MLP-input GEMM (gate/up + SwiGLU, or W1 + GELU), bracketed by HIP events on
            # the launch stream in the middle layer of `reps` further passes
            B.disco_probe_enable(shape.n_layers // 2)
            probe = []
            for _ in range(reps):
                dense()
                torch.cuda.synchronize()
                probe.append(B.disco_probe_read_ms())
            B.disco_probe_enable(-1)
            rows_in = shape.d_ff if shape.family == "A" else 2 * shape.d_ff
            gemm_flops = 2 * n * shape.d_model * rows_in
            probe_ms = sum(probe) / len(probe)
            fl = flops(shape, n)
            row = {"model": name, "n_tokens": n, "dense_ms": 1e3 * res["dense"], "blocks_ms": 1e3 * res["blocks"],
                   "speedup": res["blocks"] / res["dense"], "flops": fl, "dense_tflops": fl / res["dense"] / 1e12,
                   "frac_of_mfma_peak": fl / res["dense"] / 1e12 / MFMA_PEAK_TFLOPS,
                   "tokens_per_s": n / res["dense"],
                   "roofline": {"bound": "mfma", "achieved": gemm_flops / probe_ms / 1e9, "peak": MFMA_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": gemm_flops / probe_ms / 1e9 / MFMA_PEAK_TFLOPS, "traffic": None,
                                "kernel": "k_gemm_dense<%s> (MLP-input GEMM of the prompt pass)" % dense_kernel_args(
                                    4 if shape.family == "A" else 3, rows_in // 16, (n + 15) // 16, bf16_act),
                                "flops_per_launch": gemm_flops, "avg_launch_ms": probe_ms, "launches_timed": len(probe),
                                "note": ("algorithmic flops = matrix-unit flops (bf16 activations)" if bf16_act else
                                         "algorithmic flops; the bf16 hi + lo activation panels make the matrix unit do twice as many")}}
            out["rows"].append(row)
            log(f"[bench] prompt pass {name} n {n}: dense {row['dense_ms']:.2f} ms ({row['dense_tflops']:.0f} TFLOP/s), "
                f"blocks of 16 {row['blocks_ms']:.2f} ms, x{row['speedup']:.2f}")
            del kv, pws, ws
        del gm
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None,
                    help="timed iterations (default: every prompt to its end for the full loop, 60 for the other modes)")
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--policy", default="disco", choices=["disco", "disco-seeded", "static"],
                    help="disco: DISCO halting with the classifier TRAINED before the clock starts (labelling run on a further "
                         "prompt, disco_clf_train); disco-seeded: the untrained seeded classifier; static: fixed lookahead --gamma")
    ap.add_argument("--train-tokens", type=int, default=200, help="labelled positions of the classifier's training run")
    ap.add_argument("--gamma", type=int, default=5)
    ap.add_argument("--tau", type=float, default=0.5)
    ap.add_argument("--sl-max", type=int, default=10)
    ap.add_argument("--alpha", type=float, default=0.6)
    ap.add_argument("--prompt-len", type=int, default=None, help="prompt tokens (default 512; 2048 for --config cfg3)")
    ap.add_argument("--layers", type=int, default=0, help="debug: truncate the target (invalidates the number)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--temperature", type=float, default=0.0,
                    help="> 0: sampled draft tokens and speculative-sampling acceptance at this temperature "
                         "(no forced agreement); 0: the greedy workload")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the single timed run: static lookahead 1..sl-max and DISCO halting on the same "
                         "prompt and forcing, one JSON line with a row per policy")
    ap.add_argument("--grid", action="store_true",
                    help="with --sweep: also the trained classifier over thresholds 0.3 / 0.5 / 0.7 x lookahead caps 5 / 10 / 15")
    ap.add_argument("--prefill", action="store_true",
                    help="instead of the loop: the prompt pass of the 68M-class and the 13B-class model at 512 / 1024 / 2048 "
                         "tokens, dense pass against blocks of 16 through the verification forward; one JSON line "
                         "(--steps = repetitions of the dense pass)")
    ap.add_argument("--prefill-models", default="68m_draft,13b_target",
                    help="models of --prefill, comma separated, of 68m_draft, 13b_target, mqa_draft, 15b_mqa_target")
    ap.add_argument("--prefill-bf16-act", action="store_true",
                    help="--prefill with DISCO_PREFILL_BF16_ACTIVATIONS (activations rounded to bf16: half the matrix work)")
    ap.add_argument("--prefill-lengths", default="512,1024,2048", help="prompt lengths of --prefill (comma separated)")
    ap.add_argument("--micro", action="store_true",
                    help="instead of the loop: the draft-step micro-benchmark (68M-class shape, KV context 512 / 1024 / "
                         "2048) and the verification-block micro-benchmark (13B-class shape, context 1024, blocks of "
                         "1, 2, 4, 8, 11 tokens); one JSON line")
    ap.add_argument("--prompts", type=int, default=None,
                    help="number of prompts (seeds 1, 2, ..): the timed iterations run through them one after another, each "
                         "prompt generating --new-tokens tokens; prompt pass and forcing set-up between prompts are untimed")
    ap.add_argument("--new-tokens", type=int, default=None,
                    help="tokens generated per prompt when --prompts > 1 (then --steps 0 runs every prompt to its end)")
    ap.add_argument("--config", default="cfg4", choices=["cfg4", "cfg3"],
                    help="cfg4 (default, the headline): 13B-class target + 68M-class draft, 16 prompts of 512 tokens, 256 new "
                         "tokens each; cfg3: the multi-query code-model pair (15B-class LayerNorm / GELU target with one KV head, "
                         "12-layer draft that reuses the target's embedding table), one prompt of 2048 tokens, 128 new tokens")
    ap.add_argument("--chunk", type=int, default=0,
                    help="draft steps enqueued between two looks at the halt flag (0 = library default, >= sl-max: whole loop at once)")
    ap.add_argument("--launch-mode", type=int, default=0, choices=[0, 1, 2],
                    help="0: one launch per phase, QKV projection + attention of a layer in one launch (default); 1: one cooperative "
                         "launch per forward / draft loop; 2: one launch per phase, nothing fused (disco_set_launch_mode)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run plain device copies of known size and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    cfg3 = args.config == "cfg3"
    if args.prompt_len is None:
        args.prompt_len = 2048 if cfg3 else 512
    if args.prompts is None:
        args.prompts = 1 if cfg3 else 16
    if args.new_tokens is None:
        args.new_tokens = 128 if cfg3 else 256
    if args.sweep or args.temperature > 0 or args.micro or args.prefill:
        args.prompts = 1                      # these modes run one prompt
    run_to_end = args.steps is None and (args.prompts > 1 or cfg3) and not (args.sweep or args.temperature > 0)
    if args.steps is None:
        args.steps = 0 if run_to_end else 60
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (one process, one sequence); --gpus must be 1. "
              "The path shards by sequence across GPUs with no exchange: one process per GPU, each with its own prompts.", file=sys.stderr)
        sys.exit(2)
    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    dev = torch.device("cuda:0")

    if args.calibrate_copy:
        # 256 MiB read + 256 MiB written per launch: the counter reading of this kernel is the scale
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(10):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": True, "bytes_read_per_launch": 256 << 20, "bytes_written_per_launch": 256 << 20}))
        return

    from paper_2405_04304_amd import binding as B
    from paper_2405_04304_amd.engine import SpecEngine
    from workloads import synth as W

    B.disco_set_launch_mode(args.launch_mode)
    if args.micro:
        out = micro(B, W, dev, args.steps)
        out["launch_mode"] = args.launch_mode
        print(json.dumps(out), flush=True)
        return
    if args.prefill:
        print(json.dumps(prefill_bench(B, W, dev, args.steps, tuple(args.prefill_models.split(",")),
                                       tuple(int(x) for x in args.prefill_lengths.split(",")), args.prefill_bf16_act)), flush=True)
        return

    full_target = W.CFG3_TARGET if cfg3 else W.CFG2_TARGET
    target_shape = full_target if not args.layers else W.scaled_shape(full_target, n_layers=args.layers)
    draft_shape = W.CFG3_DRAFT if cfg3 else W.CFG1_DRAFT
    t0 = time.time()
    tw = W.make_weights(target_shape, 0, "bf16", device=dev)
    dw = W.make_weights(draft_shape, 10, "bf16", device="cpu")
    if cfg3:
        # the draft reuses the target's token embeddings: the first d_draft columns of the target's table
        dw["tok_emb"] = tw["tok_emb"][:, :draft_shape.d_model].cpu()
    clf = W.make_classifier(100)
    layers_sampled = target_shape.n_layers        # the oracle walks the whole target once (about 10 s of CPU work)
    tw_host = None
    if not args.no_cpu_baseline:
        keep = lambda k: (not k.startswith("l")) or int(k[1:k.index(".")]) < layers_sampled
        tw_host = {k: v.cpu() for k, v in tw.items() if keep(k)}
    gt = B.DiscoModel(target_shape, tw, dev)
    del tw
    torch.cuda.empty_cache()
    gd = (B.DiscoModel(draft_shape, dw, dev, tok_emb=gt.tok_emb, tok_emb_stride=target_shape.d_model) if cfg3
          else B.DiscoModel(draft_shape, dw, dev))
    log(f"[bench] weights ready in {time.time() - t0:.1f} s")

    n_iter = args.warmup + args.steps if not run_to_end else 10 ** 9
    cap = args.gamma if args.policy == "static" else args.sl_max
    max_new = min(n_iter, 10 ** 6) * (cap + 1) + 2   # enough text for every iteration at full acceptance
    prompt = W.make_prompt(1, args.prompt_len, target_shape.vocab).tolist()
    multi = args.prompts > 1 or run_to_end
    if multi:
        assert not args.sweep and args.temperature <= 0, "--prompts > 1 and --config cfg3 run the greedy loop only"
        max_new = args.new_tokens
    eng = SpecEngine(gt, gd, B.DiscoClf(clf, dev), max_ctx=args.prompt_len + max_new + 16, page_tokens=16)

    # untimed input shaping: the target's own greedy text decides which draft logits get forced
    t0 = time.time()
    n_greedy = max_new if multi else min(max_new, int(n_iter * 3.2) + 32)
    greedy = eng.greedy(prompt, n_greedy, progress=lambda i: log(f"[bench] greedy target token {i}/{n_greedy}"))
    greedy += [0] * (max_new - n_greedy)
    mask = W.make_force_mask(5, max_new, args.alpha)
    mask[n_greedy:] = False
    force = {"mask": mask, "tokens": greedy}
    log(f"[bench] prefill + {n_greedy} greedy target tokens in {time.time() - t0:.1f} s")

    policy = ({"mode": "static", "gamma": args.gamma} if args.policy == "static" else
              {"mode": "disco", "tau": args.tau, "sl_max": args.sl_max, "pos_mode": "absolute"})
    policy["chunk"] = args.chunk

    # algorithmic bytes (bf16 weights once per forward, live KV once per forward, fp32 logits)
    def fwd_bytes(s, ctx, m):
        w = sum(int(torch.tensor(sh).prod()) for n_, sh, kind in W.weight_specs(s)
                if kind == "matrix" and n_ not in ("tok_emb", "pos_emb")) * 2
        kv = s.n_layers * 2 * ctx * s.d_kv * 2
        return w + kv + m * s.n_layers * 2 * s.d_kv * 2 + m * s.vocab * 4

    if args.sweep:
        rows = []
        pols = [{"mode": "static", "gamma": g} for g in range(1, args.sl_max + 1)] + [policy]
        # upper bound (Sec. 3, oracle SL): draft until the first token that leaves the target's known text
        pols.append({"mode": "oracle", "reference": greedy, "sl_max": 15})
        # DISCO with a TRAINED classifier (Sec. 4, App. D.1): labelling run on another prompt with the same
        # forcing recipe, training on the GPU, F1 on this prompt's labelling run
        n_lab = min(n_greedy, 200)
        prompt2 = W.make_prompt(2, args.prompt_len, target_shape.vocab).tolist()
        greedy2 = eng.greedy(prompt2, n_lab)
        mask2 = W.make_force_mask(6, n_lab, args.alpha)
        f_tr, y_tr, _ = eng.label_run(prompt2, greedy2, {"mask": mask2, "tokens": greedy2})
        clf_plain, clf_trained = eng.clf, B.DiscoClf(clf, dev)
        B.disco_clf_train(f_tr, y_tr, n_lab, clf_trained.hidden, 400, 0.5, clf_trained.dev, None)
        f_va, y_va, _ = eng.label_run(prompt, greedy[:n_lab], {"mask": mask[:n_lab], "tokens": greedy})
        counts = torch.zeros(4, dtype=torch.int32, device=dev)
        B.disco_clf_eval(clf_trained, f_va, y_va, n_lab, args.tau, None, counts)
        tp, fp, fn, tn = counts.cpu().tolist()
        f1 = 2 * tp / max(2 * tp + fp + fn, 1)
        log(f"[bench] trained classifier: validation F1 {f1:.3f} (tp {tp} fp {fp} fn {fn} tn {tn})")
        pols.append({"mode": "disco", "tau": args.tau, "sl_max": args.sl_max, "pos_mode": "absolute", "classifier": "trained",
                     "validation_f1": f1})
        # the two rule-based baselines the paper compares with (Sec. 2 footnote; App. F).  The perplexity
        # threshold is tuned, as App. F says, on validation text: a few candidate values (quantiles of
        # 1 / largest probability over the labelling run of the other prompt), each timed on a short run
        pols.append({"mode": "heuristic", "start": 5, "up": 2, "down": 1, "sl_max": args.sl_max})
        inv_p = torch.sort(1.0 / f_tr[:n_lab, 0].float().cpu()).values
        best_thr, best_rate = None, 0.0
        for q in (0.2, 0.35, 0.5, 0.65, 0.8):
            thr = float(inv_p[int(q * (n_lab - 1))]) * 1.001
            eng.reset()
            eng.prefill(prompt2[:-1])
            torch.cuda.synchronize()
            t1 = time.perf_counter()
            r = eng.generate(prompt2, n_lab, {"mode": "ppl", "threshold": thr, "sl_max": args.sl_max},
                             force={"mask": mask2, "tokens": greedy2}, do_prefill=False, max_iterations=12)
            torch.cuda.synchronize()
            rate = sum(len(it["emit"]) for it in r["iterations"]) / (time.perf_counter() - t1)
            log(f"[bench] perplexity threshold {thr:.1f}: {rate:.1f} tokens/s on the validation prompt")
            if rate > best_rate:
                best_thr, best_rate = thr, rate
        pols.append({"mode": "ppl", "threshold": best_thr, "sl_max": args.sl_max})
        if args.grid:
            # threshold x lookahead-cap grid for the trained classifier (the structure of the paper's Table 5)
            pols += [{"mode": "disco", "tau": t, "sl_max": c, "pos_mode": "absolute", "classifier": "trained", "grid": True}
                     for t in (0.3, 0.5, 0.7) for c in (5, 10, 15) if (t, c) != (args.tau, args.sl_max)]
        for pol in pols:
            stamps = []

            def tick(it):
                torch.cuda.synchronize()
                stamps.append(time.perf_counter())

            eng.clf = clf_trained if pol.get("classifier") == "trained" else clf_plain
            eng.reset()
            eng.prefill(prompt[:-1])
            torch.cuda.synchronize()
            gc.collect()
            gc.disable()                      # no collector pauses inside the timed iterations
            stamps.append(time.perf_counter())
            res = eng.generate(prompt, max_new, pol, force=force, do_prefill=False, on_iteration=tick,
                               max_iterations=n_iter)
            gc.enable()
            its = res["iterations"][args.warmup:]
            dt = stamps[n_iter] - stamps[args.warmup]
            emitted = sum(len(it["emit"]) for it in its)
            drafted = sum(it["sl"] for it in its)
            ctx_mid = args.prompt_len + emitted // 2
            nbytes = len(its) * fwd_bytes(target_shape, ctx_mid, 1) + drafted * fwd_bytes(draft_shape, ctx_mid, 1)
            rows.append({"policy": {k: v for k, v in pol.items() if k != "reference"}, "sl_hist": res["sl_hist"], "iterations_per_s": len(its) / dt, "tokens_per_s": emitted / dt,
                         "tokens_per_iteration": emitted / len(its), "drafted_per_iteration": drafted / len(its),
                         "accepted_per_iteration": sum(it["n"] for it in its) / len(its),
                         "hbm_gbs": nbytes / dt / 1e9, "ms_per_iteration": 1e3 * dt / len(its),
                         "ms_per_iteration_median": 1e3 * sorted(
                             stamps[i + 1] - stamps[i] for i in range(args.warmup, n_iter))[len(its) // 2]})
            log(f"[bench] sweep {rows[-1]['policy']}: {rows[-1]['tokens_per_s']:.1f} tokens/s, {rows[-1]['iterations_per_s']:.1f} it/s")
        # the reference point of the paper's speed-ups (Table 1, row "Target"): the target decoding alone on the same prompt
        eng.reset()
        eng.prefill(prompt[:-1])
        torch.cuda.synchronize()
        t_stamps = [time.perf_counter()]

        def tick_target(it):
            torch.cuda.synchronize()
            t_stamps.append(time.perf_counter())

        eng.generate(prompt, 8 + min(args.steps, 64), {"mode": "static", "gamma": 0}, do_prefill=False, on_iteration=tick_target)
        target_tps = (len(t_stamps) - 9) / (t_stamps[-1] - t_stamps[8])
        for r in rows:
            r["speedup_vs_target_only"] = r["tokens_per_s"] / target_tps
        log(f"[bench] target alone: {target_tps:.1f} tokens/s")
        print(json.dumps({"sweep": rows, "target_only_tokens_per_s": target_tps, "steps": args.steps, "warmup": args.warmup,
                          "alpha": args.alpha, "prompt_len": args.prompt_len, "n_gpus": 1, "data": "synthetic", "dtype": "bf16"}),
              flush=True)
        return

    # DISCO's classifier is TRAINED before the clock starts (Sec. 4 "SL classifier training", App. D.1): labelling
    # run of the draft over the target's greedy text of a FURTHER prompt under the same forcing recipe, full-batch
    # training on the GPU, F1 on the first timed prompt's labelling run.  (With noise weights the seeded classifier
    # never halts: DISCO would be static lookahead at the cap.)
    clf_info = {"trained": False}
    if args.policy == "disco" and args.temperature <= 0:
        t0 = time.time()
        n_lab = min(args.train_tokens, max_new, B.TRAIN_MAX_N)
        seed_tr = 1000 + args.prompts
        prompt_tr = W.make_prompt(seed_tr, args.prompt_len, target_shape.vocab).tolist()
        greedy_tr = eng.greedy(prompt_tr, n_lab)
        mask_tr = W.make_force_mask(seed_tr, n_lab, args.alpha)
        f_tr, y_tr, _ = eng.label_run(prompt_tr, greedy_tr, {"mask": mask_tr, "tokens": greedy_tr})
        trained = B.DiscoClf(clf, dev)
        B.disco_clf_train(f_tr, y_tr, n_lab, trained.hidden, 400, 0.5, trained.dev, None)
        n_val = min(n_lab, n_greedy)
        f_va, y_va, _ = eng.label_run(prompt, greedy[:n_val], {"mask": mask[:n_val], "tokens": greedy})
        counts = torch.zeros(4, dtype=torch.int32, device=dev)
        B.disco_clf_eval(trained, f_va, y_va, n_val, args.tau, None, counts)
        tp, fp, fn, tn = counts.cpu().tolist()
        eng.clf = trained
        clf_info = {"trained": True, "train_positions": n_lab, "train_prompt_seed": seed_tr, "epochs": 400, "lr": 0.5,
                    "validation_f1": 2 * tp / max(2 * tp + fp + fn, 1), "validation_positions": n_val}
        log(f"[bench] classifier trained on {n_lab} positions in {time.time() - t0:.1f} s, validation F1 {clf_info['validation_f1']:.3f}")

    # the timed region: a hand-rolled loop over engine iterations so that exactly K are timed
    probe_layer = target_shape.n_layers // 2
    B.disco_probe_enable(probe_layer)
    probe_ms, stamps = [], []

    def on_iter(it):
        torch.cuda.synchronize()
        stamps.append(time.perf_counter())
        probe_ms.append(B.disco_probe_read_ms())
        if len(probe_ms) % 10 == 0:
            log(f"[bench] iteration {len(probe_ms)}" + (f"/{n_iter}" if n_iter < 10 ** 9 else ""))

    # Iterations run prompt after prompt until warmup + steps of them are done; the clock runs only inside
    # iterations (each is bracketed by a device synchronisation), so the prompt pass and the forcing set-up
    # of the later prompts are outside the timed region.
    its, deltas, hist = [], [], {}
    prompts_run, tokens_generated = 0, 0
    for p_idx in range(args.prompts):
        if len(its) >= n_iter:
            break
        prompts_run += 1
        if p_idx > 0:
            prompt = W.make_prompt(1 + p_idx, args.prompt_len, target_shape.vocab).tolist()
            greedy = eng.greedy(prompt, n_greedy)
            mask = W.make_force_mask(5 + p_idx, max_new, args.alpha)
            force = {"mask": mask, "tokens": greedy}
            log(f"[bench] prompt {p_idx + 1}/{args.prompts}: {len(its)} iterations so far")
        eng.reset()
        eng.prefill(prompt[:-1])
        torch.cuda.synchronize()
        gc.collect()
        gc.disable()                          # no collector pauses inside the timed iterations
        first = len(stamps)
        stamps.append(time.perf_counter())
        if args.temperature > 0:
            uni = {k: W.make_uniforms(21, max_new + 16, k) for k in ("draft", "accept", "resample")}
            res = eng.generate_sampling(prompt, max_new, policy, args.temperature, uni, do_prefill=False,
                                        on_iteration=on_iter, max_iterations=n_iter - len(its))
        else:
            res = eng.generate(prompt, max_new, policy, force=force, do_prefill=False, on_iteration=on_iter,
                               max_iterations=n_iter - len(its))
        torch.cuda.synchronize()
        gc.enable()
        its += res["iterations"]
        tokens_generated += len(res["tokens"])
        deltas += [stamps[i + 1] - stamps[i] for i in range(first, len(stamps) - 1)]
        for k, v in res["sl_hist"].items():
            hist[k] = hist.get(k, 0) + v
    B.disco_probe_enable(-1)
    # The paper's reference point (Table 1, row "Target"): the target model decoding on its own, one token per forward, on
    # the last prompt of the run.  Same library path (disco_iterate without a draft model), 8 warm-up + 48 timed tokens.
    target_only = None
    if args.temperature <= 0 and not args.layers:
        eng.reset()
        eng.prefill(prompt[:-1])
        torch.cuda.synchronize()
        t_stamps = [time.perf_counter()]

        def on_target_token(it):
            torch.cuda.synchronize()
            t_stamps.append(time.perf_counter())

        eng.generate(prompt, 56, {"mode": "static", "gamma": 0}, do_prefill=False, on_iteration=on_target_token)
        dt = (t_stamps[-1] - t_stamps[8]) / (len(t_stamps) - 9)
        target_only = {"tokens_per_s": 1.0 / dt, "ms_per_token": 1e3 * dt, "tokens_timed": len(t_stamps) - 9,
                       "kv_context": args.prompt_len + 8 + (len(t_stamps) - 9) // 2}
        log(f"[bench] target alone: {1e3 * dt:.3f} ms per token")
    if run_to_end or (multi and args.steps == 0):   # every prompt to its end
        n_iter = len(its)
        args.steps = n_iter - args.warmup
    assert len(its) == n_iter == len(deltas), (len(its), len(deltas), n_iter, "not enough text: raise --prompts or --new-tokens")
    t_timed = sum(deltas[args.warmup:])
    timed = its[args.warmup:]
    emitted = sum(len(it["emit"]) for it in timed)
    drafted = sum(it["sl"] for it in timed)
    accepted = sum(it["n"] for it in timed)
    ms_per_step = 1e3 * t_timed / args.steps
    value = emitted / t_timed

    # context of the timed iterations as they ran (KV length before the verification block)
    ctx_mid = sum(it["ctx"] for it in timed) / len(timed)
    iter_bytes = fwd_bytes(target_shape, ctx_mid, 1 + drafted / args.steps) + (drafted / args.steps) * fwd_bytes(draft_shape, ctx_mid, 1)
    # the MLP-input matrix: gate + up (SwiGLU family) or W1 (GELU family), bf16
    gemm_bytes = (1 if target_shape.family == "A" else 2) * target_shape.d_ff * target_shape.d_model * 2
    pm = [p for p in probe_ms[args.warmup:] if p > 0]
    gemm_ms = sum(pm) / len(pm)
    achieved = gemm_bytes / (gemm_ms * 1e-3) / 1e9
    # which form of the dominant kernel the timed blocks ran: one activation panel (blocks of <= 8 tokens) or two
    n_two = sum(1 for it in timed if it["sl"] + 1 > 8)
    panels = 2 if n_two * 2 > len(timed) else 1
    # measured HBM traffic of that kernel: from the counter summary of the configuration under profiles/
    traffic = gateup_traffic_bytes(panels, args.config) if not args.layers else None
    out = {
        "metric": ("accepted tokens/s at the 15B multi-query code-model pair, bf16 (verify+draft achieved HBM GB/s in roofline)" if cfg3 else
                   "accepted tokens/s at 13B/68M bf16 (verify+draft achieved HBM GB/s in roofline)"),
        "value": value, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_step_median": 1e3 * sorted(deltas[args.warmup:])[args.steps // 2],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": (("full DISCO loop, multi-query code-model pair: 15B-class target (40 layers, d 6144, 48 query heads x 128 with "
                          "one KV head, GELU 24576, LayerNorm, learned positions, vocab 49152) + 12-layer draft (d 768, 12 query heads "
                          "x 64 with one KV head, GELU 3072) that reads the first 768 columns of the target's embedding table, "
                          "bf16 weights and KV, batch 1; " if cfg3 else
                          "full DISCO loop, 13B-class target (40 layers, d 5120, 40x128 heads, SwiGLU 13824, vocab 32000) "
                          "+ 68M-class draft (2 layers, d 768), bf16 weights and KV, batch 1; ")
                         + (f"{prompts_run} random prompt(s) of {args.prompt_len} tokens (seeds 1..{prompts_run})"
                            + (f", {args.new_tokens} new tokens each" if multi else "")
                            + f": {len(its)} speculative iterations ran ({tokens_generated} tokens generated), the last "
                            + f"{args.steps} of them timed after {args.warmup} warm-up iterations; mean KV context of the timed "
                            + f"iterations {ctx_mid:.0f}; ")
                         + (f"greedy, forced acceptance {args.alpha}" if args.temperature <= 0 else
                            f"sampling at temperature {args.temperature} (speculative-sampling acceptance, caller-supplied uniforms)")),
            "prompts_run": prompts_run, "iterations_run": len(its), "tokens_generated": tokens_generated,
            "classifier": clf_info,
            "policy": policy, "target_layers": target_shape.n_layers,
            "tokens_counted": "accepted draft tokens + the target's token of each iteration",
        },
        "iterations_per_s": args.steps / t_timed,
        "tokens_per_iteration": emitted / args.steps,
        "accepted_draft_tokens_per_iteration": accepted / args.steps,
        "drafted_tokens_per_iteration": drafted / args.steps,
        "sl_hist": dict(sorted(hist.items())),
        "iteration_hbm_gbs": iter_bytes / (t_timed / args.steps) / 1e9,
        "iteration_hbm_frac": iter_bytes / (t_timed / args.steps) / 1e9 / HBM_PEAK_GBS,
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
            "traffic": traffic,
            "traffic_source": (None if traffic is None else
                               "profiles/" + TRAFFIC_FILES[args.config] + " (rocprofv3 FETCH_SIZE + WRITE_SIZE per dispatch, "
                               "scaled by a plain copy)"),
            # template arguments: panels, row tiles per workgroup (24576 rows run 96-row workgroups, 27648 rows 128-row
            # ones), epilogue, wavefronts, register buffers, deferred LayerNorm
            "kernel": ("k_gemm<%d, %d, %d, 8, %d, %s> (target %s; %d of the %d timed blocks had more than 8 tokens and ran the "
                       "two-panel form)" % (panels, 6 if cfg3 else 8, 4 if cfg3 else 3,
                                            4 if cfg3 else (2 if panels == 2 else 3), "true" if cfg3 else "false",
                                            "W1 GEMM + GELU" if cfg3 else "gate/up GEMM + SwiGLU", n_two, len(timed))),
            "bytes_per_launch": gemm_bytes, "avg_launch_ms": gemm_ms, "launches_timed": len(pm),
            "timing": f"HIP events around the launch of layer {probe_layer} in every timed verification forward",
        },
    }
    if target_only is not None:
        out["target_only"] = target_only
        out["speedup_vs_target_only"] = value / target_only["tokens_per_s"]
    if not args.no_cpu_baseline:
        g = max(1, round(drafted / args.steps))
        out["cpu_baseline"] = cpu_baseline(target_shape, draft_shape, tw_host, dw, clf, g, emitted / args.steps,
                                           args.prompt_len, layers_sampled)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
