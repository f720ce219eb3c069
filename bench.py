#!/usr/bin/env python3
"""Benchmark of the predict / verify / commit decode path on one MI355X.

Workload: the medium hourglass (d=1024, 16 heads, 4+4 / 8+8 / 16 blocks, 1027-token vocabulary, 4096x1024
condition memory), batch 1, 2000 faces = 18000 tokens of K/V context, draft block 9 ("9-9" schedule).
Weights are seeded random-init, the condition memory is N(0,1): synthetic stand-ins with the shapes of the
paper's workload (the paper measures trained models on ShapeNetV2 / gObjaverse meshes).

A step is one pass of the whole hot path: fm_draft -> fm_verify_block -> fm_commit.  Because random-init
draft heads are almost never right, the headline run uses the library's replay draft source: every head
still runs, then each draft token is replaced by the known greedy continuation with probability 0.93
(which reproduces the mean accepted lengths the paper reports for its 9-9 model) or by a wrong id.  The
native-head and sequential figures are reported next to it.

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_PEAK_TFLOPS = 2500.0   # dense fp16 / bf16
REPLAY_P = 0.93
REPLAY_SEED = 20251115


def cpu_baseline(cfg, weights, mem, seconds=20.0):
    """Times the CPU oracle (as it stands) on a bounded sample of the same workload."""
    import numpy as np
    from oracle import speculative as osp
    from oracle.hourglass import Model, SeqState
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    model = Model(cfg, weights, work=np.float64)
    budget = cfg.max_tokens
    st = SeqState(model, mem, budget)
    t0 = time.time()
    steps = 0
    while time.time() - t0 < seconds and st.P < budget:
        block = osp.draft(model, st, budget)
        _, y, a = osp.verify(model, st, block)
        osp.commit(model, st, block, y, a)
        steps += 1
    dt = time.time() - t0
    return {"value": st.P / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"first {steps} speculative steps ({st.P} tokens) of the same workload, native draft heads, "
                      f"float64 NumPy, {dt:.1f} s"}


def counter_traffic(config_index, persistent):
    """HBM bytes per launch of the dominant kernel from the committed hardware-counter summary (two rocprofv3
    --pmc runs of `bench.py --counter-pass`, scaled by a copy kernel of known size); None when there is none
    for this workload."""
    if config_index != 2 or not persistent:
        return None
    path = os.path.join(ROOT, "profiles", "k_verify_persist_config2_b1_hbm_counters.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1])
    except OSError:
        pass
    return None


def forced_fill(fm, cfg, torch, target, seed=7):
    """Bring every sequence to `target` committed tokens without a greedy stream: whole blocks of seeded random
    coordinate tokens are verified (which writes their K/V rows) and committed by force (the caller owns the
    accepted lengths it hands to fm_commit).  Deterministic: the same call leaves the same state every time."""
    tok, ln = fm.new_block()
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    gen = torch.Generator(device="cuda").manual_seed(seed)
    fm.set_draft_replay(None, 0, 0.0, 0)
    fm.set_budget(target // 9)
    while True:
        for _ in range(50):
            fm.draft(tok, ln)
            tok[:, 1:] = torch.randint(0, cfg.n_bins, (cfg.batch, cfg.block_max - 1), generator=gen,
                                       device="cuda", dtype=torch.int32)
            ln[:] = torch.where(ln > 0, torch.full_like(ln, cfg.block_max), ln)
            fm.verify_block(tok, ln, None, acc)
            fm.commit(ln)
        if int(fm.read_state()[:, 4].min()) == 1:      # every sequence has reached the budget
            return


def time_verify(fm, torch, tok, ln, acc, iters):
    """Average duration of fm_verify_block on the block in (tok, ln), HIP events on the library's stream."""
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        fm.verify_block(tok, ln, None, acc)
    ev0.record(fm.stream)
    for _ in range(iters):
        fm.verify_block(tok, ln, None, acc)
    ev1.record(fm.stream)
    torch.cuda.synchronize()
    return ev0.elapsed_time(ev1) / iters


def half_context_leg(fm, cfg, torch, mems_dev, faces, steps, warmup):
    """The decode step at half context for a configuration whose whole generation does not fit a default run
    (several sequences): forced fill to faces/2, a short native continuation to learn the greedy stream from there,
    the identical fill again, then `warmup` untimed and `steps` timed steps of draft -> verify -> commit with the
    replay draft source (p = REPLAY_P) on that continuation, and the verify pass alone for the roofline."""
    half = 9 * (faces // 2)
    # the continuation must outlast the warm-up and timed steps even if every block is accepted whole
    cont = min((steps + warmup) * cfg.block_max // 9 + 3, faces - faces // 2)

    def fill():
        for q in range(cfg.batch):
            fm.prefill_condition(q, mems_dev[q])
        forced_fill(fm, cfg, torch, half)
    fill()
    out, n, _ = fm.generate(faces // 2 + cont, True)        # native heads from the filled state
    stream, nt = out.clone(), int(n.min().item())
    fill()
    fm.set_draft_replay(stream, nt, REPLAY_P, REPLAY_SEED)
    fm.set_budget(faces // 2 + cont)
    tok, ln = fm.new_block()
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    for _ in range(warmup):
        fm.draft(tok, ln)
        fm.verify_block(tok, ln, None, acc)
        fm.commit(acc)
    torch.cuda.synchronize()
    p0 = fm.read_state()[:, 0].sum()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record(fm.stream)
    for _ in range(steps):
        fm.draft(tok, ln)
        fm.verify_block(tok, ln, None, acc)
        fm.commit(acc)
    ev1.record(fm.stream)
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1)
    state = fm.read_state()
    tokens = int(state[:, 0].sum() - p0)
    assert int(state[:, 4].max()) == 0, "the continuation was too short for the timed steps"
    fm.draft(tok, ln)
    nbytes = fm.verify_bytes()
    ms_verify = time_verify(fm, torch, tok, ln, acc, 10)
    gbs = nbytes / (ms_verify * 1e-3) / 1e9
    return {"tokens_per_s": tokens / ms * 1e3, "ms_per_step": ms / steps, "steps": steps, "tokens": tokens,
            "mean_accepted_per_sequence": tokens / steps / cfg.batch,
            "context_tokens_per_sequence": [int(v) for v in state[:, 0]],
            "roofline": {"bound": "hbm", "kernel": "verify pass at half context (all launches of fm_verify_block)" if fm.verify_path() == 0
                         else "k_verify_persist at half context (fm_verify_block)",
                         "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS,
                         "traffic": None, "algorithmic_bytes": nbytes, "ms": ms_verify}}


class _Totals:
    steps = 0
    tokens = 0
    ms_total = 0.0
    nonfinite_rows = 0


def generate_in_stages(fm, faces, what, stage=500):
    """fm_generate to `faces` faces in stages of `stage` faces (the budget is raised and the loop resumes), with a
    progress line on stderr after each: a long generation then never looks hung.  Totals over the stages."""
    tot = _Totals()
    done = 0
    while done < faces:
        done = min(done + stage, faces)
        out, n, st = fm.generate(done, True)
        tot.steps += int(st.steps)
        tot.tokens += int(st.tokens)
        tot.ms_total += float(st.ms_total)
        tot.nonfinite_rows += int(st.nonfinite_rows)
        print(f"bench: {what}: {done} / {faces} faces, {tot.steps} steps, {tot.ms_total / 1e3:.1f} s", file=sys.stderr, flush=True)
    return out, n, tot


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="timed decode steps; 0 = the whole generation")
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2)
    ap.add_argument("--faces", type=int, default=0, help="override the face budget (0 = the configuration's)")
    ap.add_argument("--draft", default="", help="override the draft counts: Dc,m,n (coordinate heads, point tokens, face tokens)")
    ap.add_argument("--batch", type=int, default=0, help="override the number of sequences of the configuration")
    ap.add_argument("--model", default="",
                    help="override width and depth: d,H,c,v,f = d_model, heads, blocks at the coordinate / point / face level "
                         "(c and v split evenly before and after the coarser level), e.g. 1536,16,4,8,12 for the paper's "
                         "model with 96-wide heads; head widths other than 64 run one launch per operator")
    ap.add_argument("--window", type=int, default=0,
                    help="sliding-window self-attention: window in coordinate tokens (multiple of 9); with --faces beyond "
                         "the configuration's budget the stream runs past one window over ring K/V caches")
    ap.add_argument("--correct", type=int, default=0,
                    help="run the correct stage (label head, vertex-sharing moves, z-y-x re-sort) in every step, with this "
                         "many historical vertices; random-init labels, so only its cost is meaningful")
    ap.add_argument("--b8-steps", type=int, default=100,
                    help="timed steps of the extra batch-8 leg (configs[3] at its full size, at half context); 0 = skip")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--gemm-sweep", action="store_true",
                    help="row sweep (16 .. 4096) of the weight-streaming GEMM kernel on the FFN up projection; prints and exits")
    ap.add_argument("--exchange-probe", action="store_true",
                    help="cost of one dependent all-to-all hand-off between resident workgroups (the step the single-launch "
                         "verify kernel repeats ~10 times per block), by workgroup count and volume; prints and exits")
    ap.add_argument("--counter-pass", action="store_true",
                    help="short run for hardware-counter collection: fill the caches to half context with forced "
                         "commits, then one 1 GiB device copy (the calibration kernel) and 5 verify passes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct

    cfg = si.CONFIGS[args.config]
    if args.draft:
        dc, m, n = (int(v) for v in args.draft.split(","))
        cfg = cfg.replace(draft_coord=dc, draft_point=m, draft_face=n)
    if args.batch:
        cfg = cfg.replace(batch=args.batch)
    if args.model:
        dm, nh, lc, lv, lf = (int(v) for v in args.model.split(","))
        cfg = cfg.replace(name=f"{cfg.name} with model {args.model}", d_model=dm, n_heads=nh, l_cpre=lc // 2, l_cpost=lc - lc // 2,
                          l_vpre=lv // 2, l_vpost=lv - lv // 2, l_face=lf)
    faces = args.faces or cfg.faces
    if args.window:
        cfg = cfg.replace(window=args.window, faces=max(faces, cfg.faces))
    print(f"bench: drawing the weights of configs[{args.config}]", file=sys.stderr, flush=True)
    weights = si.make_weights(cfg, 0)
    print("bench: weights drawn, creating the context", file=sys.stderr, flush=True)
    fm = FlashMesh(config_struct(cfg))
    fm.load_weights(si.pack_blob(cfg, weights))
    if args.correct:
        fm.set_correct(args.correct)
    if args.exchange_probe:
        rows = []
        for wgs in (256, 128, 64):
            for nbytes in (4096, 12288, 36864):
                rows.append({"workgroups": wgs, "bytes": nbytes, "us_per_round": fm.measure_exchange(wgs, nbytes)})
        rows.append({"workgroups": 2, "pingpong": True, "us_per_round_trip": fm.measure_exchange(2, 4096, True)})
        print(json.dumps({"exchange_probe": "dependent all-to-all hand-offs between resident workgroups: tagged 8-byte elements, "
                                            "agent-scope stores, agent-scope loads repeated until every tag matches", "rows": rows}))
        return
    if args.gemm_sweep:
        sweep = [fm.measure_gemm(r) for r in (8, 16, 32, 72, 128, 256, 512, 1024, 2048, 4096)]
        for e in sweep:
            e["frac_of_mfma_peak"] = e["TFLOPs"] / MFMA_PEAK_TFLOPS
            e["weight_GBs"] = 2.0 * cfg.d_model * cfg.ffn_mult * cfg.d_model / (e["ms"] * 1e-3) / 1e9
        print(json.dumps({"gemm_sweep": f"Y[rows, {cfg.ffn_mult * cfg.d_model}] = gelu(X[rows, {cfg.d_model}] W^T), k_gemm_mfma", "rows": sweep}))
        return
    mems = [si.make_memory(cfg, s) for s in range(cfg.batch)]
    mems_dev = [torch.from_numpy(m).cuda() for m in mems]

    def reset():
        for s in range(cfg.batch):
            fm.prefill_condition(s, mems_dev[s])

    if args.counter_pass:
        # The K/V caches only need the right length for the byte counters, not a greedy stream: commit whole
        # blocks of arbitrary coordinate tokens (the caller owns the accepted lengths it hands to fm_commit).
        for _ in range(4):                          # the prefill kernel several times: its counters are read off the last call
            reset()
        forced_fill(fm, cfg, torch, 9 * (faces // 2))
        fm.set_budget(faces)
        tok, ln = fm.new_block()
        acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
        fm.draft(tok, ln)
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)                              # calibration: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        for _ in range(5):
            fm.verify_block(tok, ln, None, acc)
        torch.cuda.synchronize()
        print(json.dumps({"counter_pass": True, "context_tokens": int(fm.read_state()[0, 0]),
                          "verify_algorithmic_bytes": fm.verify_bytes(), "copy_bytes_each_way": 1 << 30,
                          "verify_path": fm.verify_path()}))
        return

    if cfg.batch > 1:
        # several sequences: the whole generation does not fit a default run, so the step is timed at half context
        steps = args.steps if args.steps > 0 else 100
        leg = half_context_leg(fm, cfg, torch, mems_dev, faces, steps, args.warmup)
        measured = fm.measure_peaks()
        leg["roofline"]["frac_of_measured_read_rate"] = leg["roofline"]["achieved"] / measured["hbm_read_GBs"]
        result = {
            "metric": f"mesh tokens/sec, batch {cfg.batch} (replay drafts p={REPLAY_P}, all heads executed)",
            "value": leg["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": steps, "warmup": args.warmup,
            "ms_per_step": leg["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f16 (bf16-valued weights held as half, fp32 accumulate)", "data": "synthetic",
            "config": {"workload": f"configs[{args.config}] {cfg.name}: d={cfg.d_model}, {cfg.n_layers} blocks, batch {cfg.batch}, "
                                   f"{faces} faces per sequence, block {cfg.block_max}, timed at half context "
                                   f"({9 * (faces // 2)} tokens per sequence, reached by forced commits)",
                       "draft_source": f"replay p={REPLAY_P}", "tokens": leg["tokens"],
                       "mean_accepted_per_sequence": leg["mean_accepted_per_sequence"],
                       "context_tokens_per_sequence": leg["context_tokens_per_sequence"], "measured_on_this_gpu": measured},
            "roofline": leg["roofline"],
        }
        if not args.no_cpu:
            result["cpu_baseline"] = cpu_baseline(cfg, weights, mems[0], args.cpu_seconds)
        print(json.dumps(result))
        return

    # warm-up: W untimed steps through the step-wise entry points
    reset()
    tok, ln = fm.new_block()
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    for _ in range(args.warmup):
        fm.draft(tok, ln)
        fm.verify_block(tok, ln, None, acc)
        fm.commit(acc)
    torch.cuda.synchronize()

    # 1) native draft heads, whole generation: also yields the greedy stream the replay source needs
    reset()
    fm.set_draft_replay(None, 0, 0.0, 0)
    torch.cuda.synchronize()
    out, n, st_native = generate_in_stages(fm, faces, "native heads")
    stream = out.clone()
    n_tokens = int(n.min().item())

    # 2) headline: replay draft source, timed
    reset()
    fm.set_draft_replay(stream, n_tokens, REPLAY_P, REPLAY_SEED)
    torch.cuda.synchronize()
    t0 = time.time()
    context = None
    if args.steps > 0:
        # K timed steps at half context: the replay source at p = 1 decodes the first half of the stream, then the
        # timed steps run with the headline acceptance level
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fm.set_draft_replay(stream, n_tokens, 1.0, 0)
        fm.generate(max(faces // 2, 1), True)
        fm.set_draft_replay(stream, n_tokens, REPLAY_P, REPLAY_SEED)
        fm.set_budget(faces)
        for _ in range(args.warmup):
            fm.draft(tok, ln)
            fm.verify_block(tok, ln, None, acc)
            fm.commit(acc)
        torch.cuda.synchronize()
        p0 = fm.read_state()[:, 0].sum()
        context = int(p0)
        ev0.record()
        for _ in range(args.steps):
            fm.draft(tok, ln)
            fm.verify_block(tok, ln, None, acc)
            fm.commit(acc)
        ev1.record()
        torch.cuda.synchronize()
        ms = ev0.elapsed_time(ev1)
        steps, tokens = args.steps, int(fm.read_state()[:, 0].sum() - p0)
        same = None
    else:
        out2, n2, st = fm.generate(faces, True)
        torch.cuda.synchronize()
        ms, steps, tokens = st.ms_total, int(st.steps), int(st.tokens)
        same = bool((out2 == stream).all().item())
    wall = time.time() - t0
    hist = None if args.steps > 0 else st.hist()[: cfg.block_max + 1]
    levels = None if args.steps > 0 else {
        "coordinate_only_steps": sum(st.hist(0)), "point_level_steps": sum(st.hist(1)), "face_level_steps": sum(st.hist(2)),
        "point_acc": st.mean_verified_drafts(1), "face_acc": st.mean_verified_drafts(2),
        "ms_draft": st.ms_draft, "ms_verify": st.ms_verify, "ms_commit": st.ms_commit, "phase_samples": int(st.phase_samples)}

    # 3) plain one-token-per-step decoding of the same backbone on a prefix (the sequential baseline)
    reset()
    fm.set_draft_replay(None, 0, 0.0, 0)
    seq_faces = min(faces, 100)
    _, _, st_seq = fm.generate(seq_faces, False)

    # the one MFMA-bound piece: cross-attention K/V of all blocks from the condition memory (once per sequence)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    prefill_reps = 20
    for _ in range(3):
        fm.prefill_condition(0, mems_dev[0])
    ev0.record(fm.stream)
    for _ in range(prefill_reps):
        fm.prefill_condition(0, mems_dev[0])
    ev1.record(fm.stream)
    torch.cuda.synchronize()
    ms_prefill = ev0.elapsed_time(ev1) / prefill_reps
    prefill_flop = 2.0 * cfg.mem_len * 2 * cfg.d_model * cfg.d_model * cfg.n_layers
    prefill = {"ms": ms_prefill, "tflops": prefill_flop / (ms_prefill * 1e-3) / 1e12,
               "frac_of_mfma_peak": prefill_flop / (ms_prefill * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
               "calls_timed": prefill_reps,
               "what": "fm_prefill_condition of one sequence: K_mem, V_mem of every block (includes the memory "
                       "re-tiling and the sequence reset launches); average over back-to-back calls"}

    # roofline of the verify pass: algorithmic HBM bytes (weights once, self and cross K/V once per block)
    # over its measured duration, at the half-way point of the run, HIP events on the library's stream
    reset()
    fm.set_draft_replay(stream, n_tokens, 1.0, 0)
    _ = fm.generate(max(faces // 2, 1), True)
    fm.set_budget(faces)
    fm.draft(tok, ln)
    bytes_mid = fm.verify_bytes()
    context_roofline = int(fm.read_state()[0, 0])
    ms_verify = time_verify(fm, torch, tok, ln, acc, 20)
    achieved = bytes_mid / (ms_verify * 1e-3) / 1e9
    if fm.verify_path() == 1:
        kernel = ("k_verify_persist (whole backbone forward of the block in one launch) at half context; the timed "
                  "region is fm_verify_block = that kernel plus the block set-up, row argmax and accept kernels")
    else:
        kernel = "verify pass at half context (all launches of fm_verify_block, one per operator)"

    measured = fm.measure_peaks()
    persistent = fm.verify_path() == 1

    # batch-8 leg: the same model with 8 independent sequences (configs[3]) at its full 2000 faces per sequence, timed
    # at half context (forced fill, see half_context_leg); ragged accepted lengths come from the per-sequence replay draws
    batch8 = None
    if args.config == 2 and args.b8_steps > 0 and not args.draft and not args.window and not args.correct and not args.faces:
        cfg8 = si.CONFIGS[3]
        fm.close()
        torch.cuda.empty_cache()
        print("bench: batch-8 leg", file=sys.stderr, flush=True)
        fm8 = FlashMesh(config_struct(cfg8))
        fm8.load_weights(si.pack_blob(cfg8, weights))
        mems8 = [torch.from_numpy(si.make_memory(cfg8, q)).cuda() for q in range(cfg8.batch)]
        batch8 = half_context_leg(fm8, cfg8, torch, mems8, cfg8.faces, args.b8_steps, 5)
        batch8["workload"] = (f"configs[3] {cfg8.name}: batch {cfg8.batch}, {cfg8.faces} faces per sequence, block {cfg8.block_max}, "
                              f"{args.b8_steps} steps timed at half context (reached by forced commits)")
        batch8["roofline"]["frac_of_measured_read_rate"] = batch8["roofline"]["achieved"] / measured["hbm_read_GBs"]
        fm8.close()
        torch.cuda.empty_cache()

    result = {
        "metric": f"mesh tokens/sec, batch {cfg.batch} (replay drafts p={REPLAY_P}, all heads executed)",
        "value": tokens / ms * 1e3,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": ms / max(steps, 1),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16 (bf16-valued weights held as half, fp32 accumulate)",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.config}] {cfg.name}: d={cfg.d_model}, {cfg.n_layers} blocks, batch {cfg.batch}, "
                               f"{faces} faces ({9 * faces} tokens), block {cfg.block_max}, draft counts Dc={cfg.draft_coord} m={cfg.draft_point} n={cfg.draft_face}"
                               + (f", sliding window {cfg.window} tokens" if cfg.window else "")
                               + (f", correct stage on ({args.correct} historical vertices)" if args.correct else "")
                               + (f"; {steps} steps timed at half context ({context} tokens committed, reached with replay p=1)" if context is not None else "; whole generation timed"),
                   "draft_source": f"replay p={REPLAY_P}", "tokens": tokens, "mean_accepted": tokens / max(steps, 1),
                   "accepted_hist": hist, "per_level": levels, "stream_equals_native_run": same,
                   "nonfinite_logit_rows": int(st_native.nonfinite_rows),
                   "native_heads_tokens_per_s": st_native.tokens / st_native.ms_total * 1e3,
                   "native_heads_ms_per_step": st_native.ms_total / max(st_native.steps, 1),
                   "sequential_tokens_per_s": st_seq.tokens / st_seq.ms_total * 1e3,
                   "sequential_prefix_faces": seq_faces, "host_wall_s": wall, "prefill": prefill,
                   "measured_on_this_gpu": measured, "batch8": batch8},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": counter_traffic(args.config, persistent) if (faces == si.CONFIGS[args.config].faces and not args.window and not args.draft and not args.batch and not args.model) else None,
                     "traffic_source": "committed counter profile profiles/k_verify_persist_config2_b1_hbm_counters.txt (two rocprofv3 --pmc runs of bench.py --counter-pass at half context), not a counter of this run",
                     "context_tokens": context_roofline, "algorithmic_bytes": bytes_mid, "ms": ms_verify,
                     "frac_of_measured_read_rate": achieved / measured["hbm_read_GBs"]},
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, weights, mems[0], args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
