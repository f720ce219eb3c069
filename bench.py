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


class _Totals:
    steps = 0
    tokens = 0
    ms_total = 0.0


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
    ap.add_argument("--window", type=int, default=0,
                    help="sliding-window self-attention: window in coordinate tokens (multiple of 9); with --faces beyond "
                         "the configuration's budget the stream runs past one window over ring K/V caches")
    ap.add_argument("--correct", type=int, default=0,
                    help="run the correct stage (label head, vertex-sharing moves, z-y-x re-sort) in every step, with this "
                         "many historical vertices; random-init labels, so only its cost is meaningful")
    ap.add_argument("--b8-faces", type=int, default=150,
                    help="faces per sequence of the extra batch-8 leg (configs[3], same model as configs[2]); 0 = skip")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=20.0)
    ap.add_argument("--gemm-sweep", action="store_true",
                    help="row sweep (16 .. 4096) of the weight-streaming GEMM kernel on the FFN up projection; prints and exits")
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
        reset()
        fm.set_budget(faces)
        tok, ln = fm.new_block()
        acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
        gen = torch.Generator(device="cuda").manual_seed(7)
        target = 9 * (faces // 2)
        while int(fm.read_state()[:, 0].min()) < target:
            for _ in range(50):
                fm.draft(tok, ln)
                tok[:, 1:] = torch.randint(0, cfg.n_bins, (cfg.batch, cfg.block_max - 1), generator=gen,
                                           device="cuda", dtype=torch.int32)
                fm.verify_block(tok, ln, None, acc)
                fm.commit(ln)
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
    if args.steps > 0:
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        fm.set_budget(faces)
        p0 = fm.read_state()[:, 0].sum()
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
    hist = None if args.steps > 0 else [int(v) for v in st.acc_hist[: cfg.block_max + 1]]

    # 3) plain one-token-per-step decoding of the same backbone on a prefix (the sequential baseline)
    reset()
    fm.set_draft_replay(None, 0, 0.0, 0)
    seq_faces = min(faces, 100)
    _, _, st_seq = fm.generate(seq_faces, False)

    # the one MFMA-bound piece: cross-attention K/V of all blocks from the condition memory (once per sequence)
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fm.prefill_condition(0, mems_dev[0])
    ev0.record(fm.stream)
    for _ in range(5):
        fm.prefill_condition(0, mems_dev[0])
    ev1.record(fm.stream)
    torch.cuda.synchronize()
    ms_prefill = ev0.elapsed_time(ev1) / 5
    prefill_flop = 2.0 * cfg.mem_len * 2 * cfg.d_model * cfg.d_model * cfg.n_layers
    prefill = {"ms": ms_prefill, "tflops": prefill_flop / (ms_prefill * 1e-3) / 1e12,
               "frac_of_mfma_peak": prefill_flop / (ms_prefill * 1e-3) / 1e12 / MFMA_PEAK_TFLOPS,
               "what": "fm_prefill_condition of one sequence: K_mem, V_mem of every block (includes the memory "
                       "re-tiling and the sequence reset launches)"}

    # roofline of the verify pass: algorithmic HBM bytes (weights once, self and cross K/V once per block)
    # over its measured duration, at the half-way point of the run, HIP events on the library's stream
    reset()
    fm.set_draft_replay(stream, n_tokens, 1.0, 0)
    _ = fm.generate(max(faces // 2, 1), True)
    fm.set_budget(faces)
    fm.draft(tok, ln)
    bytes_mid = fm.verify_bytes()
    iters = 20
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(3):
        fm.verify_block(tok, ln, None, acc)
    ev0.record(fm.stream)
    for _ in range(iters):
        fm.verify_block(tok, ln, None, acc)
    ev1.record(fm.stream)
    torch.cuda.synchronize()
    ms_verify = ev0.elapsed_time(ev1) / iters
    achieved = bytes_mid / (ms_verify * 1e-3) / 1e9
    if fm.verify_path() == 1:
        kernel = ("k_verify_persist (whole backbone forward of the block in one launch) at half context; the timed "
                  "region is fm_verify_block = that kernel plus the block set-up, row argmax and accept kernels")
    else:
        kernel = "verify pass at half context (all launches of fm_verify_block, one per operator)"

    measured = fm.measure_peaks()
    persistent = fm.verify_path() == 1

    # batch-8 leg: the same model with 8 independent sequences (configs[3]) on a shortened budget, so that the
    # default run stays within minutes; ragged accepted lengths come from the per-sequence replay draws
    batch8 = None
    if args.config == 2 and args.b8_faces > 0 and not args.draft and not args.window and not args.correct:
        cfg8 = si.CONFIGS[3]
        f8 = min(args.b8_faces, cfg8.faces)
        fm.close()
        torch.cuda.empty_cache()
        fm8 = FlashMesh(config_struct(cfg8))
        fm8.load_weights(si.pack_blob(cfg8, weights))
        mems8 = [torch.from_numpy(si.make_memory(cfg8, q)).cuda() for q in range(cfg8.batch)]

        def reset8():
            for q in range(cfg8.batch):
                fm8.prefill_condition(q, mems8[q])

        reset8()
        fm8.set_draft_replay(None, 0, 0.0, 0)
        out8, n8, _ = fm8.generate(f8, True)
        stream8, nt8 = out8.clone(), int(n8.min().item())
        reset8()
        fm8.set_draft_replay(stream8, nt8, REPLAY_P, REPLAY_SEED)
        out8b, _, st8 = fm8.generate(f8, True)
        same8 = bool((out8b == stream8).all().item())
        reset8()
        fm8.set_draft_replay(stream8, nt8, 1.0, 0)
        fm8.generate(max(f8 // 2, 1), True)
        fm8.set_budget(f8)
        tok8, ln8 = fm8.new_block()
        acc8 = torch.zeros(cfg8.batch, dtype=torch.int32, device="cuda")
        fm8.draft(tok8, ln8)
        b8_bytes = fm8.verify_bytes()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for _ in range(3):
            fm8.verify_block(tok8, ln8, None, acc8)
        ev0.record(fm8.stream)
        for _ in range(10):
            fm8.verify_block(tok8, ln8, None, acc8)
        ev1.record(fm8.stream)
        torch.cuda.synchronize()
        ms8 = ev0.elapsed_time(ev1) / 10
        batch8 = {"workload": f"configs[3] {cfg8.name}: batch {cfg8.batch}, {f8} faces per sequence, block {cfg8.block_max}",
                  "tokens_per_s": st8.tokens / st8.ms_total * 1e3, "ms_per_step": st8.ms_total / max(int(st8.steps), 1),
                  "mean_accepted_per_sequence": st8.tokens / max(int(st8.steps), 1) / cfg8.batch,
                  "stream_equals_native_run": same8, "verify_ms_at_half_context": ms8,
                  "verify_algorithmic_bytes": b8_bytes, "verify_GBs": b8_bytes / (ms8 * 1e-3) / 1e9,
                  "verify_frac_of_hbm_peak": b8_bytes / (ms8 * 1e-3) / 1e9 / HBM_PEAK_GBS}
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
                               + (f", correct stage on ({args.correct} historical vertices)" if args.correct else ""),
                   "draft_source": f"replay p={REPLAY_P}", "tokens": tokens, "mean_accepted": tokens / max(steps, 1),
                   "accepted_hist": hist, "stream_equals_native_run": same,
                   "native_heads_tokens_per_s": st_native.tokens / st_native.ms_total * 1e3,
                   "native_heads_ms_per_step": st_native.ms_total / max(st_native.steps, 1),
                   "sequential_tokens_per_s": st_seq.tokens / st_seq.ms_total * 1e3,
                   "sequential_prefix_faces": seq_faces, "host_wall_s": wall, "prefill": prefill,
                   "measured_on_this_gpu": measured, "batch8": batch8},
        "roofline": {"bound": "hbm", "kernel": kernel,
                     "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": counter_traffic(args.config, persistent) if (faces == si.CONFIGS[args.config].faces and not args.window and not args.draft and not args.batch) else None,
                     "algorithmic_bytes": bytes_mid, "ms": ms_verify,
                     "frac_of_measured_read_rate": achieved / measured["hbm_read_GBs"]},
    }
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, weights, mems[0], args.cpu_seconds)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
