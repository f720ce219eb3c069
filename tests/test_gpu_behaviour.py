"""GPU tests of the decode-step contract: idempotent verify, rollback, replay accounting, error paths,
and the full-size runs with teacher-forced oracle checks."""
import os
import time

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


def _ctx(cfg, max_tokens=None):
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    w = si.make_weights(cfg, 0)
    fm = FlashMesh(config_struct(cfg, max_tokens=max_tokens))
    fm.load_weights(si.pack_blob(cfg, w))
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    return fm, w


def test_verify_is_idempotent_and_commit_is_the_only_transition():
    _need_gpu()
    cfg = si.TEST_CONFIGS["t_bf16_99"]
    print("case idempotent", flush=True)
    fm, _ = _ctx(cfg)
    tok, ln = fm.new_block()
    S, Bm, V = cfg.batch, fm.block_max, cfg.vocab
    lg1 = torch.zeros(S, Bm, V, device="cuda")
    lg2 = torch.zeros(S, Bm, V, device="cuda")
    a1 = torch.zeros(S, dtype=torch.int32, device="cuda")
    a2 = torch.zeros(S, dtype=torch.int32, device="cuda")
    for step in range(12):
        fm.draft(tok, ln)
        before = fm.read_state().copy()
        fm.verify_block(tok, ln, lg1, a1)
        # a different (wrong) block in between must leave no trace
        junk = (tok + 1) % cfg.n_bins
        junk[:, 0] = tok[:, 0]
        fm.verify_block(junk, ln, lg2, a2)
        fm.verify_block(tok, ln, lg2, a2)
        torch.cuda.synchronize()
        assert np.array_equal(fm.read_state(), before)
        L = ln.cpu().numpy()
        for s in range(S):
            assert torch.equal(lg1[s, :L[s]], lg2[s, :L[s]])
        assert torch.equal(a1, a2)
        fm.commit(a1)
        after = fm.read_state()
        assert np.array_equal(after[:, 0], before[:, 0] + a1.cpu().numpy())


def test_rollback_with_corrupted_drafts_ragged_batch():
    """Drafts = the known continuation corrupted at a per-sequence index k: accepted must equal k exactly
    and the emitted streams must not change."""
    _need_gpu()
    cfg = si.TEST_CONFIGS["t_bf16_99"]
    print("case rollback", flush=True)
    fm, _ = _ctx(cfg)
    out, n, _ = fm.generate(cfg.faces, False)
    truth = out.cpu().numpy()
    budget = 9 * cfg.faces
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    fm.set_budget(cfg.faces)
    S, Bm = cfg.batch, fm.block_max
    tok, ln = fm.new_block()
    acc = torch.zeros(S, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(3)
    P = np.zeros(S, int)
    while (P < budget).any():
        ks = rng.integers(1, Bm + 1, S)
        blk = np.zeros((S, Bm), np.int32)
        lens = np.zeros(S, np.int32)
        for s in range(S):
            if P[s] >= budget:
                continue
            L = min(Bm, budget - P[s])
            x = [cfg.bos] + list(truth[s])
            blk[s, :L] = x[P[s]:P[s] + L]
            if ks[s] < L:
                blk[s, ks[s]] = (blk[s, ks[s]] + 1) % cfg.n_bins
            lens[s] = L
        tok.copy_(torch.from_numpy(blk))
        ln.copy_(torch.from_numpy(lens))
        fm.verify_block(tok, ln, None, acc)
        fm.commit(acc)
        a = acc.cpu().numpy()
        for s in range(S):
            if lens[s]:
                assert a[s] == min(ks[s], lens[s]), (s, P[s], ks[s], lens[s], a[s])
        P += a
        st = fm.read_state()
        assert np.array_equal(st[:, 0], P)
        assert np.array_equal(st[:, 1], (P + 2) // 3) and np.array_equal(st[:, 2], (P + 8) // 9)
    assert all(fm.read_state()[:, 4] == 1)


def test_replay_accounting_matches_host_prediction():
    """With the replay draft source the whole step sequence is predictable on the host from the
    counter-based uniforms: accepted = 1 + leading kept drafts."""
    _need_gpu()
    cfg = si.TEST_CONFIGS["t_bf16_1815"]
    print("case replay", flush=True)
    fm, _ = _ctx(cfg)
    out, n, st0 = fm.generate(cfg.faces, True)
    budget = 9 * cfg.faces
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    keep, seed = 0.8, 77
    fm.set_draft_replay(out.clone(), budget, keep, seed)
    out2, n2, st = fm.generate(cfg.faces, True)
    assert torch.equal(out, out2)
    hist = np.zeros(32, int)
    steps = 0
    for s in range(cfg.batch):
        P, k = 0, 0
        while P < budget:
            L = 1 if P == 0 else min(fm.block_max, budget - P)
            a = 1
            while a < L and si.replay_uniform(seed, s, P + a) < keep:
                a += 1
            hist[a] += 1
            P += a
            k += 1
        steps = max(steps, k)
    assert st.hist() == list(hist)
    assert st.steps == steps and st.tokens == budget * cfg.batch


def test_error_paths():
    _need_gpu()
    import ctypes as C
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    cfg = si.TEST_CONFIGS["t_f32_99"]
    fm = FlashMesh(config_struct(cfg))
    tok, ln = fm.new_block()
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    lib, h = fm.lib, fm.h
    assert lib.fm_verify_block(h, tok.data_ptr(), ln.data_ptr(), None, acc.data_ptr()) == -2      # no weights
    assert b"weights" in lib.fm_last_error(h)
    blob = si.pack_blob(cfg, si.make_weights(cfg, 0))
    assert lib.fm_load_weights(h, blob.ctypes.data, blob.size - 1) == -1
    fm.load_weights(blob)
    mem = torch.from_numpy(si.make_memory(cfg, 0)).cuda()
    assert lib.fm_prefill_condition(h, cfg.batch, mem.data_ptr()) == -1
    assert lib.fm_prefill_condition(h, -1, mem.data_ptr()) == -1
    assert lib.fm_prefill_condition(h, 0, None) == -1
    out = torch.zeros(cfg.batch, cfg.max_tokens, dtype=torch.int32, device="cuda")
    assert lib.fm_generate(h, cfg.faces, 1, out.data_ptr(), ln.data_ptr(), None) == -2            # not prefilled
    assert lib.fm_set_budget(h, 0) == -1 and lib.fm_set_budget(h, cfg.faces + 1) == -1
    assert lib.fm_verify_block(h, None, ln.data_ptr(), None, acc.data_ptr()) == -1
    assert lib.fm_correct(h, tok.data_ptr(), ln.data_ptr(), None) == -2                           # stage is off
    assert lib.fm_set_correct(h, -1) == -1
    assert lib.fm_set_correct(h, 4) == 0 and lib.fm_correct(h, None, ln.data_ptr(), None) == -1
    assert lib.fm_set_correct(h, 0) == 0
    # an unprefilled sequence is simply not live; over-long and out-of-range block entries are clipped
    fm.prefill_condition(0, mem)
    tok.fill_(10 ** 6)
    tok[:, 0] = cfg.bos
    ln.fill_(1000)
    fm.verify_block(tok, ln, None, acc)
    torch.cuda.synchronize()
    a = acc.cpu().numpy()
    assert 1 <= a[0] <= fm.block_max and a[1] == 0


def test_persistent_kernel_gives_up_instead_of_hanging(monkeypatch):
    """Every wait inside the single-launch verify kernel is bounded.  With the test hook that makes the embedding
    publish under a wrong tag nothing downstream can ever arrive: all workgroups must leave after the (shortened)
    bound and the kernel itself finishes normally.  The failed pass accepts nothing and commits nothing, the host
    reports once which stage was stuck, and the context carries on with one launch per operator and still emits the
    stream of the model."""
    _need_gpu()
    cfg = si.TEST_CONFIGS["t_bf16_99_b1"]
    print("case bounded waits", flush=True)
    monkeypatch.setenv("FM_PERSIST", "0")
    ref, _ = _ctx(cfg)
    assert ref.verify_path() == 0
    want = ref.generate(cfg.faces, True)[0].cpu().numpy()
    monkeypatch.delenv("FM_PERSIST")
    monkeypatch.setenv("FM_PK_TIMEOUT_TICKS", "200000")     # 2 ms
    monkeypatch.setenv("FM_PK_TEST_SKEW", "1")
    fm, _ = _ctx(cfg)
    assert fm.verify_path() == 1
    tok, ln = fm.new_block()
    acc = torch.full((1,), 7, dtype=torch.int32, device="cuda")
    fm.draft(tok, ln)
    t0 = time.time()
    fm.verify_block(tok, ln, None, acc)
    fm.commit(acc)                                          # enqueued before the host knows: must change nothing
    with pytest.raises(RuntimeError, match="timed out"):
        fm.read_state()
    assert time.time() - t0 < 5.0
    assert int(acc[0]) == 0
    assert fm.verify_path() == 0                            # the context has left the single-launch path
    st = fm.read_state()                                    # reported once; the state is that of the last good commit
    assert tuple(st[0, :5]) == (0, 0, 0, cfg.bos, 0)
    fm.verify_block(tok, ln, None, acc)
    fm.commit(acc)
    assert int(acc[0]) == 1 and fm.read_state()[0, 0] == 1
    fm.prefill_condition(0, torch.from_numpy(si.make_memory(cfg, 0)).cuda())
    got = fm.generate(cfg.faces, True)[0].cpu().numpy()
    assert np.array_equal(got, want)
    # the whole-loop entry point meets the failure in its first interval, recovers by itself and finishes the stream
    fm2, _ = _ctx(cfg)
    assert fm2.verify_path() == 1
    out, n, stats = fm2.generate(cfg.faces, True)
    assert fm2.verify_path() == 0 and int(n[0]) == 9 * cfg.faces and stats.tokens == 9 * cfg.faces
    assert np.array_equal(out.cpu().numpy(), want)


def _teacher_forced_check(cfg, stream, tol, work, chunk=600, say=print):
    """Replays a device stream through the oracle in long blocks and applies the margin rule at every position."""
    from oracle.hourglass import Model, SeqState, forward_block
    model = Model(cfg, si.make_weights(cfg, 0), work=work)
    flips = 0
    worst = 0.0
    for s, toks in enumerate(stream):
        st = SeqState(model, si.make_memory(cfg, s), len(toks))
        x = [cfg.bos] + [int(t) for t in toks]
        nlim = cfg.n_bins if cfg.ban_specials else cfg.vocab
        while st.P < len(toks):
            B = min(chunk, len(toks) - st.P)
            lg = forward_block(model, st, x[st.P:st.P + B], long_block=True)
            ref = np.argmax(lg[:, :nlim], axis=1)
            dev = np.array(x[st.P + 1:st.P + B + 1])
            for i in np.nonzero(ref != dev)[0]:
                gap = lg[i, ref[i]] - lg[i, dev[i]]
                worst = max(worst, float(gap))
                assert gap <= tol, ("device token beyond tolerance", s, st.P + i, gap)
                flips += 1
            st.P += B
            say("  teacher-forced", s, st.P)
    return flips, worst


def test_config1_full_size_stream(say):
    """configs[1] at its full size (500 faces, 4500 tokens): replay run == native run == what the oracle
    picks at every position (teacher-forced, margin rule)."""
    _need_gpu()
    cfg = si.CONFIGS[1]
    print("case config1 full", flush=True)
    fm, _ = _ctx(cfg)
    out, n, st = fm.generate(cfg.faces, True)
    assert int(n[0]) == 4500 and st.tokens == 4500
    fm.prefill_condition(0, torch.from_numpy(si.make_memory(cfg, 0)).cuda())
    fm.set_draft_replay(out.clone(), 4500, 0.93, 5)
    out2, n2, st2 = fm.generate(cfg.faces, True)
    assert torch.equal(out, out2)
    assert st2.steps < st.steps and st2.tokens == 4500
    flips, worst = _teacher_forced_check(cfg, out.cpu().numpy(), TOL["bf16"], np.float64, say=say)
    print("config1 full: allowed flips", flips, "worst margin", worst, "steps native/replay", st.steps, st2.steps, flush=True)


def test_config1_sliding_window_stream():
    """configs[1] (4500 tokens) with a sliding window of 900 tokens (Sec. 5.1 "window size"): the stream is five
    windows long, the K/V rings of all three levels wrap (1024 / 384 / 128 positions), and the run is the
    single-launch verify kernel.  Native run == replay run == what the oracle, which keeps every key and masks,
    picks at every position (teacher-forced, margin rule)."""
    _need_gpu()
    cfg = si.CONFIGS[1].replace(window=900)
    print("case config1 window 900", flush=True)
    fm, _ = _ctx(cfg)
    assert fm.verify_path() == 1
    out, n, st = fm.generate(cfg.faces, True)
    assert int(n[0]) == 4500 and st.tokens == 4500
    fm.prefill_condition(0, torch.from_numpy(si.make_memory(cfg, 0)).cuda())
    fm.set_draft_replay(out.clone(), 4500, 0.93, 5)
    out2, n2, st2 = fm.generate(cfg.faces, True)
    assert torch.equal(out, out2)
    assert st2.steps < st.steps and st2.tokens == 4500
    fm.prefill_condition(0, torch.from_numpy(si.make_memory(cfg, 0)).cuda())
    fm.set_draft_replay(None, 0, 0.0, 0)
    out3, n3, st3 = fm.generate(cfg.faces, False)          # one token per step through the same kernels
    assert torch.equal(out, out3) and st3.steps == 4500
    flips, worst = _teacher_forced_check(cfg, out.cpu().numpy(), TOL["bf16"], np.float64)
    print("config1 window: allowed flips", flips, "worst margin", worst, "steps native/replay", st.steps, st2.steps, flush=True)
    # the window changes the model: its stream leaves the unwindowed one after the first window
    fm_all, _ = _ctx(si.CONFIGS[1])
    out_all, _, _ = fm_all.generate(cfg.faces, True)
    a, b = out.cpu().numpy()[0], out_all.cpu().numpy()[0]
    assert np.array_equal(a[:100], b[:100]) and not np.array_equal(a, b)


def test_batched_long_context_stream():
    """Eight ragged sequences of 2304 tokens at a small width: the key axis of the self-attention is cut into
    nine ranges whose partial results are merged by the second launch, and the host-side bound on the
    committed lengths decides how many of them are launched.  Native run == replay run == the oracle's
    choice at every position (teacher-forced, margin rule)."""
    _need_gpu()
    cfg = si.TEST_CONFIGS["t_bf16_99_b8long"]
    print("case batched long", flush=True)
    fm, _ = _ctx(cfg)
    assert fm.verify_path() == 0
    out, n, st = fm.generate(cfg.faces, True)
    assert [int(v) for v in n] == [cfg.max_tokens] * cfg.batch
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    fm.set_draft_replay(out.clone(), cfg.max_tokens, 0.8, 11)
    out2, n2, st2 = fm.generate(cfg.faces, True)
    assert torch.equal(out, out2) and st2.steps < st.steps
    flips, worst = _teacher_forced_check(cfg, out.cpu().numpy(), TOL["bf16"], np.float64)
    print("batched long: allowed flips", flips, "worst margin", worst, "steps native/replay", st.steps, st2.steps, flush=True)


def test_config2_full_size_stream(say):
    """configs[2] (d = 1024, 16 heads, 40 blocks, block 9) through the single-launch verify kernel: every emitted token
    against the oracle's choice at that position (teacher-forced, margin rule).  The default run stops at 800 faces
    (7200 tokens: the oracle's attention grows with the square of the length and the GPU machine allows a test suite a
    quarter of an hour); FM_LONG=1 runs the configuration's full 2000 faces (18 000 tokens, about seven minutes)."""
    _need_gpu()
    faces = si.CONFIGS[2].faces if os.environ.get("FM_LONG") == "1" else 800
    cfg = si.CONFIGS[2].replace(faces=faces)
    print("case config2", faces, "faces", flush=True)
    fm, _ = _ctx(cfg)
    assert fm.verify_path() == 1
    out, n, st = fm.generate(cfg.faces, True)
    assert int(n[0]) == 9 * faces
    say("  stream generated")
    flips, worst = _teacher_forced_check(cfg, out.cpu().numpy(), TOL["bf16"], np.float32, chunk=1200, say=say)
    print("config2: allowed flips", flips, "worst margin", worst, flush=True)


def test_streams_are_bit_reproducible_across_runs_and_modes():
    """Same seeds => same stream, run after run, and for speculative, replay and one-token decoding alike
    (the kernels never let the arithmetic of a position depend on what it is batched with)."""
    _need_gpu()
    cfg = si.CONFIGS[1]
    faces = 160
    print("case reproducible", flush=True)
    fm, _ = _ctx(cfg)
    mem = torch.from_numpy(si.make_memory(cfg, 0)).cuda()

    def run(spec, replay=None):
        fm.prefill_condition(0, mem)
        if replay is None:
            fm.set_draft_replay(None, 0, 0.0, 0)
        else:
            fm.set_draft_replay(replay, 9 * faces, 0.9, 3)
        out, n, st = fm.generate(faces, spec)
        return out.clone(), st

    ref, st = run(True)
    for _ in range(3):
        o, _ = run(True)
        assert torch.equal(o, ref)
    o, st_seq = run(False)
    assert torch.equal(o, ref) and st_seq.steps == 9 * faces
    o, st_rep = run(True, ref)
    assert torch.equal(o, ref) and st_rep.steps < st.steps


def test_config3_real_widths_at_context(say):
    """configs[3] at its real widths (d = 1024, 16 heads, 40 blocks, 8 sequences) with every sequence more than 3000
    tokens into its stream and the sequences at different lengths: the split key ranges of the self-attention and
    their merge at 16 heads x 8 sequences.  The device fills the caches by decoding with replayed drafts (ragged
    accepted lengths); the oracle is brought to the same state by teacher forcing, which also checks every token of
    the fill by the margin rule; then both run in lock step: logits, greedy tokens, accepted and committed lengths.
    The device decodes all eight sequences; the oracle follows two of them (a sampled check: its cost is per sequence)."""
    _need_gpu()
    from oracle.hourglass import Model, SeqState, forward_block
    import parity_harness
    from parity_harness import lockstep
    parity_harness.PROGRESS = say
    cfg = si.CONFIGS[3].replace(faces=420)
    S, budget = cfg.batch, 9 * cfg.faces
    print("case config3 at context", flush=True)
    fm, w = _ctx(cfg)
    assert fm.verify_path() == 0
    out, n, _ = fm.generate(cfg.faces, True)                     # the greedy streams (native heads)
    truth = out.cpu().numpy()
    say("  streams generated")
    for s in range(S):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    replay = (out.clone(), budget, 0.85, 23)
    fm.set_draft_replay(*replay)
    fm.set_budget(cfg.faces)
    tok, ln = fm.new_block()
    acc = torch.zeros(S, dtype=torch.int32, device="cuda")
    steps = 0
    while True:                                                  # ragged fill: stop once every sequence is past 3000
        for _ in range(25):
            fm.draft(tok, ln)
            fm.verify_block(tok, ln, None, acc)
            fm.commit(acc)
        steps += 25
        st_dev = fm.read_state()
        if st_dev[:, 0].min() >= 3000:
            break
        assert st_dev[:, 0].max() < budget - 200, st_dev[:, 0]
    P = [int(v) for v in st_dev[:, 0]]
    say("  device filled to", P, "in", steps, "steps")
    assert len(set(P)) > 1                                       # ragged
    model = Model(cfg, w, work=np.float32)
    nlim = cfg.n_bins
    states, flips = [], 0
    for s in range(S):
        if s not in (1, 6):            # the oracle follows two of the eight sequences (the kernels do not tell them apart)
            states.append(None)
            continue
        st = SeqState(model, si.make_memory(cfg, s), budget)
        x = [cfg.bos] + [int(t) for t in truth[s, :budget]]
        while st.P < P[s]:
            B = min(1200, P[s] - st.P)
            lg = forward_block(model, st, x[st.P:st.P + B], long_block=True)
            ref = np.argmax(lg[:, :nlim], axis=1)
            dev = np.array(x[st.P + 1:st.P + B + 1])
            for i in np.nonzero(ref != dev)[0]:
                assert lg[i, ref[i]] - lg[i, dev[i]] <= TOL["bf16"], ("fill token beyond tolerance", s, st.P + i)
                flips += 1
            st.P += B
            say("  oracle fill", s, st.P)
        st.tokens = x[:P[s]]
        st.main = x[P[s]]
        assert st.main == int(st_dev[s, 3])
        states.append(st)
    rep, _, _ = lockstep(cfg, cfg.faces, TOL["bf16"], max_steps=4, replay=replay, pair=(model, fm, states))
    parity_harness.PROGRESS = None
    print(rep, "fill flips", flips, flush=True)
    assert rep.steps == 4 and len(rep.accepted) == 4 * 2 and len(set(rep.accepted)) > 1


@pytest.mark.parametrize("name", ["t_bf16_99", "t_bf16_99_b1"])
def test_half_precision_overflow_is_counted(name):
    """Activations of the half-precision path beyond 65504 become infinities without a trap.  A run with an outlier weight
    (one FFN up projection scaled by 2^24, still bf16-valued) must say so: fm_stats.nonfinite_rows counts the verify rows
    whose logits were not finite; a healthy run counts none.  Both verify paths."""
    _need_gpu()
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    cfg = si.TEST_CONFIGS[name]
    counts = []
    for scale in (1.0, 2.0 ** 24):
        w = si.make_weights(cfg, 0)
        w["cpre.0.w1"] = w["cpre.0.w1"] * scale
        fm = FlashMesh(config_struct(cfg))
        fm.load_weights(si.pack_blob(cfg, w))
        for s in range(cfg.batch):
            fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
        out, n, st = fm.generate(4, True)
        counts.append(int(st.nonfinite_rows))
        assert int(n.min()) == 36                     # the loop still ends at the budget
    print("non-finite rows: healthy", counts[0], "with the outlier", counts[1], flush=True)
    assert counts[0] == 0 and counts[1] > 0
