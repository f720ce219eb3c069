"""GPU parity: the HIP path through the C-ABI against the CPU oracle, step by step."""
import os

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")


@pytest.mark.parametrize("name", ["t_f32_c", "t_f32_99", "t_f32_1815", "t_bf16_99", "t_bf16_1815", "t_bf16_99_b1", "t_bf16_99_b1w",
                                  "t_f32_1818", "t_bf16_1812", "t_bf16_279", "t_f32_2727", "t_bf16_c17",
                                  "t_f32_99_w36", "t_bf16_99_w36", "t_bf16_99_b1_w36", "t_bf16_1815_w72",
                                  "t_bf16_1815_b1", "t_bf16_2727_b1", "t_bf16_1815_b1_w72",
                                  "t_f32_99_noA", "t_bf16_1815_noA", "t_bf16_99_b1_noA",
                                  "t_f32_99_noB", "t_bf16_1815_noAB", "t_bf16_99_b1_noB",
                                  "t_f32_hd96", "t_f32_hd128", "t_bf16_hd96", "t_bf16_hd128"])
def test_lockstep_small_native_heads(name):
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name]
    print("case", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype])
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams)
    if name.endswith("_b1") or "_b1_" in name or name.endswith("_b1w"):
        assert fm.verify_path() == 1          # one sequence in half precision: the single-launch verify kernel
    # the device's own whole-loop entry point must emit the same streams
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out, n, st = fm.generate(cfg.faces, True)
    out, n = out.cpu().numpy(), n.cpu().numpy()
    for s in range(cfg.batch):
        assert n[s] == 9 * cfg.faces
        if rep.token_flips == 0:
            assert list(out[s, :n[s]]) == streams[s]
    assert st.tokens == 9 * cfg.faces * cfg.batch
    # plain sequential decoding of the same backbone gives the same stream (Sec. 3.3 keeps the model's output)
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out2, n2, st2 = fm.generate(cfg.faces, False)
    assert st2.steps == 9 * cfg.faces
    if cfg.dtype == "f32":
        assert np.array_equal(out2.cpu().numpy(), out)


@pytest.mark.parametrize("name", ["t_f32_99", "t_f32_1815", "t_bf16_99", "t_bf16_1815", "t_bf16_99_b1", "t_f32_2727", "t_bf16_c17",
                                  "t_bf16_1815_noAB", "t_f32_hd96", "t_bf16_hd96"])
def test_lockstep_with_correct_stage(name):
    """Predict - correct - verify (Sec. 3.2): labels from the label head, the integer correction of every draft block
    bit for bit, and a stream that the stage leaves untouched."""
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name]
    print("case correct", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype], correct_hist=6)
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams)
    if cfg.draft_point or cfg.draft_face:
        assert rep.points > 0 and rep.corrected_blocks > 0
    # whole-loop entry point with the stage on, and plain sequential decoding: the same stream
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out, n, st = fm.generate(cfg.faces, True)
    out = out.cpu().numpy()
    if rep.token_flips == 0:
        for s in range(cfg.batch):
            assert list(out[s, :9 * cfg.faces]) == streams[s]
    fm.set_correct(0)
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out2, n2, st2 = fm.generate(cfg.faces, True)
    assert np.array_equal(out2.cpu().numpy(), out)
    with pytest.raises(RuntimeError):
        fm.correct(*fm.new_block())


@pytest.mark.parametrize("name,temperature", [("t_f32_99", 1.0), ("t_f32_1815", 0.7), ("t_bf16_99", 1.0), ("t_bf16_1815", 1.3),
                                              ("t_bf16_99_b1", 1.0), ("t_f32_c", 1.0)])
def test_lockstep_sampled_decoding(name, temperature):
    """Sampled decoding with non-greedy verification: the drawn drafts, the rejection tests (accepted lengths) and the
    resampled tokens against the oracle, decision by decision, with the same counter-based uniforms on both sides."""
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name]
    print("case sampled", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype], sampling=(temperature, 17))
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams)
    # reproducible from the seed through the whole-loop entry point, and different for another seed
    def run(seed):
        fm.set_sampling(temperature, seed)
        for s in range(cfg.batch):
            fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
        return fm.generate(cfg.faces, True)[0].cpu().numpy()
    a, b, c = run(17), run(17), run(18)
    assert np.array_equal(a, b) and not np.array_equal(a, c)
    if rep.token_flips == 0 and rep.draft_flips == 0:
        for s in range(cfg.batch):
            assert list(a[s, :9 * cfg.faces]) == streams[s]
    # temperature 0 is greedy decoding again
    fm.set_sampling(0.0, 0)
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    g1 = fm.generate(cfg.faces, True)[0].cpu().numpy()
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    g2 = fm.generate(cfg.faces, False)[0].cpu().numpy()
    if cfg.dtype == "f32":
        assert np.array_equal(g1, g2)


@pytest.mark.parametrize("name", ["t_f32_1815", "t_bf16_99"])
def test_lockstep_sampled_decoding_with_correct_stage(name):
    """Tokens the correct stage rewrote are no longer draws from the stored proposal: the rejection test then treats them
    as proposals with all their mass on one token (accept with probability p(x), resample from p without x)."""
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name]
    print("case sampled + correct", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype], sampling=(1.0, 3), correct_hist=6)
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams) and rep.corrected_blocks > 0


@pytest.mark.parametrize("name", ["t_bf16_99_w36", "t_bf16_1815_b1_w72"])
def test_lockstep_everything_on(name):
    """Sliding window, correct stage and sampled decoding together, on both verify paths (three sequences per operator,
    one sequence with 18-token blocks in the single-launch kernel)."""
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name].replace(faces=60)
    print("case everything", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype], sampling=(0.9, 21), correct_hist=9)
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams)


@pytest.mark.parametrize("name", ["t_bf16_d768_h8", "t_bf16_d1024_h8"])
def test_paper_head_widths_half_precision(name, say):
    """Head widths 96 and 128 (the paper's own shapes, Sec. 5.1: d = 768 with 8 heads; 16 heads of 128 scaled to 8) on the
    half-precision path: tiled prefill GEMM into the wide-head cache layouts, MFMA attention, draft heads - every step of
    the generation in lock-step."""
    _need_gpu()
    from parity_harness import lockstep
    import parity_harness
    parity_harness.PROGRESS = say
    cfg = si.TEST_CONFIGS[name]
    print("case paper head width", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL["bf16"])
    parity_harness.PROGRESS = None
    print(rep, flush=True)
    assert all(len(s) == 9 * cfg.faces for s in streams)
    assert fm.verify_path() == 0              # the single-launch kernel is written for 64-wide heads
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out = fm.generate(cfg.faces, True)[0].cpu().numpy()
    if rep.token_flips == 0:
        for s in range(cfg.batch):
            assert list(out[s, :9 * cfg.faces]) == streams[s]


def test_config0_tiny_full_run():
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.CONFIGS[0]
    print("case config0", flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL["f32"])
    print(rep, flush=True)
    assert len(streams[0]) == 90


def test_config3_shape_short_lockstep(say):
    """configs[3] at its real widths (d=1024, 40 blocks, 8 sequences with ragged progress) for a few steps of
    lock-step decoding: draft blocks, logits, greedy tokens, accepted and committed lengths."""
    _need_gpu()
    from parity_harness import lockstep
    import parity_harness
    parity_harness.PROGRESS = say
    cfg = si.CONFIGS[3].replace(faces=40)
    print("case config3 short", flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL["bf16"], max_steps=5)
    parity_harness.PROGRESS = None
    print(rep, flush=True)
    assert rep.steps == 5 and len(rep.accepted) == 5 * cfg.batch


def test_config4_shape_short_lockstep(say):
    """configs[4] at its real widths (d=1536, 48 blocks, 4 sequences, block 18) for a few lock-step steps."""
    _need_gpu()
    from parity_harness import lockstep
    import parity_harness
    parity_harness.PROGRESS = say
    cfg = si.CONFIGS[4].replace(faces=40)
    print("case config4 short", flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL["bf16"], max_steps=4)
    parity_harness.PROGRESS = None
    print(rep, flush=True)
    assert rep.steps == 4 and len(rep.accepted) == 4 * cfg.batch


@pytest.mark.parametrize("name", ["t_f32_99", "t_bf16_99", "t_bf16_hd96", "t_bf16_d768_h8", "t_bf16_d1024_h8", "config1", "config2"])
def test_condition_kv_element_by_element(name):
    """fm_prefill_condition against the definition K_mem = W_k c, V_mem = W_v c (Sec. 3.1), every element of every block:
    the per-block launches (small memories), the tiled matrix-unit kernel (memories of whole 256-row tiles) in all three
    head widths, and the fp32 path.  Tolerance from the arithmetic: the memory is rounded to half once (2^-11 relative per
    element, the weights are exact), products are summed in fp32, and the result is rounded to half once more."""
    _need_gpu()
    from oracle.hourglass import Model
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    cfg = si.CONFIGS[int(name[-1])].replace(faces=10) if name.startswith("config") else si.TEST_CONFIGS[name]
    # configs[2] is the shape the prefill figure of the benchmark is measured on (4096 x 1024 memory, 40 blocks): every
    # element of the first and last block of each stack (the float64 reference of all 40 would take minutes)
    only = {0, 3, 4, 11, 12, 27, 28, 35, 36, 39} if name == "config2" else None
    print("case condition K/V", name, flush=True)
    w = si.make_weights(cfg, 0)
    model = Model(cfg, w)
    fm = FlashMesh(config_struct(cfg))
    fm.load_weights(si.pack_blob(cfg, w))
    half = cfg.dtype == "bf16"
    u_in, u_acc = (2.0 ** -11, 2.0 ** -24) if half else (0.0, 2.0 ** -24)
    worst = 0.0
    for s in range(cfg.batch):
        mem = si.make_memory(cfg, s)
        fm.prefill_condition(s, torch.from_numpy(mem).cuda())
        b = 0
        for st in ("cpre", "vpre", "face", "vpost", "cpost"):
            for i in range(model.layers[st]):
                pfx = f"{st}.{i}."
                if only is not None and b not in only:
                    b += 1
                    continue
                K, V = model.mem_kv(pfx, mem)                      # [M, H, hd] float64
                dk, dv = fm.debug_mem_kv(s, b)
                for ref, dev, wn in ((K, dk, "ck"), (V, dv, "cv")):
                    ref = ref.reshape(cfg.mem_len, cfg.d_model)
                    mag = np.abs(np.asarray(mem, np.float64)) @ np.abs(model.w[pfx + wn]).T      # sum of |w_k c_k| per element
                    bound = 1.05 * ((u_in + (cfg.d_model + 2) * u_acc) * mag + (u_in if half else u_acc) * np.abs(ref)) + 1e-30
                    err = np.abs(dev.astype(np.float64) - ref)
                    worst = max(worst, float((err / bound).max()))
                    assert (err <= bound).all(), (name, s, pfx, wn, float(err.max()), float((err / bound).max()))
                b += 1
    print(f"condition K/V {name}: worst error / bound = {worst:.3f}", flush=True)
    assert 0.0 < worst <= 1.0
    with pytest.raises(RuntimeError):
        fm.debug_mem_kv(0, b)


@pytest.mark.parametrize("name", ["t_f32_99", "t_bf16_99", "t_bf16_99_b1"])
def test_lockstep_eos_ends_sequences(name):
    """The degenerate end of a mesh: with the special tokens admitted (ban_specials = 0) the random-init backbone emits
    EOS somewhere in most sequences, which finishes that sequence at once (the rest of its block is dropped) while the
    others go on; blocks, accepted lengths, committed state and finished flags in lock-step with the oracle, and the
    whole-loop entry point ends every stream at the same token."""
    _need_gpu()
    from parity_harness import lockstep, make_pair
    cfg = si.TEST_CONFIGS[name].replace(ban_specials=0, faces=16)
    print("case eos", name, flush=True)
    eos_row = cfg.n_bins + 1

    def louder_eos(w):                                # a power of two: the row stays bf16-valued
        w["lm"][eos_row] = 2.0 * w["lm"][eos_row]
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype], pair=make_pair(cfg, edit_weights=louder_eos))
    print(rep, [len(s) for s in streams], flush=True)
    eos = cfg.n_bins + 1
    ended = [s for s in streams if s and s[-1] == eos and len(s) < 9 * cfg.faces]
    for s in streams:
        assert eos not in s[:-1]                      # nothing is generated behind an EOS
        assert len(s) == 9 * cfg.faces or s[-1] == eos
    assert ended, "no sequence met an EOS"
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out, n, st = fm.generate(cfg.faces, True)
    out, n = out.cpu().numpy(), n.cpu().numpy()
    if rep.token_flips == 0:
        for s in range(cfg.batch):
            assert list(out[s, :n[s]]) == streams[s]


@pytest.mark.parametrize("name", ["t_bf16_99", "t_f32_99"])
def test_lockstep_at_the_largest_batch(name):
    """64 sequences, the most fm_create accepts: every per-sequence table, flag and counter at its full length."""
    _need_gpu()
    from parity_harness import lockstep
    cfg = si.TEST_CONFIGS[name].replace(batch=64, faces=3)
    print("case batch 64", name, flush=True)
    rep, streams, fm = lockstep(cfg, cfg.faces, TOL[cfg.dtype])
    print(rep, flush=True)
    assert len(streams) == 64 and all(len(s) == 27 for s in streams)
    assert len({tuple(s) for s in streams}) > 32          # the sequences are conditioned on different memories
    for s in range(cfg.batch):
        fm.prefill_condition(s, torch.from_numpy(si.make_memory(cfg, s)).cuda())
    out, n, st = fm.generate(cfg.faces, True)
    assert st.tokens == 27 * 64
    if rep.token_flips == 0:
        out = out.cpu().numpy()
        for s in range(64):
            assert list(out[s, :27]) == streams[s]
