"""fm_prefill_condition_static: the variant of fm_prefill_condition whose staging area is a device array inside the
library image, for callers that must not allocate.  Same kernels, so the cross-attention K/V it leaves in a context -
seen through the logits of the verify passes that follow and through the emitted stream - must be bit for bit those
of the allocating entry point, and within the logit tolerance of the CPU oracle."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _ctx(cfg, static):
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    fm = FlashMesh(config_struct(cfg))
    fm.load_weights(si.pack_blob(cfg, si.make_weights(cfg, 0)))
    return fm


def _prefill(fm, cfg, static):
    for s in range(cfg.batch):
        mem = torch.from_numpy(si.make_memory(cfg, s)).cuda()
        (fm.prefill_condition_static if static else fm.prefill_condition)(s, mem)


def _steps(fm, cfg, n):
    tok, ln = fm.new_block()
    lg = torch.zeros(cfg.batch, fm.block_max, cfg.vocab, device="cuda")
    acc = torch.zeros(cfg.batch, dtype=torch.int32, device="cuda")
    out = []
    fm.set_budget(cfg.faces)
    for _ in range(n):
        fm.draft(tok, ln)
        lg.zero_()
        fm.verify_block(tok, ln, lg, acc)
        fm.commit(acc)
        out.append((tok.clone(), ln.clone(), lg.clone(), acc.clone()))
    torch.cuda.synchronize()
    return out


def test_static_prefill_matches_the_allocating_entry_point_on_two_calls_in_a_row():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    big = si.CONFIGS[1].replace(faces=20)              # 2048 x 512 memory: the tiled matrix-unit path, 2 MiB of staging
    small = si.TEST_CONFIGS["t_bf16_99"]               # 40 x 128 memory, three sequences: per-block launches
    tiny32 = si.TEST_CONFIGS["t_f32_99"]               # fp32 path
    print("case static prefill", flush=True)
    ctx = {}
    for name, cfg in (("big", big), ("small", small), ("f32", tiny32)):
        ctx[name] = (_ctx(cfg, False), _ctx(cfg, True), cfg)
    # the static calls back to back, the second and third with smaller inputs than the one before; then the allocating ones
    for name in ("big", "small", "f32"):
        _prefill(ctx[name][1], ctx[name][2], True)
    for name in ("big", "small", "f32"):
        _prefill(ctx[name][0], ctx[name][2], False)
    for name in ("big", "small", "f32"):
        ref, dut, cfg = ctx[name]
        a, b = _steps(ref, cfg, 8), _steps(dut, cfg, 8)
        for (t0, l0, g0, a0), (t1, l1, g1, a1) in zip(a, b):
            assert torch.equal(t0, t1) and torch.equal(l0, l1) and torch.equal(a0, a1), name
            assert torch.equal(g0, g1), name            # same kernels on the same K/V: bit for bit
        _prefill(ref, cfg, False)
        _prefill(dut, cfg, True)
        s0 = ref.generate(cfg.faces, True)[0]
        s1 = dut.generate(cfg.faces, True)[0]
        assert torch.equal(s0, s1), name
    # against the CPU oracle, step by step, with the static variant doing the prefill
    from parity_harness import lockstep
    for cfg, tol in ((small, 2e-2), (tiny32, 1e-4)):
        rep, streams, _ = lockstep(cfg, cfg.faces, tol, prefill="prefill_condition_static")
        print(rep, flush=True)
        assert all(len(s) == 9 * cfg.faces for s in streams)


def test_static_prefill_rejects_what_does_not_fit():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2511_15618_amd import FlashMesh
    from paper_2511_15618_amd.binding import config_struct
    # fp32 staging = mem_len * d_model * 12 bytes = 24 MiB here, beyond the 16 MiB of the static area
    cfg = si.Config("too_big", 256, 4, 32, 1, 1, 1, 1, 1, 8192, "f32", 1, 2, 2, 0, 0)
    fm = FlashMesh(config_struct(cfg))
    fm.load_weights(si.pack_blob(cfg, si.make_weights(cfg, 0)))
    mem = torch.from_numpy(si.make_memory(cfg, 0)).cuda()
    assert fm.lib.fm_prefill_condition_static(fm.h, 0, C.c_void_p(mem.data_ptr())) == -1
    assert b"static area" in fm.lib.fm_last_error(fm.h)
    assert fm.lib.fm_prefill_condition_static(fm.h, 1, C.c_void_p(mem.data_ptr())) == -1      # sequence out of range
    assert fm.lib.fm_prefill_condition_static(fm.h, 0, None) == -1
    fm.prefill_condition(0, mem)                      # the allocating entry point takes it
    out, n, _ = fm.generate(cfg.faces, True)
    assert int(n[0]) == 9 * cfg.faces
