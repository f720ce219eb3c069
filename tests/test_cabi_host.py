"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every declared symbol,
and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

import synth_inputs as si
from paper_2511_15618_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_15618_amd import build
        build.build()
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "flashmesh.h")).read()
    declared = sorted(set(re.findall(r"\b(fm_[a-z_]+)\s*\(", header)))
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == declared


def test_config_struct_matches_header_layout():
    header = open(os.path.join(ROOT, "include", "flashmesh.h")).read()
    start = header.index("typedef struct {", header.index("Plain-old-data configuration"))
    body = header[start + len("typedef struct {"):header.index("} fm_config;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        m = re.match(r"\s*(int32_t|float)\s+(.*)", decl.strip(), flags=re.S)
        if m:
            fields += [(n.strip(), m.group(1)) for n in m.group(2).split(",")]
    got = [(n, "float" if t is C.c_float else "int32_t") for n, t in binding.FmConfig._fields_]
    assert got == fields


@pytest.mark.parametrize("bad", [
    dict(d_model=100), dict(n_heads=3), dict(dtype=7), dict(max_batch=0), dict(max_batch=65), dict(max_tokens=10),
    dict(draft_point=4), dict(draft_face=12), dict(draft_coord=1), dict(draft_face=36), dict(l_face=0),
    dict(mem_len=0), dict(rope_base=1.0), dict(rms_eps=0.0), dict(window=-9), dict(window=10), dict(rules_off=4),
    dict(d_model=160),               # head width 80
])
def test_create_rejects_bad_config_without_touching_the_device(lib, bad):
    cs = binding.config_struct(si.TEST_CONFIGS["t_f32_99"])
    for k, v in bad.items():
        setattr(cs, k, v)
    h = C.c_void_p()
    assert lib.fm_create(C.byref(cs), None, C.byref(h)) == -1      # FM_EINVAL
    assert not h.value


def test_null_arguments(lib):
    assert lib.fm_create(None, None, None) == -1
    assert lib.fm_destroy(None) == -1
    assert lib.fm_draft(None, None, None) == -1
    assert lib.fm_verify_block(None, None, None, None, None) == -1
    assert lib.fm_commit(None, None) == -1
    assert lib.fm_generate(None, 1, 1, None, None, None) == -1
    assert lib.fm_load_weights(None, None, 0) == -1
    assert lib.fm_prefill_condition(None, 0, None) == -1
    assert lib.fm_last_error(None) == b"null context"
    assert lib.fm_set_correct(None, 3) == -1
    assert lib.fm_correct(None, None, None, None) == -1
    assert lib.fm_measure_gemm(None, 16, None) == -1


def test_manifest_matches_blob_size():
    for cfg in list(si.TEST_CONFIGS.values()) + si.CONFIGS[:3]:
        n = si.blob_size(cfg)
        d, ff, hf, V = cfg.d_model, 4 * cfg.d_model, cfg.hf_ffn_mult * cfg.d_model, cfg.vocab
        per_block = 3 * d + 8 * d * d + 2 * ff * d
        sp = sum(si.sp_head_counts(cfg).values()) * (d + 5 * d * d)
        hfn = (len(si.hf_coord_offsets(cfg)) + len(si.hf_vertex_offsets(cfg))) * (d + d * d + 2 * hf * d)
        assert n == V * d + cfg.n_layers * per_block + 2 * d * d + d + V * d + sp + hfn + 3 * d   # + label head


def test_replay_uniform_is_uniform_and_keyed():
    import numpy as np
    u = np.array([si.replay_uniform(5, 1, p) for p in range(1, 4001)])
    assert 0.0 <= u.min() and u.max() < 1.0 and abs(u.mean() - 0.5) < 0.03
    assert abs((u < 0.93).mean() - 0.93) < 0.02
    assert si.replay_uniform(5, 1, 10) != si.replay_uniform(5, 2, 10) != si.replay_uniform(6, 1, 10)
