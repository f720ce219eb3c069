"""ctypes binding: argument marshalling only.  Names follow include/flashmesh.h."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libflashmesh.so")

EXPORTS = ["fm_create", "fm_destroy", "fm_last_error", "fm_block_max", "fm_blob_elems", "fm_load_weights",
           "fm_prefill_condition", "fm_prefill_condition_static", "fm_draft", "fm_verify_block", "fm_commit", "fm_generate", "fm_read_state",
           "fm_set_draft_replay", "fm_set_budget", "fm_set_correct", "fm_correct", "fm_set_sampling", "fm_verify_bytes", "fm_debug_ring", "fm_debug_profile", "fm_debug_draft", "fm_debug_mem_kv",
           "fm_verify_path", "fm_measure_peaks", "fm_measure_gemm", "fm_measure_exchange"]


class LibraryMissing(RuntimeError):
    pass


class FmConfig(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "d_model", "n_heads", "ffn_mult", "n_bins", "l_cpre", "l_cpost", "l_vpre", "l_vpost", "l_face", "mem_len",
        "dtype", "max_batch", "max_tokens", "draft_coord", "draft_point", "draft_face", "hf_ffn_mult",
        "ban_specials")] + [("rope_base", C.c_float), ("rms_eps", C.c_float), ("window", C.c_int32), ("rules_off", C.c_int32)]


class FmStats(C.Structure):
    _fields_ = [("steps", C.c_int64), ("tokens", C.c_int64), ("acc_hist", (C.c_int64 * 32) * 3), ("ms_total", C.c_double),
                ("ms_draft", C.c_double), ("ms_verify", C.c_double), ("ms_commit", C.c_double), ("phase_samples", C.c_int64),
                ("nonfinite_rows", C.c_int64)]

    def hist(self, kind=None):
        """Accepted-length histogram as a list of 32 counts: kind 0 / 1 / 2 = coordinate-only / point-level / face-level
        steps, None = all steps."""
        kinds = (0, 1, 2) if kind is None else (kind,)
        return [sum(int(self.acc_hist[k][i]) for k in kinds) for i in range(32)]

    def mean_verified_drafts(self, kind):
        """Mean number of accepted draft tokens per step of that kind (the paper's Point-Acc for 1, Face-Acc for 2)."""
        h = self.hist(kind)
        n = sum(h)
        return sum((i - 1) * v for i, v in enumerate(h) if i > 0) / n if n else float("nan")


_lib = None


def load_library():
    """Load the HIP library; there is no fallback: without it nothing in this package computes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LibraryMissing(f"{LIB_PATH} not built: run `python -m paper_2511_15618_amd.build`")
    lib = C.CDLL(LIB_PATH)
    p, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.fm_create.argtypes = [C.POINTER(FmConfig), p, C.POINTER(p)]
    lib.fm_destroy.argtypes = [p]
    lib.fm_last_error.argtypes = [p]
    lib.fm_last_error.restype = C.c_char_p
    lib.fm_block_max.argtypes = [p]
    lib.fm_block_max.restype = i32
    lib.fm_blob_elems.argtypes = [p]
    lib.fm_blob_elems.restype = i64
    lib.fm_load_weights.argtypes = [p, p, C.c_size_t]
    lib.fm_prefill_condition.argtypes = [p, i32, p]
    lib.fm_prefill_condition_static.argtypes = [p, i32, p]
    lib.fm_draft.argtypes = [p, p, p]
    lib.fm_verify_block.argtypes = [p, p, p, p, p]
    lib.fm_commit.argtypes = [p, p]
    lib.fm_generate.argtypes = [p, i32, i32, p, p, C.POINTER(FmStats)]
    lib.fm_read_state.argtypes = [p, p]
    lib.fm_set_draft_replay.argtypes = [p, p, i32, i32, C.c_float, C.c_uint64]
    lib.fm_set_budget.argtypes = [p, i32]
    lib.fm_set_sampling.argtypes = [p, C.c_float, C.c_uint64]
    lib.fm_set_correct.argtypes = [p, i32]
    lib.fm_correct.argtypes = [p, p, p, p]
    lib.fm_verify_bytes.argtypes = [p, C.POINTER(C.c_double)]
    lib.fm_debug_ring.argtypes = [p, i32, p]
    lib.fm_debug_draft.argtypes = [p, i32, p]
    lib.fm_debug_mem_kv.argtypes = [p, i32, i32, p, p]
    lib.fm_debug_profile.argtypes = [p, p, i32]
    lib.fm_measure_peaks.argtypes = [p, C.POINTER(C.c_double)]
    lib.fm_measure_gemm.argtypes = [p, i32, C.POINTER(C.c_double)]
    lib.fm_measure_exchange.argtypes = [p, i32, i32, i32, C.POINTER(C.c_double)]
    lib.fm_verify_path.argtypes = [p]
    lib.fm_verify_path.restype = i32
    for n in EXPORTS:
        if n not in ("fm_last_error", "fm_block_max", "fm_blob_elems", "fm_verify_path"):
            getattr(lib, n).restype = C.c_int
    _lib = lib
    return lib


def config_struct(cfg, max_batch=None, max_tokens=None) -> FmConfig:
    """FmConfig from a synth_inputs.Config-like object (attribute access only)."""
    return FmConfig(
        d_model=cfg.d_model, n_heads=cfg.n_heads, ffn_mult=cfg.ffn_mult, n_bins=cfg.n_bins,
        l_cpre=cfg.l_cpre, l_cpost=cfg.l_cpost, l_vpre=cfg.l_vpre, l_vpost=cfg.l_vpost, l_face=cfg.l_face,
        mem_len=cfg.mem_len, dtype=1 if cfg.dtype == "bf16" else 0,
        max_batch=max_batch or cfg.batch, max_tokens=max_tokens or cfg.max_tokens,
        draft_coord=cfg.draft_coord, draft_point=cfg.draft_point, draft_face=cfg.draft_face,
        hf_ffn_mult=cfg.hf_ffn_mult, ban_specials=cfg.ban_specials, rope_base=cfg.rope_base, rms_eps=cfg.rms_eps,
        window=getattr(cfg, "window", 0), rules_off=(0 if getattr(cfg, "rule_a", 1) else 1) | (0 if getattr(cfg, "rule_b", 1) else 2))


class FlashMesh:
    """One library context.  Tensor arguments are torch CUDA tensors (int32 / float32, contiguous)."""

    def __init__(self, fm_config: FmConfig, stream=None):
        import torch
        self.lib = load_library()
        self.torch = torch
        self.cfgs = fm_config
        self.stream = stream if stream is not None else torch.cuda.current_stream()
        h = C.c_void_p()
        rc = self.lib.fm_create(C.byref(fm_config), C.c_void_p(self.stream.cuda_stream), C.byref(h))
        if rc != 0:
            raise RuntimeError(f"fm_create failed with code {rc}")
        self.h = h
        self.batch = fm_config.max_batch
        self.block_max = self.lib.fm_block_max(h)
        self.vocab = fm_config.n_bins + 3
        self.max_tokens = fm_config.max_tokens

    def _chk(self, rc, what):
        if rc != 0:
            raise RuntimeError(f"{what} failed ({rc}): {self.lib.fm_last_error(self.h).decode()}")

    @staticmethod
    def _ptr(t):
        return C.c_void_p(0 if t is None else t.data_ptr())

    def close(self):
        if self.h:
            self.lib.fm_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def blob_elems(self) -> int:
        return int(self.lib.fm_blob_elems(self.h))

    def load_weights(self, blob: np.ndarray):
        blob = np.ascontiguousarray(blob, dtype=np.float32)
        self._chk(self.lib.fm_load_weights(self.h, C.c_void_p(blob.ctypes.data), C.c_size_t(blob.size)), "fm_load_weights")

    def prefill_condition(self, seq: int, mem):
        assert mem.is_cuda and mem.dtype == self.torch.float32 and mem.is_contiguous()
        assert tuple(mem.shape) == (self.cfgs.mem_len, self.cfgs.d_model)
        self._chk(self.lib.fm_prefill_condition(self.h, seq, self._ptr(mem)), "fm_prefill_condition")

    def prefill_condition_static(self, seq: int, mem):
        assert mem.is_cuda and mem.dtype == self.torch.float32 and mem.is_contiguous()
        assert tuple(mem.shape) == (self.cfgs.mem_len, self.cfgs.d_model)
        self._chk(self.lib.fm_prefill_condition_static(self.h, seq, self._ptr(mem)), "fm_prefill_condition_static")

    def new_block(self):
        t = self.torch
        return (t.zeros(self.batch, self.block_max, dtype=t.int32, device="cuda"),
                t.zeros(self.batch, dtype=t.int32, device="cuda"))

    def draft(self, block_tok, block_len):
        self._chk(self.lib.fm_draft(self.h, self._ptr(block_tok), self._ptr(block_len)), "fm_draft")

    def verify_block(self, block_tok, block_len, logits, accepted):
        self._chk(self.lib.fm_verify_block(self.h, self._ptr(block_tok), self._ptr(block_len), self._ptr(logits),
                                           self._ptr(accepted)), "fm_verify_block")

    def commit(self, accepted):
        self._chk(self.lib.fm_commit(self.h, self._ptr(accepted)), "fm_commit")

    def generate(self, max_faces: int, speculative: bool = True):
        t = self.torch
        out = t.zeros(self.batch, self.max_tokens, dtype=t.int32, device="cuda")
        n = t.zeros(self.batch, dtype=t.int32, device="cuda")
        st = FmStats()
        self._chk(self.lib.fm_generate(self.h, max_faces, 1 if speculative else 0, self._ptr(out), self._ptr(n),
                                       C.byref(st)), "fm_generate")
        return out, n, st

    def read_state(self) -> np.ndarray:
        out = np.zeros((self.batch, 6), np.int32)
        self._chk(self.lib.fm_read_state(self.h, C.c_void_p(out.ctypes.data)), "fm_read_state")
        return out

    def set_draft_replay(self, stream, n_valid: int, keep_prob: float, seed: int):
        if stream is None:
            self._chk(self.lib.fm_set_draft_replay(self.h, None, 0, 0, 0.0, 0), "fm_set_draft_replay")
        else:
            assert stream.dtype == self.torch.int32 and stream.is_cuda and stream.is_contiguous()
            self._keep = stream
            self._chk(self.lib.fm_set_draft_replay(self.h, self._ptr(stream), stream.shape[1], n_valid,
                                                   C.c_float(keep_prob), C.c_uint64(seed)), "fm_set_draft_replay")

    def set_sampling(self, temperature: float, seed: int):
        self._chk(self.lib.fm_set_sampling(self.h, C.c_float(temperature), C.c_uint64(seed)), "fm_set_sampling")

    def set_correct(self, hist_vertices: int):
        self._chk(self.lib.fm_set_correct(self.h, hist_vertices), "fm_set_correct")

    def correct(self, block_tok, block_len, labels_out=None):
        self._chk(self.lib.fm_correct(self.h, self._ptr(block_tok), self._ptr(block_len), self._ptr(labels_out)), "fm_correct")

    def set_budget(self, max_faces: int):
        self._chk(self.lib.fm_set_budget(self.h, max_faces), "fm_set_budget")

    def debug_ring(self, which: int) -> np.ndarray:
        size = (32, 16, 8, 16, 32, 16, 8)[which]
        out = np.zeros((self.batch, size, self.cfgs.d_model), np.float32)
        self._chk(self.lib.fm_debug_ring(self.h, which, C.c_void_p(out.ctypes.data)), "fm_debug_ring")
        return out

    def keep_draft_rows(self, on: bool = True):
        self._chk(self.lib.fm_debug_draft(self.h, -1 if on else -2, None), "fm_debug_draft")

    def debug_draft(self, which: int) -> np.ndarray:
        cfgs = self.cfgs
        if which == 0:
            shape = (self.batch, self.block_max, self.vocab)
        elif which == 1:
            shape = (self.batch, max(cfgs.draft_point // 3 - 1, 1), 3)
        else:
            shape = (self.batch, max(cfgs.draft_face // 3 - (0 if cfgs.rules_off & 2 else 1), 1), 3)
        out = np.zeros(shape, np.float32)
        self._chk(self.lib.fm_debug_draft(self.h, which, C.c_void_p(out.ctypes.data)), "fm_debug_draft")
        return out

    def debug_mem_kv(self, seq: int, block: int):
        k = np.zeros((self.cfgs.mem_len, self.cfgs.d_model), np.float32)
        v = np.zeros_like(k)
        self._chk(self.lib.fm_debug_mem_kv(self.h, seq, block, C.c_void_p(k.ctypes.data), C.c_void_p(v.ctypes.data)), "fm_debug_mem_kv")
        return k, v

    def debug_profile(self, n: int = 1024) -> np.ndarray:
        out = np.zeros(n, np.uint64)
        self._chk(self.lib.fm_debug_profile(self.h, C.c_void_p(out.ctypes.data), n), "fm_debug_profile")
        return out

    def measure_peaks(self) -> dict:
        v = (C.c_double * 3)()
        self._chk(self.lib.fm_measure_peaks(self.h, v), "fm_measure_peaks")
        return {"hbm_read_GBs": v[0], "hbm_copy_GBs": v[1], "mfma_f16_TFLOPs": v[2]}

    def measure_gemm(self, rows: int) -> dict:
        out = (C.c_double * 2)()
        self._chk(self.lib.fm_measure_gemm(self.h, rows, out), "fm_measure_gemm")
        return {"rows": rows, "ms": out[0], "TFLOPs": out[1]}

    def measure_exchange(self, workgroups: int, nbytes: int, pingpong: bool = False) -> float:
        """Microseconds per dependent all-to-all hand-off between `workgroups` resident workgroups."""
        out = C.c_double()
        self._chk(self.lib.fm_measure_exchange(self.h, workgroups, nbytes, 1 if pingpong else 0, C.byref(out)), "fm_measure_exchange")
        return out.value

    def verify_path(self) -> int:
        return int(self.lib.fm_verify_path(self.h))

    def verify_bytes(self) -> float:
        v = C.c_double()
        self._chk(self.lib.fm_verify_bytes(self.h, C.byref(v)), "fm_verify_bytes")
        return v.value
