"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds NONE of the method's arithmetic: it only names the model
configurations, lists the parameter tensors in manifest order, draws them from
seeded NumPy generators, rounds them to bf16 where a configuration asks for
bf16 storage, and provides the counter-based uniform generator that the
synthetic "replay" draft source uses.  Both sides import it; neither side
imports the other.

The paper's evaluation uses trained 0.5-3.4 B parameter hourglass models on
ShapeNetV2 / gObjaverse meshes (Sec. 5.1 "Datasets", Table 1).  Neither weights
nor meshes are available, so every input here is random-init and seeded, with
the shapes of the paper's workloads: 9 coordinate tokens per face, 3 per
vertex (Supp. "Hourglass Transformer"), one attention window of context
(18K / 36K tokens, Sec. 5.1 "Implementary details").
"""
from __future__ import annotations

import dataclasses
import numpy as np

HEAD_DIM = 64
N_SPECIAL = 3  # BOS, EOS, PAD follow the coordinate bins


@dataclasses.dataclass(frozen=True)
class Config:
    name: str
    d_model: int
    n_heads: int
    n_bins: int
    l_cpre: int
    l_cpost: int
    l_vpre: int
    l_vpost: int
    l_face: int
    mem_len: int
    dtype: str            # "f32" | "bf16"
    batch: int
    faces: int            # generation budget per sequence
    draft_coord: int      # Dc: coordinate-level SP heads
    draft_point: int      # m : nominal point-level tokens (multiple of 3, 0 = off)
    draft_face: int       # n : nominal face-level tokens (multiple of 9, 0 = off)
    ffn_mult: int = 4
    hf_ffn_mult: int = 4
    ban_specials: int = 1
    rope_base: float = 10000.0
    rms_eps: float = 1e-6
    window: int = 0       # self-attention window in coordinate tokens (multiple of 9); 0 = the whole context
    rule_a: int = 1       # supplement "Optimizations", rule (A): no point-level prediction where a face-level one fires
    rule_b: int = 1       # rule (B): the point / face levels leave their first three tokens to the coordinate level

    @property
    def vocab(self) -> int:
        return self.n_bins + N_SPECIAL

    @property
    def bos(self) -> int:
        return self.n_bins

    @property
    def eos(self) -> int:
        return self.n_bins + 1

    @property
    def pad(self) -> int:
        return self.n_bins + 2

    @property
    def max_tokens(self) -> int:
        return 9 * self.faces

    def level_window(self, lvl: str) -> int:
        """Window at level "c" / "v" / "f" in that level's own positions (0 = unbounded): the same span of the
        mesh at every level."""
        return self.window // {"c": 1, "v": 3, "f": 9}[lvl]

    @property
    def block_max(self) -> int:
        """Largest verify block: main token plus drafts."""
        return max(1 + self.draft_coord, self.draft_point, self.draft_face, 1)

    @property
    def n_layers(self) -> int:
        return self.l_cpre + self.l_cpost + self.l_vpre + self.l_vpost + self.l_face

    def replace(self, **kw) -> "Config":
        return dataclasses.replace(self, **kw)


# The five benchmark configurations (index = position in the benchmark list).
CONFIGS = [
    Config("tiny", 256, 4, 128, 2, 2, 2, 2, 4, 256, "f32", 1, 10, 3, 0, 0),
    Config("small", 512, 8, 1024, 2, 2, 4, 4, 8, 2048, "bf16", 1, 500, 2, 9, 9),
    Config("medium", 1024, 16, 1024, 4, 4, 8, 8, 16, 4096, "bf16", 1, 2000, 2, 9, 9),
    Config("medium_b8", 1024, 16, 1024, 4, 4, 8, 8, 16, 4096, "bf16", 8, 2000, 2, 9, 9),
    Config("large_b4", 1536, 24, 1024, 4, 4, 8, 8, 24, 4096, "bf16", 4, 4000, 2, 15, 18),
]

# Small shapes for CPU-side tests and quick parity runs (not benchmark lines).
TEST_CONFIGS = {
    "t_f32_c": Config("t_f32_c", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 1, 6, 3, 0, 0),
    "t_f32_99": Config("t_f32_99", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 6, 2, 9, 9),
    "t_f32_1815": Config("t_f32_1815", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 8, 2, 15, 18),
    "t_bf16_99": Config("t_bf16_99", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 3, 12, 2, 9, 9),
    "t_bf16_99_b1": Config("t_bf16_99_b1", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 12, 2, 9, 9),
    "t_bf16_99_b1w": Config("t_bf16_99_b1w", 256, 4, 64, 2, 1, 2, 2, 3, 100, "bf16", 1, 30, 2, 9, 9),
    "t_bf16_99_b8long": Config("t_bf16_99_b8long", 256, 4, 64, 2, 1, 2, 2, 3, 100, "bf16", 8, 256, 2, 9, 9),
    # draft-count variants of the paper's sweep (face-point counts 18-18, 18-12, 27-9, 27-27) and coordinate-only heads
    "t_f32_1818": Config("t_f32_1818", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 10, 2, 18, 18),
    "t_bf16_1812": Config("t_bf16_1812", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 2, 10, 2, 12, 18),
    "t_bf16_279": Config("t_bf16_279", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 12, 2, 9, 27),
    "t_f32_2727": Config("t_f32_2727", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 12, 2, 27, 27),
    "t_bf16_c17": Config("t_bf16_c17", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 2, 8, 17, 0, 0),
    # rule (A) of the supplement switched off: the point level also fires at face split nodes (three levels overlap there)
    "t_f32_99_noA": Config("t_f32_99_noA", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 6, 2, 9, 9, rule_a=0),
    "t_bf16_1815_noA": Config("t_bf16_1815_noA", 192, 3, 64, 1, 2, 2, 2, 2, 72, "bf16", 2, 14, 2, 15, 18, rule_a=0),
    # rule (B) off as well: HF sets for the first three coordinate offsets and the vertex offset 0
    "t_f32_99_noB": Config("t_f32_99_noB", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 6, 2, 9, 9, rule_b=0),
    "t_bf16_1815_noAB": Config("t_bf16_1815_noAB", 192, 3, 64, 1, 2, 2, 2, 2, 72, "bf16", 2, 14, 2, 15, 18, rule_a=0, rule_b=0),
    "t_bf16_99_b1_noB": Config("t_bf16_99_b1_noB", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 12, 2, 9, 9, rule_b=0),
    # head widths of the paper's own models (Sec. 5.1: d = 768 / 1536 / 2048 with 8 / 16 heads, i.e. 96 and 128 per head;
    # 4-8-12 and 4-10-18 blocks per level), scaled down in width and depth, in both storage types; the last two keep
    # the paper's d = 768 with 8 heads, and 8 heads of 128, at a few blocks, with a condition memory of whole GEMM tiles
    "t_f32_hd96": Config("t_f32_hd96", 192, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 6, 2, 9, 9),
    "t_f32_hd128": Config("t_f32_hd128", 256, 2, 32, 2, 2, 3, 2, 3, 24, "f32", 1, 6, 2, 15, 18),
    "t_bf16_hd96": Config("t_bf16_hd96", 192, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 2, 8, 2, 9, 9),
    "t_bf16_hd128": Config("t_bf16_hd128", 256, 2, 32, 2, 2, 3, 2, 3, 40, "bf16", 1, 8, 2, 15, 18),
    "t_bf16_d768_h8": Config("t_bf16_d768_h8", 768, 8, 128, 1, 1, 1, 1, 2, 256, "bf16", 2, 6, 2, 9, 9),
    "t_bf16_d1024_h8": Config("t_bf16_d1024_h8", 1024, 8, 128, 1, 1, 1, 1, 1, 256, "bf16", 1, 5, 2, 15, 18),
    "t_bf16_99_b1_noA": Config("t_bf16_99_b1_noA", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 12, 2, 9, 9, rule_a=0),
    "t_bf16_1815": Config("t_bf16_1815", 192, 3, 64, 1, 2, 2, 2, 2, 72, "bf16", 2, 14, 2, 15, 18),
    # blocks longer than 16 tokens at one sequence (two row groups at the coordinate level of the single-launch verify kernel)
    "t_bf16_1815_b1": Config("t_bf16_1815_b1", 256, 4, 64, 2, 1, 2, 2, 3, 100, "bf16", 1, 30, 2, 15, 18),
    "t_bf16_2727_b1": Config("t_bf16_2727_b1", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 24, 2, 27, 27),
    "t_bf16_1815_b1_w72": Config("t_bf16_1815_b1_w72", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 150, 2, 15, 18, window=72),
    # sliding window: streams long enough that the K/V rings (multiples of 128 positions) wrap at all three levels
    "t_f32_99_w36": Config("t_f32_99_w36", 128, 2, 32, 1, 2, 1, 2, 2, 24, "f32", 2, 150, 2, 9, 9, window=36),
    "t_bf16_99_w36": Config("t_bf16_99_w36", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 3, 150, 2, 9, 9, window=36),
    "t_bf16_99_b1_w36": Config("t_bf16_99_b1_w36", 128, 2, 32, 1, 2, 1, 2, 2, 40, "bf16", 1, 150, 2, 9, 9, window=36),
    "t_bf16_1815_w72": Config("t_bf16_1815_w72", 192, 3, 64, 1, 2, 2, 2, 2, 72, "bf16", 2, 150, 2, 15, 18, window=72),
}

STACKS = ("cpre", "vpre", "face", "vpost", "cpost")


def stack_layers(cfg: Config) -> dict:
    return {"cpre": cfg.l_cpre, "vpre": cfg.l_vpre, "face": cfg.l_face,
            "vpost": cfg.l_vpost, "cpost": cfg.l_cpost}


def sp_head_counts(cfg: Config) -> dict:
    """Number of SP heads per level: coordinate Dc, point m/3-1, face n/9-1."""
    return {"c": cfg.draft_coord,
            "v": max(cfg.draft_point // 3 - 1, 0),
            "f": max(cfg.draft_face // 9 - 1, 0)}


def hf_coord_offsets(cfg: Config) -> range:
    """Coordinate offsets t that own an HF parameter set (under rule (B) offsets 0..2 are left to the coordinate level)."""
    return range(3 if cfg.rule_b else 0, max(cfg.draft_point, cfg.draft_face))


def hf_vertex_offsets(cfg: Config) -> range:
    """Vertex offsets j (from the face split node) that own a vertex-level HF parameter set."""
    return range(1 if cfg.rule_b else 0, cfg.draft_face // 3) if cfg.draft_face else range(0)


def manifest(cfg: Config):
    """Parameter tensors in blob order: (name, shape, kind, fan_in).

    Linear weights are in the mathematical layout [out, in] (y = W x)."""
    d, ff, hf, V = cfg.d_model, cfg.ffn_mult * cfg.d_model, cfg.hf_ffn_mult * cfg.d_model, cfg.vocab
    out = [("emb", (V, d), "emb", 0)]
    for st in STACKS:
        for i in range(stack_layers(cfg)[st]):
            p = f"{st}.{i}."
            out += [(p + "g1", (d,), "gain", 0)]
            out += [(p + n, (d, d), "lin", d) for n in ("wq", "wk", "wv", "wo")]
            out += [(p + "g2", (d,), "gain", 0)]
            out += [(p + n, (d, d), "lin", d) for n in ("cq", "ck", "cv", "co")]
            out += [(p + "g3", (d,), "gain", 0), (p + "w1", (ff, d), "lin", d), (p + "w2", (d, ff), "lin", ff)]
    out += [("short_cv", (d, d), "lin", d), ("short_vf", (d, d), "lin", d)]
    out += [("gf", (d,), "gain", 0), ("lm", (V, d), "lin", d)]
    for lvl, cnt in sp_head_counts(cfg).items():
        for k in range(1, cnt + 1):
            p = f"sp.{lvl}.{k}."
            out += [(p + "g", (d,), "gain", 0)]
            out += [(p + n, (d, d), "lin", d) for n in ("wq", "wo", "cq", "co", "lin")]
    for lvl, offs in (("c", hf_coord_offsets(cfg)), ("v", hf_vertex_offsets(cfg))):
        for t in offs:
            p = f"hf.{lvl}.{t}."
            out += [(p + "g", (d,), "gain", 0), (p + "wq", (d, d), "lin", d),
                    (p + "w1", (hf, d), "lin", d), (p + "w2", (d, hf), "lin", hf)]
    out += [("label", (3, d), "lin", d)]     # label head of the correct stage: historical / new / intra-batch
    return out


def blob_size(cfg: Config) -> int:
    return sum(int(np.prod(s)) for _, s, _, _ in manifest(cfg))


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    y = ((u + r) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return y.view(np.float32).reshape(x.shape)


def make_weights(cfg: Config, seed: int = 0, gain_jitter: float = 0.0) -> dict:
    """Random-init parameters: linear ~ N(0,1)/sqrt(fan_in), embedding ~ N(0,1), gains 1
    (or 1 + gain_jitter*N(0,1) so that tests can tell the gains apart)."""
    w = {}
    for idx, (name, shape, kind, fan_in) in enumerate(manifest(cfg)):
        rng = np.random.default_rng([seed, idx])
        if kind == "gain":
            a = np.ones(shape, np.float32)
            if gain_jitter:
                a = a + gain_jitter * rng.standard_normal(shape, dtype=np.float32)
        else:
            a = rng.standard_normal(shape, dtype=np.float32)
            if kind == "lin":
                a *= np.float32(1.0 / np.sqrt(fan_in))
            if cfg.dtype == "bf16":
                a = bf16_round(a)
        w[name] = a
    return w


def pack_blob(cfg: Config, w: dict) -> np.ndarray:
    """Concatenate the tensors in manifest order into one flat float32 array."""
    out = np.empty(blob_size(cfg), np.float32)
    o = 0
    for name, shape, _, _ in manifest(cfg):
        n = int(np.prod(shape))
        out[o:o + n] = w[name].reshape(-1)
        o += n
    return out


def make_memory(cfg: Config, seq: int) -> np.ndarray:
    """Condition memory [mem_len, d_model] ~ N(0,1), one seed per sequence."""
    return np.random.default_rng(1000 + seq).standard_normal((cfg.mem_len, cfg.d_model), dtype=np.float32)


_M64 = (1 << 64) - 1


def replay_uniform(seed: int, seq: int, pos: int) -> float:
    """Counter-based uniform in [0,1) keyed by (seed, sequence, absolute token position).

    splitmix64 finaliser over a 64-bit key, top 24 bits.  The device side
    implements the same integer recipe, so both sides draw identical numbers."""
    z = (seed * 0x9E3779B97F4A7C15 + seq * 0xBF58476D1CE4E5B9 + pos * 0x94D049BB133111EB + 0x2545F4914F6CDD1D) & _M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
    z = z ^ (z >> 31)
    return (z >> 40) / float(1 << 24)
