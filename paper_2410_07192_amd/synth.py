"""Seeded synthetic inputs shared by the tests, the benchmark and the CPU checker.

Nothing in this module performs any of the method's arithmetic: it only draws
random numbers with the shapes and distributions of the workloads and, for the
bf16 workloads, rounds them to bf16-representable values (an input-format
conversion, so that both sides start from identical numbers).

Weight layout produced here is the mathematical one, y = x @ W + b with
W of shape [in_features, out_features].
"""
from __future__ import annotations

from dataclasses import dataclass, asdict
import numpy as np


@dataclass(frozen=True)
class ModelShape:
    """Transformer shape of a fill job (or of the emulated main-job stage)."""
    n_layers: int
    d_model: int
    n_heads: int
    d_ff: int
    seq_len: int
    batch: int            # sequences per microbatch
    vocab: int = 0        # 0: hidden states are given directly (no embedding)
    causal: bool = False
    dtype: str = "bf16"   # "f32" or "bf16"
    eps: float = 1e-5

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_heads

    @property
    def tokens(self) -> int:
        return self.batch * self.seq_len

    def asdict(self):
        return asdict(self)


# The five workloads.  Index = position in the benchmark description (0-based).
WORKLOADS = {
    "cfg1": ModelShape(1, 256, 4, 1024, 128, 4, 0, False, "f32"),
    "cfg2": ModelShape(12, 768, 12, 3072, 512, 32, 30522, False, "bf16"),
    "cfg3": ModelShape(24, 2048, 16, 8192, 1024, 16, 50257, True, "bf16"),
    "cfg4": ModelShape(12, 1024, 16, 4096, 1024, 8, 50257, True, "bf16"),
    "cfg5": ModelShape(3, 8192, 64, 32768, 2048, 1, 0, True, "bf16"),
}

# 1F1B schedule parameters per workload: (p, m, t_f ns, t_b ns, free bytes)
GIB = 1 << 30
SCHEDULES = {
    "cfg1": (4, 8, 2_000_000, 4_000_000, 2 * GIB),
    "cfg2": (8, 16, 15_000_000, 30_000_000, 24 * GIB),
    "cfg4": (16, 32, 15_000_000, 30_000_000, 16 * GIB),
}

LAYER_PARAM_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                     "ln2_g", "ln2_b", "w_1", "b_1", "w_2", "b_2")


def layer_param_shapes(d: int, f: int):
    return {
        "ln1_g": (d,), "ln1_b": (d,),
        "w_qkv": (d, 3 * d), "b_qkv": (3 * d,),
        "w_o": (d, d), "b_o": (d,),
        "ln2_g": (d,), "ln2_b": (d,),
        "w_1": (d, f), "b_1": (f,),
        "w_2": (f, d), "b_2": (d,),
    }


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    r = ((u + bias) & np.uint32(0xFFFF0000)).astype(np.uint32)
    return r.view(np.float32)


def _draw(rng, shape, std, mean=0.0, dtype="bf16"):
    a = rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)
    return round_to_bf16(a) if dtype == "bf16" else a


def make_layer_params(shape: ModelShape, layer: int, seed: int = 0, std: float = 0.02):
    """Parameters of one layer: every matrix, bias and LayerNorm shift ~ N(0, std^2);
    LayerNorm scales ~ 1 + N(0, std^2), so that no term is trivially zero or one."""
    rng = np.random.default_rng([seed, 7, layer])
    out = {}
    for name, shp in layer_param_shapes(shape.d_model, shape.d_ff).items():
        mean = 1.0 if name.endswith("_g") else 0.0
        out[name] = _draw(rng, shp, std, mean, shape.dtype)
    return out


def make_model_params(shape: ModelShape, seed: int = 0, std: float = 0.02):
    """Embeddings (when vocab > 0), all layers and the final LayerNorm."""
    rng = np.random.default_rng([seed, 11])
    p = {"layers": [make_layer_params(shape, l, seed, std) for l in range(shape.n_layers)]}
    if shape.vocab > 0:
        p["tok_emb"] = _draw(rng, (shape.vocab, shape.d_model), std, 0.0, shape.dtype)
        p["pos_emb"] = _draw(rng, (shape.seq_len, shape.d_model), std, 0.0, shape.dtype)
    p["lnf_g"] = _draw(rng, (shape.d_model,), std, 1.0, shape.dtype)
    p["lnf_b"] = _draw(rng, (shape.d_model,), std, 0.0, shape.dtype)
    return p


def make_hidden(shape: ModelShape, seed: int = 1, batch: int | None = None):
    """Hidden states ~ N(0,1), [batch, seq, d]."""
    rng = np.random.default_rng([seed, 13])
    b = shape.batch if batch is None else batch
    return _draw(rng, (b, shape.seq_len, shape.d_model), 1.0, 0.0, shape.dtype)


def make_token_ids(shape: ModelShape, seed: int = 1, batch: int | None = None):
    """Token ids uniform over the vocabulary, int32 [batch, seq]."""
    rng = np.random.default_rng([seed, 17])
    b = shape.batch if batch is None else batch
    return rng.integers(0, shape.vocab, size=(b, shape.seq_len), dtype=np.int32)


def make_planner_instance(seed: int, n_nodes: int, n_bubbles: int,
                          max_dur: int = 1000, max_mem: int = 100):
    """Random integer instance (B, M, F) for planner parity tests."""
    rng = np.random.default_rng([seed, 19])
    B = rng.integers(1, 4 * max_dur, size=n_bubbles).tolist()
    M = rng.integers(max_mem // 2, 2 * max_mem, size=n_bubbles).tolist()
    F = [(int(rng.integers(1, max_dur)), int(rng.integers(1, max_mem))) for _ in range(n_nodes)]
    return [int(b) for b in B], [int(x) for x in M], F
