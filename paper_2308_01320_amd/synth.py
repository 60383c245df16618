"""Seeded synthetic inputs: model dimensions, random weights, random prompts.

This module holds no arithmetic of the generation method itself.  It only
draws numbers and names shapes, so that the CPU oracle's tests and the HIP
path's tests can be fed the very same arrays.  It imports neither of them.

Workload shapes follow the paper's generation benchmark (Section 5.3 (I):
a 256-token prompt followed by 256 generated tokens, the actor run once per
generated token) on OPT-shaped decoders (Section 2, Tables 1-3 name the
OPT family from 1.3B to 175B).
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class ModelDims:
    """Dimensions of an OPT-style decoder and of one generation job."""

    name: str
    n_layers: int
    hidden: int
    n_heads: int
    ffn: int
    vocab: int
    max_positions: int
    batch: int
    prompt_len: int
    gen_len: int
    dtype: str  # "f32" or "bf16": storage type of weights / KV cache
    sampling: str  # "greedy" or "gumbel"
    pos_offset: int = 0
    ln_eps: float = 1e-5

    @property
    def head_dim(self) -> int:
        return self.hidden // self.n_heads

    def sliced(self, **kw) -> "ModelDims":
        """Same layer shape, fewer layers / smaller job (parity fixtures)."""
        return replace(self, **kw)


# The five workloads the benchmark definition names (index = config number).
CONFIGS = {
    "tiny": ModelDims("tiny", 2, 256, 4, 1024, 1024, 128, 4, 32, 16, "f32", "greedy"),
    "opt-1.3b": ModelDims("opt-1.3b", 24, 2048, 32, 8192, 50272, 2048, 32, 256, 256, "bf16", "gumbel"),
    "opt-6.7b": ModelDims("opt-6.7b", 32, 4096, 32, 16384, 50272, 2048, 16, 256, 256, "bf16", "greedy"),
    "opt-13b": ModelDims("opt-13b", 40, 5120, 40, 20480, 50272, 2048, 32, 256, 256, "bf16", "gumbel"),
    "opt-66b": ModelDims("opt-66b", 64, 9216, 72, 36864, 50272, 2048, 8, 256, 256, "bf16", "greedy"),
}

LAYER_TENSORS = (
    "ln1_g", "ln1_b", "wqkv", "bqkv", "wo", "bo",
    "ln2_g", "ln2_b", "w1", "b1", "w2", "b2",
)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16-representable fp32 (ties to even)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def layer_shapes(d: ModelDims) -> Dict[str, tuple]:
    H, F = d.hidden, d.ffn
    return {
        "ln1_g": (H,), "ln1_b": (H,),
        "wqkv": (3 * H, H), "bqkv": (3 * H,),
        "wo": (H, H), "bo": (H,),
        "ln2_g": (H,), "ln2_b": (H,),
        "w1": (F, H), "b1": (F,),
        "w2": (H, F), "b2": (H,),
    }


def make_weights(d: ModelDims, seed: int = 0, tied: bool = True, std: float = 0.02) -> dict:
    """Random-init weights as fp32 numpy arrays, drawn in a fixed tensor order.

    Matrices, embeddings and biases ~ N(0, std); LayerNorm gains 1 + N(0, std),
    LayerNorm shifts N(0, std), so that a dropped bias or affine term changes
    the output.  For dtype "bf16" every value is rounded to a bf16-representable
    fp32, so both sides start from identical numbers.

    Returns {"tok_emb", "pos_emb", "lnf_g", "lnf_b", "lm_head", "layers": [..]}.
    With tied=True, "lm_head" is the same array object as "tok_emb".
    """
    rng = np.random.default_rng(seed)

    def draw(shape, mean=0.0):
        a = (rng.standard_normal(shape, dtype=np.float32) * np.float32(std) + np.float32(mean)).astype(np.float32)
        return round_to_bf16(a) if d.dtype == "bf16" else a

    w = {}
    w["tok_emb"] = draw((d.vocab, d.hidden))
    w["pos_emb"] = draw((d.max_positions + d.pos_offset, d.hidden))
    layers = []
    for _ in range(d.n_layers):
        lw = {}
        for name, shape in layer_shapes(d).items():
            lw[name] = draw(shape, mean=1.0 if name.endswith("_g") else 0.0)
        layers.append(lw)
    w["layers"] = layers
    w["lnf_g"] = draw((d.hidden,), mean=1.0)
    w["lnf_b"] = draw((d.hidden,))
    w["lm_head"] = w["tok_emb"] if tied else draw((d.vocab, d.hidden))
    return w


def make_prompts(d: ModelDims, seed: int = 1234, batch: int | None = None, prompt_len: int | None = None) -> np.ndarray:
    """Prompt token ids [B, S], i.i.d. uniform on [0, vocab), int32."""
    rng = np.random.default_rng(seed)
    B = d.batch if batch is None else batch
    S = d.prompt_len if prompt_len is None else prompt_len
    return rng.integers(0, d.vocab, size=(B, S), dtype=np.int32)


def device_weights(d, torch, seed=0, std=0.02, tile=None):
    """Random-init bf16 weights generated on the device, tensor by tensor (the full-size models do not
    fit host memory).  tile: optional callable applied to every GEMM matrix (and the LM head) as soon as
    it is drawn, the row-major original then dropped -- a caller that hands the engine pre-tiled matrices
    passes the binding's tiling call here, so that no matrix ever exists twice."""
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    dt = torch.bfloat16

    def draw(shape, mean=0.0):
        t = torch.randn(shape, generator=g, device="cuda", dtype=torch.float32)
        return (t * std + mean).to(dt).contiguous()

    def mat(shape):
        m = draw(shape)
        if tile is None:
            return m
        t = tile(m)
        torch.cuda.synchronize()
        return t

    H, F = d.hidden, d.ffn
    w = {"tok_emb": draw((d.vocab, H)), "pos_emb": draw((d.max_positions + d.pos_offset, H)), "layers": []}
    for _ in range(d.n_layers):
        w["layers"].append({
            "ln1_g": draw((H,), 1.0), "ln1_b": draw((H,)), "wqkv": mat((3 * H, H)), "bqkv": draw((3 * H,)),
            "wo": mat((H, H)), "bo": draw((H,)), "ln2_g": draw((H,), 1.0), "ln2_b": draw((H,)),
            "w1": mat((F, H)), "b1": draw((F,)), "w2": mat((H, F)), "b2": draw((H,))})
    w["lnf_g"], w["lnf_b"] = draw((H,), 1.0), draw((H,))
    w["lm_head"] = tile(w["tok_emb"]) if tile is not None else w["tok_emb"]
    return w
