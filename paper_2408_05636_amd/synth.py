"""Seeded synthetic inputs: model shapes, random-init weights, prefixes.

This module serves both the HIP path and the CPU oracle's tests.  It holds
none of the method's arithmetic: no forward pass, no softmax, no sampling,
no acceptance rule and no counter-based uniforms -- only shapes and seeded
draws of weights and prompt tokens.

The paper evaluates trained GPT-2 XL / GPT-Neo / Vicuna targets with an MDLM
drafter on text prompts (Evaluation, Experimental Setup); none of those are
available here, so random-init models of the same *shapes* and uniform random
prompts stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Tuple

import numpy as np


@dataclass(frozen=True)
class ModelConfig:
    arch: str            # "gpt2" (LayerNorm, bias, GELU, learned positions) | "llama" (RMSNorm, RoPE, GQA, SwiGLU)
    dtype: str           # "f32" | "bf16": storage type of matrices and embeddings
    n_layer: int
    d_model: int
    n_head: int
    n_kv_head: int
    d_ff: int
    vocab: int           # output classes; the drafter's mask token has id == vocab
    n_ctx: int
    bidirectional: bool  # True: diffusion drafter (non-causal, mask row, timestep embedding)
    norm_eps: float = 1e-5
    rope_theta: float = 500000.0

    @property
    def d_head(self) -> int:
        return self.d_model // self.n_head

    @property
    def d_kv(self) -> int:
        return self.n_kv_head * self.d_head

    @property
    def vocab_pad(self) -> int:
        """Leading dimension of logit / probability rows and row count of the stored LM head."""
        return (self.vocab + 255) // 256 * 256


def gpt2_shape(dtype, n_layer, d, heads, d_ff, vocab, n_ctx, bidirectional):
    return ModelConfig("gpt2", dtype, n_layer, d, heads, heads, d_ff, vocab, n_ctx, bidirectional)


# The five workloads.  (target, drafter, prefix_len, gamma, T, batch)
def workload(name: str):
    if name == "tiny":          # 2-layer d=128 fp32 pair, vocab 512 + mask
        t = gpt2_shape("f32", 2, 128, 4, 512, 512, 1024, False)
        d = gpt2_shape("f32", 2, 128, 4, 512, 512, 1024, True)
        return dict(target=t, drafter=d, prefix_len=32, gamma=8, T=4, batch=1)
    if name == "gpt2s":         # GPT-2-small-shaped pair, bf16
        t = gpt2_shape("bf16", 12, 768, 12, 3072, 50257, 1024, False)
        d = gpt2_shape("bf16", 12, 768, 12, 3072, 50257, 1024, True)
        return dict(target=t, drafter=d, prefix_len=256, gamma=16, T=8, batch=1)
    if name == "gpt2xl":        # GPT-2-XL-shaped target, small drafter
        t = gpt2_shape("bf16", 48, 1600, 25, 6400, 50257, 1024, False)
        d = gpt2_shape("bf16", 12, 768, 12, 3072, 50257, 1024, True)
        return dict(target=t, drafter=d, prefix_len=512, gamma=16, T=8, batch=1)
    if name == "gpt2xl_b16":    # batched, ragged prefixes U[128,768]
        w = workload("gpt2xl")
        w.update(batch=16, prefix_len=(128, 768), gamma=16, T=4)
        return w
    if name == "llama8b":       # Llama-3-8B-shaped target
        t = ModelConfig("llama", "bf16", 32, 4096, 32, 8, 14336, 128256, 2048, False)
        d = gpt2_shape("bf16", 12, 768, 12, 3072, 128256, 2048, True)
        return dict(target=t, drafter=d, prefix_len=1024, gamma=32, T=8, batch=1)
    if name == "llama8b_b8":    # the same pair, eight sequences
        w = workload("llama8b")
        w.update(batch=8)
        return w
    raise KeyError(name)


def shrink(cfg: ModelConfig, **kw) -> ModelConfig:
    """Same architecture with some dimensions replaced (layer cuts, small vocab for tests)."""
    return replace(cfg, **kw)


# --------------------------------------------------------------------------
# Parameter inventory.  Order is the storage order of the flat weight buffer.
# role: "embed"/"matrix" are stored in cfg.dtype; "gain"/"bias" always fp32.
# --------------------------------------------------------------------------
def weight_specs(cfg: ModelConfig) -> List[Tuple[str, Tuple[int, ...], str]]:
    d, F = cfg.d_model, cfg.d_ff
    specs: List[Tuple[str, Tuple[int, ...], str]] = []
    n_embed_rows = cfg.vocab + (1 if cfg.bidirectional else 0)
    specs.append(("wte", (n_embed_rows, d), "embed"))
    if cfg.arch == "gpt2":
        specs.append(("wpe", (cfg.n_ctx, d), "embed"))
    if cfg.bidirectional:
        specs += [("t_w1", (d, d), "matrix"), ("t_b1", (d,), "bias"),
                  ("t_w2", (d, d), "matrix"), ("t_b2", (d,), "bias")]
    for i in range(cfg.n_layer):
        p = f"l{i}."
        if cfg.arch == "gpt2":
            specs += [(p + "ln1_g", (d,), "gain"), (p + "ln1_b", (d,), "bias"),
                      (p + "w_qkv", (d + 2 * cfg.d_kv, d), "matrix"), (p + "b_qkv", (d + 2 * cfg.d_kv,), "bias"),
                      (p + "w_o", (d, d), "matrix"), (p + "b_o", (d,), "bias"),
                      (p + "ln2_g", (d,), "gain"), (p + "ln2_b", (d,), "bias"),
                      (p + "w_fc", (F, d), "matrix"), (p + "b_fc", (F,), "bias"),
                      (p + "w_proj", (d, F), "matrix"), (p + "b_proj", (d,), "bias")]
        else:
            specs += [(p + "ln1_g", (d,), "gain"),
                      (p + "w_qkv", (d + 2 * cfg.d_kv, d), "matrix"),
                      (p + "w_o", (d, d), "matrix"),
                      (p + "ln2_g", (d,), "gain"),
                      (p + "w_gate", (F, d), "matrix"),
                      (p + "w_up", (F, d), "matrix"),
                      (p + "w_proj", (d, F), "matrix")]
    specs.append(("lnf_g", (d,), "gain"))
    if cfg.arch == "gpt2":
        specs.append(("lnf_b", (d,), "bias"))
    specs.append(("w_head", (cfg.vocab, d), "matrix"))
    return specs


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """fp32 array -> nearest bf16 value (ties to even), returned as fp32.  (Finite inputs well below
    the largest fp32: the rounding increment is added in 32-bit arithmetic.)"""
    u = np.array(x, dtype=np.float32, order="C", copy=True).view(np.uint32)
    bias = (u >> np.uint32(16)) & np.uint32(1)
    bias += np.uint32(0x7FFF)
    u += bias
    u &= np.uint32(0xFFFF0000)
    return u.view(np.float32).reshape(np.shape(x))


def gen_tensor(cfg: ModelConfig, seed: int, index: int, shape, role: str) -> np.ndarray:
    """One parameter tensor.  Matrices, embeddings and biases ~ N(0, 0.02^2); norm gains
    1 + N(0, 0.02^2).  Values of "embed"/"matrix" tensors are rounded to the storage type so
    that every consumer sees exactly the stored numbers."""
    rng = np.random.Generator(np.random.Philox(seed=np.random.SeedSequence([int(seed), int(index)])))
    w = rng.standard_normal(size=shape, dtype=np.float32) * np.float32(0.02)
    if role == "gain":
        w = w + np.float32(1.0)
    if role in ("embed", "matrix") and cfg.dtype == "bf16":
        w = round_to_bf16(w)
    return w


def gen_weights(cfg: ModelConfig, seed: int, threads: int = 1) -> Dict[str, np.ndarray]:
    """All parameter tensors of a model.  Every tensor has a generator of its own (seed, tensor index), so the
    values do not depend on `threads` (numpy's generators release the interpreter lock while they fill)."""
    specs = list(enumerate(weight_specs(cfg)))
    if threads <= 1:
        return {name: gen_tensor(cfg, seed, i, shape, role) for i, (name, shape, role) in specs}
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=threads) as ex:
        vals = list(ex.map(lambda it: gen_tensor(cfg, seed, it[0], it[1][1], it[1][2]), specs))
    return {name: v for (_, (name, _, _)), v in zip(specs, vals)}


def gen_prefix(vocab: int, length: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed=np.random.SeedSequence([int(seed), 0x70726566])))
    return rng.integers(0, vocab, size=length, dtype=np.int32)


def gen_prefix_lengths(batch: int, lo: int, hi: int, seed: int) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(seed=np.random.SeedSequence([int(seed), 0x6C656E73])))
    return rng.integers(lo, hi + 1, size=batch, dtype=np.int32)


def gen_prob_rows(rows: int, vocab: int, seed: int, sharp: float = 1.0) -> np.ndarray:
    """Random logits rows (fp32) for kernel-level tests of sampling and acceptance."""
    rng = np.random.Generator(np.random.Philox(seed=np.random.SeedSequence([int(seed), 0x726F7773])))
    return (rng.standard_normal(size=(rows, vocab), dtype=np.float32) * np.float32(sharp))
