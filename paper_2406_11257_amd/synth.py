"""Seeded synthetic checkpoints shaped like the models the paper compresses.

This module only draws random inputs; it holds none of the method's
arithmetic.  It serves the tests, the benchmark and the CPU oracle alike, so
that both sides always see the same bytes.  The real Pythia / PanGu
checkpoints of the paper's Sec. 4 are not available; these stand in for them.

Per tensor (fields drawn from independent streams):
    W_prev = fp32( N(0, 0.02^2) )
    W      = W_prev +fp32 fp32(noise),  noise ~ Laplace(0, b)  (or b * Student-t(3))
    m      = fp32( N(0, (5e-5)^2) )                         first Adam moment
    v      = fp32( m^2 * lognormal(0, 1) + 1e-16 )          second Adam moment
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 20240611
ALPHA, BETA, NBITS, LLOYD_ITERS = 5e-5, 2.0, 4, 10


@dataclass(frozen=True)
class TensorSpec:
    name: str
    n: int
    kind: str          # "embed", "norm", "attn", "mlp"


def gpt_neox_layout(d_model: int, layers: int, ffn: int, vocab: int) -> list[TensorSpec]:
    t = [TensorSpec("embed_in.weight", vocab * d_model, "embed")]
    for i in range(layers):
        p = f"layers.{i}."
        t += [
            TensorSpec(p + "input_layernorm.weight", d_model, "norm"),
            TensorSpec(p + "input_layernorm.bias", d_model, "norm"),
            TensorSpec(p + "post_attention_layernorm.weight", d_model, "norm"),
            TensorSpec(p + "post_attention_layernorm.bias", d_model, "norm"),
            TensorSpec(p + "attention.query_key_value.weight", 3 * d_model * d_model, "attn"),
            TensorSpec(p + "attention.query_key_value.bias", 3 * d_model, "attn"),
            TensorSpec(p + "attention.dense.weight", d_model * d_model, "attn"),
            TensorSpec(p + "attention.dense.bias", d_model, "attn"),
            TensorSpec(p + "mlp.dense_h_to_4h.weight", ffn * d_model, "mlp"),
            TensorSpec(p + "mlp.dense_h_to_4h.bias", ffn, "mlp"),
            TensorSpec(p + "mlp.dense_4h_to_h.weight", d_model * ffn, "mlp"),
            TensorSpec(p + "mlp.dense_4h_to_h.bias", d_model, "mlp"),
        ]
    t += [TensorSpec("final_layer_norm.weight", d_model, "norm"),
          TensorSpec("final_layer_norm.bias", d_model, "norm"),
          TensorSpec("embed_out.weight", vocab * d_model, "embed")]
    return t


def llama_layout(d_model: int, layers: int, ffn: int, vocab: int) -> list[TensorSpec]:
    t = [TensorSpec("embed_tokens.weight", vocab * d_model, "embed")]
    for i in range(layers):
        p = f"layers.{i}."
        t += [TensorSpec(p + f"self_attn.{x}_proj.weight", d_model * d_model, "attn")
              for x in ("q", "k", "v", "o")]
        t += [TensorSpec(p + "mlp.gate_proj.weight", ffn * d_model, "mlp"),
              TensorSpec(p + "mlp.up_proj.weight", ffn * d_model, "mlp"),
              TensorSpec(p + "mlp.down_proj.weight", d_model * ffn, "mlp"),
              TensorSpec(p + "input_layernorm.weight", d_model, "norm"),
              TensorSpec(p + "post_attention_layernorm.weight", d_model, "norm")]
    t += [TensorSpec("norm.weight", d_model, "norm"),
          TensorSpec("lm_head.weight", vocab * d_model, "embed")]
    return t


@dataclass(frozen=True)
class Config:
    cid: int
    name: str
    tensors: tuple

    @property
    def total(self) -> int:
        return sum(t.n for t in self.tensors)


def config(cid: int) -> Config:
    if cid == 0:
        return Config(0, "pythia-14m", tuple(gpt_neox_layout(128, 6, 512, 50304)))
    if cid in (1, 4):
        return Config(cid, "pythia-410m", tuple(gpt_neox_layout(1024, 24, 4096, 50304)))
    if cid == 2:
        return Config(2, "pythia-1.4b", tuple(gpt_neox_layout(2048, 24, 8192, 50304)))
    if cid == 3:
        return Config(3, "llama-7b", tuple(llama_layout(4096, 32, 11008, 32000)))
    raise ValueError(cid)


def noise_recipe(cid: int, idx: int, spec: TensorSpec) -> tuple[str, float]:
    """(distribution, scale) of the weight update for tensor ``idx``."""
    if cid == 1 and spec.kind in ("embed", "norm"):
        return "laplace", 3e-5
    if cid == 2 and idx % 5 == 0:
        return "student3", 1e-4
    return "laplace", 1e-4


def _rng(cid: int, step: int, idx: int, fld: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(
        np.random.SeedSequence([BASE_SEED, cid, step, idx, fld])))


def draw_noise(cid, step, idx, spec, n=None) -> np.ndarray:
    n = spec.n if n is None else n
    dist, scale = noise_recipe(cid, idx, spec)
    g = _rng(cid, step, idx, 1)
    if dist == "laplace":
        return g.laplace(0.0, scale, n).astype(np.float32)
    return (g.standard_t(3, n) * scale).astype(np.float32)


def draw_moments(cid, step, idx, spec, n=None):
    n = spec.n if n is None else n
    m = (_rng(cid, step, idx, 2).standard_normal(n) * 5e-5).astype(np.float32)
    ln = _rng(cid, step, idx, 3).lognormal(0.0, 1.0, n)
    v = (m.astype(np.float64) ** 2 * ln + 1e-16).astype(np.float32)
    return m, v


def draw_tensor(cid: int, idx: int, spec: TensorSpec, step: int = 0, n=None):
    """(W_prev, W, m, v) fp32 numpy arrays for one tensor of one step.
    ``n`` overrides the length (used to take a bounded sample of a huge tensor)."""
    n = spec.n if n is None else n
    Wp = (_rng(cid, step, idx, 0).standard_normal(n) * 0.02).astype(np.float32)
    W = (Wp + draw_noise(cid, step, idx, spec, n)).astype(np.float32)
    m, v = draw_moments(cid, step, idx, spec, n)
    return Wp, W, m, v


def torch_draw_tensor(cid: int, idx: int, spec: TensorSpec, device, step: int = 0):
    """Same recipe drawn with torch's generator on ``device`` (for checkpoints too
    large to draw on the host in reasonable time).  The values differ from
    ``draw_tensor``; whoever needs them on both sides copies them."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((BASE_SEED * 1000003 + cid * 10007 + step * 1009 + idx) & 0x7FFFFFFFFFFF)
    n = spec.n
    Wp = torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, 0.02, generator=g)
    dist, scale = noise_recipe(cid, idx, spec)
    u = torch.empty(n, dtype=torch.float32, device=device).uniform_(-0.5, 0.5, generator=g)
    if dist == "laplace":
        noise = -scale * torch.sign(u) * torch.log1p(-2.0 * u.abs().clamp_(max=0.49999997))
    else:   # Student-t(3) = N / sqrt(chi2_3 / 3)
        z = torch.empty(n, dtype=torch.float32, device=device).normal_(generator=g)
        chi = torch.zeros(n, dtype=torch.float32, device=device)
        for _ in range(3):
            chi += torch.empty(n, dtype=torch.float32, device=device).normal_(generator=g) ** 2
        noise = scale * z / torch.sqrt(chi.clamp_(min=1e-12) / 3.0)
        del z, chi
    W = Wp + noise
    del noise, u
    m = torch.empty(n, dtype=torch.float32, device=device).normal_(0.0, 5e-5, generator=g)
    ln = torch.empty(n, dtype=torch.float32, device=device).normal_(generator=g).exp_()
    v = m * m * ln + 1e-16
    del ln
    return Wp, W, m, v
