"""Seeded synthetic inputs for the Fleet decode step.

Data only: shapes, seeds, distributions and the bf16 storage format.  None of
the method's arithmetic lives here.  Both the HIP path and the CPU oracle are
fed from these generators (the HIP path gets device tensors, the oracle gets
host ``uint16`` views of the same values).

Recipe (stands in for the trained Qwen3-8B weights and the 64-in/1024-out
generation workload of the paper's evaluation, which are not available):
  * weight matrices  ~ N(0, 0.02), rounded to bf16
  * norm gains       = bf16(1 + N(0, 0.02))  (ln1, ln2, q_norm, k_norm, final)
  * input hidden     ~ N(0, 1), bf16
  * KV cache         ~ N(0, 1), bf16, filled for every slot below max_seq
  * positions        fixed, or uniform integers in [lo, hi]
Matrices are [out_features, in_features] row-major.
"""
from __future__ import annotations

import dataclasses

import numpy as np
import torch


@dataclasses.dataclass(frozen=True)
class Shape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    max_batch: int
    max_seq: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e6

    def asdict(self) -> dict:
        return dataclasses.asdict(self)

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim


def reduced_shape(max_batch: int = 1, max_seq: int = 129, n_layers: int = 1,
                  vocab: int = 0) -> Shape:
    """One reduced Qwen3-style layer: hidden 1024, 8 Q / 2 KV heads x 128, FFN 3072."""
    return Shape(n_layers, 1024, 8, 2, 128, 3072, vocab, max_batch, max_seq)


def qwen3_8b_shape(max_batch: int, max_seq: int, n_layers: int = 36,
                   vocab: int = 151936) -> Shape:
    """Qwen3-8B: hidden 4096, 32 Q / 8 KV heads x 128, FFN 12288, 36 layers."""
    return Shape(n_layers, 4096, 32, 8, 128, 12288, vocab, max_batch, max_seq)


class Gen:
    """Seeded tensor source on one device (``cpu`` or ``cuda``)."""

    def __init__(self, seed: int, device: str = "cpu"):
        self.device = torch.device(device)
        self.g = torch.Generator(device=self.device)
        self.g.manual_seed(seed)

    def normal_bf16(self, shape, std: float, mean: float = 0.0) -> torch.Tensor:
        """bf16(mean + N(0, std)), generated in fp32 chunks to bound memory."""
        out = torch.empty(shape, dtype=torch.bfloat16, device=self.device)
        flat = out.view(-1)
        step = 1 << 26
        for s in range(0, flat.numel(), step):
            e = min(flat.numel(), s + step)
            t = torch.randn(e - s, generator=self.g, device=self.device, dtype=torch.float32)
            flat[s:e] = (t * std + mean).to(torch.bfloat16)
        return out

    def randint(self, lo: int, hi: int, n: int) -> torch.Tensor:
        """n integers uniform in [lo, hi], int32."""
        return torch.randint(lo, hi + 1, (n,), generator=self.g, device=self.device,
                             dtype=torch.int32)


PER_LAYER = ("ln1", "wqkv", "q_norm", "k_norm", "wo", "ln2", "wgu", "wdown")


def make_weights(shape: Shape, gen: Gen, with_embed: bool = False) -> dict:
    """Random-init weights of the given architecture (dict of bf16 tensors)."""
    H, hd, F = shape.hidden, shape.head_dim, shape.ffn
    w = {k: [] for k in PER_LAYER}
    for _ in range(shape.n_layers):
        w["ln1"].append(gen.normal_bf16((H,), 0.02, 1.0))
        w["wqkv"].append(gen.normal_bf16((shape.qkv_rows, H), 0.02))
        w["q_norm"].append(gen.normal_bf16((hd,), 0.02, 1.0))
        w["k_norm"].append(gen.normal_bf16((hd,), 0.02, 1.0))
        w["wo"].append(gen.normal_bf16((H, shape.q_dim), 0.02))
        w["ln2"].append(gen.normal_bf16((H,), 0.02, 1.0))
        w["wgu"].append(gen.normal_bf16((2 * F, H), 0.02))
        w["wdown"].append(gen.normal_bf16((H, F), 0.02))
    if shape.vocab > 0:
        w["final_norm"] = gen.normal_bf16((H,), 0.02, 1.0)
        w["lm_head"] = gen.normal_bf16((shape.vocab, H), 0.02)
        if with_embed:
            # unit scale, like the hidden states that enter a step otherwise: with rows of
            # N(0, 0.02) the residual stream of a two-layer model is all branch output, and the
            # oracle's own result moves by up to 0.015 x RMS when only its fp32 summation order
            # is reversed -- no room under a 2e-2 x RMS bar for a second implementation
            w["embed"] = gen.normal_bf16((shape.vocab, H), 1.0)
    return w


def make_hidden(shape: Shape, batch: int, gen: Gen) -> torch.Tensor:
    return gen.normal_bf16((batch, shape.hidden), 1.0)


def make_kv_cache(shape: Shape, gen: Gen):
    """(k_cache, v_cache), bf16 [n_layers, max_batch, n_kv, max_seq, head_dim] ~ N(0,1)."""
    dims = (shape.n_layers, shape.max_batch, shape.n_kv_heads, shape.max_seq, shape.head_dim)
    return gen.normal_bf16(dims, 1.0), gen.normal_bf16(dims, 1.0)


def to_host_u16(t: torch.Tensor) -> np.ndarray:
    """Host uint16 view (bf16 bit patterns) of a bf16 tensor."""
    assert t.dtype == torch.bfloat16
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def weights_to_host(w: dict) -> dict:
    out = {}
    for k, v in w.items():
        out[k] = [to_host_u16(a) for a in v] if isinstance(v, list) else to_host_u16(v)
    return out


def bf16_bits_to_f32(u16: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to fp32 (format conversion only)."""
    return (u16.astype(np.uint32) << 16).view(np.float32)
