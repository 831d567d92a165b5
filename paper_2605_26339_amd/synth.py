"""Seeded synthetic inputs for the QAM-W codec: weight matrices, activation RMS vectors
and the model-shaped weight sets the benchmark and the parity tests run on.

This module holds no arithmetic of the method.  It only draws random inputs with the
shapes and value distributions of the workloads:

  * W[i, j] = g[i, j] * rho[i],  g ~ N(0, 1),  rho[i] ~ LogNormal(0, row_sigma)
  * activation RMS a[j] ~ LogNormal(0, 1), floor(0.01 * d_in) channels (chosen without
    replacement) multiplied by 20

Host generation uses numpy's Philox counter-based generator, device generation a seeded
torch.Generator; a row generated on the device is read back by whoever needs it on the
host, it is never regenerated there.
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass

import numpy as np

# ------------------------------------------------------------------------------ shapes
# (name, d_out, d_in, activation site).  Matrices that read the same activations share
# one activation-RMS vector per layer.
_TINYLLAMA = [("q", 2048, 2048, "attn_in"), ("k", 256, 2048, "attn_in"), ("v", 256, 2048, "attn_in"),
              ("o", 2048, 2048, "o_in"), ("gate", 5632, 2048, "mlp_in"), ("up", 5632, 2048, "mlp_in"),
              ("down", 2048, 5632, "down_in")]
_LLAMA2_7B = [("q", 4096, 4096, "attn_in"), ("k", 4096, 4096, "attn_in"), ("v", 4096, 4096, "attn_in"),
              ("o", 4096, 4096, "o_in"), ("gate", 11008, 4096, "mlp_in"), ("up", 11008, 4096, "mlp_in"),
              ("down", 4096, 11008, "down_in")]
_LLAMA2_13B = [("q", 5120, 5120, "attn_in"), ("k", 5120, 5120, "attn_in"), ("v", 5120, 5120, "attn_in"),
               ("o", 5120, 5120, "o_in"), ("gate", 13824, 5120, "mlp_in"), ("up", 13824, 5120, "mlp_in"),
               ("down", 5120, 13824, "down_in")]


@dataclass(frozen=True)
class Workload:
    name: str
    config_id: int
    layers: int
    matrices: tuple          # per layer: (name, d_out, d_in, site)
    dtype: str               # "f32" or "bf16": storage type of W handed to encode
    bits: int
    block: int
    row_sigma: float
    alpha: float = 0.3

    @property
    def K(self) -> int:
        return 1 << self.bits

    def n_weights(self) -> int:
        return self.layers * sum(m[1] * m[2] for m in self.matrices)

    def n_pairs(self) -> int:
        return self.n_weights() // 2


WORKLOADS = {
    "c0_single_2048": Workload("c0_single_2048", 0, 1, (("q", 2048, 2048, "attn_in"),), "f32", 11, 128, 0.5),
    "c1_tinyllama_1.1b": Workload("c1_tinyllama_1.1b", 1, 22, tuple(_TINYLLAMA), "f32", 11, 128, 0.5),
    "c2_llama2_7b_b11": Workload("c2_llama2_7b_b11", 2, 32, tuple(_LLAMA2_7B), "bf16", 11, 128, 0.5),
    "c3_llama2_7b_b7": Workload("c3_llama2_7b_b7", 3, 32, tuple(_LLAMA2_7B), "bf16", 7, 256, 1.0),
    "c4_llama2_13b_b11": Workload("c4_llama2_13b_b11", 4, 40, tuple(_LLAMA2_13B), "bf16", 11, 128, 0.5),
}


def seed_for(config_id: int, layer: int, tag: str) -> int:
    """64-bit seed from (config, layer, tag) by SHA-256 of their text form."""
    h = hashlib.sha256(f"qamw-synth/{config_id}/{layer}/{tag}".encode()).digest()
    return int.from_bytes(h[:8], "little")


# ------------------------------------------------------------------------------ host side
def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed & (2**64 - 1)))


def weight_host(seed: int, d_out: int, d_in: int, row_sigma: float = 0.5) -> np.ndarray:
    """fp32 [d_out][d_in], Gaussian entries times a log-normal row scale."""
    rng = _rng(seed)
    rho = np.exp(rng.standard_normal(d_out) * row_sigma).astype(np.float32)
    g = rng.standard_normal((d_out, d_in), dtype=np.float32)
    return g * rho[:, None]


def act_rms_host(seed: int, d_in: int) -> np.ndarray:
    """fp32 [d_in] activation RMS with 1% outlier channels."""
    rng = _rng(seed)
    a = np.exp(rng.standard_normal(d_in))
    n_out = int(0.01 * d_in)
    if n_out > 0:
        pick = rng.choice(d_in, size=n_out, replace=False)
        a[pick] *= 20.0
    return a.astype(np.float32)


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round an fp32 array to bf16 storage (uint16 bit patterns) with torch's cast."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


# ------------------------------------------------------------------------------ device side
def weight_device(seed: int, d_out: int, d_in: int, row_sigma: float, dtype: str, device="cuda"):
    """Same distribution generated on the device with a seeded torch.Generator.
    dtype "f32" -> torch.float32, "bf16" -> torch.bfloat16 (rounded to nearest even)."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(seed & (2**63 - 1))
    rho = torch.exp(torch.randn(d_out, device=device, generator=gen) * row_sigma)
    w = torch.randn(d_out, d_in, device=device, generator=gen)
    w.mul_(rho[:, None])
    return w if dtype == "f32" else w.to(torch.bfloat16)
