"""Seeded synthetic inputs for the Spark-FFN decode path.

This module holds input recipes only -- shapes, distributions, seeds, storage rounding --
and none of the method's arithmetic.  It is the one module that both the CPU oracle's
tests and the HIP path's tests / benchmark draw from, so that both sides see byte-identical
arrays.

Recipes (the paper measured on trained weights and real prompts, which are not available;
only its shapes and the Gaussian-at-initialisation distribution of Section 4 / Fig.3 are
reproduced):
  * FFN weights: i.i.d. N(0, 1/d_model), stored neuron-major, rounded once (RNE) to the
    storage dtype; layer l of a stack uses seed ``base_seed + l``.
  * token vectors: i.i.d. N(0, 1), rounded once to the activation dtype.
  * top-k rows (training / prefill shape): row i ~ N(mu_i, sigma_i^2) with
    mu_i ~ U(-1, 1), sigma_i ~ U(0.5, 2); each entry is replaced with probability 0.01 by
    mu_i + sigma_i * t, t ~ Student-t with 3 degrees of freedom (heavy-tailed outliers).
"""
from __future__ import annotations

from dataclasses import dataclass

import torch


@dataclass(frozen=True)
class FFNShape:
    name: str
    d_model: int
    d_ff: int
    r: int
    k: int

    @property
    def r2(self) -> int:
        return self.d_model - self.r

    def weight_elems(self) -> int:
        return self.d_ff * (2 * self.d_model)


TINY = FFNShape("tiny", 256, 1024, 128, 82)
GEMMA2_2B = FFNShape("gemma2-2b", 2304, 9216, 1024, 737)
GEMMA2_9B = FFNShape("gemma2-9b", 3584, 14336, 1536, 1147)
# The layer the paper itself trains (Section 4: d_ff = 13824, k = 1106, r = 1024).
PAPER_2B = FFNShape("spark-paper-2b", 2304, 13824, 1024, 1106)
# A deliberately awkward shape for ragged-tail coverage (nothing divides anything).
RAGGED = FFNShape("ragged", 328, 1000, 136, 77)

SHAPES = {s.name: s for s in (TINY, GEMMA2_2B, GEMMA2_9B, PAPER_2B, RAGGED)}


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def ffn_layer(shape: FFNShape, seed: int, dtype=torch.bfloat16, device="cpu"):
    """Neuron-major weights (K1n[d_ff, r], K2n[d_ff, d_model-r], Vn[d_ff, d_model])."""
    g = _gen(seed, device)
    scale = float(shape.d_model) ** -0.5

    def draw(cols):
        w = torch.randn(shape.d_ff, cols, generator=g, device=device, dtype=torch.float32)
        return (w * scale).to(dtype).contiguous()

    return draw(shape.r), draw(shape.r2), draw(shape.d_model)


def ffn_stack(shape: FFNShape, n_layers: int, base_seed: int = 1000, dtype=torch.bfloat16,
              device="cpu"):
    return [ffn_layer(shape, base_seed + l, dtype, device) for l in range(n_layers)]


def tokens(shape: FFNShape, batch: int, seed: int, dtype=torch.bfloat16, device="cpu"):
    """q[batch, d_model] ~ N(0, 1), rounded once to ``dtype``."""
    g = _gen(seed, device)
    q = torch.randn(batch, shape.d_model, generator=g, device=device, dtype=torch.float32)
    return q.to(dtype).contiguous()


def attn_caches(n_ctx: int, d_attn: int, r: int, seed: int, dtype=torch.bfloat16, device="cpu"):
    """Token-major caches of one key / value head: k1c[n_ctx, r], k2c[n_ctx, d_attn - r] with
    keys ~ N(0, 1 / d_attn), vc[n_ctx, d_attn] ~ N(0, 1), each rounded once to ``dtype``."""
    g = _gen(seed, device)
    scale = float(d_attn) ** -0.5

    def draw(cols, sc):
        w = torch.randn(n_ctx, cols, generator=g, device=device, dtype=torch.float32)
        return (w * sc).to(dtype).contiguous()

    return draw(r, scale), draw(d_attn - r, scale), draw(d_attn, 1.0)


def attn_queries(n_heads: int, group: int, d_attn: int, seed: int, dtype=torch.bfloat16, device="cpu"):
    """q[n_heads, group, d_attn] ~ N(0, 1), rounded once to ``dtype``."""
    g = _gen(seed, device)
    q = torch.randn(n_heads, group, d_attn, generator=g, device=device, dtype=torch.float32)
    return q.to(dtype).contiguous()


def topk_rows(rows: int, n: int, seed: int = 4242, dtype=torch.float32, device="cpu",
              outlier_prob: float = 0.01, chunk: int = 1024):
    """Activation matrix for the standalone row-wise statistical top-k."""
    g = _gen(seed, device)
    mu = torch.rand(rows, 1, generator=g, device=device) * 2.0 - 1.0
    sigma = torch.rand(rows, 1, generator=g, device=device) * 1.5 + 0.5
    out = torch.empty(rows, n, dtype=dtype, device=device)
    for lo in range(0, rows, chunk):
        hi = min(rows, lo + chunk)
        m = hi - lo
        z = torch.randn(m, n, generator=g, device=device)
        if outlier_prob > 0:
            pick = torch.rand(m, n, generator=g, device=device) < outlier_prob
            num = torch.randn(m, n, generator=g, device=device)
            chi = torch.randn(m, n, 3, generator=g, device=device).square_().sum(-1)
            t3 = num / torch.sqrt(chi / 3.0)
            z = torch.where(pick, t3, z)
        out[lo:hi] = (mu[lo:hi] + sigma[lo:hi] * z).to(dtype)
    return out


def grad_rows(rows: int, n: int, seed: int = 5151, dtype=torch.float32, device="cpu"):
    """Upstream gradient for the backward pass of the row-wise top-k: i.i.d. N(0, 1), rounded once."""
    g = _gen(seed, device)
    return torch.randn(rows, n, generator=g, device=device, dtype=torch.float32).to(dtype).contiguous()


def quantize_rows_fp8(w: torch.Tensor):
    """Per-row symmetric quantisation of a weight matrix to OCP E4M3 codes: ``scale = max|row| / 448``
    rounded to 8 significant bits (bf16), ``code = round_to_nearest_even(w / scale)``.  Returns
    (codes uint8 [rows, cols], scales float32 [rows]) on the device of ``w``; an input generator."""
    w = w.detach().to(torch.float32)
    amax = w.abs().amax(dim=1)
    scale = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
    scale = scale.to(torch.bfloat16).to(torch.float32)
    # a scale rounded down would push the row's largest entry past 448: step it up one bf16 ulp
    low = scale * 448.0 < amax
    scale = torch.where(low, (scale.to(torch.bfloat16).view(torch.int16) + 1).view(torch.bfloat16).to(torch.float32), scale)
    codes = (w / scale[:, None]).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
    return codes.contiguous(), scale.contiguous()


def quantize_rows_int8(w: torch.Tensor):
    """Per-row symmetric quantisation to signed 8-bit codes: ``scale = max|row| / 127`` rounded up to 8
    significant bits (bf16), ``code = round_to_nearest_even(w / scale)`` in -127..127.  Returns (codes
    as uint8 bytes [rows, cols], scales float32 [rows]) on the device of ``w``; an input generator."""
    w = w.detach().to(torch.float32)
    amax = w.abs().amax(dim=1)
    scale = torch.where(amax > 0, amax / 127.0, torch.ones_like(amax))
    scale = scale.to(torch.bfloat16).to(torch.float32)
    low = scale * 127.0 < amax
    scale = torch.where(low, (scale.to(torch.bfloat16).view(torch.int16) + 1).view(torch.bfloat16).to(torch.float32), scale)
    codes = torch.round(w / scale[:, None]).clamp(-127, 127).to(torch.int8).view(torch.uint8)
    return codes.contiguous(), scale.contiguous()


def to_oracle(t: torch.Tensor):
    """Exact float32 view of a stored tensor for the CPU oracle (bf16 -> fp32 is exact)."""
    return t.detach().to("cpu").to(torch.float32).numpy()
