"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module holds model *shapes* and random-number recipes only: no norm, no
attention, no mask, no sampling arithmetic lives here.  Both sides receive the
very same bytes (weights, prompts, K/V fills) and compute on them separately.

Shapes follow the backbones the paper continues pre-training from (Setup,
"Model initialization"): Qwen2.5-1.5B-like and Qwen3-8B-like decoders, plus a
tiny model the oracle finishes in seconds.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import torch


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    tied_embeddings: bool
    rope_base: float = 10000.0
    rms_eps: float = 1e-6

    @property
    def mask_token_id(self) -> int:
        # The paper does not say which id the mask token has; the last id of
        # the vocabulary is reserved for it and prompts never contain it.
        return self.vocab - 1

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def with_layers(self, n_layers: int) -> "ModelShape":
        return replace(self, n_layers=n_layers, name=f"{self.name}-{n_layers}L")


TINY = ModelShape("tiny", 2, 128, 4, 4, 32, 512, 512, False)
# A second small shape with grouped-query attention and head_dim 128 so that
# the bf16 MFMA kernels (which need head_dim 128) can be checked end to end
# against the oracle in seconds.
SMALL_GQA = ModelShape("small-gqa", 2, 256, 4, 2, 128, 512, 2048, False)
SHAPE_1P5B = ModelShape("1.5b-shape", 28, 1536, 12, 2, 128, 8960, 151936, True)
SHAPE_8B = ModelShape("8b-shape", 36, 4096, 32, 8, 128, 12288, 151936, False)

SHAPES = {s.name: s for s in (TINY, SMALL_GQA, SHAPE_1P5B, SHAPE_8B)}


def _gen(seed: int, device: str = "cpu") -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def make_weights(shape: ModelShape, seed: int, dtype: torch.dtype = torch.float32,
                 device: str = "cpu", std: float = 0.02) -> Dict[str, object]:
    """Random-init weights: every matrix ~ N(0, std^2), norm gains = 1.

    Matrices are [out_features, in_features] row-major.  With ``dtype=bfloat16``
    the values are drawn in fp32 and rounded once; both sides then hold the
    same bf16 values.  The draw order is fixed (embed, lm_head, then per layer
    wq, wk, wv, wo, w_gate, w_up, w_down), so a given (shape, seed, device
    kind) always yields the same bytes.
    """
    g = _gen(seed, device)

    def mat(rows: int, cols: int) -> torch.Tensor:
        w = torch.empty(rows, cols, dtype=torch.float32, device=device)
        w.normal_(0.0, std, generator=g)
        return w.to(dtype)

    d = shape.d_model
    w: Dict[str, object] = {}
    w["embed"] = mat(shape.vocab, d)
    w["lm_head"] = None if shape.tied_embeddings else mat(shape.vocab, d)
    w["final_norm"] = torch.ones(d, dtype=dtype, device=device)
    layers: List[Dict[str, torch.Tensor]] = []
    for _ in range(shape.n_layers):
        layers.append({
            "attn_norm": torch.ones(d, dtype=dtype, device=device),
            "wq": mat(shape.q_dim, d),
            "wk": mat(shape.kv_dim, d),
            "wv": mat(shape.kv_dim, d),
            "wo": mat(d, shape.q_dim),
            "ffn_norm": torch.ones(d, dtype=dtype, device=device),
            "w_gate": mat(shape.d_ff, d),
            "w_up": mat(shape.d_ff, d),
            "w_down": mat(d, shape.d_ff),
        })
    w["layers"] = layers
    return w


def weights_to(w: Dict[str, object], dtype: Optional[torch.dtype] = None,
               device: Optional[str] = None) -> Dict[str, object]:
    """Copy a weight dictionary to another dtype/device (values unchanged when widening)."""
    def cv(t):
        if t is None:
            return None
        return t.to(device=device if device is not None else t.device,
                    dtype=dtype if dtype is not None else t.dtype)
    out = {k: cv(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: cv(v) for k, v in lw.items()} for lw in w["layers"]]
    return out


def make_prompt(shape: ModelShape, length: int, seed: int, batch: int = 1) -> torch.Tensor:
    """Uniform random token ids in [0, vocab-2] (the mask id never appears), int32 [batch, length]."""
    g = _gen(seed)
    return torch.randint(0, shape.vocab - 1, (batch, length), generator=g, dtype=torch.int64).to(torch.int32)


def make_drafts(shape: ModelShape, k: int, seed: int, batch: int = 1) -> torch.Tensor:
    """Arbitrary draft tokens, int32 [batch, k]."""
    g = _gen(seed)
    return torch.randint(0, shape.vocab - 1, (batch, k), generator=g, dtype=torch.int64).to(torch.int32)


def make_normal(size, seed: int, dtype: torch.dtype = torch.float32, std: float = 1.0) -> torch.Tensor:
    """N(0, std^2) tensor drawn in fp32 on the CPU and rounded once to ``dtype``."""
    g = _gen(seed)
    t = torch.empty(*size, dtype=torch.float32)
    t.normal_(0.0, std, generator=g)
    return t.to(dtype)


def make_acceptance_lengths(k: int, steps: int, mean: float, seed: int) -> torch.Tensor:
    """Seeded per-step acceptance lengths in [1, k] whose average is close to ``mean``.

    Stands in for the tokens-per-forward mix a trained model shows (the paper's
    Table 2 reports the averages); lengths are binomial around the mean so that
    short and long acceptances both occur.
    """
    g = _gen(seed)
    p = (mean - 1.0) / max(k - 1, 1)
    draws = (torch.rand(steps, k - 1, generator=g) < p).sum(dim=1) + 1
    return draws.to(torch.int32)


def shuffled_page_table(n_pages_needed: int, n_pages_total: int, seed: int) -> torch.Tensor:
    """A random injective map logical page -> physical page, int32 [n_pages_needed]."""
    g = _gen(seed)
    perm = torch.randperm(n_pages_total, generator=g)[:n_pages_needed]
    return perm.to(torch.int32)
