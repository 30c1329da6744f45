"""Correlated-Gaussian K/V activations, sampled codebooks and queries.

Recipe (stands in for LLaMA / Mistral K/V activations, which are not
available offline; it keeps the two properties of those activations that the
paper's Section 3.1 and Section 2.3 report: strong correlation between
neighbouring channels and a few large-magnitude key channels):

* ``x = A z + bias`` with ``z ~ N(0, I_D)``; ``A`` is block diagonal, every
  8x8 block being the Cholesky factor of ``0.3 I + 0.7 11^T`` (unit variance,
  pairwise correlation 0.7 inside a block, none across blocks).  Groups of
  8, 4 or 2 contiguous channels never straddle a block.
* ``bias ~ N(0, 1)`` per channel, drawn once per (config, layer, K or V).
* keys only: ``round(0.04 D)`` channels picked by a seeded permutation are
  multiplied by 10 after the bias is added.
* a codebook ``[G, 2^b, c]`` is the group-wise slicing of ``2^b`` fresh samples
  of the same recipe (same bias, same outlier channels): sampled, not learned.
* queries are i.i.d. ``N(0, 1)``.
* everything is rounded to fp16 once, on the host.

Seeds: ``numpy.random.SeedSequence([240503917, cfg_id, layer, stream])`` with
the stream ids listed in ``STREAMS``.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict

import numpy as np

ROOT_SEED = 240503917
BLOCK = 8
RHO = 0.7
OUTLIER_FRACTION = 0.04
OUTLIER_SCALE = 10.0

STREAMS = {
    "k_data": 0,
    "v_data": 1,
    "k_centroids": 2,
    "v_centroids": 3,
    "q": 4,
    "k_bias": 5,
    "v_bias": 6,
    "k_outliers": 7,
}


@dataclass(frozen=True)
class WorkloadConfig:
    cfg_id: int
    name: str
    c: int            # channels per coupled group
    b: int            # bits per code
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int      # cached tokens per sequence
    layers: int
    encode_tokens: int  # tokens per sequence handed to one cq_encode call

    @property
    def kv_channels(self) -> int:
        return self.n_kv_heads * self.head_dim

    @property
    def n_groups(self) -> int:
        return self.kv_channels // self.c

    @property
    def n_centroids(self) -> int:
        return 1 << self.b


CONFIGS: Dict[int, WorkloadConfig] = {
    1: WorkloadConfig(1, "CQ-8c8b/b1/ctx1024", 8, 8, 1, 32, 32, 128, 1024, 1, 1024),
    2: WorkloadConfig(2, "CQ-4c8b/b16/ctx4096/32layers", 4, 8, 16, 32, 32, 128, 4096, 32, 1),
    3: WorkloadConfig(3, "CQ-2c8b/b64/ctx8192", 2, 8, 64, 32, 32, 128, 8192, 1, 512),
    4: WorkloadConfig(4, "CQ-8c10b/gqa32:8/b32/ctx16384", 8, 10, 32, 32, 8, 128, 16384, 1, 1),
    5: WorkloadConfig(5, "CQ-8c8b/b4/ctx131072", 8, 8, 4, 32, 32, 128, 131072, 1, 32768),
}


def _rng(cfg_id: int, layer: int, stream: str, extra: int = 0) -> np.random.Generator:
    seq = np.random.SeedSequence([ROOT_SEED, cfg_id, layer, STREAMS[stream], extra])
    return np.random.default_rng(seq)


def mixing_block() -> np.ndarray:
    """Lower-triangular 8x8 factor L with L L^T = 0.3 I + 0.7 11^T."""
    cov = (1.0 - RHO) * np.eye(BLOCK) + RHO * np.ones((BLOCK, BLOCK))
    return np.linalg.cholesky(cov)


@dataclass(frozen=True)
class TensorRecipe:
    """Per (config, layer, K|V) constants of the generator."""
    cfg_id: int
    layer: int
    which: str              # "k" or "v"
    channels: int
    bias: np.ndarray        # [D] float64
    channel_scale: np.ndarray  # [D] float64: 10 on key outlier channels, else 1


def tensor_recipe(cfg_id: int, layer: int, which: str, channels: int) -> TensorRecipe:
    assert which in ("k", "v")
    assert channels % BLOCK == 0
    bias = _rng(cfg_id, layer, f"{which}_bias").standard_normal(channels)
    scale = np.ones(channels)
    if which == "k":
        n_out = int(round(OUTLIER_FRACTION * channels))
        perm = _rng(cfg_id, layer, "k_outliers").permutation(channels)
        scale[perm[:n_out]] = OUTLIER_SCALE
    return TensorRecipe(cfg_id, layer, which, channels, bias, scale)


def _draw(recipe: TensorRecipe, n: int, rng: np.random.Generator) -> np.ndarray:
    d = recipe.channels
    z = rng.standard_normal((n, d // BLOCK, BLOCK))
    x = z @ mixing_block().T            # row vectors: x_blk = L z_blk
    x = x.reshape(n, d) + recipe.bias
    x *= recipe.channel_scale
    return x


def sample_activations(recipe: TensorRecipe, n_tokens: int, chunk: int = 0) -> np.ndarray:
    """fp16 ``[n_tokens, D]``; ``chunk`` picks an independent stream (e.g. per sequence)."""
    rng = _rng(recipe.cfg_id, recipe.layer, f"{recipe.which}_data", chunk)
    return _draw(recipe, n_tokens, rng).astype(np.float16)


def sample_codebook(recipe: TensorRecipe, c: int, b: int) -> np.ndarray:
    """fp16 ``[G, 2^b, c]``: entry j of group g is channels [g c, g c + c) of sample j."""
    rng = _rng(recipe.cfg_id, recipe.layer, f"{recipe.which}_centroids")
    k = 1 << b
    s = _draw(recipe, k, rng)                       # [K, D]
    g = recipe.channels // c
    cb = s.reshape(k, g, c).transpose(1, 0, 2)      # [G, K, c]
    return np.ascontiguousarray(cb).astype(np.float16)


def sample_query(cfg_id: int, layer: int, batch: int, n_q_heads: int, head_dim: int) -> np.ndarray:
    rng = _rng(cfg_id, layer, "q")
    return rng.standard_normal((batch, n_q_heads, head_dim)).astype(np.float16)


def sample_activations_torch(recipe: TensorRecipe, n_tokens: int, seed: int, device):
    """Same recipe drawn on ``device`` with torch's generator (different stream,
    same distribution): for throughput runs whose inputs are too large to
    ship from the host.  Returns fp16 ``[n_tokens, D]``."""
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed((ROOT_SEED * 1000003 + recipe.cfg_id * 10007 + recipe.layer * 101 + seed) % (2**63 - 1))
    d = recipe.channels
    lmat = torch.tensor(mixing_block(), dtype=torch.float32, device=device)
    z = torch.randn((n_tokens, d // BLOCK, BLOCK), generator=gen, device=device, dtype=torch.float32)
    x = (z @ lmat.T).reshape(n_tokens, d)
    x += torch.tensor(recipe.bias, dtype=torch.float32, device=device)
    x *= torch.tensor(recipe.channel_scale, dtype=torch.float32, device=device)
    return x.to(torch.float16)
