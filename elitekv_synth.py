"""Seeded synthetic inputs for the EliteKV decode hot path.

This module only draws random arrays of the right shapes and scales.  It holds
none of the method's arithmetic (no projection, no rotation, no attention), so
that the CPU oracle and the HIP path can both be fed from it without sharing
any code of the method itself.

Workload recipe (LLaMA2-shaped, Section 4.1 of the paper names LLaMA2-7B and
LLaMA2-13B as the models; the (r, d_c) pairs follow the cache-size formula of
Section 3.2 "J-LRD": 2*r*n_h + d_c elements per token per layer):

  x            ~ N(0, 1)            [T, d]         token hidden states
  W_ke, W_dkv  ~ N(0, 1/d)          [d, n_h, 2r], [d, d_c]
  W_uk, W_uv   ~ N(0, 1/d_c)        [d_c, n_h, d_h-2r], [d_c, n_h, d_h]
  q            ~ N(0, 1)            [B, n_h, d_h]  (the q projection is off-path)
  I_h          = r distinct chunk indices in [0, d_h/2) per head, unsorted

With these variances the latent c = x W_dkv, the elite keys and the
reconstructed key dims are all ~N(0,1) per element and the logits
q.k/sqrt(d_h) are ~N(0,1): the softmax is neither flat nor one-hot.

All draws are float64 from numpy's PCG64 and are cast to the I/O dtype exactly
once by the caller; the same cast arrays go to the GPU and (upcast) to the
oracle.
"""
from __future__ import annotations

from dataclasses import dataclass, asdict

import numpy as np

SEED_BASE = 1586 * 10


@dataclass(frozen=True)
class Config:
    """One workload: model dims, batch, context and I/O dtype name."""
    name: str
    index: int          # position in the benchmark's config list (seed offset)
    d_model: int
    n_heads: int
    head_dim: int
    r: int              # elite chunks per head
    d_c: int            # joint latent rank
    batch: int
    context: int        # cached tokens per batch row that the query attends to
    dtype: str          # "fp32" or "bf16"
    rope_base: float = 10000.0
    prefill: int = 0    # tokens of one prefill-append call (config 4)
    d_ck: int = 0       # separated latents (S-LRD): d_c = d_ck + d_cv, the first d_ck columns are c^k; 0 = joint

    def as_dict(self):
        return asdict(self)


# configs[k] of the benchmark definition, k = 0..4
CONFIGS = {
    "tiny_fp32": Config("tiny_fp32", 0, 128, 4, 32, 2, 64, 1, 129, "fp32"),
    "7b_25_b8_s4096": Config("7b_25_b8_s4096", 1, 4096, 32, 128, 8, 1536, 8, 4096, "bf16"),
    "7b_25_b1_s32768": Config("7b_25_b1_s32768", 2, 4096, 32, 128, 8, 1536, 1, 32768, "bf16"),
    "13b_25_b16_s8192": Config("13b_25_b16_s8192", 3, 5120, 40, 128, 8, 1920, 16, 8192, "bf16"),
    "7b_12_b64_s2048": Config("7b_12_b64_s2048", 4, 4096, 32, 128, 4, 768, 64, 2048, "bf16",
                              prefill=2048),
    # the separated low-rank variant at the same cache size as configs 2 and 1 (the paper prints no
    # (d_ck, d_cv); these give the value side the larger share / an even split)
    "7b_25_slrd_b1_s32768": Config("7b_25_slrd_b1_s32768", 5, 4096, 32, 128, 8, 1536, 1, 32768, "bf16", d_ck=576),
    "7b_25_slrd_b8_s4096": Config("7b_25_slrd_b8_s4096", 6, 4096, 32, 128, 8, 1536, 8, 4096, "bf16", d_ck=768),
}


def rng_for(cfg_index: int, stream: int = 0) -> np.random.Generator:
    """PCG64 generator for config `cfg_index`; `stream` separates independent uses."""
    return np.random.Generator(np.random.PCG64([SEED_BASE + cfg_index, stream]))


def draw_elite_idx(rng, n_heads: int, head_dim: int, r: int) -> np.ndarray:
    """[n_h, r] int32: r distinct chunk indices per head, in random (unsorted) order."""
    out = np.empty((n_heads, r), dtype=np.int32)
    for h in range(n_heads):
        out[h] = rng.choice(head_dim // 2, size=r, replace=False)
    return out


def draw_weights(rng, d_model, n_heads, head_dim, r, d_c):
    """The four weight blocks of the J-LRD parameterisation, float64, natural layouts."""
    W_ke = rng.standard_normal((d_model, n_heads, 2 * r)) / np.sqrt(d_model)
    W_dkv = rng.standard_normal((d_model, d_c)) / np.sqrt(d_model)
    W_uk = rng.standard_normal((d_c, n_heads, head_dim - 2 * r)) / np.sqrt(d_c)
    W_uv = rng.standard_normal((d_c, n_heads, head_dim)) / np.sqrt(d_c)
    return W_ke, W_dkv, W_uk, W_uv


def draw_hidden(rng, tokens: int, d_model: int) -> np.ndarray:
    return rng.standard_normal((tokens, d_model))


def draw_query(rng, batch: int, n_heads: int, head_dim: int) -> np.ndarray:
    return rng.standard_normal((batch, n_heads, head_dim))


def draw_cache_planes(rng, rows: int, n_heads: int, r: int, d_c: int):
    """Timing-only fill: N(0,1) elite-key and latent planes.

    A rotation leaves an isotropic Gaussian isotropic, so these have the same
    distribution as planes produced by a real append under the recipe above.
    """
    ke = rng.standard_normal((rows, n_heads, 2 * r))
    c = rng.standard_normal((rows, d_c))
    return ke, c


def problem(cfg: Config, tokens: int | None = None, batch: int | None = None):
    """All host-side inputs of one config as a dict of float64 / int arrays.

    `tokens` hidden states are drawn for ONE batch row's context (default
    cfg.context); callers that need several rows draw again with another stream.
    """
    rng = rng_for(cfg.index)
    B = cfg.batch if batch is None else batch
    T = cfg.context if tokens is None else tokens
    idx = draw_elite_idx(rng, cfg.n_heads, cfg.head_dim, cfg.r)
    W_ke, W_dkv, W_uk, W_uv = draw_weights(rng, cfg.d_model, cfg.n_heads, cfg.head_dim,
                                           cfg.r, cfg.d_c)
    q = draw_query(rng, B, cfg.n_heads, cfg.head_dim)
    x = draw_hidden(rng, T, cfg.d_model)
    return dict(elite_idx=idx, W_ke=W_ke, W_dkv=W_dkv, W_uk=W_uk, W_uv=W_uv, q=q, x=x)
