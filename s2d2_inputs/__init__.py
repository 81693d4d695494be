"""Seeded synthetic inputs for the S2D2 draft+verify step.

This module serves both the CPU oracle and the HIP path with *data only*: model
shapes, random-init weights, prefix token ids, synthetic KV-cache contents,
page tables and synthetic logit pairs.  It contains none of the method's
arithmetic (no forward pass, no sampling rule, no acceptance rule) and imports
neither the oracle nor the HIP binding.

Everything is generated on the CPU with numpy's Philox bit generator keyed by
(seed, tensor name), so every tensor can be regenerated independently and
identically on any machine.  Tensors are returned as CPU torch tensors in the
storage dtype of the configuration (bf16 or fp32); both sides up-cast from
those same bits.
"""
from __future__ import annotations

import os
import zlib
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Dict, Optional, Tuple

import numpy as np
import torch

WEIGHT_STD = 0.02  # N(0, 0.02) random init for every projection / embedding


@dataclass(frozen=True)
class ModelCfg:
    """Shape of a pre-norm decoder (RMSNorm, RoPE, GQA, SwiGLU or MoE-SwiGLU)."""

    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    n_experts: int = 0
    top_k: int = 0
    d_expert: int = 0
    dtype: str = "bf16"  # storage dtype of weights and KV cache: "bf16" | "f32"
    rope_theta: float = 1.0e6
    rms_eps: float = 1.0e-6
    right_shifted: bool = False  # the output at position i-1 is the distribution of token i (else: of the [MASK] at i)

    @property
    def mask_id(self) -> int:
        return self.vocab - 1

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.bfloat16 if self.dtype == "bf16" else torch.float32

    @property
    def is_moe(self) -> bool:
        return self.n_experts > 0

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def n_params(self) -> int:
        d, D = self.d_model, self.head_dim
        per = d * self.qkv_rows + self.n_q_heads * D * d
        if self.is_moe:
            per += d * self.n_experts + self.n_experts * 3 * d * self.d_expert
        else:
            per += 3 * d * self.d_ffn
        return per * self.n_layers + d * self.vocab  # unembedding counted, embedding gather is not


@dataclass(frozen=True)
class Workload:
    """One benchmark / parity configuration: a model shape plus the step's batch shape."""

    cfg: ModelCfg
    batch: int
    prefix_min: int
    prefix_max: int
    block: int
    taus: Tuple[float, ...] = (0.9,)
    page_size: int = 16
    steps: int = 1
    synthetic_kv: bool = True  # False: the prefix cache comes from a real causal prefill


CONFIGS: Dict[int, Workload] = {
    1: Workload(ModelCfg("tiny-f32", 2, 256, 4, 2, 64, 768, 4096, dtype="f32"),
                batch=1, prefix_min=128, prefix_max=128, block=4, synthetic_kv=False),
    2: Workload(ModelCfg("dense-1.7b", 28, 2048, 16, 8, 128, 6144, 151936),
                batch=1, prefix_min=512, prefix_max=512, block=4, steps=64, synthetic_kv=False),
    3: Workload(ModelCfg("dense-4b", 36, 2560, 32, 8, 128, 9728, 151936),
                batch=8, prefix_min=1024, prefix_max=4096, block=8, taus=(0.7, 0.8, 0.9, 0.95)),
    4: Workload(ModelCfg("dense-8b", 36, 4096, 32, 8, 128, 12288, 151936),
                batch=16, prefix_min=8192, prefix_max=8192, block=16, page_size=16),
    5: Workload(ModelCfg("moe-16b", 20, 2048, 16, 4, 128, 0, 157184, n_experts=64, top_k=8, d_expert=1024),
                batch=32, prefix_min=2048, prefix_max=2048, block=32),
}


def shrink(cfg: ModelCfg, **kw) -> ModelCfg:
    """Same architecture with some dimensions replaced (used for fast parity cases)."""
    return replace(cfg, **kw)


def _workers() -> int:
    return max(1, min(16, os.cpu_count() or 1))


def _rng(seed: int, name: str) -> np.random.Generator:
    key = (int(seed) & 0xFFFFFFFF) | (zlib.crc32(name.encode()) << 32)
    return np.random.Generator(np.random.Philox(key=key))


def _normal(seed: int, name: str, shape, std: float, dtype: torch.dtype) -> torch.Tensor:
    g = _rng(seed, name)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    return torch.from_numpy(a).to(dtype)


def tensor_names(cfg: ModelCfg):
    names = ["embed", "unembed", "norm_f"]
    for l in range(cfg.n_layers):
        names += [f"l{l}.norm1", f"l{l}.wqkv", f"l{l}.wo", f"l{l}.norm2"]
        if cfg.is_moe:
            names += [f"l{l}.router", f"l{l}.e_wgu", f"l{l}.e_wdown"]
        else:
            names += [f"l{l}.wgu", f"l{l}.wdown"]
    return names


def gen_tensor(cfg: ModelCfg, seed: int, name: str, unembed_gain: float = 1.0,
               norm_jitter: float = 0.0) -> torch.Tensor:
    """One named weight tensor.

    Layouts ("out, in", the input dimension contiguous):
      embed   [V, d]            unembed [V, d] (scaled by `unembed_gain`)
      norm*   [d] fp32 gains (1, or 1 + norm_jitter*N(0,1) for tests)
      wqkv    [(Hq+2Hkv)*D, d]  rows: all query heads, then key heads, then value heads
      wo      [d, Hq*D]
      wgu     [2, F, d]         [0] = gate projection, [1] = up projection
      wdown   [d, F]
      router  [E, d]            N(0, 1/d): router logits are ~N(0,1) on a unit-RMS input
      e_wgu   [E, 2, Fe, d]     e_wdown [E, d, Fe]
    """
    d, D, dt = cfg.d_model, cfg.head_dim, cfg.torch_dtype
    base = name.split(".")[-1]
    if base in ("norm1", "norm2", "norm_f"):
        g = torch.ones(d, dtype=torch.float32)
        if norm_jitter:
            g = g + _normal(seed, name, (d,), norm_jitter, torch.float32)
        return g
    if base == "embed":
        return _normal(seed, name, (cfg.vocab, d), WEIGHT_STD, dt)
    if base == "unembed":
        return _normal(seed, name, (cfg.vocab, d), WEIGHT_STD * unembed_gain, dt)
    if base == "wqkv":
        return _normal(seed, name, (cfg.qkv_rows, d), WEIGHT_STD, dt)
    if base == "wo":
        return _normal(seed, name, (d, cfg.n_q_heads * D), WEIGHT_STD, dt)
    if base == "wgu":
        return _normal(seed, name, (2, cfg.d_ffn, d), WEIGHT_STD, dt)
    if base == "wdown":
        return _normal(seed, name, (d, cfg.d_ffn), WEIGHT_STD, dt)
    if base == "router":
        return _normal(seed, name, (cfg.n_experts, d), d ** -0.5, dt)
    if base == "e_wgu":
        return _normal(seed, name, (cfg.n_experts, 2, cfg.d_expert, d), WEIGHT_STD, dt)
    if base == "e_wdown":
        return _normal(seed, name, (cfg.n_experts, d, cfg.d_expert), WEIGHT_STD, dt)
    raise KeyError(name)


def calibrate_unembed_gain(cfg: ModelCfg, seed: int = 0, probe_rows: int = 48,
                           target_median: float = 0.55) -> float:
    """Scalar gain on the N(0,0.02) unembedding so that top-1 probabilities are spread out.

    After the final RMSNorm (gains 1) a hidden row has unit RMS, and the unembedding is
    independent of it, so each logit is N(0, (gain*0.02)^2 * d).  The gain is found by a
    seeded bisection on iid Gaussian probe rows such that the median top-1 softmax
    probability is `target_median`; with a vocabulary this large the top-1 probability of
    individual rows then spreads over roughly 0.1 ... 0.99.
    """
    g = _rng(seed, "gain-probe")
    z = g.standard_normal(size=(probe_rows, cfg.vocab)).astype(np.float64)

    def median_top1(sigma: float) -> float:
        x = z * sigma
        x -= x.max(axis=1, keepdims=True)
        p = 1.0 / np.exp(x).sum(axis=1)
        return float(np.median(p))

    lo, hi = 0.1, 40.0
    for _ in range(40):
        mid = 0.5 * (lo + hi)
        if median_top1(mid) < target_median:
            lo = mid
        else:
            hi = mid
    sigma = 0.5 * (lo + hi)
    return sigma / (WEIGHT_STD * cfg.d_model ** 0.5)


def gen_weights(cfg: ModelCfg, seed: int = 0, unembed_gain: Optional[float] = None,
                norm_jitter: float = 0.0) -> Dict[str, torch.Tensor]:
    if unembed_gain is None:
        unembed_gain = calibrate_unembed_gain(cfg, seed)
    names = tensor_names(cfg)
    # every tensor has its own keyed generator, so the tensors can be drawn concurrently
    with ThreadPoolExecutor(max_workers=_workers()) as ex:
        w = dict(zip(names, ex.map(lambda n: gen_tensor(cfg, seed, n, unembed_gain, norm_jitter), names)))
    w["__unembed_gain__"] = torch.tensor(unembed_gain, dtype=torch.float64)
    return w


def gen_prefix_lengths(wl: Workload, seed: int = 0, batch: Optional[int] = None) -> np.ndarray:
    n = wl.batch if batch is None else batch
    g = _rng(seed, "prefix-len")
    return g.integers(wl.prefix_min, wl.prefix_max + 1, size=n).astype(np.int32)


def gen_prefix_ids(cfg: ModelCfg, length: int, seed: int = 0, seq: int = 0) -> np.ndarray:
    """Prefix token ids, uniform on [0, V-2] (the last id is [MASK])."""
    g = _rng(seed, f"prefix-ids-{seq}")
    return g.integers(0, cfg.vocab - 1, size=length).astype(np.int32)


def kv_sigma(cfg: ModelCfg) -> float:
    """Std of a key/value element under random init: unit-RMS input times N(0,0.02) weights."""
    return WEIGHT_STD * cfg.d_model ** 0.5


def gen_page_table(n_seq: int, pages_per_seq: int, seed: int = 0) -> np.ndarray:
    """[n_seq, pages_per_seq] int32: a seeded random permutation of the physical pages."""
    g = _rng(seed, "page-table")
    perm = g.permutation(n_seq * pages_per_seq).astype(np.int32)
    return perm.reshape(n_seq, pages_per_seq)


def gen_synth_kv_pages(cfg: ModelCfg, n_pages: int, page_size: int, seed: int = 0,
                       layer: int = 0, which: str = "k") -> torch.Tensor:
    """Synthetic cache contents for one layer: [n_pages, Hkv, page_size, D] iid N(0, kv_sigma^2).

    Stands in for the post-RoPE keys / values of a real prefix (the prefill is not on the
    hot path); rounded to the cache dtype.
    """
    return _normal(seed, f"synthkv-{which}-{layer}",
                   (n_pages, cfg.n_kv_heads, page_size, cfg.head_dim), kv_sigma(cfg), cfg.torch_dtype)


def gen_logit_pairs(rows: int, vocab: int, seed: int = 0, agree_frac: float = 0.76,
                    eps: float = 0.35) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Synthetic (draft, verifier) fp32 logit rows for the vocabulary kernels alone.

    Rows come from a two-component mixture shaped like the paper's Table 7 quadrants:
    about `agree_frac` of the rows have verifier logits equal to the draft logits plus a
    small perturbation (ratio q/p mostly above 0.5), the rest have an independent verifier
    row (ratio far below 0.5).  The per-row logit scale is uniform on [3.5, 8], which spreads
    the top-1 probability over roughly 0.1 ... 0.99 for vocabularies of 10^5 entries.
    Returns (draft [rows,V] f32, verifier [rows,V] f32, agree [rows] bool).
    """
    g = _rng(seed, "logit-pairs")
    sigma = g.uniform(3.5, 8.0, size=(rows, 1)).astype(np.float32)
    draft = g.standard_normal(size=(rows, vocab), dtype=np.float32) * sigma
    agree = g.uniform(size=rows) < agree_frac
    ver = np.empty_like(draft)
    for r in range(rows):
        if agree[r]:
            ver[r] = draft[r] + np.float32(eps) * g.standard_normal(size=vocab, dtype=np.float32)
        else:
            ver[r] = g.standard_normal(size=vocab, dtype=np.float32) * sigma[r]
    return draft, ver, agree
