"""Seeded synthetic inputs shaped like the paper's LLaMA-family workloads.

This module only draws random numbers and rounds them to the storage type; it contains none
of the method's arithmetic, so both the CPU oracle's tests and the GPU path's tests may use it.

The paper serves LLaMA2-13B / 70B in bf16 on a public instruction dataset (Section 6.1); no
dataset or trained weight is available here, so Gaussian tensors of the same shapes stand in:
projection weights ~ N(0, 0.02^2), norm gains 1 + 0.02 N(0,1), activations and cached K/V
~ N(0,1), integer lengths uniform on a closed range, token counts Poisson(64) times a burst
factor.  For bf16 configurations every tensor is rounded once (round-to-nearest-even) and the
rounded values, widened to fp32, are what both sides consume.

Generator: torch.Generator (CPU, Philox/MT as shipped) seeded with `seed`; tensors are drawn in
the fixed order wq, wk, wv, wo, wgate, wup, wdown, g1, g2 (weights) and lens, x, k_cache,
v_cache (inputs, from seed + 1).
"""
from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch


@dataclass(frozen=True)
class Config:
    name: str
    kind: str            # "decoder_layer" | "linear" | "attn_block" | "ffn_block" (the layer's two halves)
    dtype: str           # "f32" | "bf16"
    hidden: int = 0
    n_q_heads: int = 0
    n_kv_heads: int = 0
    head_dim: int = 0
    intermediate: int = 0
    rms_eps: float = 1e-5
    rope_base: float = 10000.0
    in_features: int = 0     # linear
    out_features: int = 0    # linear
    mode: str = "prefill"    # "prefill" | "decode" | "linear"
    n_seqs: int = 0          # sequences (decoder layer) or token rows (linear)
    seq_pad: int = 1         # padded prompt length (prefill)
    len_lo: int = 0          # prompt length (prefill) or cached length (decode), inclusive range
    len_hi: int = 0
    replicas: tuple = (1,)
    n_layers: int = 1        # consecutive decoder layers in the module (a run)

    @property
    def cache_cap(self) -> int:
        """Slots per (sequence, kv head): longest cached length + the appended token,
        rounded up to a multiple of 64."""
        return ((self.len_hi + 1 + 63) // 64) * 64


CONFIGS = {
    # the five benchmark configurations
    "C1": Config("C1-tiny-f32-prefill", "decoder_layer", "f32", 256, 4, 4, 64, 688,
                 mode="prefill", n_seqs=4, seq_pad=32, len_lo=32, len_hi=32, replicas=(1, 2)),
    "C2": Config("C2-llama2-7b-decode", "decoder_layer", "bf16", 4096, 32, 32, 128, 11008,
                 mode="decode", n_seqs=32, len_lo=1024, len_hi=1024, replicas=(1, 2, 4)),
    "C3": Config("C3-llama2-13b-prefill", "decoder_layer", "bf16", 5120, 40, 40, 128, 13824,
                 mode="prefill", n_seqs=8, seq_pad=512, len_lo=256, len_hi=512, replicas=(1, 2)),
    "C4": Config("C4-llama2-70b-gqa-decode", "decoder_layer", "bf16", 8192, 64, 8, 128, 28672,
                 mode="decode", n_seqs=64, len_lo=512, len_hi=2048, replicas=(1, 2)),
    "C5": Config("C5-down-proj-bursty", "linear", "bf16", in_features=11008, out_features=4096,
                 mode="linear", n_seqs=64, replicas=(1, 2, 4)),
}


def scaled(cfg: Config, **kw) -> Config:
    """Same structure, other sizes (for parity cases the oracle finishes in seconds)."""
    return replace(cfg, **kw)


def _round(t: torch.Tensor, dtype: str) -> torch.Tensor:
    if dtype == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    return t


def _randn(g, shape, dtype, std=1.0, mean=0.0):
    t = torch.randn(shape, generator=g, dtype=torch.float32)
    if std != 1.0:
        t.mul_(std)
    if mean != 0.0:
        t.add_(mean)
    return _round(t, dtype).numpy()


def make_weights(cfg: Config, seed: int = 0) -> dict:
    """fp32 numpy arrays holding storage-type-representable values; matrices are [out, in]."""
    g = torch.Generator().manual_seed(seed)
    if cfg.kind == "linear":
        return {"w": _randn(g, (cfg.out_features, cfg.in_features), cfg.dtype, 0.02)}
    if cfg.n_layers > 1:   # a run of layers: a list, drawn layer after layer from the one generator
        return [_layer_weights(cfg, g) for _ in range(cfg.n_layers)]
    return _layer_weights(cfg, g)


def _layer_weights(cfg: Config, g) -> dict:
    H, d = cfg.hidden, cfg.head_dim
    QD, KD, I = cfg.n_q_heads * d, cfg.n_kv_heads * d, cfg.intermediate
    w = {}
    for name, shape in (("wq", (QD, H)), ("wk", (KD, H)), ("wv", (KD, H)), ("wo", (H, QD)),
                        ("wgate", (I, H)), ("wup", (I, H)), ("wdown", (H, I))):
        w[name] = _randn(g, shape, cfg.dtype, 0.02)
    w["g1"] = _randn(g, (H,), cfg.dtype, 0.02, 1.0)
    w["g2"] = _randn(g, (H,), cfg.dtype, 0.02, 1.0)
    return w


@dataclass
class Inputs:
    x: np.ndarray                       # prefill [B,S,H]; decode [B,H]; linear [T,in]
    lens: Optional[np.ndarray] = None   # int32 [B]
    k_cache: Optional[np.ndarray] = None  # decode: [B, n_kv, cap, d], slots < lens[b] filled
    v_cache: Optional[np.ndarray] = None


def make_inputs(cfg: Config, seed: int = 0, lens=None, x_std: float = 1.0, k_std: float = 1.0) -> Inputs:
    """lens: fixed lengths instead of drawn ones (each within [0 or 1, len_hi]); x_std / k_std:
    standard deviation of the activations / of the cached keys (1 in the benchmark configurations;
    parity cases use a small x_std so that the module's output is dominated by what its kernels
    add to the residual stream, and a larger k_std for sharply peaked attention weights)."""
    g = torch.Generator().manual_seed(seed + 1)
    if cfg.kind == "linear":
        return Inputs(x=_randn(g, (cfg.n_seqs, cfg.in_features), cfg.dtype, x_std))
    if cfg.kind == "ffn_block":   # independent token rows
        return Inputs(x=_randn(g, (cfg.n_seqs, cfg.hidden), cfg.dtype, x_std))
    B, H = cfg.n_seqs, cfg.hidden
    drawn = torch.randint(cfg.len_lo, cfg.len_hi + 1, (B,), generator=g, dtype=torch.int64)
    if lens is None:
        lens = drawn.to(torch.int32).numpy()
    else:
        lens = np.asarray(lens, dtype=np.int32).copy()
        if lens.shape != (B,) or lens.min() < 0 or lens.max() > cfg.len_hi:
            raise ValueError("lens: one value in [0, len_hi] per sequence")
    if cfg.mode == "prefill":
        return Inputs(x=_randn(g, (B, cfg.seq_pad, H), cfg.dtype, x_std), lens=lens)
    x = _randn(g, (B, H), cfg.dtype, x_std)
    shape = (B, cfg.n_kv_heads, cfg.cache_cap, cfg.head_dim)
    if cfg.n_layers > 1:
        shape = (cfg.n_layers,) + shape    # one cache per layer of the run
    k = _randn(g, shape, cfg.dtype, k_std)
    v = _randn(g, shape, cfg.dtype)
    # slots at and beyond the cached length are not part of the input: zero them so that a
    # reader of a wrong slot is caught
    for b in range(B):
        k[..., b, :, lens[b]:, :] = 0.0
        v[..., b, :, lens[b]:, :] = 0.0
    return Inputs(x=x, lens=lens, k_cache=k, v_cache=v)


# ---- bursty single-projection load (benchmark configuration 4) ------------------------------------
def bursty_token_counts(seed: int = 0, n_batches: int = 200, lam: float = 64.0):
    """Per batch: n = max(1, Poisson(lam)) * f with f uniform on {1, 4, 16}, i.i.d."""
    g = torch.Generator().manual_seed(seed + 2)
    base = torch.poisson(torch.full((n_batches,), lam), generator=g).clamp_(min=1).to(torch.int64)
    burst = torch.tensor([1, 4, 16])[torch.randint(0, 3, (n_batches,), generator=g)]
    return [int(v) for v in (base * burst)]


def replicas_for_tokens(n: int) -> int:
    """Harness policy for the bursty load: 1 replica below 128 tokens, 2 below 512, else 4."""
    return 1 if n < 128 else (2 if n < 512 else 4)
