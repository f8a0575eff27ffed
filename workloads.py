"""Seeded synthetic inputs for the VCAS linear-backward path.

Serves both the CPU oracle's tests and the GPU library's tests / benchmark.
Holds no arithmetic of the method itself: only shapes, keep-ratio schedules
and random tensors with the value structure of the paper's workloads
(transformer linear layers at finetuning batch sizes, per-sample gradient
norms that are heavy-tailed as in the paper's Fig. 3).

Tensors are returned as numpy arrays: fp32 as ``float32``; bf16 as ``uint16``
bit patterns (round-to-nearest-even from the fp32 draw).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F32, BF16 = 0, 1


@dataclass(frozen=True)
class LayerSpec:
    """One linear layer's backward problem."""
    name: str
    dtype: int          # F32 or BF16
    N: int              # batch
    T: int              # tokens per sample
    K_in: int
    K_out: int
    rho: float          # data keep ratio
    nu: float           # token keep ratio
    layer: int          # Philox layer id
    seed: int = 0       # Philox seed
    gen_seed: int = 0   # input generator seed
    sample_sigma: float = 1.0   # LogNormal sigma of the per-sample scale (0 = none)
    token_sigma: float = 0.0    # LogNormal sigma of the per-token scale (0 = none)

    @property
    def R(self) -> int:
        return self.N * self.T


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even fp32 -> bf16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_layer(spec: LayerSpec):
    """Returns (G[R,K_out], X[R,K_in], W[K_out,K_in]) for one layer."""
    rng = np.random.Generator(np.random.PCG64([spec.gen_seed, spec.layer, 0x5CA5]))
    N, T = spec.N, spec.T
    X = rng.standard_normal((N * T, spec.K_in), dtype=np.float32)
    W = rng.standard_normal((spec.K_out, spec.K_in), dtype=np.float32) * np.float32(0.02)
    G = rng.standard_normal((N, T, spec.K_out), dtype=np.float32)
    if spec.sample_sigma > 0:
        s = np.exp(spec.sample_sigma * rng.standard_normal(N)).astype(np.float32)
        G *= s[:, None, None]
    if spec.token_sigma > 0:
        u = np.exp(spec.token_sigma * rng.standard_normal((N, T))).astype(np.float32)
        G *= u[:, :, None]
    G = G.reshape(N * T, spec.K_out)
    if spec.dtype == BF16:
        return f32_to_bf16_bits(G), f32_to_bf16_bits(X), f32_to_bf16_bits(W)
    return G, X, W


def _stack(name, dtype, N, T, hidden, ffn, blocks, rho_top, rho_bottom, nu,
           sample_sigma, token_sigma, gen_seed=0, seed=0, fused_qkv=False):
    """Encoder-style stack: per block Q, K, V, out-proj (h->h), FFN up (h->ffn),
    FFN down (ffn->h).  Block `blocks-1` is the top (nearest the loss); the data
    keep ratio is interpolated linearly from rho_top there to rho_bottom at
    block 0, and is shared by the six linears of a block.  fused_qkv: the three
    projections as one h->3h linear under a single SampleA mask."""
    shapes = [("q", hidden, hidden), ("k", hidden, hidden), ("v", hidden, hidden),
              ("o", hidden, hidden), ("up", hidden, ffn), ("down", ffn, hidden)]
    if fused_qkv:
        shapes = [("qkv", hidden, 3 * hidden)] + shapes[3:]
    out = []
    for b in range(blocks):
        f = b / (blocks - 1) if blocks > 1 else 1.0
        rho = rho_bottom + (rho_top - rho_bottom) * f
        for j, (nm, kin, kout) in enumerate(shapes):
            out.append(LayerSpec(f"{name}.b{b}.{nm}", dtype, N, T, kin, kout, float(rho), nu,
                                 layer=b * 6 + j, seed=seed, gen_seed=gen_seed,
                                 sample_sigma=sample_sigma, token_sigma=token_sigma))
    return out


def config(name: str):
    """The benchmark configurations, as lists of LayerSpec in backward order
    (top block first)."""
    if name == "single_fp32":
        return [LayerSpec("single_fp32", F32, 8, 128, 768, 768, 0.5, 0.5, layer=0, seed=0,
                          sample_sigma=1.0)]
    if name == "bert_base":
        ls = _stack("bert_base", BF16, 32, 128, 768, 3072, 12, 1.0, 0.3, 0.5, 1.0, 0.5)
    elif name == "bert_base_fused_qkv":
        ls = _stack("bert_base_fused_qkv", BF16, 32, 128, 768, 3072, 12, 1.0, 0.3, 0.5, 1.0, 0.5, fused_qkv=True)
    elif name == "bert_large":
        ls = _stack("bert_large", BF16, 32, 512, 1024, 4096, 24, 1.0, 0.25, 0.4, 1.0, 0.5)
    elif name == "vit_b16":
        ls = _stack("vit_b16", BF16, 64, 197, 768, 3072, 12, 0.3, 0.3, 0.5, 1.5, 0.0)
    elif name.startswith("gpt2_medium"):
        # "gpt2_medium:0.5:0.25" selects one (rho, nu) point of the sweep
        parts = name.split(":")
        rho = float(parts[1]) if len(parts) > 1 else 0.5
        nu = float(parts[2]) if len(parts) > 2 else 0.5
        ls = _stack("gpt2_medium", BF16, 16, 1024, 1024, 4096, 24, rho, rho, nu, 0.0, 0.5)
    else:
        raise KeyError(name)
    return sorted(ls, key=lambda s: -s.layer)


CONFIG_NAMES = ["single_fp32", "bert_base", "bert_large", "vit_b16", "gpt2_medium", "bert_base_fused_qkv"]


def small_cases():
    """Parity cases the oracle finishes in seconds: several tiles, ragged tails,
    both dtypes, degenerate keep ratios."""
    c = []
    k = 0
    for dtype in (F32, BF16):
        for (N, T, kin, kout, rho, nu, ss, ts) in [
            (8, 128, 768, 768, 0.5, 0.5, 1.0, 0.0),     # configs[0] shape
            (5, 37, 264, 136, 0.6, 0.5, 1.0, 0.5),      # nothing a multiple of a tile
            (3, 197, 320, 200, 0.7, 0.3, 1.5, 0.0),     # ViT token count
            (16, 64, 128, 512, 1.0, 1.0, 1.0, 0.5),     # keep everything
            (16, 64, 512, 128, 1.0, 0.25, 1.0, 0.5),    # token sampling only
            (12, 50, 256, 256, 0.1, 0.5, 2.0, 0.5),     # almost everything dropped
            (1, 300, 136, 264, 0.5, 0.5, 0.0, 1.0),     # a single sample
        ]:
            c.append(LayerSpec(f"small{k}", dtype, N, T, kin, kout, rho, nu, layer=k, seed=1234 + k,
                               gen_seed=99, sample_sigma=ss, token_sigma=ts))
            k += 1
    return c
