"""Seeded synthetic inputs for the Self-Indexing KV cache decode path.

This module only draws random numbers and rounds them to 16-bit storage; it
holds none of the method's arithmetic and is the one piece of code the CPU
oracle's callers and the HIP library's callers share.  The tensors stand in
for the GQA key/value caches of the paper's Llama-3.1-8B / Qwen2.5-14B decode
workloads (section "Experimental Setup"), which need model weights and
benchmark data that are not available here.

Every tensor is drawn in fp32 from numpy's Generator(PCG64(seed)), rounded to
nearest-even into the configuration's 16-bit type and returned as raw uint16
bit patterns, so both sides read identical bits.
"""
from dataclasses import dataclass, replace

import numpy as np


@dataclass(frozen=True)
class Config:
    name: str
    batch: int
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    context: int          # tokens resident before the first decode step
    top_k: int
    dtype: str            # "fp16" | "bf16"
    sigma: str            # "unit" | "lognormal" (per-channel std ~ LogNormal(0, 0.5))
    outlier_frac: float   # fraction of channels scaled up (count = ceil(frac * D))
    outlier_count: int    # explicit channel count, used when outlier_frac == 0
    outlier_scale: float
    seed: int
    append: bool          # quantise-append one new key per head per step
    steps: int            # decode steps the workload describes


CONFIGS = {
    "C1": Config("C1 tiny decode 4K", 1, 1, 4, 128, 4096, 256, "fp16", "unit", 0.0, 4, 10.0, 0, False, 1),
    "C2": Config("C2 Llama-3-8B-shaped layer decode 32K", 1, 8, 32, 128, 32768, 1024, "bf16",
                 "lognormal", 0.01, 0, 8.0, 1, False, 1),
    "C3": Config("C3 long context 128K with append", 1, 8, 32, 128, 131072, 2048, "bf16",
                 "lognormal", 0.01, 0, 8.0, 2, True, 1),
    "C4": Config("C4 large batch 32x16K", 32, 8, 32, 128, 16384, 512, "bf16",
                 "lognormal", 0.01, 0, 8.0, 3, False, 1),
    "C5": Config("C5 prefill-compress + 16 decode steps 4x64K GQA8", 4, 8, 64, 128, 65536, 1536, "bf16",
                 "lognormal", 0.02, 0, 10.0, 4, True, 16),
    # the shape the paper's module-timing table is quoted on ("16K token input with batch size 10", 7.5 % of the
    # tokens kept), on a Llama-3-8B-shaped layer: context for the paper's numbers, not one of the five workloads
    "T4": Config("T4 module-timing shape 10x16K, 7.5 % kept", 10, 8, 32, 128, 16384, 1229, "bf16",
                 "lognormal", 0.01, 0, 8.0, 5, False, 1),
}


def scaled(cfg: Config, **kw) -> Config:
    """A copy of a configuration with some fields replaced (reduced test sizes)."""
    return replace(cfg, **kw)


def to_bits(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 values to nearest-even fp16 / bf16 and return the uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).view(np.uint16)
    if dtype == "bf16":
        u = x.view(np.uint32)
        bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
        return ((u + bias) >> 16).astype(np.uint16)
    raise ValueError(dtype)


def from_bits(bits: np.ndarray, dtype: str) -> np.ndarray:
    """Exact fp32 view of fp16 / bf16 bit patterns (for building torch tensors or checks)."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if dtype == "fp16":
        return bits.view(np.float16).astype(np.float32)
    if dtype == "bf16":
        return (bits.astype(np.uint32) << 16).view(np.float32)
    raise ValueError(dtype)


def channel_scales(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    """Per (kv head, channel) standard deviation including outlier channels; shared by the batch."""
    H, D = cfg.n_kv_heads, cfg.head_dim
    if cfg.sigma == "lognormal":
        s = rng.lognormal(0.0, 0.5, size=(H, D)).astype(np.float32)
    else:
        s = np.ones((H, D), np.float32)
    n_out = cfg.outlier_count if cfg.outlier_frac == 0 else int(np.ceil(cfg.outlier_frac * D))
    for h in range(H):
        ch = rng.permutation(D)[:n_out]
        s[h, ch] *= np.float32(cfg.outlier_scale)
    return s


def _normal(rng, shape):
    return rng.standard_normal(size=shape, dtype=np.float32)


def make_cache(cfg: Config, capacity: int = None, channel_offset_std: float = 0.0, layer: int = 0):
    """K, V as uint16 bits [B, Hkv, capacity, D]; rows at or beyond cfg.context are zero.

    channel_offset_std > 0 adds a per (kv head, channel) constant ~ N(0, std^2) to K so that
    the channel-mean path is exercised (the benchmark configurations are zero-mean).
    `layer` picks an independent draw of the same recipe (distinct cache-resident copies).
    """
    B, H, L, D = cfg.batch, cfg.n_kv_heads, cfg.context, cfg.head_dim
    cap = L if capacity is None else int(capacity)
    assert cap >= L
    root = np.random.SeedSequence([cfg.seed, layer])
    struct_ss, *seq_ss = root.spawn(1 + B)
    srng = np.random.Generator(np.random.PCG64(struct_ss))
    sk = channel_scales(cfg, srng)
    sv = channel_scales(cfg, srng)
    off = (srng.standard_normal(size=(H, D)).astype(np.float32) * np.float32(channel_offset_std)
           if channel_offset_std > 0 else np.zeros((H, D), np.float32))
    K = np.zeros((B, H, cap, D), np.uint16)
    V = np.zeros((B, H, cap, D), np.uint16)
    for b in range(B):
        rng = np.random.Generator(np.random.PCG64(seq_ss[b]))
        for h in range(H):
            K[b, h, :L] = to_bits(_normal(rng, (L, D)) * sk[h] + off[h], cfg.dtype)
            V[b, h, :L] = to_bits(_normal(rng, (L, D)) * sv[h], cfg.dtype)
    return K, V


def make_step_inputs(cfg: Config, step: int, layer: int = 0):
    """q [B, Hq, D] and the new key/value rows [B, Hkv, D] of one decode step, as uint16 bits."""
    B, H, D = cfg.batch, cfg.n_kv_heads, cfg.head_dim
    root = np.random.SeedSequence([cfg.seed, layer, 7919, step])
    rng = np.random.Generator(np.random.PCG64(root))
    q = to_bits(_normal(rng, (B, cfg.n_q_heads, D)), cfg.dtype)
    srng = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, layer]).spawn(1 + B)[0]))
    sk = channel_scales(cfg, srng)
    sv = channel_scales(cfg, srng)
    k_new = to_bits(_normal(rng, (B, H, D)) * sk, cfg.dtype)
    v_new = to_bits(_normal(rng, (B, H, D)) * sv, cfg.dtype)
    return q, k_new, v_new


def algorithmic_bytes(cfg: Config, context: int = None) -> dict:
    """Bytes one decode step must read: the 1-bit code plane plus the gathered 16-bit K/V rows."""
    L = cfg.context if context is None else context
    codes = cfg.batch * cfg.n_kv_heads * L * (cfg.head_dim // 8)
    gathered = cfg.batch * cfg.n_q_heads * min(cfg.top_k, L) * 2 * cfg.head_dim * 2
    return {"codes": codes, "gathered": gathered, "total": codes + gathered}
