"""Seeded synthetic inputs for the decoder-layer hot path.

This module is shared by the tests, the benchmark and the smoke check; it feeds the same
numbers to the HIP path and to the CPU oracle.  It holds no arithmetic of the layer itself:
only the named shape presets, the random draws, the one-time rounding of the draws to the
storage dtype, and the bit-level bf16 <-> float conversions needed to hand one set of values
to both sides.

Recipe (stands in for LLaMA-2 style layers trained on text, paper section "Experimental
Setup": token content does not change cost or numerics class):
  x, dY ~ N(0, 1)          shape [B, S, H]
  weight matrices ~ N(0, sigma_w), sigma_w = 0.02 (a standard deviation)
  RMSNorm gains = 1
Every tensor gets its own counter-based stream keyed by (seed, tensor id, layer, micro-batch),
so a tensor does not change when another one is resized.  Values are drawn in fp32 and
rounded once (round-to-nearest-even) to the storage dtype; those rounded values are what
both sides see.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

F32 = 0
BF16 = 1


@dataclass(frozen=True)
class LayerConfig:
    """Shape of one decoder layer and its micro-batch (symbols B, S, H of the paper's Table 1)."""
    name: str
    dtype: int          # F32 or BF16: storage type of activations and weights
    B: int
    S: int
    H: int
    n_heads: int
    head_dim: int
    I: int              # SwiGLU intermediate width
    rope_theta: float = 10000.0
    rms_eps: float = 1e-6
    sigma_w: float = 0.02
    n_layers: int = 1
    n_microbatches: int = 1

    @property
    def T(self) -> int:
        return self.B * self.S

    def with_(self, **kw) -> "LayerConfig":
        return replace(self, **kw)


CONFIGS = {
    "C1": LayerConfig("C1", F32, 1, 128, 64, 4, 16, 176),
    "C2": LayerConfig("C2", BF16, 1, 8192, 4096, 32, 128, 11008),
    "C3": LayerConfig("C3", BF16, 1, 32768, 4096, 32, 128, 11008),
    "C4": LayerConfig("C4", BF16, 2, 16384, 5120, 40, 128, 13824, n_layers=4),
    "C5": LayerConfig("C5", BF16, 1, 16384, 8192, 64, 128, 22016, n_microbatches=4),
}

# tensor ids for the random streams
_ID_X, _ID_DY, _ID_WQKV, _ID_WO, _ID_WGU, _ID_WD = range(6)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 -> bf16 (nearest, ties to even); returns the 16-bit patterns as uint16."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(a32: np.ndarray, dtype: int) -> np.ndarray:
    """fp32 draws -> storage array (float32, or uint16 holding bf16 bit patterns)."""
    return f32_to_bf16_bits(a32) if dtype == BF16 else np.ascontiguousarray(a32, dtype=np.float32)


def to_f64(stored: np.ndarray, dtype: int) -> np.ndarray:
    """storage array -> the exact same values in fp64 (what the oracle consumes)."""
    if dtype == BF16:
        return bf16_bits_to_f32(stored).astype(np.float64)
    return np.asarray(stored, dtype=np.float32).astype(np.float64)


def _normal(seed: int, tid: int, layer: int, mb: int, shape, scale: float) -> np.ndarray:
    rng = np.random.Generator(np.random.Philox(key=[(seed << 20) ^ (tid << 16) ^ (layer << 8) ^ mb, 0x7A77]))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def make_activations(cfg: LayerConfig, seed: int = 0, mb: int = 0):
    """(x, dY), each [B, S, H] in storage dtype."""
    shp = (cfg.B, cfg.S, cfg.H)
    x = to_storage(_normal(seed, _ID_X, 0, mb, shp, 1.0), cfg.dtype)
    dy = to_storage(_normal(seed, _ID_DY, 0, mb, shp, 1.0), cfg.dtype)
    return x, dy


def make_weights(cfg: LayerConfig, seed: int = 0, layer: int = 0, sigma_w: float | None = None, gamma_jitter: float = 0.0):
    """Named weight tensors of one layer in storage dtype.

    Row order of the fused matrices: w_qkv = [Q rows; K rows; V rows] (each H rows, head-major),
    w_gate_up = [gate rows; up rows] (each I rows).  All matrices are [out, in] row-major.
    gamma_jitter > 0 perturbs the gains away from 1 (test-only, so a dropped gain is visible).
    """
    s = cfg.sigma_w if sigma_w is None else sigma_w
    H, I = cfg.H, cfg.I
    w = {
        "w_qkv": _normal(seed, _ID_WQKV, layer, 0, (3 * H, H), s),
        "w_o": _normal(seed, _ID_WO, layer, 0, (H, H), s),
        "w_gate_up": _normal(seed, _ID_WGU, layer, 0, (2 * I, H), s),
        "w_down": _normal(seed, _ID_WD, layer, 0, (H, I), s),
    }
    g1 = np.ones(H, dtype=np.float32)
    g2 = np.ones(H, dtype=np.float32)
    if gamma_jitter:
        g1 = g1 + _normal(seed, 6, layer, 0, (H,), gamma_jitter)
        g2 = g2 + _normal(seed, 7, layer, 0, (H,), gamma_jitter)
    w["gamma_attn"] = g1
    w["gamma_mlp"] = g2
    return {k: to_storage(v, cfg.dtype) for k, v in w.items()}


def device_normal(shape, seed: int, std: float = 1.0, dtype=None):
    """A seeded N(0, std) tensor drawn directly in GPU memory (for operands too large to draw on
    the host and upload in a test): fp32 draws rounded once to `dtype` (torch.bfloat16 unless
    given).  Both sides see the stored values: the HIP path reads the tensor, the oracle the
    slices of it that are copied back."""
    import torch
    gen = torch.Generator(device="cuda")
    gen.manual_seed(int(seed))
    t = torch.empty(tuple(shape), dtype=torch.float32, device="cuda")
    t.normal_(0.0, float(std), generator=gen)
    return t.to(torch.bfloat16 if dtype is None else dtype)


def weights_to_f64(w: dict, dtype: int) -> dict:
    return {k: to_f64(v, dtype) for k, v in w.items()}


CHUNK_ORDER = ("gamma_attn", "w_qkv", "w_o", "gamma_mlp", "w_gate_up", "w_down")


def pack_chunk(w: dict, offsets: dict, total_elems: int, dtype: int) -> np.ndarray:
    """Flat weight chunk in storage dtype; offsets are element offsets reported by the library."""
    out = np.zeros(total_elems, dtype=np.uint16 if dtype == BF16 else np.float32)
    for k in CHUNK_ORDER:
        v = w[k].reshape(-1)
        out[offsets[k]:offsets[k] + v.size] = v
    return out


def unpack_shard(flat: np.ndarray, offsets: dict, cfg: LayerConfig) -> dict:
    """Split a flat fp32 gradient shard (same element offsets as the chunk) into named tensors."""
    H, I = cfg.H, cfg.I
    shapes = {"gamma_attn": (H,), "w_qkv": (3 * H, H), "w_o": (H, H), "gamma_mlp": (H,),
              "w_gate_up": (2 * I, H), "w_down": (H, I)}
    return {k: flat[offsets[k]:offsets[k] + int(np.prod(shapes[k]))].reshape(shapes[k]) for k in CHUNK_ORDER}
