"""Test harness: moves seeded inputs to the GPU, calls the HIP path through its binding, brings
results back; and runs the CPU oracle on the very same stored values."""
from __future__ import annotations

import numpy as np

from paper_2511_09741_amd import inputs as I

TOL = {I.F32: 1e-4, I.BF16: 2e-2}   # tensor-scale max error bar per storage dtype


def tensor_scale_err(got, ref, floor: float = 0.0) -> float:
    """max_i |got_i - ref_i| / max(max_i |ref_i|, floor)  (element-wise relative error is ill-posed
    at ref ~ 0; `floor` is for tensors whose exact value is identically zero)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if not np.all(np.isfinite(got)):
        return float("inf")
    denom = max(float(np.max(np.abs(ref))), floor)
    num = float(np.max(np.abs(got - ref)))
    return num / denom if denom > 0 else num


# ----------------------------------------------------------------------------- host <-> device
def to_dev(arr: np.ndarray, dtype: int):
    """storage array (float32, or uint16 bf16 bits) -> torch tensor on cuda:0 of the matching type."""
    import torch
    if dtype == I.BF16:
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def from_dev(t) -> np.ndarray:
    """torch tensor (bf16 or fp32) -> fp64 numpy."""
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def empty_dev(shape, dtype: int):
    import torch
    return torch.empty(shape, dtype=torch.bfloat16 if dtype == I.BF16 else torch.float32, device="cuda")


class DeviceLayer:
    """Buffers of one layer on the GPU and the fwd/bwd calls on them (through the C ABI)."""

    def __init__(self, taw, cfg: I.LayerConfig, flags: int = 0):
        import torch
        self.taw, self.cfg = taw, cfg
        self.desc = taw.desc_from_config(cfg, flags)
        self.layout = taw.taw_layer_weight_layout(self.desc)
        self.ctx = torch.empty(taw.taw_layer_ctx_bytes(self.desc), dtype=torch.uint8, device="cuda")
        self.ws_bytes = taw.taw_layer_workspace_bytes(self.desc)
        self.ws = torch.empty(self.ws_bytes, dtype=torch.uint8, device="cuda")
        self.rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
        taw.taw_rope_table_init(self.desc, self.rope)
        self.G = torch.zeros(self.layout["total_elems"], dtype=torch.float32, device="cuda")
        self.chunk = None

    def set_weights(self, w: dict):
        flat = I.pack_chunk(w, self.layout, self.layout["total_elems"], self.cfg.dtype)
        self.chunk = to_dev(flat, self.cfg.dtype)

    def fwd(self, x_dev):
        y = empty_dev(tuple(x_dev.shape), self.cfg.dtype)
        self.taw.taw_layer_fwd(self.desc, self.chunk, self.rope, x_dev, y, self.ctx, self.ws, self.ws_bytes)
        return y

    def bwd(self, x_dev, dy_dev):
        dx = empty_dev(tuple(x_dev.shape), self.cfg.dtype)
        self.taw.taw_layer_bwd(self.desc, self.chunk, self.rope, x_dev, dy_dev, self.ctx, dx, self.G, self.ws, self.ws_bytes)
        return dx

    def grads(self) -> dict:
        import torch
        torch.cuda.synchronize()
        flat = self.G.cpu().numpy()
        return {k: v.astype(np.float64) for k, v in I.unpack_shard(flat, self.layout, self.cfg).items()}


def run_gpu_layer(taw, cfg, seed=0, sigma_w=None, gamma_jitter=0.0):
    import torch
    w = I.make_weights(cfg, seed, sigma_w=sigma_w, gamma_jitter=gamma_jitter)
    x, dy = I.make_activations(cfg, seed)
    L = DeviceLayer(taw, cfg)
    L.set_weights(w)
    xd, dyd = to_dev(x, cfg.dtype), to_dev(dy, cfg.dtype)
    y = L.fwd(xd)
    dx = L.bwd(xd, dyd)
    torch.cuda.synchronize()
    return from_dev(y), from_dev(dx), L.grads()


def run_oracle_layer(cfg, seed=0, sigma_w=None, gamma_jitter=0.0):
    from oracle import decoder_layer as O
    w = I.weights_to_f64(I.make_weights(cfg, seed, sigma_w=sigma_w, gamma_jitter=gamma_jitter), cfg.dtype)
    x, dy = I.make_activations(cfg, seed)
    x64, dy64 = I.to_f64(x, cfg.dtype), I.to_f64(dy, cfg.dtype)
    y, cache = O.layer_fwd(w, x64, cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    dx, G = O.layer_bwd(w, cache, dy64)
    return y, dx, G, cache


def check_layer(taw, cfg, seed=0, sigma_w=None, gamma_jitter=0.0, tol=None, verbose=True):
    tol = TOL[cfg.dtype] if tol is None else tol
    y, dx, G = run_gpu_layer(taw, cfg, seed, sigma_w, gamma_jitter)
    yr, dxr, Gr, _ = run_oracle_layer(cfg, seed, sigma_w, gamma_jitter)
    errs = {"y": tensor_scale_err(y, yr), "dx": tensor_scale_err(dx, dxr)}
    for k in Gr:
        errs["G." + k] = tensor_scale_err(G[k], Gr[k])
    if verbose:
        print(f"[{cfg.name} seed={seed} sigma_w={sigma_w}] " + " ".join(f"{k}={v:.2e}" for k, v in errs.items()), flush=True)
    bad = {k: v for k, v in errs.items() if not v <= tol}
    assert not bad, f"tensor-scale error above {tol}: {bad}"
    return errs
