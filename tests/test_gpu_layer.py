"""Parity of the whole layer (forward + backward through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

from paper_2511_09741_amd import inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_c1_fp32_tiny_layer(taw, seed):
    """BASELINE config 1: fp32, B=1 S=128 H=64, 4 heads x 16, I=176; tensor-scale error <= 1e-4."""
    U.check_layer(taw, I.CONFIGS["C1"], seed=seed)


def test_c1_shapes_with_peaked_attention_and_nontrivial_gains(taw):
    """At sigma_w = 0.02 the scores are nearly flat; sigma_w = 0.5 makes the softmax peaked, and
    gains away from 1 make a dropped gamma visible."""
    U.check_layer(taw, I.CONFIGS["C1"], seed=3, sigma_w=0.5, gamma_jitter=0.3, tol=2e-4)


@pytest.mark.parametrize("B,S,H,nh,I_", [(2, 37, 48, 3, 40), (1, 1, 32, 2, 24), (3, 65, 64, 4, 100), (1, 200, 30, 3, 50)])
def test_fp32_ragged_shapes(taw, B, S, H, nh, I_):
    """Generic kernels on shapes that are no multiple of any tile or vector width (S=1 included)."""
    cfg = I.LayerConfig("ragged", I.F32, B, S, H, nh, H // nh, I_)
    U.check_layer(taw, cfg, seed=4, sigma_w=0.3, gamma_jitter=0.2, tol=2e-4)


def test_bf16_storage_on_generic_kernels(taw):
    """bf16 storage with head_dim 16: no MFMA kernel takes it, the generic path must."""
    cfg = I.LayerConfig("bf16-generic", I.BF16, 2, 48, 64, 4, 16, 88)
    U.check_layer(taw, cfg, seed=5, sigma_w=0.2, gamma_jitter=0.2)


def test_accumulate_flag_adds_into_the_shard(taw):
    import torch
    cfg = I.CONFIGS["C1"]
    w = I.make_weights(cfg, 0)
    x, dy = I.make_activations(cfg, 0)
    L = U.DeviceLayer(taw, cfg, flags=taw.TAW_ACCUMULATE)
    L.set_weights(w)
    xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
    L.fwd(xd)
    L.G.fill_(7.0)                       # padding and payload start at a known value
    L.bwd(xd, dyd)
    L.bwd(xd, dyd)
    g2 = L.grads()
    L2 = U.DeviceLayer(taw, cfg, flags=0)
    L2.set_weights(w)
    L2.fwd(xd)
    L2.G.fill_(7.0)
    L2.bwd(xd, dyd)
    g1 = L2.grads()
    for k in g1:
        assert U.tensor_scale_err(g2[k] - 7.0, 2 * g1[k]) < 1e-5, k
    # the padding between sub-tensors is never written
    flat = L2.G.cpu().numpy()
    mask = np.ones(flat.size, bool)
    shapes = {"gamma_attn": 64, "w_qkv": 192 * 64, "w_o": 64 * 64, "gamma_mlp": 64, "w_gate_up": 352 * 64, "w_down": 64 * 176}
    for k, n in shapes.items():
        mask[L2.layout[k]:L2.layout[k] + n] = False
    assert np.all(flat[mask] == 7.0)
    torch.cuda.synchronize()


def test_microbatch_accumulation_matches_oracle_sum(taw):
    """Same weights, independent micro-batches, G accumulated across them (config 5's pattern at tiny size)."""
    from oracle import decoder_layer as O
    cfg = I.CONFIGS["C1"]
    w = I.make_weights(cfg, 0, sigma_w=0.2)
    w64 = I.weights_to_f64(w, cfg.dtype)
    L = U.DeviceLayer(taw, cfg, flags=taw.TAW_ACCUMULATE)
    L.set_weights(w)
    Gsum = None
    for mb in range(4):
        x, dy = I.make_activations(cfg, 0, mb=mb)
        xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
        y = L.fwd(xd)
        dx = L.bwd(xd, dyd)
        yr, cache = O.layer_fwd(w64, I.to_f64(x, cfg.dtype), cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
        dxr, G = O.layer_bwd(w64, cache, I.to_f64(dy, cfg.dtype))
        assert U.tensor_scale_err(U.from_dev(y), yr) < 1e-4 and U.tensor_scale_err(U.from_dev(dx), dxr) < 1e-4
        Gsum = G if Gsum is None else {k: O.grad_accum(Gsum[k], G[k]) for k in G}
    got = L.grads()
    for k in Gsum:
        assert U.tensor_scale_err(got[k], Gsum[k]) < 1e-4, k


@pytest.mark.parametrize("B,S,nh,I_,sigma", [(1, 256, 2, 384, 0.02), (2, 333, 2, 392, 0.05), (1, 1024, 4, 1408, 0.02), (1, 77, 1, 136, 0.1)])
def test_bf16_layer_on_mfma_kernels(taw, B, S, nh, I_, sigma):
    """bf16, head_dim 128: the MFMA GEMM and attention kernels carry the layer.  Sizes span several
    tiles and leave ragged tails in tokens, widths and the SwiGLU dimension."""
    cfg = I.LayerConfig("bf16-mfma", I.BF16, B, S, nh * 128, nh, 128, I_, sigma_w=sigma)
    U.check_layer(taw, cfg, seed=B + S, gamma_jitter=0.1)
