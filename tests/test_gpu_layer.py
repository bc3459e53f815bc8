"""Parity of the whole layer (forward + backward through the C ABI) against the CPU oracle."""
import numpy as np
import pytest

from paper_2511_09741_amd import inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_c1_fp32_tiny_layer(taw, seed):
    """The smallest stated configuration: fp32, B=1 S=128 H=64, 4 heads x 16, I=176; tensor-scale error <= 1e-4."""
    U.check_layer(taw, I.CONFIGS["C1"], seed=seed)


def test_c1_shapes_with_peaked_attention_and_nontrivial_gains(taw):
    """At sigma_w = 0.02 the scores are nearly flat; sigma_w = 0.5 makes the softmax peaked, and
    gains away from 1 make a dropped gamma visible."""
    U.check_layer(taw, I.CONFIGS["C1"], seed=3, sigma_w=0.5, gamma_jitter=0.3)


@pytest.mark.parametrize("B,S,H,nh,I_", [(2, 37, 48, 3, 40), (1, 1, 32, 2, 24), (3, 65, 64, 4, 100), (1, 200, 30, 3, 50)])
def test_fp32_ragged_shapes(taw, B, S, H, nh, I_):
    """Generic kernels on shapes that are no multiple of any tile or vector width (S=1 included)."""
    cfg = I.LayerConfig("ragged", I.F32, B, S, H, nh, H // nh, I_)
    U.check_layer(taw, cfg, seed=4, sigma_w=0.3, gamma_jitter=0.2)


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


@pytest.mark.parametrize("B,S,nh,I_,sigma", [(1, 256, 2, 384, 0.02), (2, 333, 2, 392, 0.05), (1, 1024, 4, 1408, 0.02), (1, 77, 1, 136, 0.1),
                                             (1, 256, 2, 400, 0.02), (16, 48, 2, 384, 0.05)])
def test_bf16_layer_on_mfma_kernels(taw, B, S, nh, I_, sigma):
    """bf16, head_dim 128: the MFMA GEMM and attention kernels carry the layer.  Sizes span several
    tiles and leave ragged tails in tokens, widths and the SwiGLU dimension.  The backward linears run
    pairwise in one grid when the token count and the widths are multiples of 32 (first, third and last
    case; the fifth with 2 I = 800, which takes the 32-deep input-gradient loop) and one by one otherwise.
    Where the token count is a multiple of 256 the qkv projection rotates q and k in its epilogue; the
    last case has sequences of 48 tokens, so the positions wrap inside the 32-row blocks of that epilogue."""
    cfg = I.LayerConfig("bf16-mfma", I.BF16, B, S, nh * 128, nh, 128, I_, sigma_w=sigma)
    U.check_layer(taw, cfg, seed=B + S, gamma_jitter=0.1)


@pytest.mark.parametrize("H,nh,B,S", [(1024, 8, 4, 512), (2048, 16, 2, 384)])
def test_bf16_layer_at_the_widths_of_the_papers_throughput_table(taw, H, nh, B, S):
    """The narrower models of the paper's throughput table (Experiments, Throughput and Memory Usage: H = 1024 and 2048,
    heads of 128, I = 8H/3 rounded up to 256, micro-batches of several sequences): whole layer against the oracle, every
    element, at a reduced sequence length.  The first case has 2048 tokens: all four of its weight gradients are computed in
    3 - 4 ranges of tokens and summed by the second kernel, as at the table's own sizes."""
    cfg = I.LayerConfig(f"table-{H}", I.BF16, B, S, H, nh, 128, (8 * H // 3 + 255) // 256 * 256)
    T = B * S
    cut = [taw.taw_op_linear_bwd_scratch_floats(T, N, K) > 0 for N, K in ((H, cfg.I), (2 * cfg.I, H), (H, H), (3 * H, H))]
    assert all(cut) == (H == 1024)
    U.check_layer(taw, cfg, seed=H + S)


def test_bf16_layer_with_the_other_forms_of_the_attention_backward(taw):
    """TAW_ATTN_BWD_FUSED (one kernel, dQ partial sums in private slots inside the workspace) and TAW_ATTN_BWD_RECOMPUTE
    (two kernels, the scores recomputed, nothing extra in the workspace) against the oracle, beside the default (two
    kernels, dS handed over through the workspace); same tolerance, they differ in summation order at most."""
    cfg = I.LayerConfig("bf16-fused-bwd", I.BF16, 2, 1100, 512, 4, 128, 1408, sigma_w=0.05)
    w = I.make_weights(cfg, 7, gamma_jitter=0.1)
    x, dy = I.make_activations(cfg, 7)
    w64 = I.weights_to_f64(w, cfg.dtype)
    from oracle import decoder_layer as O
    yr, cache = O.layer_fwd(w64, I.to_f64(x, cfg.dtype), cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    dxr, Gr = O.layer_bwd(w64, cache, I.to_f64(dy, cfg.dtype))
    ws = {f: taw.taw_layer_workspace_bytes(taw.desc_from_config(cfg, f)) for f in (0, taw.TAW_ATTN_BWD_FUSED, taw.TAW_ATTN_BWD_RECOMPUTE)}
    assert ws[taw.TAW_ATTN_BWD_RECOMPUTE] < ws[0] and ws[taw.TAW_ATTN_BWD_RECOMPUTE] < ws[taw.TAW_ATTN_BWD_FUSED]
    for flags in (taw.TAW_ATTN_BWD_FUSED, taw.TAW_ATTN_BWD_RECOMPUTE, 0):
        L = U.DeviceLayer(taw, cfg, flags=flags)
        L.set_weights(w)
        xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
        L.fwd(xd)
        dx = L.bwd(xd, dyd)
        assert U.tensor_scale_err(U.from_dev(dx), dxr) < U.TOL[cfg.dtype]
        G = L.grads()
        for k in Gr:
            assert U.tensor_scale_err(G[k], Gr[k]) < U.TOL[cfg.dtype], (flags, k)


def test_four_chained_layers_with_staged_weights(taw):
    """Config 4's pattern at reduced width (bf16, MFMA kernels): forward through layers 0..3, backward
    3..0, every layer's weights arriving through taw_weight_stage into one of two staging buffers on a
    side stream (ready / consumed events).  The oracle chains the same four layers in fp64; the device
    passes bf16 activations between layers.  Compared: the last output, the gradient of the first
    input and all four gradient shards."""
    import torch
    from oracle import decoder_layer as O
    nl = 4
    cfg = I.LayerConfig("chain", I.BF16, 2, 320, 256, 2, 128, 392, sigma_w=0.05, n_layers=nl)
    ws = [I.make_weights(cfg, 0, layer=l, gamma_jitter=0.1) for l in range(nl)]
    x, dy = I.make_activations(cfg, 0)
    # ---- oracle
    w64 = [I.weights_to_f64(w, cfg.dtype) for w in ws]
    a, caches = I.to_f64(x, cfg.dtype), []
    for l in range(nl):
        a, c = O.layer_fwd(w64[l], a, cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
        caches.append(c)
    y_ref = a
    g, G_ref = I.to_f64(dy, cfg.dtype), [None] * nl
    for l in reversed(range(nl)):
        g, G_ref[l] = O.layer_bwd(w64[l], caches[l], g)
    dx_ref = g
    # ---- device
    desc = taw.desc_from_config(cfg, 0)
    lay = taw.taw_layer_weight_layout(desc)
    P = lay["total_elems"]
    store = [U.to_dev(I.pack_chunk(w, lay, P, cfg.dtype), cfg.dtype) for w in ws]      # the owners' copies
    stage = [torch.empty_like(store[0]) for _ in range(2)]
    ctx = [torch.empty(taw.taw_layer_ctx_bytes(desc), dtype=torch.uint8, device="cuda") for _ in range(nl)]
    wsb = taw.taw_layer_workspace_bytes(desc)
    wsp = torch.empty(wsb, dtype=torch.uint8, device="cuda")
    rope = torch.empty(cfg.S * (cfg.head_dim // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, rope)
    G = [torch.zeros(P, dtype=torch.float32, device="cuda") for _ in range(nl)]
    compute, side = torch.cuda.current_stream(), torch.cuda.Stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    order = list(range(nl)) + list(reversed(range(nl)))          # layer whose weights each step needs
    for b in range(2):
        consumed[b].record(compute)
    taw.taw_weight_stage(stage[0], store[order[0]], P * 2, side, consumed[0], ready[0])
    acts = [U.to_dev(x, cfg.dtype)]
    grad = U.to_dev(dy, cfg.dtype)
    for i, l in enumerate(order):
        buf = i & 1
        if i + 1 < len(order):                                    # next step's weights into the other buffer
            taw.taw_weight_stage(stage[buf ^ 1], store[order[i + 1]], P * 2, side, consumed[buf ^ 1], ready[buf ^ 1])
        compute.wait_event(ready[buf])
        if i < nl:
            y = torch.empty_like(acts[0])
            taw.taw_layer_fwd(desc, stage[buf], rope, acts[l], y, ctx[l], wsp, wsb, compute)
            acts.append(y)
        else:
            dx = torch.empty_like(grad)
            taw.taw_layer_bwd(desc, stage[buf], rope, acts[l], grad, ctx[l], dx, G[l], wsp, wsb, compute)
            grad = dx
        consumed[buf].record(compute)
    torch.cuda.synchronize()
    e_y, e_dx = U.tensor_scale_err(U.from_dev(acts[nl]), y_ref), U.tensor_scale_err(U.from_dev(grad), dx_ref)
    print(f"4 chained layers: y={e_y:.2e} dx={e_dx:.2e}", flush=True)
    assert e_y < 2e-2 and e_dx < 2e-2
    for l in range(nl):
        got = {k: v.astype(np.float64) for k, v in I.unpack_shard(G[l].cpu().numpy(), lay, cfg).items()}
        for k in G_ref[l]:
            e = U.tensor_scale_err(got[k], G_ref[l][k])
            assert e < 2e-2, (l, k, e)


def test_bf16_microbatch_accumulation_with_staging(taw):
    """Config 5's pattern at reduced width (bf16, MFMA kernels): one layer, four micro-batches, the
    weight gradients accumulated by the backward's epilogue into the fp32 shard, while the next
    layer's chunk is staged on a side stream."""
    import torch
    from oracle import decoder_layer as O
    cfg = I.LayerConfig("mb4", I.BF16, 1, 384, 256, 2, 128, 520, sigma_w=0.05, n_microbatches=4)
    w = I.make_weights(cfg, 0, gamma_jitter=0.1)
    w64 = I.weights_to_f64(w, cfg.dtype)
    L = U.DeviceLayer(taw, cfg, flags=taw.TAW_ACCUMULATE)
    L.set_weights(w)
    nxt = U.to_dev(I.pack_chunk(I.make_weights(cfg, 0, layer=1), L.layout, L.layout["total_elems"], cfg.dtype), cfg.dtype)
    staged = torch.empty_like(nxt)
    side = torch.cuda.Stream()
    taw.taw_weight_stage(staged, nxt, nxt.numel() * 2, side, None, None)
    Gsum = None
    for mb in range(4):
        x, dy = I.make_activations(cfg, 0, mb=mb)
        xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
        y = L.fwd(xd)
        dx = L.bwd(xd, dyd)
        yr, cache = O.layer_fwd(w64, I.to_f64(x, cfg.dtype), cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
        dxr, G = O.layer_bwd(w64, cache, I.to_f64(dy, cfg.dtype))
        assert U.tensor_scale_err(U.from_dev(y), yr) < 2e-2 and U.tensor_scale_err(U.from_dev(dx), dxr) < 2e-2
        Gsum = G if Gsum is None else {k: O.grad_accum(Gsum[k], G[k]) for k in G}
    got = L.grads()
    for k in Gsum:
        assert U.tensor_scale_err(got[k], Gsum[k]) < 2e-2, k
    torch.cuda.synchronize()
    assert torch.equal(staged, nxt)


@pytest.mark.parametrize("cfg", [I.CONFIGS["C1"], I.LayerConfig("recompute-bf16", I.BF16, 2, 333, 256, 2, 128, 392, sigma_w=0.05)],
                         ids=["fp32", "bf16"])
def test_recompute_mode_gives_the_same_results(taw, cfg):
    """Activation checkpointing (TAW_RECOMPUTE): the forward keeps only x, the backward rebuilds the
    intermediates in the workspace.  Results against the oracle as in the default mode, and bit-identical
    to the default mode's own results (the same kernels on the same values)."""
    import torch
    w = I.make_weights(cfg, 3, gamma_jitter=0.1)
    x, dy = I.make_activations(cfg, 3)
    xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
    outs = []
    for flags in (0, taw.TAW_RECOMPUTE):
        L = U.DeviceLayer(taw, cfg, flags=flags)
        L.set_weights(w)
        y = L.fwd(xd)
        L.ws.fill_(0x5A)                    # nothing of the forward may survive in the workspace
        dx = L.bwd(xd, dyd)
        torch.cuda.synchronize()
        outs.append((y, dx, L.G.clone()))
    assert taw.taw_layer_ctx_bytes(taw.desc_from_config(cfg, taw.TAW_RECOMPUTE)) == 0
    for a, b in zip(outs[0], outs[1]):
        assert torch.equal(a, b)
    w64 = I.weights_to_f64(w, cfg.dtype)
    from oracle import decoder_layer as O
    yr, cache = O.layer_fwd(w64, I.to_f64(x, cfg.dtype), cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    dxr, _ = O.layer_bwd(w64, cache, I.to_f64(dy, cfg.dtype))
    assert U.tensor_scale_err(U.from_dev(outs[1][0]), yr) < U.TOL[cfg.dtype]
    assert U.tensor_scale_err(U.from_dev(outs[1][1]), dxr) < U.TOL[cfg.dtype]
