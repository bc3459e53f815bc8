"""Parity at the sizes the benchmark runs, in the launch configuration it times (the layer calls
and the kernel entry points of the C ABI on the C2 .. C5 shapes).

C2 (T = 8192) is small enough for the complete fp64 oracle: every output is compared element by
element.  At the C3, C4 and C5 widths the oracle evaluates sampled outputs one by one from the
plain definition: rows of y and the tail of dx of the whole layer; 8 x 8 blocks of every GEMM
output (the forward projections, the rotated qkv projection, and the paired input-gradient /
weight-gradient launch of every backward linear); attention rows and the tail of the attention
gradients, with and without the rotary backward; rows of the row-wise kernels; the RMSNorm gain
gradient over all tokens.  Large operands of the kernel-level cases are drawn on the device by the
seeded generator of the inputs module and only the slices the oracle needs come back to the host.
"""
import numpy as np
import pytest

from oracle import decoder_layer as O
from paper_2511_09741_amd import inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu

C3 = I.CONFIGS["C3"]
BF = I.BF16
TOL = U.TOL[BF]
WIDTHS = ["C3", "C4", "C5"]       # H = 4096 / 5120 / 8192, 32 / 40 / 64 heads, I = 11008 / 13824 / 22016, B = 1 / 2 / 1


def f64(t):
    """device tensor (any slice) -> fp64 numpy"""
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def test_c2_layer_against_the_complete_oracle(taw):
    """One forward + backward of the C2 layer, every element of y, dx and the six gradient tensors."""
    U.check_layer(taw, I.CONFIGS["C2"], seed=0)


@pytest.mark.parametrize("width", ["C3", "C4", "C5"])
def test_layer_sampled_rows_and_backward_tail(taw, width):
    """The whole layer at the widths of C3, C4 and C5 through taw_layer_fwd and taw_layer_bwd: y at sampled token rows
    (first, last, both sides of tile boundaries) of the last batch element and dx at its last 256 positions, which the
    oracle obtains from the plain definition as a closed sub-problem (a query's gradient needs its own row of
    probabilities; keys at u >= t0 are seen by the queries t >= t0 only)."""
    import torch
    cfg = I.CONFIGS[width]
    w = I.make_weights(cfg, 0)
    x, dy = I.make_activations(cfg, 0)
    L = U.DeviceLayer(taw, cfg)
    L.set_weights(w)
    xd, dyd = U.to_dev(x, cfg.dtype), U.to_dev(dy, cfg.dtype)
    y = L.fwd(xd)
    dx = L.bwd(xd, dyd)
    torch.cuda.synchronize()
    b = cfg.B - 1
    w64 = I.weights_to_f64(w, cfg.dtype)
    del w
    x64 = I.to_f64(x[b], cfg.dtype)
    S = cfg.S
    rows = np.array([0, 1, 63, 64, 255, 256, 4097, S // 2 - 1, S // 2, S - 257, S - 1])
    yr = O.layer_fwd_rows(w64, x64, rows, cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    e_y = U.tensor_scale_err(f64(y[b, torch.from_numpy(rows).cuda()]), yr)
    print(f"{width} y rows: {e_y:.2e}", flush=True)
    assert e_y < TOL
    t0 = S - 256
    dxr = O.layer_bwd_tail(w64, x64, I.to_f64(dy[b], cfg.dtype), t0, cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    e_dx = U.tensor_scale_err(f64(dx[b, t0:]), dxr)
    print(f"{width} dx tail (last 256 positions): {e_dx:.2e}", flush=True)
    assert e_dx < TOL


def _blocks(rng, M, N, n=6, bs=8):
    """index blocks: the four corners of the output (first / last tiles) and n random interior ones; column
    starts are even, so a block holds whole rotary pairs"""
    r = [np.arange(0, bs), np.arange(M - bs, M)]
    c = [np.arange(0, bs), np.arange(N - bs, N)]
    out = [(a, b) for a in r for b in c]
    for _ in range(n):
        i, j = int(rng.integers(0, M - bs)), 2 * int(rng.integers(0, (N - bs) // 2))
        out.append((np.arange(i, i + bs), np.arange(j, j + bs)))
    return out


def _idx(a):
    import torch
    return torch.from_numpy(np.asarray(a)).cuda()


def _block_err(pairs):
    """tensor-scale error over a list of (got, ref) blocks of one output"""
    worst = max(float(np.max(np.abs(g - r))) for g, r in pairs)
    scale = max(float(np.max(np.abs(r))) for _, r in pairs)
    return worst / scale


def _fwd_gemms(cfg):
    T, H, Iw = cfg.T, cfg.H, cfg.I
    return [("o_proj+res", T, H, H, True), ("gate_up", T, 2 * Iw, H, False), ("down+res", T, H, Iw, True)]


@pytest.mark.parametrize("width", WIDTHS)
def test_forward_gemms_sampled_blocks(taw, width):
    """The forward projections (C = A B^T, with the residual where the layer has one) at the layer's
    shapes: sampled 8 x 8 output blocks against fp64 dot products."""
    import torch
    cfg = I.CONFIGS[width]
    for name, M, N, K, res in _fwd_gemms(cfg):
        A = I.device_normal((M, K), seed=11, std=1.0)
        B = I.device_normal((N, K), seed=12, std=0.02)
        C = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
        R = I.device_normal((M, N), seed=14, std=1.0) if res else None
        taw.taw_op_gemm(BF, taw.TAW_GEMM_NT, M, N, K, A, K, B, K, C, N, BF, 0, R, N, taw.TAW_IMPL_MFMA)
        torch.cuda.synchronize()
        rng = np.random.default_rng(M + N + K)
        pairs = []
        for rows, cols in _blocks(rng, M, N):
            ri, ci = _idx(rows), _idx(cols)
            ref = f64(A[ri, :]) @ f64(B[ci, :]).T
            if res:
                ref = ref + f64(R[ri][:, ci])
            pairs.append((f64(C[ri][:, ci]), ref))
        err = _block_err(pairs)
        print(f"{width} gemm {name} {M}x{N}x{K}: {err:.2e}", flush=True)
        assert err < TOL
        del A, B, C, R


@pytest.mark.parametrize("width", WIDTHS)
def test_qkv_projection_with_rotary_epilogue_sampled_blocks(taw, width):
    """qkv = xn Wqkv^T with q and k rotated by position, as the forward runs it (the rotation sits in the
    GEMM's epilogue at these shapes): sampled blocks against fp64 dot products rotated by the oracle's angles.
    With B = 2 the positions restart at the second batch element."""
    import torch
    cfg = I.CONFIGS[width]
    T, H, S, d = cfg.T, cfg.H, cfg.S, cfg.head_dim
    xn = I.device_normal((T, H), seed=15, std=1.0)
    Wq = I.device_normal((3 * H, H), seed=16, std=0.02)
    qkv = torch.empty((T, 3 * H), dtype=torch.bfloat16, device="cuda")
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(taw.desc_from_config(cfg, 0), table)
    taw.taw_op_qkv_rope(BF, cfg.B, S, cfg.n_heads, d, xn, Wq, qkv, table, taw.TAW_IMPL_MFMA)
    torch.cuda.synchronize()
    phi = O.rope_angles(S, d, cfg.rope_theta)
    rng = np.random.default_rng(T + H)
    blocks = _blocks(rng, T, 3 * H, n=8)
    blocks.append((np.arange(S - 4, S + 4) % T, np.arange(H - 4, H + 4)))       # across the batch boundary (B = 2) and the q | k boundary
    pairs = []
    for rows, cols in blocks:
        ri, ci = _idx(rows), _idx(cols)
        raw = f64(xn[ri, :]) @ f64(Wq[ci, :]).T
        ref = raw.copy()
        for a in range(0, len(cols), 2):
            c0 = int(cols[a])
            if c0 >= 2 * H:
                continue                                                       # v is not rotated
            ang = phi[rows % S, (c0 % d) // 2]
            ref[:, a] = raw[:, a] * np.cos(ang) - raw[:, a + 1] * np.sin(ang)
            ref[:, a + 1] = raw[:, a] * np.sin(ang) + raw[:, a + 1] * np.cos(ang)
        pairs.append((f64(qkv[ri][:, ci]), ref))
    err = _block_err(pairs)
    print(f"{width} qkv + rotary: {err:.2e}", flush=True)
    assert err < TOL


def _bwd_linears(cfg):
    T, H, Iw = cfg.T, cfg.H, cfg.I
    return [("down", T, H, Iw), ("gate_up", T, 2 * Iw, H), ("o_proj", T, H, H), ("qkv", T, 3 * H, H)]    # (name, T, N = out, K = in)


@pytest.mark.parametrize("width", WIDTHS)
def test_backward_linears_paired_launch_sampled_blocks(taw, width):
    """Every linear's backward as taw_layer_bwd launches it (the input gradient dx = dy W and the
    weight gradient G += dy^T x in one grid): sampled blocks of both outputs against fp64 dot products;
    G starts from random values and is accumulated into."""
    import torch
    cfg = I.CONFIGS[width]
    for name, T, N, K in _bwd_linears(cfg):
        dyy = I.device_normal((T, N), seed=17, std=1.0)
        W = I.device_normal((N, K), seed=18, std=0.02)
        x = I.device_normal((T, K), seed=19, std=1.0)
        G = I.device_normal((N, K), seed=20, std=1.0, dtype=torch.float32)
        G0 = G.clone()
        dx = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
        taw.taw_op_linear_bwd(BF, T, N, K, dyy, W, x, dx, G, 1, taw.TAW_IMPL_MFMA)
        torch.cuda.synchronize()
        rng = np.random.default_rng(T + N + K)
        p_dx, p_g = [], []
        for rows, cols in _blocks(rng, T, K):
            ri, ci = _idx(rows), _idx(cols)
            p_dx.append((f64(dx[ri][:, ci]), f64(dyy[ri, :]) @ f64(W[:, ci])))
        for rows, cols in _blocks(rng, N, K):
            ri, ci = _idx(rows), _idx(cols)
            p_g.append((f64(G[ri][:, ci]), f64(dyy[:, ri]).T @ f64(x[:, ci]) + f64(G0[ri][:, ci])))
        e_dx, e_g = _block_err(p_dx), _block_err(p_g)
        print(f"{width} linear backward {name} T={T} N={N} K={K}: dx={e_dx:.2e} G={e_g:.2e}", flush=True)
        assert e_dx < TOL and e_g < 1e-4
        del dyy, W, x, G, G0, dx


@pytest.mark.parametrize("T,N,K", [(2080, 256, 256), (4096, 264, 520), (65536, 1024, 1024), (65536, 1024, 2816), (65536, 2048, 2048), (65536, 6144, 2048)],
                         ids=lambda v: str(v))
def test_backward_linear_weight_gradient_cut_along_tokens(taw, T, N, K):
    """Narrow linears (the 1024- and 2048-wide models of the paper's throughput table, and two small ragged shapes): the
    weight gradient computed in ranges of tokens and summed by a second kernel.  Sampled blocks of G and dx against fp64
    dot products, with and without accumulation; the same call twice gives the same bits; and the uncut launch (no
    scratch) agrees to fp32 summation order."""
    import torch
    n_scr = taw.taw_op_linear_bwd_scratch_floats(T, N, K)
    assert n_scr > 0 and n_scr % (N * K) == 0 and 2 <= n_scr // (N * K) <= 32
    scratch = torch.full((n_scr,), float("nan"), dtype=torch.float32, device="cuda")     # stale contents must not matter
    dyy = I.device_normal((T, N), seed=27, std=1.0)
    W = I.device_normal((N, K), seed=28, std=0.02)
    x = I.device_normal((T, K), seed=29, std=1.0)
    G0 = I.device_normal((N, K), seed=30, std=1.0, dtype=torch.float32)
    dx = torch.empty((T, K), dtype=torch.bfloat16, device="cuda")
    rng = np.random.default_rng(T + N + K)
    for accumulate in (1, 0):
        G = G0.clone()
        taw.taw_op_linear_bwd(BF, T, N, K, dyy, W, x, dx, G, accumulate, taw.TAW_IMPL_MFMA, scratch=scratch)
        G_again, dx_again = G0.clone(), torch.empty_like(dx)
        taw.taw_op_linear_bwd(BF, T, N, K, dyy, W, x, dx_again, G_again, accumulate, taw.TAW_IMPL_MFMA, scratch=scratch)
        G_uncut = G0.clone()
        taw.taw_op_linear_bwd(BF, T, N, K, dyy, W, x, dx_again, G_uncut, accumulate, taw.TAW_IMPL_MFMA)
        torch.cuda.synchronize()
        assert torch.equal(G, G_again) and torch.equal(dx, dx_again)
        scale = float(G_uncut.abs().max())
        assert float((G - G_uncut).abs().max()) < 2e-5 * scale
        p_dx, p_g = [], []
        for rows, cols in _blocks(rng, T, K):
            ri, ci = _idx(rows), _idx(cols)
            p_dx.append((f64(dx[ri][:, ci]), f64(dyy[ri, :]) @ f64(W[:, ci])))
        for rows, cols in _blocks(rng, N, K):
            ri, ci = _idx(rows), _idx(cols)
            p_g.append((f64(G[ri][:, ci]), f64(dyy[:, ri]).T @ f64(x[:, ci]) + accumulate * f64(G0[ri][:, ci])))
        e_dx, e_g = _block_err(p_dx), _block_err(p_g)
        print(f"linear backward, cut into {n_scr // (N * K)}: T={T} N={N} K={K} accumulate={accumulate}: dx={e_dx:.2e} G={e_g:.2e}", flush=True)
        assert e_dx < TOL and e_g < 1e-4


@pytest.mark.parametrize("width,form", [(w, 5) for w in WIDTHS] + [("C3", 2), ("C3", 3), ("C4", 3)],
                         ids=[w + "-stored" for w in WIDTHS] + ["C3-split", "C3-fused", "C4-fused"])
def test_attention_sampled(taw, width, form):
    """Attention at the layer's shape (all heads, all batch elements in one launch): o and lse at
    sampled (batch, head, row); dq, dk, dv on the last 300 positions, once as gradients of the q, k
    passed in and once through the rotary backward (rope_table given).  The backward with stored dS (form 5, what
    taw_layer_bwd runs) at every width, where it must also equal the pair that recomputes the scores bit for bit
    over the whole of dq, dk, dv (the two contract in the same order); that pair (form 2) against the oracle at one width;
    the fused form with dQ slots (form 3) at two (16 and 4 key blocks per worker)."""
    import torch
    cfg = I.CONFIGS[width]
    B, S, nh, d = cfg.B, cfg.S, cfg.n_heads, cfg.head_dim
    H = nh * d
    qkv = I.device_normal((B * S, 3 * H), seed=21, std=0.5)
    dO = I.device_normal((B * S, H), seed=22, std=1.0)
    o = torch.empty((B * S, H), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    taw.taw_op_attn_fwd(BF, B, S, nh, d, qkv, o, lse, taw.TAW_IMPL_MFMA)
    dqkv = torch.empty_like(qkv)
    dqkv_rot = torch.empty_like(qkv)
    scratch = torch.empty(taw.taw_op_attn_bwd_scratch_floats(B, S, nh), dtype=torch.float32, device="cuda")
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(taw.desc_from_config(cfg, 0), table)
    taw.taw_op_attn_bwd(BF, B, S, nh, d, qkv, o, dO, lse, dqkv, scratch, None, form)
    taw.taw_op_attn_bwd(BF, B, S, nh, d, qkv, o, dO, lse, dqkv_rot, scratch, table, form)
    torch.cuda.synchronize()
    if form == 5:
        other = torch.empty_like(qkv)
        taw.taw_op_attn_bwd(BF, B, S, nh, d, qkv, o, dO, lse, other, scratch, table, 2)
        torch.cuda.synchronize()
        assert torch.equal(other, dqkv_rot)
        del other
    rows = np.array([0, 1, 63, 64, 255, 256, 257, 8191, 8192, S // 2 + 3617, S - 1 - 256, S - 1])
    t0 = S - 300
    phi = O.rope_angles(S, d, cfg.rope_theta)
    for b, h in ((0, 0), (B - 1, nh // 2 - 3), (B - 1, nh - 1)):
        sl = slice(b * S, (b + 1) * S)
        q, k, v = (f64(qkv[sl, p * H + h * d: p * H + (h + 1) * d]) for p in range(3))
        o_r, lse_r = O.attention_fwd_rows(q[rows], k, v, rows)
        e_o = U.tensor_scale_err(f64(o[sl, h * d:(h + 1) * d])[rows], o_r)
        e_l = float(np.max(np.abs(f64(lse.view(B, nh, S)[b, h])[rows] - lse_r)))
        dq_r, dk_r, dv_r = O.attention_bwd_tail(q, k, v, f64(dO[sl, h * d:(h + 1) * d]), t0)
        got = [f64(dqkv[b * S + t0:(b + 1) * S, p * H + h * d: p * H + (h + 1) * d]) for p in range(3)]
        e_dq, e_dk, e_dv = (U.tensor_scale_err(g, r) for g, r in zip(got, (dq_r, dk_r, dv_r)))
        got = [f64(dqkv_rot[b * S + t0:(b + 1) * S, p * H + h * d: p * H + (h + 1) * d]) for p in range(3)]
        rot = [O.rope_apply(z[None, :, None, :], phi[t0:], inverse=True)[0, :, 0, :] for z in (dq_r, dk_r)]
        e_rq, e_rk, e_rv = (U.tensor_scale_err(g, r) for g, r in zip(got, (rot[0], rot[1], dv_r)))
        print(f"{width} attention b={b} h={h}: o={e_o:.2e} lse={e_l:.2e} dq={e_dq:.2e} dk={e_dk:.2e} dv={e_dv:.2e} "
              f"| rotary backward: dq={e_rq:.2e} dk={e_rk:.2e} dv={e_rv:.2e}", flush=True)
        assert e_o < TOL and e_l < 2e-2 and e_dq < TOL and e_dk < TOL and e_dv < TOL
        assert e_rq < TOL and e_rk < TOL and e_rv < TOL


@pytest.mark.parametrize("width", WIDTHS)
def test_rmsnorm_sampled_rows_and_full_gain_gradient(taw, width):
    """RMSNorm forward / backward over all tokens at the layer's width (H = 5120 and 8192 take the
    kernel's LDS column-sum path): sampled token rows against the oracle, and the gain gradient
    (a sum over all tokens) in full."""
    import torch
    cfg = I.CONFIGS[width]
    T, H = cfg.T, cfg.H
    rows = np.array([0, 1, 3, 4, 1023, 1024, 2047, 2048, T // 2 + 1, T - 4, T - 1])
    ri = _idx(rows)
    x = I.device_normal((T, H), seed=31, std=1.0)
    gam = (I.device_normal((H,), seed=32, std=0.1, dtype=torch.float32) + 1.0).to(torch.bfloat16)
    out = torch.empty_like(x)
    r = torch.empty(T, dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_fwd(BF, T, H, x, gam, cfg.rms_eps, out, r)
    torch.cuda.synchronize()
    ref, r_ref = O.rmsnorm_fwd(f64(x[ri]), f64(gam), cfg.rms_eps)
    assert U.tensor_scale_err(f64(out[ri]), ref) < 1e-2
    assert U.tensor_scale_err(f64(r[ri]), r_ref) < 1e-5
    dout = I.device_normal((T, H), seed=33, std=1.0)
    dres = I.device_normal((T, H), seed=34, std=1.0)
    dz = torch.empty_like(x)
    dgam = torch.zeros(H, dtype=torch.float32, device="cuda")
    scratch = torch.empty(taw.taw_op_rmsnorm_bwd_scratch_floats(H), dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_bwd(BF, T, H, dout, x, r, gam, dres, dz, dgam, 0, scratch)
    torch.cuda.synchronize()
    dz_ref, _ = O.rmsnorm_bwd(f64(dout[ri]), f64(x[ri]), r_ref, f64(gam))
    e_dz = U.tensor_scale_err(f64(dz[ri]), dz_ref + f64(dres[ri]))
    dg_ref = np.zeros(H)
    for s0 in range(0, T, 4096):                      # column sums over all tokens, a slab at a time (the oracle's own r)
        xs, ds = f64(x[s0:s0 + 4096]), f64(dout[s0:s0 + 4096])
        _, rs = O.rmsnorm_fwd(xs, f64(gam), cfg.rms_eps)
        dg_ref += O.rmsnorm_bwd(ds, xs, rs, f64(gam))[1]
    e_dg = U.tensor_scale_err(f64(dgam), dg_ref)
    print(f"{width} rmsnorm H={H} T={T}: dz={e_dz:.2e} dgamma={e_dg:.2e}", flush=True)
    assert e_dz < 1e-2 and e_dg < 1e-3


@pytest.mark.parametrize("width", WIDTHS)
def test_rope_and_swiglu_sampled_rows(taw, width):
    """The standalone rotary kernel (forward) and SwiGLU forward / backward at the layer's shapes."""
    import torch
    cfg = I.CONFIGS[width]
    T, H, Iw, S, d = cfg.T, cfg.H, cfg.I, cfg.S, cfg.head_dim
    rows = np.array([0, 1, 3, 4, 1023, 1024, T // 2 + 1, T - 4, T - 1])
    ri = _idx(rows)
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(taw.desc_from_config(cfg, 0), table)
    qkv = I.device_normal((T, 3 * H), seed=35, std=1.0)
    before = f64(qkv[ri])
    taw.taw_op_rope(BF, cfg.B, S, 2 * H, d, qkv, 3 * H, table, 0)
    torch.cuda.synchronize()
    phi = O.rope_angles(S, d, cfg.rope_theta)[rows % S]    # the sampled rows' own positions
    z = before[:, :2 * H].reshape(len(rows), 2 * cfg.n_heads, d)
    ref = np.empty_like(z)
    c, s_ = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    ref[..., 0::2] = z[..., 0::2] * c - z[..., 1::2] * s_
    ref[..., 1::2] = z[..., 0::2] * s_ + z[..., 1::2] * c
    got = f64(qkv[ri])
    assert U.tensor_scale_err(got[:, :2 * H], ref.reshape(len(rows), 2 * H)) < 1e-2
    assert np.array_equal(got[:, 2 * H:], before[:, 2 * H:])             # v untouched
    del qkv
    gu = I.device_normal((T, 2 * Iw), seed=36, std=1.5)
    da = I.device_normal((T, Iw), seed=37, std=1.0)
    a = torch.empty((T, Iw), dtype=torch.bfloat16, device="cuda")
    dgu = torch.empty_like(gu)
    taw.taw_op_swiglu_fwd(BF, T, Iw, gu, a)
    taw.taw_op_swiglu_bwd(BF, T, Iw, da, gu, dgu)
    torch.cuda.synchronize()
    g, u = f64(gu[ri])[:, :Iw], f64(gu[ri])[:, Iw:]
    assert U.tensor_scale_err(f64(a[ri]), O.swiglu_fwd(g, u)) < 1e-2
    dg, du = O.swiglu_bwd(f64(da[ri]), g, u)
    assert U.tensor_scale_err(f64(dgu[ri]), np.concatenate([dg, du], axis=1)) < 1e-2


@pytest.mark.parametrize("width", ["C3", "C5"])
def test_grad_accum_at_chunk_size(taw, width):
    """taw_grad_accum over a whole chunk (202 M elements at the 7B width, 810 M at the 70B width),
    fp32 and bf16 sources."""
    import torch
    desc = taw.desc_from_config(I.CONFIGS[width], 0)
    P = taw.taw_layer_weight_layout(desc)["total_elems"]
    G = I.device_normal((P,), seed=41, std=1.0, dtype=torch.float32)
    for src_dt, tdt in ((taw.TAW_F32, torch.float32), (taw.TAW_BF16, torch.bfloat16)):
        g = I.device_normal((P,), seed=42, std=1.0, dtype=tdt)
        G0 = G.clone()
        taw.taw_grad_accum(G, g, src_dt, P, 0.25)
        torch.cuda.synchronize()
        for part in (slice(0, 5_000_000), slice(P - 5_000_000, P)):     # the head of the chunk and its tail, element by element
            ref = O.grad_accum(f64(G0[part]), f64(g[part]), 0.25)
            assert U.tensor_scale_err(f64(G[part]), ref) < 1e-6
        del g, G0
