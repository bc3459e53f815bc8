"""Parity at the sizes the benchmark runs, in the launch configuration it times (the layer calls
and the kernel entry points of the C ABI on the C2 / C3 shapes).

C2 (T = 8192) is small enough for the complete fp64 oracle: every output is compared element
by element.  At C3 (T = 32768) the oracle evaluates sampled outputs one by one from the plain
definition: rows of y; blocks of GEMM outputs; attention rows and the tail of the attention
gradients; rows of the row-wise kernels; column sums over all tokens.  Large inputs for the
kernel-level cases are drawn on the device by the seeded generator of the inputs module and
only the slices the oracle needs come back to the host.
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


def f64(t):
    """device tensor (any slice) -> fp64 numpy"""
    import torch
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def test_c2_layer_against_the_complete_oracle(taw):
    """One forward + backward of the C2 layer, every element of y, dx and the six gradient tensors."""
    U.check_layer(taw, I.CONFIGS["C2"], seed=0)


def test_c3_forward_sampled_rows(taw):
    """y of the C3 layer at sampled token rows (first, last, both sides of tile boundaries)."""
    import torch
    cfg = C3
    w = I.make_weights(cfg, 0)
    x, _ = I.make_activations(cfg, 0)
    L = U.DeviceLayer(taw, cfg)
    L.set_weights(w)
    y = L.fwd(U.to_dev(x, cfg.dtype))
    torch.cuda.synchronize()
    rows = np.array([0, 1, 63, 64, 255, 256, 4097, 16383, 16384, 32511, 32767])
    yr = O.layer_fwd_rows(I.weights_to_f64(w, cfg.dtype), I.to_f64(x, cfg.dtype)[0], rows, cfg.n_heads, cfg.rope_theta, cfg.rms_eps)
    err = U.tensor_scale_err(f64(y[0, torch.from_numpy(rows).cuda()]), yr)
    print(f"C3 y rows: {err:.2e}", flush=True)
    assert err < TOL


def _blocks(rng, M, N, n=6, bs=8):
    """index blocks: the four corners of the output (first / last tiles) and n random interior ones"""
    r = [np.arange(0, bs), np.arange(M - bs, M)]
    c = [np.arange(0, bs), np.arange(N - bs, N)]
    out = [(a, b) for a in r for b in c]
    for _ in range(n):
        i, j = int(rng.integers(0, M - bs)), int(rng.integers(0, N - bs))
        out.append((np.arange(i, i + bs), np.arange(j, j + bs)))
    return out


T3, H3, I3 = C3.T, C3.H, C3.I
GEMMS_C3 = [  # (name, mode, M, N, K, fp32 out + accumulate, residual)
    ("qkv", 0, T3, 3 * H3, H3, False, False),
    ("o_proj+res", 0, T3, H3, H3, False, True),
    ("gate_up", 0, T3, 2 * I3, H3, False, False),
    ("down+res", 0, T3, H3, I3, False, True),
    ("d_a", 1, T3, I3, H3, False, False),
    ("d_hn", 1, T3, H3, 2 * I3, False, False),
    ("d_xn", 1, T3, H3, 3 * H3, False, False),
    ("G.w_down", 2, H3, I3, T3, True, False),
    ("G.w_gate_up", 2, 2 * I3, H3, T3, True, False),
    ("G.w_qkv", 2, 3 * H3, H3, T3, True, False),
]


@pytest.mark.parametrize("name,mode,M,N,K,f32acc,res", GEMMS_C3, ids=[g[0] for g in GEMMS_C3])
def test_c3_gemm_sampled_blocks(taw, name, mode, M, N, K, f32acc, res):
    """The C3 layer's GEMM shapes: sampled 8 x 8 output blocks against fp64 dot products."""
    import torch
    a_shape = (K, M) if mode == 2 else (M, K)
    b_shape = (N, K) if mode == 0 else (K, N)
    A = I.device_normal(a_shape, seed=11, std=1.0)
    B = I.device_normal(b_shape, seed=12, std=0.02 if mode != 2 else 1.0)
    c_dt = torch.float32 if f32acc else torch.bfloat16
    C = I.device_normal((M, N), seed=13, std=1.0, dtype=c_dt) if f32acc else torch.empty((M, N), dtype=c_dt, device="cuda")
    C0 = C.clone() if f32acc else None
    R = I.device_normal((M, N), seed=14, std=1.0) if res else None
    taw.taw_op_gemm(BF, mode, M, N, K, A, a_shape[1], B, b_shape[1], C, N, taw.TAW_F32 if f32acc else BF, int(f32acc), R, N, taw.TAW_IMPL_MFMA)
    torch.cuda.synchronize()
    rng = np.random.default_rng(M + N + K)
    worst, scale = 0.0, 0.0
    for rows, cols in _blocks(rng, M, N):
        ri, ci = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
        a = f64(A[:, ri]).T if mode == 2 else f64(A[ri, :])
        b = f64(B[ci, :]).T if mode == 0 else f64(B[:, ci])
        ref = a @ b
        if f32acc:
            ref = ref + f64(C0[ri][:, ci])
        if res:
            ref = ref + f64(R[ri][:, ci])
        got = f64(C[ri][:, ci])
        worst = max(worst, float(np.max(np.abs(got - ref))))
        scale = max(scale, float(np.max(np.abs(ref))))
    err = worst / scale
    print(f"C3 gemm {name}: {err:.2e}", flush=True)
    assert err < (1e-4 if f32acc else TOL)


def test_c3_attention_sampled(taw):
    """Attention at the C3 shape: o and lse at sampled (head, row) pairs; dq, dk, dv on the last 300
    positions (dq of a query needs its own row of probabilities only; a key at u >= t0 is seen by the
    queries t >= t0 only)."""
    import torch
    B, S, nh, d = 1, C3.S, C3.n_heads, C3.head_dim
    H = nh * d
    qkv = I.device_normal((S, 3 * H), seed=21, std=0.5)
    dO = I.device_normal((S, H), seed=22, std=1.0)
    o = torch.empty((S, H), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    taw.taw_op_attn_fwd(BF, B, S, nh, d, qkv, o, lse, taw.TAW_IMPL_MFMA)
    dqkv = torch.empty_like(qkv)
    scratch = torch.empty(taw.taw_op_attn_bwd_scratch_floats(B, S, nh), dtype=torch.float32, device="cuda")
    taw.taw_op_attn_bwd(BF, B, S, nh, d, qkv, o, dO, lse, dqkv, scratch, None, taw.TAW_IMPL_MFMA)
    torch.cuda.synchronize()
    rows = np.array([0, 1, 63, 64, 255, 256, 257, 8191, 8192, 20000, 32767 - 256, 32767])
    t0 = S - 300
    for h in (0, 13, 31):
        q, k, v = (f64(qkv[:, p * H + h * d: p * H + (h + 1) * d]) for p in range(3))
        o_r, lse_r = O.attention_fwd_rows(q[rows], k, v, rows)
        e_o = U.tensor_scale_err(f64(o[:, h * d:(h + 1) * d])[rows], o_r)
        e_l = float(np.max(np.abs(f64(lse.view(nh, S)[h])[rows] - lse_r)))
        dq_r, dk_r, dv_r = O.attention_bwd_tail(q, k, v, f64(dO[:, h * d:(h + 1) * d]), t0)
        got = [f64(dqkv[t0:, p * H + h * d: p * H + (h + 1) * d]) for p in range(3)]
        e_dq, e_dk, e_dv = (U.tensor_scale_err(g, r) for g, r in zip(got, (dq_r, dk_r, dv_r)))
        print(f"C3 attention head {h}: o={e_o:.2e} lse={e_l:.2e} dq={e_dq:.2e} dk={e_dk:.2e} dv={e_dv:.2e}", flush=True)
        assert e_o < TOL and e_l < 2e-2 and e_dq < TOL and e_dk < TOL and e_dv < TOL


def test_c3_rowwise_kernels_sampled(taw):
    """RMSNorm forward / backward, rotary embedding and SwiGLU at the C3 shapes: sampled token rows
    against the oracle, and the RMSNorm gain gradient (a sum over all 32768 tokens) in full."""
    import torch
    T, H, Iw, S, d = C3.T, C3.H, C3.I, C3.S, C3.head_dim
    rows = np.array([0, 1, 3, 4, 1023, 1024, 16385, 32764, 32767])
    ri = torch.from_numpy(rows).cuda()
    x = I.device_normal((T, H), seed=31, std=1.0)
    gam = I.device_normal((H,), seed=32, std=0.1) + 1.0
    gam = gam.to(torch.bfloat16)
    out = torch.empty_like(x)
    r = torch.empty(T, dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_fwd(BF, T, H, x, gam, C3.rms_eps, out, r)
    torch.cuda.synchronize()
    ref, r_ref = O.rmsnorm_fwd(f64(x[ri]), f64(gam), C3.rms_eps)
    assert U.tensor_scale_err(f64(out[ri]), ref) < 1e-2
    assert U.tensor_scale_err(f64(r[ri]), r_ref) < 1e-5
    # backward: dz rows and the complete dgamma (the oracle's own r for every row)
    dout = I.device_normal((T, H), seed=33, std=1.0)
    dres = I.device_normal((T, H), seed=34, std=1.0)
    dz = torch.empty_like(x)
    dgam = torch.zeros(H, dtype=torch.float32, device="cuda")
    scratch = torch.empty(taw.taw_op_rmsnorm_bwd_scratch_floats(H), dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_bwd(BF, T, H, dout, x, r, gam, dres, dz, dgam, 0, scratch)
    torch.cuda.synchronize()
    dz_ref, _ = O.rmsnorm_bwd(f64(dout[ri]), f64(x[ri]), r_ref, f64(gam))
    assert U.tensor_scale_err(f64(dz[ri]), dz_ref + f64(dres[ri])) < 1e-2
    dg_ref = np.zeros(H)
    for t0 in range(0, T, 4096):                      # column sums over all tokens, a slab at a time
        xs, ds = f64(x[t0:t0 + 4096]), f64(dout[t0:t0 + 4096])
        _, rs = O.rmsnorm_fwd(xs, f64(gam), C3.rms_eps)
        dg_ref += O.rmsnorm_bwd(ds, xs, rs, f64(gam))[1]
    assert U.tensor_scale_err(f64(dgam), dg_ref) < 1e-3
    # rotary embedding on q | k of a [T, 3H] matrix, forward then inverse
    desc = taw.desc_from_config(C3, 0)
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, table)
    qkv = I.device_normal((T, 3 * H), seed=35, std=1.0)
    before = f64(qkv[ri])
    taw.taw_op_rope(BF, C3.B, S, 2 * H, d, qkv, 3 * H, table, 0)
    torch.cuda.synchronize()
    phi = O.rope_angles(S, d, C3.rope_theta)[rows]       # the sampled rows' own positions (B = 1: row = position)
    z = before[:, :2 * H].reshape(len(rows), 2 * C3.n_heads, d)
    ref = np.empty_like(z)
    c, s_ = np.cos(phi)[:, None, :], np.sin(phi)[:, None, :]
    ref[..., 0::2] = z[..., 0::2] * c - z[..., 1::2] * s_
    ref[..., 1::2] = z[..., 0::2] * s_ + z[..., 1::2] * c
    got = f64(qkv[ri])
    assert U.tensor_scale_err(got[:, :2 * H], ref.reshape(len(rows), 2 * H)) < 1e-2
    assert np.array_equal(got[:, 2 * H:], before[:, 2 * H:])             # v untouched
    # SwiGLU forward / backward
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


def test_grad_accum_at_chunk_size(taw):
    """taw_grad_accum over a whole 7B-shaped chunk (202 M elements), fp32 and bf16 sources."""
    import torch
    desc = taw.desc_from_config(C3, 0)
    P = taw.taw_layer_weight_layout(desc)["total_elems"]
    G = I.device_normal((P,), seed=41, std=1.0, dtype=torch.float32)
    for src_dt, tdt in ((taw.TAW_F32, torch.float32), (taw.TAW_BF16, torch.bfloat16)):
        g = I.device_normal((P,), seed=42, std=1.0, dtype=tdt)
        G0 = G.clone()
        taw.taw_grad_accum(G, g, src_dt, P, 0.25)
        torch.cuda.synchronize()
        sl = slice(P - 5_000_000, P)                     # the tail of the chunk and ...
        for part in (slice(0, 5_000_000), sl):           # ... its head, element by element
            ref = O.grad_accum(f64(G0[part]), f64(g[part]), 0.25)
            assert U.tensor_scale_err(f64(G[part]), ref) < 1e-6
