"""Each kernel on its own against the matching step of the oracle, through the C ABI."""
import numpy as np
import pytest

from oracle import decoder_layer as O
from paper_2511_09741_amd import inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu


def draw(rng, shape, dtype, scale=1.0):
    """random values already representable in the storage dtype: (storage array, fp64 values)"""
    a = (scale * rng.standard_normal(shape)).astype(np.float32)
    st = I.to_storage(a, dtype)
    return st, I.to_f64(st, dtype)


GEMM_SHAPES = [(64, 64, 64), (200, 136, 72), (8, 8, 8), (257, 264, 520), (1, 8, 16), (300, 40, 1000)]


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("M,N,K", GEMM_SHAPES)
def test_gemm_generic(taw, dtype, mode, M, N, K):
    _gemm_case(taw, dtype, mode, M, N, K, taw.TAW_IMPL_GENERIC, seed=M + N + K + mode)


def _gemm_case(taw, dtype, mode, M, N, K, impl, seed=0, c_f32=False, accumulate=False, residual=False):
    import torch
    rng = np.random.default_rng(seed)
    a_shape = (K, M) if mode == 2 else (M, K)
    b_shape = (N, K) if mode == 0 else (K, N)
    A, A64 = draw(rng, a_shape, dtype)
    B, B64 = draw(rng, b_shape, dtype)
    opA = A64.T if mode == 2 else A64
    opB = B64.T if mode == 0 else B64
    ref = opA @ opB
    c_dtype = I.F32 if c_f32 else dtype
    Cd = U.empty_dev((M, N), c_dtype)
    if accumulate:
        C0, C064 = draw(rng, (M, N), c_dtype, 3.0)
        Cd.copy_(U.to_dev(C0, c_dtype))
        ref = ref + C064
    Rd = None
    if residual:
        R, R64 = draw(rng, (M, N), c_dtype, 2.0)
        Rd = U.to_dev(R, c_dtype)
        ref = ref + R64
    Ad, Bd = U.to_dev(A, dtype), U.to_dev(B, dtype)
    taw.taw_op_gemm(dtype, mode, M, N, K, Ad, a_shape[1], Bd, b_shape[1], Cd, N, c_dtype, int(accumulate), Rd, N, impl)
    torch.cuda.synchronize()
    tol = 2e-2 if (dtype == I.BF16 and not c_f32) else 1e-4
    err = U.tensor_scale_err(U.from_dev(Cd), ref)
    assert err < tol, err
    return err


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
def test_gemm_generic_epilogues(taw, dtype):
    _gemm_case(taw, dtype, 0, 100, 72, 64, taw.TAW_IMPL_GENERIC, residual=True)
    _gemm_case(taw, dtype, 2, 72, 40, 333, taw.TAW_IMPL_GENERIC, c_f32=True, accumulate=True)
    _gemm_case(taw, dtype, 2, 72, 40, 333, taw.TAW_IMPL_GENERIC, c_f32=True, accumulate=False)


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("T,H", [(5, 64), (130, 4096), (33, 100), (7, 1000), (2, 8192 if True else 0)])
def test_rmsnorm_fwd_bwd(taw, dtype, T, H):
    import torch
    if dtype == I.F32 and H > 4096:
        H = 4096
    rng = np.random.default_rng(T * H)
    x, x64 = draw(rng, (T, H), dtype)
    g, g64 = draw(rng, (H,), dtype, 0.3)
    g64 = g64 + 1.0
    g = I.to_storage((g64).astype(np.float32), dtype); g64 = I.to_f64(g, dtype)
    dout, dout64 = draw(rng, (T, H), dtype)
    dres, dres64 = draw(rng, (T, H), dtype)
    eps = 1e-6
    xd, gd = U.to_dev(x, dtype), U.to_dev(g, dtype)
    out = U.empty_dev((T, H), dtype)
    r = torch.empty(T, dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_fwd(dtype, T, H, xd, gd, eps, out, r)
    ref, rref = O.rmsnorm_fwd(x64, g64, eps)
    tol = U.TOL[dtype]
    assert U.tensor_scale_err(U.from_dev(out), ref) < tol
    assert U.tensor_scale_err(U.from_dev(r), rref) < 1e-5
    # backward with the oracle's r (fp32-rounded) so the op is tested on its own
    r32 = torch.from_numpy(rref.astype(np.float32)).cuda()
    dz = U.empty_dev((T, H), dtype)
    dgam = torch.full((H,), 5.0, dtype=torch.float32, device="cuda")
    scratch = torch.empty(taw.taw_op_rmsnorm_bwd_scratch_floats(H), dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_bwd(dtype, T, H, U.to_dev(dout, dtype), xd, r32, gd, U.to_dev(dres, dtype), dz, dgam, 1, scratch)
    dzr, dgr = O.rmsnorm_bwd(dout64, x64, rref, g64)
    assert U.tensor_scale_err(U.from_dev(dz), dzr + dres64) < tol
    assert U.tensor_scale_err(U.from_dev(dgam) - 5.0, dgr) < 1e-4
    taw.taw_op_rmsnorm_bwd(dtype, T, H, U.to_dev(dout, dtype), xd, r32, gd, None, dz, dgam, 0, scratch)
    assert U.tensor_scale_err(U.from_dev(dz), dzr) < tol
    assert U.tensor_scale_err(U.from_dev(dgam), dgr) < 1e-4


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("B,S,nh,d", [(2, 33, 3, 16), (1, 300, 2, 128), (1, 5, 2, 6)])
def test_rope_forward_and_inverse(taw, dtype, B, S, nh, d):
    import torch
    rng = np.random.default_rng(S + d)
    H = nh * d
    z, z64 = draw(rng, (B * S, 3 * H), dtype)
    desc = taw.make_desc(dtype, B, S, H, nh, d, 8, 10000.0)
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, table)
    phi = O.rope_angles(S, d, 10000.0)
    tab = U.from_dev(table).reshape(S, d // 2, 2)
    assert np.max(np.abs(tab[..., 0] - np.cos(phi))) < 1e-7 and np.max(np.abs(tab[..., 1] - np.sin(phi))) < 1e-7
    zd = U.to_dev(z, dtype)
    taw.taw_op_rope(dtype, B, S, 2 * H, d, zd, 3 * H, table, 0)
    ref = z64.copy()
    for part in range(2):
        blk = z64[:, part * H:(part + 1) * H].reshape(B, S, nh, d)
        ref[:, part * H:(part + 1) * H] = O.rope_apply(blk, phi).reshape(B * S, H)
    got = U.from_dev(zd)
    assert U.tensor_scale_err(got, ref) < (1e-2 if dtype == I.BF16 else 1e-6)
    assert np.array_equal(got[:, 2 * H:], z64[:, 2 * H:])          # v untouched
    taw.taw_op_rope(dtype, B, S, 2 * H, d, zd, 3 * H, table, 1)
    assert U.tensor_scale_err(U.from_dev(zd), z64) < (2e-2 if dtype == I.BF16 else 1e-6)


def test_rope_table_accuracy_at_long_context(taw):
    """Angles up to 32767 rad: the table must stay at fp32 rounding accuracy (fp64 evaluation)."""
    import torch
    S, d = 32768, 128
    desc = taw.make_desc(I.BF16, 1, S, 4096, 32, d, 11008)
    table = torch.empty(S * (d // 2) * 2, dtype=torch.float32, device="cuda")
    taw.taw_rope_table_init(desc, table)
    rows = np.array([0, 1, 1000, 20000, 32767])
    tab = U.from_dev(table).reshape(S, d // 2, 2)[rows]
    phi = O.rope_angles(S, d, 10000.0)[rows]
    assert np.max(np.abs(tab[..., 0] - np.cos(phi))) < 1e-6 and np.max(np.abs(tab[..., 1] - np.sin(phi))) < 1e-6


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("T,I_", [(7, 176), (129, 1000), (3, 11008), (5, 37)])
def test_swiglu_fwd_bwd(taw, dtype, T, I_):
    rng = np.random.default_rng(T + I_)
    gu, gu64 = draw(rng, (T, 2 * I_), dtype, 2.0)
    da, da64 = draw(rng, (T, I_), dtype)
    a = U.empty_dev((T, I_), dtype)
    dgu = U.empty_dev((T, 2 * I_), dtype)
    gud = U.to_dev(gu, dtype)
    taw.taw_op_swiglu_fwd(dtype, T, I_, gud, a)
    taw.taw_op_swiglu_bwd(dtype, T, I_, U.to_dev(da, dtype), gud, dgu)
    g, u = gu64[:, :I_], gu64[:, I_:]
    tol = 1e-2 if dtype == I.BF16 else 1e-5
    assert U.tensor_scale_err(U.from_dev(a), O.swiglu_fwd(g, u)) < tol
    dg, du = O.swiglu_bwd(da64, g, u)
    assert U.tensor_scale_err(U.from_dev(dgu), np.concatenate([dg, du], axis=1)) < tol


def _attn_case(taw, dtype, B, S, nh, d, impl, seed=0, scale=1.0, bwd_impl=None):
    import torch
    rng = np.random.default_rng(seed)
    H = nh * d
    qkv, qkv64 = draw(rng, (B * S, 3 * H), dtype, scale)
    dO, dO64 = draw(rng, (B * S, H), dtype)
    q, k, v = (qkv64[:, i * H:(i + 1) * H].reshape(B, S, nh, d) for i in range(3))
    oref = O.attention_fwd(q, k, v)
    qkvd = U.to_dev(qkv, dtype)
    o = U.empty_dev((B * S, H), dtype)
    lse = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    taw.taw_op_attn_fwd(dtype, B, S, nh, d, qkvd, o, lse, impl)
    tol = U.TOL[dtype]
    e_o = U.tensor_scale_err(U.from_dev(o), oref.reshape(B * S, H))
    # log-sum-exp of the scaled scores: the oracle's own (pinned) row-wise form, every row of every head
    lref = np.empty((B, nh, S))
    for b in range(B):
        for h in range(nh):
            _, lref[b, h] = O.attention_fwd_rows(q[b, :, h], k[b, :, h], v[b, :, h], np.arange(S))
    e_l = float(np.max(np.abs(U.from_dev(lse).reshape(B, nh, S) - lref)))
    # backward from the stored (storage-rounded) forward output of the oracle, so bwd is tested on its own
    o_st = I.to_storage(oref.reshape(B * S, H).astype(np.float32), dtype)
    o64 = I.to_f64(o_st, dtype).reshape(B, S, nh, d)
    dq, dk, dv = O.attention_bwd(q, k, v, o64, dO64.reshape(B, S, nh, d))
    dref = np.concatenate([dq.reshape(B * S, H), dk.reshape(B * S, H), dv.reshape(B * S, H)], axis=1)
    lse_ref32 = torch.from_numpy(lref.astype(np.float32).reshape(-1)).cuda()
    dqkv = U.empty_dev((B * S, 3 * H), dtype)
    scratch = torch.empty(taw.taw_op_attn_bwd_scratch_floats(B, S, nh), dtype=torch.float32, device="cuda")
    taw.taw_op_attn_bwd(dtype, B, S, nh, d, qkvd, U.to_dev(o_st, dtype), U.to_dev(dO, dtype), lse_ref32, dqkv, scratch, None, impl if bwd_impl is None else bwd_impl)
    got = U.from_dev(dqkv)
    # at S = 1 the exact dq and dk are identically zero: measure them on the scale of dv
    fl = 1e-3 * float(np.max(np.abs(dref[:, 2 * H:])))
    e_dq = U.tensor_scale_err(got[:, :H], dref[:, :H], floor=fl)
    e_dk = U.tensor_scale_err(got[:, H:2 * H], dref[:, H:2 * H], floor=fl)
    e_dv = U.tensor_scale_err(got[:, 2 * H:], dref[:, 2 * H:])
    print(f"attn dtype={dtype} B={B} S={S} nh={nh} d={d} impl={impl}: o={e_o:.2e} lse={e_l:.2e} dq={e_dq:.2e} dk={e_dk:.2e} dv={e_dv:.2e}", flush=True)
    assert e_o < tol and e_l < (2e-2 if dtype == I.BF16 else 1e-4)
    assert e_dq < tol and e_dk < tol and e_dv < tol


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("B,S,nh,d", [(1, 128, 4, 16), (2, 67, 3, 8), (1, 1, 2, 16), (1, 130, 1, 128)])
def test_attention_generic(taw, dtype, B, S, nh, d):
    _attn_case(taw, dtype, B, S, nh, d, taw.TAW_IMPL_GENERIC, seed=S)


@pytest.mark.parametrize("src_dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("n", [0, 1, 3, 4, 1027, 13490, 1 << 20])      # 13490: whole workgroups, a partly filled one and a scalar tail
def test_grad_accum(taw, src_dtype, n):
    import torch
    rng = np.random.default_rng(n + 1)
    G0 = rng.standard_normal(n + 8).astype(np.float32)
    g, g64 = draw(rng, (n + 8,), src_dtype)
    Gd = torch.from_numpy(G0.copy()).cuda()
    taw.taw_grad_accum(Gd, U.to_dev(g, src_dtype), src_dtype, n, 0.25)
    got = U.from_dev(Gd)
    ref = O.grad_accum(G0[:n].astype(np.float64), g64[:n], 0.25)
    assert np.max(np.abs(got[:n] - ref), initial=0.0) < 1e-6
    assert np.array_equal(got[n:], G0[n:].astype(np.float64))        # nothing past n_elems is touched


def test_weight_stage_double_buffer(taw):
    """Chunks staged on a side stream, ordered against the compute stream by the two events."""
    import torch
    n = 1 << 22
    shards = [torch.full((n,), float(j + 1), dtype=torch.float32, device="cuda") for j in range(4)]
    bufs = [torch.zeros(n, dtype=torch.float32, device="cuda") for _ in range(2)]
    sums = torch.zeros(4, dtype=torch.float32, device="cuda")
    copy_stream = torch.cuda.Stream()
    compute = torch.cuda.current_stream()
    ready = [torch.cuda.Event() for _ in range(2)]
    consumed = [torch.cuda.Event() for _ in range(2)]
    torch.cuda.synchronize()
    taw.taw_weight_stage(bufs[0], shards[0], n * 4, copy_stream, None, ready[0])
    for j in range(4):
        if j + 1 < 4:
            nb = (j + 1) & 1
            taw.taw_weight_stage(bufs[nb], shards[j + 1], n * 4, copy_stream, consumed[nb] if j >= 1 else None, ready[nb])
        compute.wait_event(ready[j & 1])
        sums[j] = bufs[j & 1].sum() / n          # "the layer" reads its weights
        consumed[j & 1].record(compute)
    torch.cuda.synchronize()
    assert sums.cpu().tolist() == [1.0, 2.0, 3.0, 4.0]
    taw.taw_weight_stage(None, None, 0, copy_stream, None, ready[0])   # bytes == 0 only handles the events
    torch.cuda.synchronize()


# ----------------------------------------------------------------------------- MFMA kernels (bf16)
# K % 64 == 0 runs the 64-deep pipelined kernel (1, 2, 3 and many K steps), K % 32 == 0 the 32-deep one,
# any other K the register-staged kernel
MFMA_GEMM_SHAPES = {
    0: [(256, 256, 64), (8, 8, 8), (300, 520, 136), (257, 263, 72), (1000, 264, 4104), (512, 768, 1024), (1, 3, 8),
        (300, 520, 96), (257, 263, 128), (264, 520, 192), (300, 264, 160), (1000, 264, 4096), (5, 3, 32)],
    1: [(256, 256, 64), (8, 8, 8), (300, 520, 136), (257, 264, 72), (1000, 264, 4104), (512, 768, 1024), (1, 8, 8),
        (300, 520, 96), (257, 264, 128), (264, 520, 192), (300, 264, 160), (1000, 264, 4096), (5, 8, 32)],
    2: [(256, 256, 64), (8, 8, 8), (304, 520, 133), (264, 256, 77), (1000, 264, 4100), (512, 768, 1024), (8, 8, 1),
        (304, 520, 96), (264, 256, 128), (264, 520, 192), (304, 264, 160), (1000, 264, 4096), (8, 8, 32)],
}


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_gemm_mfma_shapes(taw, mode):
    """Several tiles, ragged tails in M, N and K, and degenerate sizes; bf16 output."""
    for (M, N, K) in MFMA_GEMM_SHAPES[mode]:
        err = _gemm_case(taw, I.BF16, mode, M, N, K, taw.TAW_IMPL_MFMA, seed=M + N + K)
        print(f"mfma gemm mode={mode} {M}x{N}x{K}: err={err:.2e}", flush=True)


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_gemm_mfma_epilogues(taw, mode):
    for shp in ((520, 264, 200) if mode != 2 else (520, 264, 203), (520, 264, 192), (520, 264, 160)):   # one per kernel
        _gemm_case(taw, I.BF16, mode, *shp, taw.TAW_IMPL_MFMA, residual=True)
        _gemm_case(taw, I.BF16, mode, *shp, taw.TAW_IMPL_MFMA, c_f32=True)
        _gemm_case(taw, I.BF16, mode, *shp, taw.TAW_IMPL_MFMA, c_f32=True, accumulate=True)
        _gemm_case(taw, I.BF16, mode, *shp, taw.TAW_IMPL_MFMA, c_f32=True, accumulate=True, residual=True)


def test_gemm_mfma_fp32_output_is_accurate(taw):
    """With fp32 output the only error left is the accumulation order: far below bf16 rounding."""
    for mode in (0, 1, 2):
        err = _gemm_case(taw, I.BF16, mode, 264, 512, 2048, taw.TAW_IMPL_MFMA, c_f32=True, seed=mode)
        assert err < 2e-6, (mode, err)


# the forms of the MFMA backward: the split dK/dV + dQ pair, fused with private dQ slots, fused with atomics, and the split
# pair whose dK/dV kernel stores dS for the dQ kernel
BWD_FORMS = {"split": 2, "fused": 3, "atomic": 4, "stored": 5}


@pytest.mark.parametrize("form", list(BWD_FORMS))
@pytest.mark.parametrize("B,S,nh", [(1, 64, 1), (1, 256, 2), (2, 333, 2), (1, 1, 1), (1, 1000, 1), (1, 130, 3), (1, 2081, 2), (3, 520, 1), (4, 2304, 16)])
def test_attention_mfma(taw, B, S, nh, form):
    """Tiled online-softmax kernels: several query/key tiles, ragged S, S = 1, more than one head and batch; every
    form of the backward (2081 keys: nine key blocks dealt to several workers per head in the fused form, each adding
    into its slot more than once; 520: a last query block with rows beyond the sequence; 4 x 16 heads x 2304: four workers per head with up to three key blocks each)."""
    _attn_case(taw, I.BF16, B, S, nh, 128, taw.TAW_IMPL_MFMA, seed=S + nh, bwd_impl=BWD_FORMS[form])


@pytest.mark.parametrize("form", list(BWD_FORMS))
def test_attention_mfma_peaked_scores(taw, form):
    """Scores of order 10: the running maximum moves a lot between key tiles."""
    _attn_case(taw, I.BF16, 1, 700, 2, 128, taw.TAW_IMPL_MFMA, seed=9, scale=3.0, bwd_impl=BWD_FORMS[form])


@pytest.mark.parametrize("form", ["fused", "stored"])
def test_attention_backward_forms_without_atomics_are_reproducible(taw, form):
    """The fused backward with slots adds its dQ partial sums in a fixed order, and the form with stored dS reads back only
    what it wrote: two runs over scratch with different stale contents give the same bits."""
    import torch
    B, S, nh, d = 2, 1500, 3, 128
    H = nh * d
    qkv = I.device_normal((B * S, 3 * H), seed=5, std=0.7)
    dO = I.device_normal((B * S, H), seed=6, std=1.0)
    o = torch.empty((B * S, H), dtype=torch.bfloat16, device="cuda")
    lse = torch.empty(B * nh * S, dtype=torch.float32, device="cuda")
    taw.taw_op_attn_fwd(I.BF16, B, S, nh, d, qkv, o, lse, taw.TAW_IMPL_MFMA)
    outs = []
    for fill in (0.0, 1e30):
        scratch = torch.full((taw.taw_op_attn_bwd_scratch_floats(B, S, nh),), fill, dtype=torch.float32, device="cuda")   # stale contents must not matter
        dqkv = torch.empty_like(qkv)
        taw.taw_op_attn_bwd(I.BF16, B, S, nh, d, qkv, o, dO, lse, dqkv, scratch, None, BWD_FORMS[form])
        torch.cuda.synchronize()
        outs.append(dqkv)
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("dtype", [I.F32, I.BF16])
@pytest.mark.parametrize("n", [1, 7, 4096, 4499, 1 << 20])           # 4499: whole workgroups, a partly filled one and a scalar tail
def test_optimizer_step(taw, dtype, n):
    """Three AdamW steps over a shard against the oracle: master weights, both moments, the chunk in its
    storage type, and the zeroed gradient shard."""
    import torch
    rng = np.random.default_rng(n)
    w = rng.standard_normal(n).astype(np.float32)
    master = torch.from_numpy(w.copy()).cuda()
    m = torch.zeros(n, dtype=torch.float32, device="cuda")
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    chunk = U.empty_dev((n,), dtype)
    w64, m64, v64 = w.astype(np.float64), np.zeros(n), np.zeros(n)
    hp = dict(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-6, weight_decay=0.1, grad_scale=0.25)
    for t in range(1, 4):
        g = rng.standard_normal(n).astype(np.float32)
        G = torch.from_numpy(g.copy()).cuda()
        taw.taw_optimizer_step(chunk, dtype, master, m, v, G, n, t, zero_grad=(t == 3), **hp)
        w64, m64, v64 = O.adamw_step(w64, m64, v64, g.astype(np.float64), t, hp["lr"], hp["beta1"], hp["beta2"], hp["eps"],
                                     hp["weight_decay"], hp["grad_scale"])
        torch.cuda.synchronize()
        assert torch.count_nonzero(G).item() == (0 if t == 3 else np.count_nonzero(g))
    assert U.tensor_scale_err(U.from_dev(master), w64) < 1e-6
    assert U.tensor_scale_err(U.from_dev(m), m64) < 1e-6 and U.tensor_scale_err(U.from_dev(v), v64) < 1e-6
    assert U.tensor_scale_err(U.from_dev(chunk), w64) < (4e-3 if dtype == I.BF16 else 1e-6)
    if dtype == I.BF16:   # the chunk is exactly the master weights rounded to bf16
        assert np.array_equal(I.to_storage(master.cpu().numpy(), dtype), chunk.view(torch.int16).cpu().numpy().view(np.uint16))
