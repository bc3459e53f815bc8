"""The entry point that allocates nothing (taw_op_rmsnorm_bwd_static: partial sums in a static device
array inside the library) against the existing entry point with a caller-owned scratch, through the
C ABI.  Two calls in a row on one GPU, the second with a smaller input: the array keeps the first
call's contents, and they must not leak into the second call's results."""
import numpy as np
import pytest

from oracle import decoder_layer as O
from paper_2511_09741_amd import inputs as I
from tests import util as U

pytestmark = pytest.mark.gpu


def _case(taw, dtype, T, H, seed, with_res, accumulate):
    import torch
    tdt = torch.bfloat16 if dtype == I.BF16 else torch.float32
    z = I.device_normal((T, H), seed=seed, std=1.0, dtype=tdt)
    dout = I.device_normal((T, H), seed=seed + 1, std=1.0, dtype=tdt)
    dres = I.device_normal((T, H), seed=seed + 2, std=1.0, dtype=tdt) if with_res else None
    gam = (I.device_normal((H,), seed=seed + 3, std=0.1, dtype=torch.float32) + 1.0).to(tdt)
    out = torch.empty_like(z)
    r = torch.empty(T, dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_fwd(dtype, T, H, z, gam, 1e-6, out, r)
    dg0 = I.device_normal((H,), seed=seed + 4, std=1.0, dtype=torch.float32)
    # existing entry point, caller-owned scratch
    dz_a, dg_a = torch.empty_like(z), dg0.clone()
    scratch = torch.empty(taw.taw_op_rmsnorm_bwd_scratch_floats(H), dtype=torch.float32, device="cuda")
    taw.taw_op_rmsnorm_bwd(dtype, T, H, dout, z, r, gam, dres, dz_a, dg_a, accumulate, scratch)
    # the entry point under test: every buffer exists before the call, nothing is allocated from here on
    dz_b, dg_b = torch.empty_like(z), dg0.clone()
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    taw.taw_op_rmsnorm_bwd_static(dtype, T, H, dout, z, r, gam, dres, dz_b, dg_b, accumulate)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(dz_a, dz_b), "dz differs from the existing entry point's"
    assert torch.equal(dg_a, dg_b), "dgamma differs from the existing entry point's"
    # and both are right: sampled rows and the full gain gradient against the oracle
    f64 = lambda t: t.detach().to(torch.float32).cpu().numpy().astype(np.float64)
    rows = np.unique(np.array([0, 1, T // 3, T // 2, T - 2, T - 1]) % T)
    ri = torch.from_numpy(rows).cuda()
    _, r_ref = O.rmsnorm_fwd(f64(z[ri]), f64(gam), 1e-6)
    dz_ref, _ = O.rmsnorm_bwd(f64(dout[ri]), f64(z[ri]), r_ref, f64(gam))
    if with_res:
        dz_ref = dz_ref + f64(dres[ri])
    assert U.tensor_scale_err(f64(dz_b[ri]), dz_ref) < (1e-2 if dtype == I.BF16 else 1e-5)
    dg_ref = np.zeros(H)
    for s0 in range(0, T, 4096):
        zs, ds = f64(z[s0:s0 + 4096]), f64(dout[s0:s0 + 4096])
        _, rs = O.rmsnorm_fwd(zs, f64(gam), 1e-6)
        dg_ref += O.rmsnorm_bwd(ds, zs, rs, f64(gam))[1]
    if accumulate:
        dg_ref = dg_ref + f64(dg0)
    assert U.tensor_scale_err(f64(dg_b), dg_ref) < 1e-3


def test_static_scratch_entry_point_matches_the_existing_one(taw):
    """A large call (all 512 partial rows of the static array written, H = 8192: the LDS column-sum path), then a
    smaller one (fewer rows, narrower: most of the array still holds the first call's sums), then fp32."""
    _case(taw, I.BF16, 6000, 8192, seed=100, with_res=True, accumulate=0)
    _case(taw, I.BF16, 37, 1024, seed=200, with_res=False, accumulate=1)
    _case(taw, I.BF16, 3, 4096, seed=300, with_res=True, accumulate=0)
    _case(taw, I.F32, 515, 1000, seed=400, with_res=True, accumulate=1)


def test_static_scratch_entry_point_rejects_what_it_cannot_hold(taw):
    ok = 0x10000
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_rmsnorm_bwd_static(I.BF16, 8, 8200, ok, ok, ok, ok, None, ok, ok, 0)
    assert e.value.status == taw.TAW_ERR_WORKSPACE
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_rmsnorm_bwd_static(I.BF16, 8, 1024, ok, None, ok, ok, None, ok, ok, 0)
    assert e.value.status == taw.TAW_ERR_NULL
    taw.taw_op_rmsnorm_bwd_static(I.BF16, 0, 1024, None, None, None, None, None, None, None, 0)     # no rows: nothing to do
