"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
headers declare, computes the chunk layout, and rejects bad arguments before any launch."""
import ctypes as C
import os
import re

import pytest

import paper_2511_09741_amd.binding as taw
from paper_2511_09741_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(taw.LIB_PATH):
        from paper_2511_09741_amd.build import build
        build()
    return taw.load()


def declared_functions():
    names = []
    for h in sorted(f for f in os.listdir(os.path.join(ROOT, "include")) if f.endswith(".h")):
        src = open(os.path.join(ROOT, "include", h)).read()
        src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
        names += re.findall(r"\b(taw_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) == 38
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/ but not exported"
    assert set(names) == set(taw.EXPORTS)


def test_status_strings(lib):
    assert taw.taw_status_string(0) == "TAW_OK"
    assert taw.taw_status_string(-5) == "TAW_ERR_WORKSPACE"
    assert taw.taw_status_string(-99) == "TAW_ERR_UNKNOWN"


def test_weight_layout_matches_the_papers_parameter_count(lib):
    """A layer holds 4H^2 + 3HI matrix parameters (about 12 H^2, Theoretical Analysis) + 2H gains."""
    d = taw.desc_from_config(I.CONFIGS["C2"])
    L = taw.taw_layer_weight_layout(d)
    H, I_ = 4096, 11008
    assert L["total_elems"] == 4 * H * H + 3 * H * I_ + 2 * H == 202_383_360
    assert abs(L["total_elems"] / (12 * H * H) - 1) < 0.01
    assert [L[k] for k in taw.LAYOUT_FIELDS[:-1]] == sorted(L[k] for k in taw.LAYOUT_FIELDS[:-1])
    assert L["w_qkv"] == H and L["w_o"] == H + 3 * H * H
    # tiny config: sub-tensors are padded to 128-element boundaries and do not overlap
    c1 = I.CONFIGS["C1"]
    L1 = taw.taw_layer_weight_layout(taw.desc_from_config(c1))
    sizes = {"gamma_attn": 64, "w_qkv": 192 * 64, "w_o": 64 * 64, "gamma_mlp": 64, "w_gate_up": 352 * 64, "w_down": 64 * 176}
    end = 0
    for k in taw.LAYOUT_FIELDS[:-1]:
        assert L1[k] % 128 == 0 and L1[k] >= end
        end = L1[k] + sizes[k]
    assert L1["total_elems"] >= end and L1["total_elems"] % 128 == 0
    assert sum(sizes.values()) == 50_304


def test_ctx_and_workspace_sizes(lib):
    d = taw.desc_from_config(I.CONFIGS["C3"], taw.TAW_ATTN_BWD_RECOMPUTE)      # without the dS hand-over of the default attention backward
    ctx, ws = taw.taw_layer_ctx_bytes(d), taw.taw_layer_workspace_bytes(d)
    T, H, I_ = 32768, 4096, 11008
    assert ctx >= 2 * T * (7 * H + 3 * I_) and ctx < 5 * 2**30
    assert ws >= 2 * T * (7 * H + 3 * I_) and ws < 5 * 2**30
    assert taw.taw_layer_ctx_bytes(taw.desc_from_config(I.CONFIGS["C3"])) == ctx
    bad = taw.make_desc(1, 1, 128, 100, 3, 32, 64)
    assert taw.taw_layer_ctx_bytes(bad) == 0 and taw.taw_layer_workspace_bytes(bad) == 0


def test_recompute_mode_moves_the_cache_into_the_workspace(lib):
    """TAW_RECOMPUTE: nothing is kept between forward and backward; the workspace grows by exactly
    what the cache would have held, and the calls insist on that size before launching anything."""
    cfg = I.CONFIGS["C2"]
    d0, d1 = taw.desc_from_config(cfg), taw.desc_from_config(cfg, taw.TAW_RECOMPUTE)
    assert taw.taw_layer_ctx_bytes(d1) == 0
    assert taw.taw_layer_workspace_bytes(d1) == taw.taw_layer_workspace_bytes(d0) + taw.taw_layer_ctx_bytes(d0)
    ok = 0x10000
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_bwd(d1, ok, ok, ok, ok + 4096, None, ok + 8192, ok, ok, taw.taw_layer_workspace_bytes(d0))
    assert e.value.status == taw.TAW_ERR_WORKSPACE       # ctx may be NULL, the workspace may not be the small one


@pytest.mark.parametrize("kw,code", [
    (dict(H=100), taw.TAW_ERR_SHAPE), (dict(S=0), taw.TAW_ERR_SHAPE), (dict(B=-1), taw.TAW_ERR_SHAPE),
    (dict(dtype=7), taw.TAW_ERR_DTYPE), (dict(head_dim=15, n_heads=4, H=60), taw.TAW_ERR_SHAPE),
    (dict(flags=16), taw.TAW_ERR_SHAPE), (dict(flags=4 | 8), taw.TAW_ERR_SHAPE), (dict(rope_theta=0.0), taw.TAW_ERR_SHAPE),
])
def test_bad_descriptors_are_rejected(lib, kw, code):
    base = dict(dtype=0, B=1, S=128, H=64, n_heads=4, head_dim=16, I=176)
    base.update(kw)
    d = taw.make_desc(**base)
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_weight_layout(d)
    assert e.value.status == code
    assert taw.taw_last_error()


def test_layer_calls_validate_before_launching(lib):
    d = taw.desc_from_config(I.CONFIGS["C1"])
    ws = taw.taw_layer_workspace_bytes(d)
    ok = 0x10000  # a 16-byte aligned fake address; every call below must fail before using it
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_fwd(d, None, ok, ok, ok + 4096, ok, ok, ws)
    assert e.value.status == taw.TAW_ERR_NULL
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_fwd(d, ok, ok, ok + 4, ok + 4096, ok, ok, ws)
    assert e.value.status == taw.TAW_ERR_ALIGN
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_fwd(d, ok, ok, ok, ok + 4096, ok, ok, ws - 1)
    assert e.value.status == taw.TAW_ERR_WORKSPACE
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_fwd(d, ok, ok, ok, ok, ok, ok, ws)
    assert e.value.status == taw.TAW_ERR_SHAPE           # y aliases x
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_bwd(d, ok, ok, ok, ok + 4096, ok, ok + 8192, None, ok, ws)
    assert e.value.status == taw.TAW_ERR_NULL
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_bwd(d, ok, ok, ok, ok + 4096, ok, ok + 4096, ok, ok, ws)
    assert e.value.status == taw.TAW_ERR_SHAPE           # dx aliases dy
    big = taw.make_desc(0, 1, 8192, 64, 4, 16, 176)       # fp32 has no MFMA attention; generic takes S <= 4096
    with pytest.raises(taw.TawError) as e:
        taw.taw_layer_fwd(big, ok, ok, ok, ok + 4096, ok, ok, taw.taw_layer_workspace_bytes(big))
    assert e.value.status == taw.TAW_ERR_UNSUPPORTED


def test_grad_accum_and_stage_validation(lib):
    ok = 0x10000
    taw.taw_grad_accum(None, None, taw.TAW_F32, 0)          # n = 0 is a no-op
    with pytest.raises(taw.TawError) as e:
        taw.taw_grad_accum(ok, ok + 8, taw.TAW_F32, 16)
    assert e.value.status == taw.TAW_ERR_ALIGN
    with pytest.raises(taw.TawError) as e:
        taw.taw_grad_accum(ok, ok + 16, taw.TAW_F32, 16)
    assert e.value.status == taw.TAW_ERR_SHAPE           # overlap
    with pytest.raises(taw.TawError) as e:
        taw.taw_grad_accum(ok, ok + 4096, 5, 16)
    assert e.value.status == taw.TAW_ERR_DTYPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_weight_stage(ok, ok + 4096, 24)
    assert e.value.status == taw.TAW_ERR_SHAPE           # not a multiple of 16
    with pytest.raises(taw.TawError) as e:
        taw.taw_weight_stage(None, ok, 32)
    assert e.value.status == taw.TAW_ERR_NULL
    with pytest.raises(taw.TawError) as e:
        taw.taw_weight_stage(ok, ok + 16, 32)
    assert e.value.status == taw.TAW_ERR_SHAPE           # overlap


def test_optimizer_step_validation(lib):
    ok = 0x10000
    with pytest.raises(taw.TawError) as e:
        taw.taw_optimizer_step(ok, 1, ok + 4096, ok + 8192, ok + 12288, ok + 16384, 16, 0)
    assert e.value.status == taw.TAW_ERR_SHAPE            # steps are 1-based
    with pytest.raises(taw.TawError) as e:
        taw.taw_optimizer_step(ok, 1, ok + 16, ok + 8192, ok + 12288, ok + 16384, 16, 1)
    assert e.value.status == taw.TAW_ERR_SHAPE            # chunk and master overlap
    with pytest.raises(taw.TawError) as e:
        taw.taw_optimizer_step(ok, 5, ok + 4096, ok + 8192, ok + 12288, ok + 16384, 16, 1)
    assert e.value.status == taw.TAW_ERR_DTYPE
    taw.taw_optimizer_step(None, 1, None, None, None, None, 0, 1)     # n = 0: nothing to do, nothing touched


def test_op_validation(lib):
    ok = 0x10000
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_gemm(taw.TAW_BF16, 5, 8, 8, 8, ok, 8, ok, 8, ok, 8, taw.TAW_BF16)
    assert e.value.status == taw.TAW_ERR_SHAPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_gemm(taw.TAW_BF16, taw.TAW_GEMM_NT, 8, 8, 8, ok, 4, ok, 8, ok, 8, taw.TAW_BF16)
    assert e.value.status == taw.TAW_ERR_SHAPE           # lda < K
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_gemm(taw.TAW_F32, taw.TAW_GEMM_NT, 8, 8, 8, ok, 8, ok, 8, ok, 8, taw.TAW_F32, impl=taw.TAW_IMPL_MFMA)
    assert e.value.status == taw.TAW_ERR_UNSUPPORTED
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_attn_fwd(taw.TAW_F32, 1, 16, 2, 16, ok, ok, ok, impl=taw.TAW_IMPL_MFMA)
    assert e.value.status == taw.TAW_ERR_UNSUPPORTED
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_rope(taw.TAW_F32, 1, 16, 24, 16, ok, 24, ok)
    assert e.value.status == taw.TAW_ERR_SHAPE           # ncols not a multiple of head_dim
    # the paired backward of a linear, the rotated qkv projection, the rotary argument of the attention backward
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_linear_bwd(taw.TAW_F32, 8, 8, 8, ok, ok, ok, ok, ok, 0, taw.TAW_IMPL_MFMA)
    assert e.value.status == taw.TAW_ERR_UNSUPPORTED     # fp32 has no MFMA kernel
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_linear_bwd(taw.TAW_BF16, 8, 8, 8, ok, None, ok, ok, ok)
    assert e.value.status == taw.TAW_ERR_NULL
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_linear_bwd(taw.TAW_BF16, 8, -1, 8, ok, ok, ok, ok, ok)
    assert e.value.status == taw.TAW_ERR_SHAPE
    taw.taw_op_linear_bwd(taw.TAW_BF16, 8, 8, 0, None, None, None, None, None)     # K = 0: both outputs are empty
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_qkv_rope(taw.TAW_BF16, 1, 16, 2, 15, ok, ok, ok, ok)
    assert e.value.status == taw.TAW_ERR_SHAPE           # odd head_dim
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_qkv_rope(taw.TAW_BF16, 1, 16, 2, 16, ok, ok, ok, None)
    assert e.value.status == taw.TAW_ERR_NULL            # the table is required here
    with pytest.raises(taw.TawError) as e:
        taw.taw_op_attn_bwd(taw.TAW_BF16, 1, 16, 2, 128, ok, ok, ok, ok, ok, ok, ok + 4)
    assert e.value.status == taw.TAW_ERR_ALIGN           # rope_table given but misaligned


def test_diag_validation(lib):
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_mfma_loop(7)
    assert e.value.status == taw.TAW_ERR_SHAPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_mfma_loop(taw.TAW_DIAG_MFMA_LDS_LOADS)          # needs a source buffer
    assert e.value.status == taw.TAW_ERR_NULL
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_lds_read_rate(0, 5)
    assert e.value.status == taw.TAW_ERR_SHAPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_dq_update_rate(0x10000, 1000, 32, 0)            # S must be a multiple of 256
    assert e.value.status == taw.TAW_ERR_SHAPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_issue_rate(3, 0, 4)
    assert e.value.status == taw.TAW_ERR_SHAPE
    assert taw.taw_diag_store_cost_bytes() == 256 * 8 * 65536
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_store_cost(0x10000, 1 << 20, 8, 16, 1)                  # the buffer must hold every wavefront's window
    assert e.value.status == taw.TAW_ERR_WORKSPACE
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_store_cost(0x10000, taw.taw_diag_store_cost_bytes(), 8, 32, 1)
    assert e.value.status == taw.TAW_ERR_SHAPE
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_issue_rate(0, 0, 3)                             # 0, 2, 4 or 8 vector instructions per slot
    assert e.value.status == taw.TAW_ERR_SHAPE


@pytest.mark.parametrize("tiles_m,tiles_n", [(1, 1), (3, 5), (16, 16), (17, 19), (7, 300), (300, 7), (33, 33), (128, 48), (128, 86), (86, 16), (16, 43), (32, 8)])
def test_gemm_tile_order_is_a_bijection_that_keeps_concurrent_tiles_together(lib, tiles_m, tiles_n):
    rows, cols = taw.taw_diag_gemm_tile_order(tiles_m, tiles_n)
    n = tiles_m * tiles_n
    assert len(rows) == n and sorted(zip(rows, cols)) == [(r, c) for r in range(tiles_m) for c in range(tiles_n)]
    # ids of one block of 256 run at about the same time, id b on XCD b % 8: count the distinct operand panels
    # (tile rows + tile columns) each full block touches, chip-wide and per XCD
    per_xcd = []
    for r0 in range(0, n - 255, 256):
        blk = range(r0, r0 + 256)
        chip = len({rows[b] for b in blk}) + len({cols[b] for b in blk})
        assert chip <= 64, (r0, chip)          # a 16 x 16 block has 32; ragged edges split a block over up to 3 pieces
        for x in range(8):
            mine = [b for b in blk if b % 8 == x]
            per_xcd.append(len({rows[b] for b in mine}) + len({cols[b] for b in mine}))
    if per_xcd:                                # 8 x 4 has 12; a block that straddles a ragged edge has more
        assert sum(per_xcd) / len(per_xcd) <= 16 and max(per_xcd) <= 40, (max(per_xcd), sum(per_xcd) / len(per_xcd))
    if tiles_m % 16 == 0 and tiles_n % 16 == 0:
        for r0 in range(0, n, 256):
            blk = range(r0, r0 + 256)
            assert len({rows[b] for b in blk}) == 16 and len({cols[b] for b in blk}) == 16
            for x in range(8):
                mine = [b for b in blk if b % 8 == x]
                assert len({rows[b] for b in mine}) == 8 and len({cols[b] for b in mine}) == 4
    with pytest.raises(taw.TawError) as e:
        taw.taw_diag_gemm_tile_order(0, 4)
    assert e.value.status == taw.TAW_ERR_SHAPE


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(taw, "_lib", None)
    monkeypatch.setattr(taw, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        taw.load()


def test_linear_bwd_scratch_rule(lib):
    """The weight gradient is cut only where it has too few tiles for its share of the chip: never at the 4096- and
    5120-wide layers, at most 32 ranges of at least 512 tokens elsewhere, nothing for empty or tiny problems."""
    f = taw.taw_op_linear_bwd_scratch_floats
    for T in (8192, 32768, 65536):
        for H, Iw in ((4096, 11008), (5120, 13824)):
            for N, K in ((H, Iw), (2 * Iw, H), (H, H), (3 * H, H)):
                assert f(T, N, K) == 0
    for T, N, K in ((65536, 1024, 1024), (65536, 1024, 2816), (65536, 3072, 1024), (65536, 2048, 2048), (2080, 256, 256), (1 << 20, 8, 8)):
        n = f(T, N, K)
        assert n > 0 and n % (N * K) == 0
        splits = n // (N * K)
        assert 2 <= splits <= 32 and T // splits >= 512 - 64
    for T, N, K in ((0, 8, 8), (8, 0, 8), (-1, 8, 8), (256, 256, 256), (1023, 8, 8)):
        assert f(T, N, K) == 0


def test_workspace_size_follows_the_attention_backward_form(lib):
    """The default backward hands dS over through the workspace: S * S bytes per (batch, head), counted in blocks of 256
    (sum over query blocks ib of 256 (ib + 1) keys x 256 rows x 2 bytes); TAW_ATTN_BWD_RECOMPUTE needs none of it; layers
    that cannot take the matrix-core attention (fp32, or heads other than 128) never pay for it."""
    for name in ("C2", "C3", "C4", "C5"):
        cfg = I.CONFIGS[name]
        full = taw.taw_layer_workspace_bytes(taw.desc_from_config(cfg, 0))
        lean = taw.taw_layer_workspace_bytes(taw.desc_from_config(cfg, taw.TAW_ATTN_BWD_RECOMPUTE))
        nqt = (cfg.S + 255) // 256
        assert full - lean == cfg.B * cfg.n_heads * (nqt * (nqt + 1) // 2) * 256 * 256 * 2
    c1 = I.CONFIGS["C1"]
    assert taw.taw_layer_workspace_bytes(taw.desc_from_config(c1, 0)) == taw.taw_layer_workspace_bytes(taw.desc_from_config(c1, taw.TAW_ATTN_BWD_RECOMPUTE))


@pytest.mark.parametrize("S", [1, 255, 256, 257, 1100, 4096])
def test_stored_ds_layout(lib, S):
    """The dS hand-over of the default attention backward, as the kernels address it: the 2 KiB units of a (batch, head) tile
    its region exactly (no gap, no overlap, query block ib holding 256 (ib + 1) keys x 256 rows), and a wavefront of the reading
    kernel (one 32-row group) finds its units for consecutive key groups at consecutive addresses; the 128 slots of a unit are a
    permutation, each store instruction (one piece of all 64 lanes) fills one contiguous KiB, and the 16 slots a
    half-wavefront of the reader touches in one transposing read (4 consecutive keys x 2 lane halves x 2 pieces) fall into 16
    different 16-byte bank groups; positions map back to the accumulator's row order."""
    L = taw.taw_diag_attn_ds_layout(S)
    nqt = (S + 255) // 256
    assert L["pair_bytes"] == sum(256 * (ib + 1) * 256 * 2 for ib in range(nqt))
    offs = L["unit_offsets"]
    assert sorted(offs) == list(range(0, L["pair_bytes"], 2048))
    k = 0
    for ib in range(nqt):
        for s in range(8):
            run = offs[k:k + 8 * (ib + 1)]
            assert run == list(range(run[0], run[0] + 2048 * len(run), 2048))
            k += len(run)
    slots = L["slots"]
    assert sorted(slots) == list(range(128))
    for tt in range(2):
        assert sorted(slots[(2 * tt + hh) * 32 + kk] for hh in range(2) for kk in range(32)) == list(range(64 * tt, 64 * tt + 64))
    for k4 in range(8):
        group = [slots[(2 * tt + hh) * 32 + 4 * k4 + j] for tt in range(2) for hh in range(2) for j in range(4)]
        assert sorted(x % 16 for x in group) == list(range(16))
    # position p = 16 hh + 8 tt + e holds accumulator register 8 tt + e of lane half hh, i.e. row 8 (r // 4) + 4 hh + r % 4
    for hh in range(2):
        for tt in range(2):
            for e in range(8):
                r = 8 * tt + e
                assert L["rows"][16 * hh + 8 * tt + e] == 8 * (r // 4) + 4 * hh + r % 4
    assert sorted(L["rows"]) == list(range(32))
