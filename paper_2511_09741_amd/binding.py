"""ctypes binding over libtaw.so: the same names as include/taw.h and include/taw_ops.h.

Argument marshalling only.  Device buffers are torch tensors (torch owns device memory and
streams); every function takes their data pointers, calls the C entry point and raises TawError
on a non-zero status.  There is no fallback: if the library is missing, load() raises.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtaw.so")

TAW_F32, TAW_BF16 = 0, 1
TAW_ACCUMULATE = 1
TAW_RECOMPUTE = 2
TAW_ATTN_BWD_FUSED = 4
TAW_ATTN_BWD_RECOMPUTE = 8
TAW_IMPL_AUTO, TAW_IMPL_GENERIC, TAW_IMPL_MFMA, TAW_IMPL_MFMA_FUSED, TAW_IMPL_MFMA_ATOMIC, TAW_IMPL_MFMA_STORED = 0, 1, 2, 3, 4, 5
TAW_GEMM_NT, TAW_GEMM_NN, TAW_GEMM_TN = 0, 1, 2
TAW_OK = 0
TAW_ERR_NULL, TAW_ERR_SHAPE, TAW_ERR_DTYPE, TAW_ERR_ALIGN, TAW_ERR_WORKSPACE, TAW_ERR_UNSUPPORTED, TAW_ERR_HIP = -1, -2, -3, -4, -5, -6, -7

LAYOUT_FIELDS = ("gamma_attn", "w_qkv", "w_o", "gamma_mlp", "w_gate_up", "w_down", "total_elems")


class taw_layer_desc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B", C.c_int32), ("S", C.c_int32), ("H", C.c_int32),
                ("n_heads", C.c_int32), ("head_dim", C.c_int32), ("I", C.c_int32),
                ("rope_theta", C.c_float), ("rms_eps", C.c_float), ("flags", C.c_uint32)]


class taw_weight_layout(C.Structure):
    _fields_ = [(f, C.c_size_t) for f in LAYOUT_FIELDS]


class taw_adamw_desc(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("grad_scale", C.c_float), ("step", C.c_int32), ("zero_grad", C.c_int32)]


class taw_diag_rate(C.Structure):
    _fields_ = [("tflops", C.c_double), ("clock_ghz", C.c_double), ("mfma_busy", C.c_double), ("ms", C.c_double)]


class taw_sched_desc(C.Structure):
    _fields_ = [("P", C.c_int32), ("D", C.c_int32), ("L", C.c_int32), ("N", C.c_int32)]


class TawError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name} ({status}): {detail}")
        self.status = status


_lib = None

_vp, _i32, _i64, _sz, _f = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
_dp = C.POINTER(taw_layer_desc)
_SIGS = {
    "taw_layer_weight_layout": (C.c_int, [_dp, C.POINTER(taw_weight_layout)]),
    "taw_layer_ctx_bytes": (_sz, [_dp]),
    "taw_layer_workspace_bytes": (_sz, [_dp]),
    "taw_rope_table_init": (C.c_int, [_dp, _vp, _vp]),
    "taw_layer_fwd": (C.c_int, [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "taw_layer_bwd": (C.c_int, [_dp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "taw_grad_accum": (C.c_int, [_vp, _vp, _i32, _sz, _f, _vp]),
    "taw_weight_stage": (C.c_int, [_vp, _vp, _sz, _vp, _vp, _vp]),
    "taw_optimizer_step": (C.c_int, [C.POINTER(taw_adamw_desc), _vp, _i32, _vp, _vp, _vp, _vp, _sz, _vp]),
    "taw_sched_owner": (C.c_int, [C.POINTER(taw_sched_desc), _i32, C.POINTER(_i32), C.POINTER(_i32)]),
    "taw_sched_step": (C.c_int, [C.POINTER(taw_sched_desc), _i32, _i32] + [C.POINTER(_i32)] * 4),
    "taw_sched_update_step": (C.c_int, [C.POINTER(taw_sched_desc), _i32, C.POINTER(_i32)]),
    "taw_sched_bubble_ratio": (C.c_int, [C.POINTER(taw_sched_desc), C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "taw_sched_comm_elems": (C.c_int, [_i32, _i32, _i32, _i32] + [C.POINTER(C.c_double)] * 3),
    "taw_diag_mfma_loop": (C.c_int, [_i32, _i32, _vp, _sz, C.POINTER(taw_diag_rate)]),
    "taw_diag_lds_read_rate": (C.c_int, [_i32, _i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "taw_diag_dq_update_rate": (C.c_int, [_vp, _i32, _i32, _i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "taw_diag_gemm_tile_order": (C.c_int, [_i32, _i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "taw_diag_issue_rate": (C.c_int, [_i32, _i32, _i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]),
    "taw_diag_attn_ds_layout": (C.c_int, [_i32, C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.POINTER(C.c_int32), C.POINTER(C.c_int32)]),
    "taw_diag_store_cost_bytes": (C.c_size_t, []),
    "taw_diag_store_cost": (C.c_int, [_vp, C.c_size_t, _i32, _i32, _i32, C.POINTER(C.c_double)]),
    "taw_status_string": (C.c_char_p, [C.c_int]),
    "taw_last_error": (C.c_char_p, []),
    "taw_op_gemm": (C.c_int, [_i32, _i32, _i64, _i64, _i64, _vp, _i64, _vp, _i64, _vp, _i64, _i32, _i32, _vp, _i64, _i32, _vp]),
    "taw_op_rmsnorm_fwd": (C.c_int, [_i32, _i64, _i32, _vp, _vp, _f, _vp, _vp, _vp]),
    "taw_op_rmsnorm_bwd_scratch_floats": (_sz, [_i32]),
    "taw_op_attn_bwd_scratch_floats": (_sz, [_i32, _i32, _i32]),
    "taw_op_rmsnorm_bwd": (C.c_int, [_i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _vp]),
    "taw_op_rmsnorm_bwd_static": (C.c_int, [_i32, _i64, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]),
    "taw_op_rope": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _vp, _i64, _vp, _i32, _vp]),
    "taw_op_swiglu_fwd": (C.c_int, [_i32, _i64, _i32, _vp, _vp, _vp]),
    "taw_op_swiglu_bwd": (C.c_int, [_i32, _i64, _i32, _vp, _vp, _vp, _vp]),
    "taw_op_attn_fwd": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _i32, _vp]),
    "taw_op_attn_bwd": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _i32, _vp]),
    "taw_op_qkv_rope": (C.c_int, [_i32, _i32, _i32, _i32, _i32, _vp, _vp, _vp, _vp, _i32, _vp]),
    "taw_op_linear_bwd_scratch_floats": (C.c_size_t, [_i64, _i64, _i64]),
    "taw_op_linear_bwd": (C.c_int, [_i32, _i64, _i64, _i64, _vp, _vp, _vp, _vp, _vp, _i32, _vp, _i32, _vp]),
}
EXPORTS = tuple(_SIGS)


def load():
    """Loads libtaw.so (built by paper_2511_09741_amd.build).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not found: build it with `python -m paper_2511_09741_amd.build`; "
                              "there is no fallback path")
        # torch first: it brings its own HIP runtime (soname libamdhip64.so.7) and the loader then
        # binds libtaw.so to that one; two HIP runtimes in one process do not both see the GPU.
        import torch  # noqa: F401
        lib = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGS.items():
            fn = getattr(lib, name)
            fn.restype, fn.argtypes = res, args
        _lib = lib
    return _lib


def _check(status: int):
    if status != TAW_OK:
        lib = load()
        raise TawError(status, lib.taw_status_string(status).decode(), lib.taw_last_error().decode())


def _p(t):
    """Device (or host) pointer of a torch tensor, None -> NULL, int passes through."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream


def make_desc(dtype, B, S, H, n_heads, head_dim, I, rope_theta=10000.0, rms_eps=1e-6, flags=0) -> taw_layer_desc:
    return taw_layer_desc(dtype, B, S, H, n_heads, head_dim, I, rope_theta, rms_eps, flags)


def desc_from_config(cfg, flags=0) -> taw_layer_desc:
    return make_desc(cfg.dtype, cfg.B, cfg.S, cfg.H, cfg.n_heads, cfg.head_dim, cfg.I, cfg.rope_theta, cfg.rms_eps, flags)


# ----------------------------------------------------------------------------- taw.h
def taw_layer_weight_layout(desc) -> dict:
    out = taw_weight_layout()
    _check(load().taw_layer_weight_layout(C.byref(desc), C.byref(out)))
    return {f: int(getattr(out, f)) for f in LAYOUT_FIELDS}


def taw_layer_ctx_bytes(desc) -> int:
    return int(load().taw_layer_ctx_bytes(C.byref(desc)))


def taw_layer_workspace_bytes(desc) -> int:
    return int(load().taw_layer_workspace_bytes(C.byref(desc)))


def taw_rope_table_init(desc, rope_table, stream=None):
    _check(load().taw_rope_table_init(C.byref(desc), _p(rope_table), _stream(stream)))


def taw_layer_fwd(desc, W_chunk, rope_table, x, y, ctx, workspace, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(load().taw_layer_fwd(C.byref(desc), _p(W_chunk), _p(rope_table), _p(x), _p(y), _p(ctx), _p(workspace),
                                workspace_bytes, _stream(stream)))


def taw_layer_bwd(desc, W_chunk, rope_table, x, dy, ctx, dx, G_shard, workspace, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    _check(load().taw_layer_bwd(C.byref(desc), _p(W_chunk), _p(rope_table), _p(x), _p(dy), _p(ctx), _p(dx), _p(G_shard),
                                _p(workspace), workspace_bytes, _stream(stream)))


# ---- schedule model (host only)
def _sched_check(rc):
    if rc != 0:
        raise ValueError("taw_sched: invalid arguments")


def taw_sched_owner(P, D, L, layer):
    """(device, group) that owns `layer`."""
    d, dev, grp = taw_sched_desc(P, D, L, 1), _i32(), _i32()
    _sched_check(load().taw_sched_owner(C.byref(d), layer, C.byref(dev), C.byref(grp)))
    return dev.value, grp.value


def taw_sched_step(P, D, L, group, t):
    """dict(phase, layer, master, prefetch_from) of `group` at step t."""
    d = taw_sched_desc(P, D, L, 1)
    ph, la, ma, pf = _i32(), _i32(), _i32(), _i32()
    _sched_check(load().taw_sched_step(C.byref(d), group, t, C.byref(ph), C.byref(la), C.byref(ma), C.byref(pf)))
    return {"phase": ph.value, "layer": la.value, "master": ma.value, "prefetch_from": pf.value}


def taw_sched_update_step(P, D, L, layer):
    d, t = taw_sched_desc(P, D, L, 1), _i32()
    _sched_check(load().taw_sched_update_step(C.byref(d), layer, C.byref(t)))
    return t.value


def taw_sched_bubble_ratio(P, D, L, N):
    d, a, b = taw_sched_desc(P, D, L, N), C.c_double(), C.c_double()
    _sched_check(load().taw_sched_bubble_ratio(C.byref(d), C.byref(a), C.byref(b)))
    return a.value, b.value


def taw_sched_comm_elems(P, B, S, H):
    a, b, c = C.c_double(), C.c_double(), C.c_double()
    _sched_check(load().taw_sched_comm_elems(P, B, S, H, C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def taw_optimizer_step(W_chunk, chunk_dtype, master, m, v, G_shard, n_elems, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8,
                       weight_decay=0.0, grad_scale=1.0, zero_grad=False, stream=None):
    d = taw_adamw_desc(lr, beta1, beta2, eps, weight_decay, grad_scale, step, int(zero_grad))
    _check(load().taw_optimizer_step(C.byref(d), _p(W_chunk), chunk_dtype, _p(master), _p(m), _p(v), _p(G_shard), n_elems,
                                     _stream(stream)))


def taw_grad_accum(G_dst, g_src, src_dtype, n_elems, scale=1.0, stream=None):
    _check(load().taw_grad_accum(_p(G_dst), _p(g_src), src_dtype, n_elems, scale, _stream(stream)))


def taw_weight_stage(dst_buf, src_shard, nbytes, copy_stream=None, wait_event=None, ready_event=None):
    we = wait_event.cuda_event if hasattr(wait_event, "cuda_event") else wait_event
    re = ready_event.cuda_event if hasattr(ready_event, "cuda_event") else ready_event
    _check(load().taw_weight_stage(_p(dst_buf), _p(src_shard), nbytes, _stream(copy_stream), we, re))


def taw_status_string(status: int) -> str:
    return load().taw_status_string(status).decode()


def taw_last_error() -> str:
    return load().taw_last_error().decode()


# ----------------------------------------------------------------------------- taw_ops.h
def taw_op_gemm(dtype, mode, M, N, K, A, lda, B, ldb, Cout, ldc, c_dtype, accumulate=0, R=None, ldr=0,
                impl=TAW_IMPL_AUTO, stream=None):
    _check(load().taw_op_gemm(dtype, mode, M, N, K, _p(A), lda, _p(B), ldb, _p(Cout), ldc, c_dtype, accumulate, _p(R), ldr,
                              impl, _stream(stream)))


def taw_op_rmsnorm_fwd(dtype, T, H, x, gamma, eps, out, r, stream=None):
    _check(load().taw_op_rmsnorm_fwd(dtype, T, H, _p(x), _p(gamma), eps, _p(out), _p(r), _stream(stream)))


def taw_op_rmsnorm_bwd_scratch_floats(H) -> int:
    return int(load().taw_op_rmsnorm_bwd_scratch_floats(H))


def taw_op_rmsnorm_bwd(dtype, T, H, dout, z, r, gamma, dres, dz, dgamma, accumulate, scratch, stream=None):
    _check(load().taw_op_rmsnorm_bwd(dtype, T, H, _p(dout), _p(z), _p(r), _p(gamma), _p(dres), _p(dz), _p(dgamma), accumulate,
                                     _p(scratch), _stream(stream)))


def taw_op_rmsnorm_bwd_static(dtype, T, H, dout, z, r, gamma, dres, dz, dgamma, accumulate, stream=None):
    _check(load().taw_op_rmsnorm_bwd_static(dtype, T, H, _p(dout), _p(z), _p(r), _p(gamma), _p(dres), _p(dz), _p(dgamma), accumulate,
                                            _stream(stream)))


def taw_op_rope(dtype, B, S, ncols, head_dim, z, ld, rope_table, inverse=0, stream=None):
    _check(load().taw_op_rope(dtype, B, S, ncols, head_dim, _p(z), ld, _p(rope_table), inverse, _stream(stream)))


def taw_op_swiglu_fwd(dtype, T, I, gu, a, stream=None):
    _check(load().taw_op_swiglu_fwd(dtype, T, I, _p(gu), _p(a), _stream(stream)))


def taw_op_swiglu_bwd(dtype, T, I, da, gu, dgu, stream=None):
    _check(load().taw_op_swiglu_bwd(dtype, T, I, _p(da), _p(gu), _p(dgu), _stream(stream)))


def taw_op_attn_fwd(dtype, B, S, n_heads, head_dim, qkv, o, lse, impl=TAW_IMPL_AUTO, stream=None):
    _check(load().taw_op_attn_fwd(dtype, B, S, n_heads, head_dim, _p(qkv), _p(o), _p(lse), impl, _stream(stream)))


def taw_op_attn_bwd_scratch_floats(B, S, n_heads) -> int:
    return int(load().taw_op_attn_bwd_scratch_floats(B, S, n_heads))


def taw_op_attn_bwd(dtype, B, S, n_heads, head_dim, qkv, o, dO, lse, dqkv, scratch, rope_table=None, impl=TAW_IMPL_AUTO, stream=None):
    _check(load().taw_op_attn_bwd(dtype, B, S, n_heads, head_dim, _p(qkv), _p(o), _p(dO), _p(lse), _p(dqkv), _p(scratch),
                                  _p(rope_table), impl, _stream(stream)))


def taw_op_qkv_rope(dtype, B, S, n_heads, head_dim, xn, w_qkv, qkv, rope_table, impl=TAW_IMPL_AUTO, stream=None):
    _check(load().taw_op_qkv_rope(dtype, B, S, n_heads, head_dim, _p(xn), _p(w_qkv), _p(qkv), _p(rope_table), impl, _stream(stream)))


def taw_op_linear_bwd_scratch_floats(T, N, K):
    return int(load().taw_op_linear_bwd_scratch_floats(T, N, K))


def taw_op_linear_bwd(dtype, T, N, K, dy, W, x, dx, G, accumulate=0, impl=TAW_IMPL_AUTO, stream=None, scratch=None):
    _check(load().taw_op_linear_bwd(dtype, T, N, K, _p(dy), _p(W), _p(x), _p(dx), _p(G), accumulate, _p(scratch), impl, _stream(stream)))


# ----------------------------------------------------------------------------- taw_diag.h (each call waits for its kernel)
TAW_DIAG_MFMA_RANDOM, TAW_DIAG_MFMA_ZERO, TAW_DIAG_MFMA_LDS, TAW_DIAG_MFMA_LDS_LOADS = 0, 1, 2, 3


def taw_diag_mfma_loop(kind, iters=20000, src=None) -> dict:
    out = taw_diag_rate()
    nbytes = 0 if src is None else src.numel() * src.element_size()
    _check(load().taw_diag_mfma_loop(kind, iters, _p(src), nbytes, C.byref(out)))
    return {"TFLOPs": out.tflops, "clock_GHz": out.clock_ghz, "mfma_busy": out.mfma_busy, "ms": out.ms}


def taw_diag_lds_read_rate(instr, waves) -> dict:
    a, b = C.c_double(), C.c_double()
    _check(load().taw_diag_lds_read_rate(instr, waves, C.byref(a), C.byref(b)))
    return {"bytes_per_clock_per_cu": a.value, "clock_GHz": b.value}


def taw_diag_dq_update_rate(buf, S, n_heads, mode) -> dict:
    a, b = C.c_double(), C.c_double()
    _check(load().taw_diag_dq_update_rate(_p(buf), S, n_heads, mode, C.byref(a), C.byref(b)))
    return {"updates_per_s": a.value, "ms": b.value}


def taw_diag_gemm_tile_order(tiles_m, tiles_n):
    """(rows, cols): lists with the output tile of every workgroup id of a tiles_m x tiles_n GEMM grid.  Host only."""
    n = max(int(tiles_m) * int(tiles_n), 1)
    rows, cols = (C.c_int32 * n)(), (C.c_int32 * n)()
    _check(load().taw_diag_gemm_tile_order(tiles_m, tiles_n, rows, cols))
    return list(rows), list(cols)


def taw_diag_attn_ds_layout(S) -> dict:
    nqt = (S + 255) // 256
    n = 32 * nqt * (nqt + 1)
    pair = C.c_int64()
    offs = (C.c_int64 * max(n, 1))()
    slots = (C.c_int32 * 128)()
    rows = (C.c_int32 * 32)()
    _check(load().taw_diag_attn_ds_layout(S, C.byref(pair), offs, slots, rows))
    return {"pair_bytes": pair.value, "unit_offsets": list(offs)[:n], "slots": list(slots), "rows": list(rows)}


def taw_diag_store_cost_bytes() -> int:
    return int(load().taw_diag_store_cost_bytes())


def taw_diag_store_cost(buf, buf_bytes, waves, mfmas, stores) -> float:
    a = C.c_double()
    _check(load().taw_diag_store_cost(_p(buf), buf_bytes, waves, mfmas, stores, C.byref(a)))
    return a.value


def taw_diag_issue_rate(mode, kind, nvalu) -> dict:
    a, b = C.c_double(), C.c_double()
    _check(load().taw_diag_issue_rate(mode, kind, nvalu, C.byref(a), C.byref(b)))
    return {"cycles_per_slot_mfma_wave": a.value, "cycles_per_slot_last_wave": b.value}
