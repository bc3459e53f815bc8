// C-ABI front end: argument validation, weight-chunk layout, ctx/workspace partition and the
// kernel sequence of the layer's forward and backward pass.  Host code only; every arithmetic
// step is a kernel from the other files of this directory.
#include <algorithm>
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstring>
#include <cstdarg>
#include <cmath>
#include <mutex>

#include "../../include/taw.h"
#include "../../include/taw_ops.h"
#include "taw_internal.h"

using namespace taw;

// ------------------------------------------------------------------------------ error reporting
static thread_local char g_err[512] = "";

static int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

static int hip_fail(int hip_code, const char* what) {
  return fail(TAW_ERR_HIP, "%s: %s", what, hipGetErrorString((hipError_t)hip_code));
}

extern "C" const char* taw_status_string(int status) {
  switch (status) {
    case TAW_OK: return "TAW_OK";
    case TAW_ERR_NULL: return "TAW_ERR_NULL";
    case TAW_ERR_SHAPE: return "TAW_ERR_SHAPE";
    case TAW_ERR_DTYPE: return "TAW_ERR_DTYPE";
    case TAW_ERR_ALIGN: return "TAW_ERR_ALIGN";
    case TAW_ERR_WORKSPACE: return "TAW_ERR_WORKSPACE";
    case TAW_ERR_UNSUPPORTED: return "TAW_ERR_UNSUPPORTED";
    case TAW_ERR_HIP: return "TAW_ERR_HIP";
    default: return "TAW_ERR_UNKNOWN";
  }
}

extern "C" const char* taw_last_error(void) { return g_err; }

static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

#define TAW_REQUIRE_PTR(p) do { if (!(p)) return fail(TAW_ERR_NULL, "%s is NULL", #p); } while (0)
#define TAW_REQUIRE_ALIGNED(p) do { if (!aligned16(p)) return fail(TAW_ERR_ALIGN, "%s is not 16-byte aligned", #p); } while (0)
#define TAW_LAUNCH(call, what) do { int e_ = (call); if (e_) return hip_fail(e_, what); } while (0)

// ------------------------------------------------------------------------------ descriptor
static int check_desc(const taw_layer_desc* d) {
  if (!d) return fail(TAW_ERR_NULL, "desc is NULL");
  if (d->dtype != TAW_F32 && d->dtype != TAW_BF16) return fail(TAW_ERR_DTYPE, "dtype %d is neither TAW_F32 nor TAW_BF16", d->dtype);
  if (d->B <= 0 || d->S <= 0 || d->H <= 0 || d->n_heads <= 0 || d->head_dim <= 0 || d->I <= 0)
    return fail(TAW_ERR_SHAPE, "non-positive dimension (B=%d S=%d H=%d n_heads=%d head_dim=%d I=%d)", d->B, d->S, d->H, d->n_heads, d->head_dim, d->I);
  if ((int64_t)d->n_heads * d->head_dim != d->H)
    return fail(TAW_ERR_SHAPE, "H=%d != n_heads*head_dim=%d*%d", d->H, d->n_heads, d->head_dim);
  if (d->head_dim % 2) return fail(TAW_ERR_SHAPE, "head_dim=%d is odd", d->head_dim);
  if ((int64_t)d->B * d->S > (int64_t)1 << 24) return fail(TAW_ERR_SHAPE, "B*S=%lld exceeds 2^24 tokens", (long long)d->B * d->S);
  if (!(d->rms_eps >= 0.f)) return fail(TAW_ERR_SHAPE, "rms_eps must be >= 0");
  if (!(d->rope_theta > 0.f)) return fail(TAW_ERR_SHAPE, "rope_theta must be > 0");
  if (d->flags & ~(TAW_ACCUMULATE | TAW_RECOMPUTE | TAW_ATTN_BWD_FUSED | TAW_ATTN_BWD_RECOMPUTE)) return fail(TAW_ERR_SHAPE, "unknown flag bits 0x%x", d->flags);
  if ((d->flags & TAW_ATTN_BWD_FUSED) && (d->flags & TAW_ATTN_BWD_RECOMPUTE)) return fail(TAW_ERR_SHAPE, "TAW_ATTN_BWD_FUSED and TAW_ATTN_BWD_RECOMPUTE name two different forms");
  return TAW_OK;
}

// which kernel family each step of the layer uses
struct Plan {
  bool mfma_gemm;   // all GEMMs of the layer on the bf16 MFMA kernel
  bool mfma_attn;   // attention on the bf16 MFMA kernels
};

static int make_plan(const taw_layer_desc* d, Plan* p) {
  const int64_t T = (int64_t)d->B * d->S;
  p->mfma_gemm = d->dtype == TAW_BF16 && d->H % 8 == 0 && d->I % 8 == 0 &&
                 gemm_mfma_supported(DT_BF16, GEMM_NT, T, 3 * (int64_t)d->H, d->H, d->H, d->H, 3 * (int64_t)d->H, DT_BF16, 0);
  p->mfma_attn = attn_mfma_supported(d->dtype, d->S, d->n_heads, d->head_dim);
  if (!rmsnorm_supported(d->dtype, d->H))
    return fail(TAW_ERR_UNSUPPORTED, "RMSNorm kernels hold a row in registers: H=%d is too wide for them", d->H);
  if (!p->mfma_attn && !attn_generic_supported(d->S, d->head_dim))
    return fail(TAW_ERR_UNSUPPORTED, "no attention kernel for S=%d head_dim=%d dtype=%d (MFMA kernel: bf16, head_dim 128; generic kernel: S <= 4096)",
                d->S, d->head_dim, d->dtype);
  return TAW_OK;
}

extern "C" int taw_layer_weight_layout(const taw_layer_desc* desc, taw_weight_layout* out) {
  int rc = check_desc(desc);
  if (rc) return rc;
  TAW_REQUIRE_PTR(out);
  const size_t H = desc->H, I = desc->I;
  size_t off = 0;
  auto place = [&](size_t n) { size_t o = off; off = round_up(off + n, 128); return o; };
  out->gamma_attn = place(H);
  out->w_qkv = place(3 * H * H);
  out->w_o = place(H * H);
  out->gamma_mlp = place(H);
  out->w_gate_up = place(2 * I * H);
  out->w_down = place(H * I);
  out->total_elems = off;
  return TAW_OK;
}

// ------------------------------------------------------------------------------ ctx / workspace partition
struct Carve {
  char* base; size_t off;
  explicit Carve(void* b) : base(static_cast<char*>(b)), off(0) {}
  void* take(size_t bytes) { void* p = base ? base + off : nullptr; off += round_up(bytes, 256); return p; }
};

struct Ctx {       // saved by the forward for the backward
  void *xn, *qkv, *o, *h, *hn, *gu, *a; float *lse, *r1, *r2; size_t bytes;
};
struct Work {      // scratch of the backward (the forward needs none of it)
  void *da, *dgu, *dhn, *dh, *dO, *dqkv, *dxn; float *D, *partials, *splitk; size_t bytes;
};

// fp32 elements of partial weight gradients the backward of the linear y[T,N] = x[T,K] W^T needs (0: its weight gradient is not cut)
static size_t linear_bwd_scratch_floats(int64_t T, int64_t N, int64_t K) {
  if (T <= 0 || N <= 0 || K <= 0) return 0;
  int64_t chunk;
  const int sp = gemm_dual_splits(T, N, K, &chunk);
  return sp > 1 ? (size_t)sp * (size_t)N * (size_t)K : 0;
}

// which form of the MFMA attention backward the layer runs
static int attn_bwd_form_of(const taw_layer_desc* d) {
  return (d->flags & TAW_ATTN_BWD_FUSED) ? ATTN_BWD_FUSED : (d->flags & TAW_ATTN_BWD_RECOMPUTE) ? ATTN_BWD_SPLIT : ATTN_BWD_STORED;
}

static Ctx carve_ctx(const taw_layer_desc* d, void* base) {
  const size_t e = dt_size(d->dtype), T = (size_t)d->B * d->S, H = d->H, I = d->I;
  Carve c(base); Ctx x;
  x.xn = c.take(T * H * e); x.qkv = c.take(T * 3 * H * e); x.o = c.take(T * H * e); x.h = c.take(T * H * e);
  x.hn = c.take(T * H * e); x.gu = c.take(T * 2 * I * e); x.a = c.take(T * I * e);
  x.lse = (float*)c.take((size_t)d->B * d->n_heads * d->S * 4); x.r1 = (float*)c.take(T * 4); x.r2 = (float*)c.take(T * 4);
  x.bytes = c.off;
  return x;
}

static Work carve_work(const taw_layer_desc* d, void* base) {
  const size_t e = dt_size(d->dtype), T = (size_t)d->B * d->S, H = d->H, I = d->I;
  Carve c(base); Work w;
  w.da = c.take(T * I * e); w.dgu = c.take(T * 2 * I * e); w.dhn = c.take(T * H * e); w.dh = c.take(T * H * e);
  w.dO = c.take(T * H * e); w.dqkv = c.take(T * 3 * H * e); w.dxn = c.take(T * H * e);
  w.D = (float*)c.take(attn_bwd_mfma_scratch_floats(d->B, d->S, d->n_heads, attn_mfma_supported(d->dtype, d->S, d->n_heads, d->head_dim) ? attn_bwd_form_of(d) : ATTN_BWD_SPLIT) * 4);   // covers the generic kernel's B*nh*S too
  w.partials = (float*)c.take((size_t)rmsnorm_bwd_partial_rows() * H * 4);
  size_t sk = linear_bwd_scratch_floats((int64_t)T, (int64_t)H, (int64_t)I);                  // down
  sk = std::max(sk, linear_bwd_scratch_floats((int64_t)T, (int64_t)(2 * I), (int64_t)H));     // gate, up
  sk = std::max(sk, linear_bwd_scratch_floats((int64_t)T, (int64_t)H, (int64_t)H));           // output projection
  sk = std::max(sk, linear_bwd_scratch_floats((int64_t)T, (int64_t)(3 * H), (int64_t)H));     // q, k, v
  w.splitk = (float*)c.take(sk * 4);
  w.bytes = c.off;
  return w;
}

// With TAW_RECOMPUTE nothing is kept between the calls: the forward's intermediates live in the
// workspace, in front of the backward's scratch, and the backward rebuilds them there first.
static size_t ctx_bytes_of(const taw_layer_desc* d) { return (d->flags & TAW_RECOMPUTE) ? 0 : carve_ctx(d, nullptr).bytes; }
static size_t workspace_bytes_of(const taw_layer_desc* d) {
  return carve_work(d, nullptr).bytes + ((d->flags & TAW_RECOMPUTE) ? carve_ctx(d, nullptr).bytes : 0);
}

extern "C" size_t taw_layer_ctx_bytes(const taw_layer_desc* desc) {
  if (check_desc(desc)) return 0;
  return ctx_bytes_of(desc);
}
extern "C" size_t taw_layer_workspace_bytes(const taw_layer_desc* desc) {
  if (check_desc(desc)) return 0;
  return workspace_bytes_of(desc);
}

// ------------------------------------------------------------------------------ op dispatch helpers
static int gemm(const Plan& p, int dtype, int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                int64_t ldb, void* C, int64_t ldc, int c_dtype, int accumulate, const void* R, int64_t ldr, hipStream_t st) {
  if (p.mfma_gemm && gemm_mfma_supported(dtype, mode, M, N, K, lda, ldb, ldc, c_dtype, ldr))
    return launch_gemm_mfma(mode, M, N, K, A, lda, B, ldb, C, ldc, c_dtype, accumulate, R, ldr, st);
  return launch_gemm_generic(dtype, mode, M, N, K, A, lda, B, ldb, C, ldc, c_dtype, accumulate, R, ldr, st);
}

// Backward of a linear y[T,N] = x[T,K] W[N,K]^T given dy: dx[T,K] = dy W (NN) and G[N,K] (+)= dy^T x (TN).
// The two are independent; on the MFMA path they share one grid, and where the weight gradient has too few tiles to
// fill its share of the chip it is cut along T into partial products in `part` (linear_bwd_scratch_floats elements;
// nullptr: never cut), summed in a fixed order by a second kernel: the result does not depend on scheduling.
static int linear_bwd(const Plan& p, int dtype, int64_t T, int64_t N, int64_t K, const void* dy, const void* W, const void* x,
                      void* dx, float* G, int accumulate, float* part, hipStream_t st) {
  if (p.mfma_gemm && gemm_mfma_supported(dtype, GEMM_NN, T, K, N, N, K, K, dtype, 0) &&
      gemm_mfma_supported(dtype, GEMM_TN, N, K, T, N, K, K, DT_F32, 0) && gemm_mfma_dual_supported(T, N)) {
    int64_t chunk = T;
    const int sp = part ? gemm_dual_splits(T, N, K, &chunk) : 1;
    return launch_gemm_mfma_dual(N, K, T, dy, N, x, K, G, K, accumulate, T, K, N, dy, N, W, K, dx, K, part, sp, chunk, st);
  }
  int rc = gemm(p, dtype, GEMM_NN, T, K, N, dy, N, W, K, dx, K, dtype, 0, nullptr, 0, st);
  if (rc) return rc;
  return gemm(p, dtype, GEMM_TN, N, K, T, dy, N, x, K, G, K, DT_F32, accumulate, nullptr, 0, st);
}

static const char* at(const void* base, size_t elem_off, int dtype) { return static_cast<const char*>(base) + elem_off * dt_size(dtype); }

// ------------------------------------------------------------------------------ rope table
extern "C" int taw_rope_table_init(const taw_layer_desc* desc, float* rope_table, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  TAW_REQUIRE_PTR(rope_table);
  TAW_REQUIRE_ALIGNED(rope_table);
  TAW_LAUNCH(launch_rope_table(desc->S, desc->head_dim, (double)desc->rope_theta, rope_table, (hipStream_t)stream), "rope table kernel");
  return TAW_OK;
}

// ------------------------------------------------------------------------------ forward
// The forward's kernel sequence into the intermediates `c`; y == nullptr stops after the SwiGLU
// (all the backward needs when it rebuilds the intermediates).
static int run_fwd(const taw_layer_desc* desc, const Plan& p, const taw_weight_layout& L, const void* W_chunk, const float* rope_table,
                   const void* x, void* y, const Ctx& c, hipStream_t st) {
  const int dt = desc->dtype;
  const int64_t T = (int64_t)desc->B * desc->S, H = desc->H, I = desc->I;
  // xn = rmsnorm(x; gamma_attn)
  TAW_LAUNCH(launch_rmsnorm_fwd(dt, T, (int)H, x, at(W_chunk, L.gamma_attn, dt), desc->rms_eps, c.xn, c.r1, st), "rmsnorm_fwd(attn)");
  // qkv = xn Wqkv^T, q and k (the first 2H columns) rotated: in the GEMM's epilogue where its tiles allow it
  if (p.mfma_gemm && dt == DT_BF16 && desc->head_dim == 128 && gemm_mfma_supported(dt, GEMM_NT, T, 3 * H, H, H, H, 3 * H, dt, 0) &&
      gemm_mfma_rope_supported(T, 3 * H, H, 2 * H, desc->S)) {
    TAW_LAUNCH(launch_gemm_mfma_nt_rope(T, 3 * H, H, c.xn, H, at(W_chunk, L.w_qkv, dt), H, c.qkv, 3 * H, rope_table, desc->S, 2 * H, st),
               "gemm qkv + rope");
  } else {
    TAW_LAUNCH(gemm(p, dt, GEMM_NT, T, 3 * H, H, c.xn, H, at(W_chunk, L.w_qkv, dt), H, c.qkv, 3 * H, dt, 0, nullptr, 0, st), "gemm qkv");
    TAW_LAUNCH(launch_rope(dt, desc->B, desc->S, (int)(2 * H), desc->head_dim, c.qkv, 3 * H, rope_table, 0, st), "rope");
  }
  // o = causal softmax attention
  if (p.mfma_attn) TAW_LAUNCH(launch_attn_fwd_mfma(desc->B, desc->S, desc->n_heads, c.qkv, c.o, c.lse, st), "attention fwd (mfma)");
  else TAW_LAUNCH(launch_attn_fwd_generic(dt, desc->B, desc->S, desc->n_heads, desc->head_dim, c.qkv, c.o, c.lse, st), "attention fwd (generic)");
  // h = x + o Wo^T
  TAW_LAUNCH(gemm(p, dt, GEMM_NT, T, H, H, c.o, H, at(W_chunk, L.w_o, dt), H, c.h, H, dt, 0, x, H, st), "gemm o-proj");
  // hn = rmsnorm(h; gamma_mlp)
  TAW_LAUNCH(launch_rmsnorm_fwd(dt, T, (int)H, c.h, at(W_chunk, L.gamma_mlp, dt), desc->rms_eps, c.hn, c.r2, st), "rmsnorm_fwd(mlp)");
  // gu = hn Wgu^T ; a = silu(g) u
  TAW_LAUNCH(gemm(p, dt, GEMM_NT, T, 2 * I, H, c.hn, H, at(W_chunk, L.w_gate_up, dt), H, c.gu, 2 * I, dt, 0, nullptr, 0, st), "gemm gate/up");
  TAW_LAUNCH(launch_swiglu_fwd(dt, T, (int)I, c.gu, c.a, st), "swiglu_fwd");
  // y = h + a Wd^T
  if (y) TAW_LAUNCH(gemm(p, dt, GEMM_NT, T, H, I, c.a, I, at(W_chunk, L.w_down, dt), I, y, H, dt, 0, c.h, H, st), "gemm down");
  return TAW_OK;
}

extern "C" int taw_layer_fwd(const taw_layer_desc* desc, const void* W_chunk, const float* rope_table, const void* x, void* y,
                             void* ctx, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const bool recompute = (desc->flags & TAW_RECOMPUTE) != 0;
  TAW_REQUIRE_PTR(W_chunk); TAW_REQUIRE_PTR(rope_table); TAW_REQUIRE_PTR(x); TAW_REQUIRE_PTR(y);
  if (!recompute) TAW_REQUIRE_PTR(ctx);
  TAW_REQUIRE_PTR(workspace);
  TAW_REQUIRE_ALIGNED(W_chunk); TAW_REQUIRE_ALIGNED(rope_table); TAW_REQUIRE_ALIGNED(x); TAW_REQUIRE_ALIGNED(y);
  TAW_REQUIRE_ALIGNED(ctx); TAW_REQUIRE_ALIGNED(workspace);
  if (x == y) return fail(TAW_ERR_SHAPE, "y must not alias x");
  if (workspace_bytes < workspace_bytes_of(desc))
    return fail(TAW_ERR_WORKSPACE, "workspace_bytes=%zu < required %zu", workspace_bytes, workspace_bytes_of(desc));
  Plan p;
  rc = make_plan(desc, &p);
  if (rc) return rc;
  taw_weight_layout L;
  taw_layer_weight_layout(desc, &L);
  return run_fwd(desc, p, L, W_chunk, rope_table, x, y, carve_ctx(desc, recompute ? workspace : ctx), (hipStream_t)stream);
}

// ------------------------------------------------------------------------------ backward
extern "C" int taw_layer_bwd(const taw_layer_desc* desc, const void* W_chunk, const float* rope_table, const void* x, const void* dy,
                             const void* ctx, void* dx, float* G_shard, void* workspace, size_t workspace_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const bool recompute = (desc->flags & TAW_RECOMPUTE) != 0;
  TAW_REQUIRE_PTR(W_chunk); TAW_REQUIRE_PTR(rope_table); TAW_REQUIRE_PTR(x); TAW_REQUIRE_PTR(dy);
  if (!recompute) TAW_REQUIRE_PTR(ctx);
  TAW_REQUIRE_PTR(dx); TAW_REQUIRE_PTR(G_shard); TAW_REQUIRE_PTR(workspace);
  TAW_REQUIRE_ALIGNED(W_chunk); TAW_REQUIRE_ALIGNED(rope_table); TAW_REQUIRE_ALIGNED(x); TAW_REQUIRE_ALIGNED(dy);
  TAW_REQUIRE_ALIGNED(ctx); TAW_REQUIRE_ALIGNED(dx); TAW_REQUIRE_ALIGNED(G_shard); TAW_REQUIRE_ALIGNED(workspace);
  if (dx == dy || dx == x) return fail(TAW_ERR_SHAPE, "dx must not alias dy or x");
  if (workspace_bytes < workspace_bytes_of(desc))
    return fail(TAW_ERR_WORKSPACE, "workspace_bytes=%zu < required %zu", workspace_bytes, workspace_bytes_of(desc));
  Plan p;
  rc = make_plan(desc, &p);
  if (rc) return rc;
  taw_weight_layout L;
  taw_layer_weight_layout(desc, &L);
  const hipStream_t st = (hipStream_t)stream;
  const int dt = desc->dtype;
  const int acc = (desc->flags & TAW_ACCUMULATE) ? 1 : 0;
  const int64_t T = (int64_t)desc->B * desc->S, H = desc->H, I = desc->I;
  // the saved intermediates, or (TAW_RECOMPUTE) the front of the workspace, rebuilt here from x
  const Ctx c = carve_ctx(desc, recompute ? workspace : const_cast<void*>(ctx));
  const Work w = carve_work(desc, static_cast<char*>(workspace) + (recompute ? c.bytes : 0));
  if (recompute) {
    rc = run_fwd(desc, p, L, W_chunk, rope_table, x, nullptr, c, st);
    if (rc) return rc;
  }

  // y = h + a Wd^T :  da = dy Wd ;  G.Wd (+)= dy^T a
  TAW_LAUNCH(linear_bwd(p, dt, T, H, I, dy, at(W_chunk, L.w_down, dt), c.a, w.da, G_shard + L.w_down, acc, w.splitk, st), "gemm da, G.w_down");
  // a = silu(g) u
  TAW_LAUNCH(launch_swiglu_bwd(dt, T, (int)I, w.da, c.gu, w.dgu, st), "swiglu_bwd");
  // gu = hn Wgu^T :  dhn = dgu Wgu ;  G.Wgu (+)= dgu^T hn
  TAW_LAUNCH(linear_bwd(p, dt, T, 2 * I, H, w.dgu, at(W_chunk, L.w_gate_up, dt), c.hn, w.dhn, G_shard + L.w_gate_up, acc, w.splitk, st), "gemm dhn, G.w_gate_up");
  // hn = rmsnorm(h) :  dh = dy + rmsnorm_bwd(dhn) ;  G.gamma_mlp
  TAW_LAUNCH(launch_rmsnorm_bwd(dt, T, (int)H, w.dhn, c.h, c.r2, at(W_chunk, L.gamma_mlp, dt), dy, w.dh, G_shard + L.gamma_mlp, acc, w.partials, st), "rmsnorm_bwd(mlp)");
  // h = x + o Wo^T :  do = dh Wo ;  G.Wo (+)= dh^T o
  TAW_LAUNCH(linear_bwd(p, dt, T, H, H, w.dh, at(W_chunk, L.w_o, dt), c.o, w.dO, G_shard + L.w_o, acc, w.splitk, st), "gemm do, G.w_o");
  // attention backward
  // attention backward, then the rotary backward on dq, dk (the MFMA kernels apply it to their accumulators before storing)
  if (p.mfma_attn) {
    TAW_LAUNCH(launch_attn_bwd_mfma(desc->B, desc->S, desc->n_heads, c.qkv, c.o, w.dO, c.lse, w.D, w.dqkv, rope_table,
                                    attn_bwd_form_of(desc), st), "attention bwd (mfma)");
  } else {
    TAW_LAUNCH(launch_attn_rowdot(dt, desc->B, desc->S, desc->n_heads, desc->head_dim, c.o, H, w.dO, H, w.D, st), "attention row dot");
    TAW_LAUNCH(launch_attn_bwd_generic(dt, desc->B, desc->S, desc->n_heads, desc->head_dim, c.qkv, w.dO, c.lse, w.D, w.dqkv, st), "attention bwd (generic)");
    TAW_LAUNCH(launch_rope(dt, desc->B, desc->S, (int)(2 * H), desc->head_dim, w.dqkv, 3 * H, rope_table, 1, st), "rope bwd");
  }
  // qkv = xn Wqkv^T :  dxn = dqkv Wqkv ;  G.Wqkv (+)= dqkv^T xn
  TAW_LAUNCH(linear_bwd(p, dt, T, 3 * H, H, w.dqkv, at(W_chunk, L.w_qkv, dt), c.xn, w.dxn, G_shard + L.w_qkv, acc, w.splitk, st), "gemm dxn, G.w_qkv");
  // xn = rmsnorm(x) :  dx = dh + rmsnorm_bwd(dxn) ;  G.gamma_attn
  TAW_LAUNCH(launch_rmsnorm_bwd(dt, T, (int)H, w.dxn, x, c.r1, at(W_chunk, L.gamma_attn, dt), w.dh, dx, G_shard + L.gamma_attn, acc, w.partials, st), "rmsnorm_bwd(attn)");
  return TAW_OK;
}

// ------------------------------------------------------------------------------ grad accumulation / staging
extern "C" int taw_grad_accum(float* G_dst, const void* g_src, int32_t src_dtype, size_t n_elems, float scale, void* stream) {
  if (src_dtype != TAW_F32 && src_dtype != TAW_BF16) return fail(TAW_ERR_DTYPE, "src_dtype %d is neither TAW_F32 nor TAW_BF16", src_dtype);
  if (n_elems == 0) return TAW_OK;
  TAW_REQUIRE_PTR(G_dst); TAW_REQUIRE_PTR(g_src);
  TAW_REQUIRE_ALIGNED(G_dst); TAW_REQUIRE_ALIGNED(g_src);
  const char* a = reinterpret_cast<const char*>(G_dst);
  const char* b = static_cast<const char*>(g_src);
  if (a < b + n_elems * dt_size(src_dtype) && b < a + n_elems * 4) return fail(TAW_ERR_SHAPE, "G_dst and g_src overlap");
  TAW_LAUNCH(launch_grad_accum(G_dst, g_src, src_dtype, n_elems, scale, (hipStream_t)stream), "grad_accum kernel");
  return TAW_OK;
}

extern "C" int taw_optimizer_step(const taw_adamw_desc* opt, void* W_chunk, int32_t chunk_dtype, float* master, float* m, float* v,
                                  float* G_shard, size_t n_elems, void* stream) {
  if (!opt) return fail(TAW_ERR_NULL, "opt is NULL");
  if (chunk_dtype != TAW_F32 && chunk_dtype != TAW_BF16) return fail(TAW_ERR_DTYPE, "chunk_dtype %d is neither TAW_F32 nor TAW_BF16", chunk_dtype);
  if (opt->step < 1) return fail(TAW_ERR_SHAPE, "step=%d must be >= 1", opt->step);
  if (!(opt->beta1 >= 0.f && opt->beta1 < 1.f) || !(opt->beta2 >= 0.f && opt->beta2 < 1.f) || !(opt->eps >= 0.f))
    return fail(TAW_ERR_SHAPE, "need 0 <= beta1, beta2 < 1 and eps >= 0");
  if (n_elems == 0) return TAW_OK;
  TAW_REQUIRE_PTR(W_chunk); TAW_REQUIRE_PTR(master); TAW_REQUIRE_PTR(m); TAW_REQUIRE_PTR(v); TAW_REQUIRE_PTR(G_shard);
  TAW_REQUIRE_ALIGNED(W_chunk); TAW_REQUIRE_ALIGNED(master); TAW_REQUIRE_ALIGNED(m); TAW_REQUIRE_ALIGNED(v); TAW_REQUIRE_ALIGNED(G_shard);
  const char* ptrs[5] = {static_cast<const char*>(W_chunk), reinterpret_cast<const char*>(master), reinterpret_cast<const char*>(m),
                         reinterpret_cast<const char*>(v), reinterpret_cast<const char*>(G_shard)};
  const size_t lens[5] = {n_elems * dt_size(chunk_dtype), n_elems * 4, n_elems * 4, n_elems * 4, n_elems * 4};
  for (int a = 0; a < 5; ++a)
    for (int b = a + 1; b < 5; ++b)
      if (ptrs[a] < ptrs[b] + lens[b] && ptrs[b] < ptrs[a] + lens[a]) return fail(TAW_ERR_SHAPE, "optimizer arrays overlap");
  const double b1c = 1.0 - pow((double)opt->beta1, (double)opt->step), b2c = 1.0 - pow((double)opt->beta2, (double)opt->step);
  TAW_LAUNCH(launch_adamw(chunk_dtype, W_chunk, master, m, v, G_shard, n_elems, opt->lr, opt->beta1, opt->beta2, opt->eps, opt->weight_decay,
                          (float)b1c, (float)b2c, opt->grad_scale, opt->zero_grad, (hipStream_t)stream), "adamw kernel");
  return TAW_OK;
}

extern "C" int taw_weight_stage(void* dst_buf, const void* src_shard, size_t bytes, void* copy_stream, void* wait_event, void* ready_event) {
  if (bytes % 16) return fail(TAW_ERR_SHAPE, "bytes=%zu is not a multiple of 16", bytes);
  if (bytes) {
    TAW_REQUIRE_PTR(dst_buf); TAW_REQUIRE_PTR(src_shard);
    TAW_REQUIRE_ALIGNED(dst_buf); TAW_REQUIRE_ALIGNED(src_shard);
    const char* a = static_cast<const char*>(dst_buf);
    const char* b = static_cast<const char*>(src_shard);
    if (a < b + bytes && b < a + bytes) return fail(TAW_ERR_SHAPE, "dst_buf and src_shard overlap");
  }
  const hipStream_t st = (hipStream_t)copy_stream;
  if (wait_event) {
    hipError_t e = hipStreamWaitEvent(st, (hipEvent_t)wait_event, 0);
    if (e != hipSuccess) return hip_fail((int)e, "hipStreamWaitEvent");
  }
  if (bytes) TAW_LAUNCH(launch_stage_copy(dst_buf, src_shard, bytes, st), "stage copy kernel");
  if (ready_event) {
    hipError_t e = hipEventRecord((hipEvent_t)ready_event, st);
    if (e != hipSuccess) return hip_fail((int)e, "hipEventRecord");
  }
  return TAW_OK;
}

// ------------------------------------------------------------------------------ kernel-level entry points
static int check_dtype(int32_t dt) {
  if (dt != TAW_F32 && dt != TAW_BF16) return fail(TAW_ERR_DTYPE, "dtype %d is neither TAW_F32 nor TAW_BF16", dt);
  return TAW_OK;
}

extern "C" int taw_op_gemm(int32_t dtype, int32_t mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                           int64_t ldb, void* C, int64_t ldc, int32_t c_dtype, int32_t accumulate, const void* R, int64_t ldr,
                           int32_t impl, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (c_dtype != dtype && c_dtype != TAW_F32) return fail(TAW_ERR_DTYPE, "c_dtype must equal dtype or be TAW_F32");
  if (mode < TAW_GEMM_NT || mode > TAW_GEMM_TN) return fail(TAW_ERR_SHAPE, "unknown gemm mode %d", mode);
  if (M < 0 || N < 0 || K < 0) return fail(TAW_ERR_SHAPE, "negative dimension");
  if (M == 0 || N == 0) return TAW_OK;
  TAW_REQUIRE_PTR(C); TAW_REQUIRE_ALIGNED(C);
  if (K > 0) { TAW_REQUIRE_PTR(A); TAW_REQUIRE_PTR(B); TAW_REQUIRE_ALIGNED(A); TAW_REQUIRE_ALIGNED(B); }
  if (R) TAW_REQUIRE_ALIGNED(R);
  const int64_t a_min = mode == TAW_GEMM_TN ? M : K, b_min = mode == TAW_GEMM_NT ? K : N;
  if (lda < a_min || ldb < b_min || ldc < N || (R && ldr < N)) return fail(TAW_ERR_SHAPE, "leading dimension smaller than the row length");
  const hipStream_t st = (hipStream_t)stream;
  const bool can = gemm_mfma_supported(dtype, mode, M, N, K, lda, ldb, ldc, c_dtype, R ? ldr : 0);
  if (impl == TAW_IMPL_MFMA && !can) return fail(TAW_ERR_UNSUPPORTED, "MFMA GEMM needs bf16 and M, N, K, strides multiples of 8");
  if (impl != TAW_IMPL_GENERIC && can)
    TAW_LAUNCH(launch_gemm_mfma(mode, M, N, K, A, lda, B, ldb, C, ldc, c_dtype, accumulate, R, ldr, st), "gemm (mfma)");
  else
    TAW_LAUNCH(launch_gemm_generic(dtype, mode, M, N, K, A, lda, B, ldb, C, ldc, c_dtype, accumulate, R, ldr, st), "gemm (generic)");
  return TAW_OK;
}

extern "C" int taw_op_rmsnorm_fwd(int32_t dtype, int64_t T, int32_t H, const void* x, const void* gamma, float eps, void* out,
                                  float* r, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || H <= 0) return fail(TAW_ERR_SHAPE, "bad shape T=%lld H=%d", (long long)T, H);
  if (!rmsnorm_supported(dtype, H)) return fail(TAW_ERR_UNSUPPORTED, "H=%d too wide for the RMSNorm kernels", H);
  if (T == 0) return TAW_OK;
  TAW_REQUIRE_PTR(x); TAW_REQUIRE_PTR(gamma); TAW_REQUIRE_PTR(out); TAW_REQUIRE_PTR(r);
  TAW_REQUIRE_ALIGNED(x); TAW_REQUIRE_ALIGNED(gamma); TAW_REQUIRE_ALIGNED(out); TAW_REQUIRE_ALIGNED(r);
  TAW_LAUNCH(launch_rmsnorm_fwd(dtype, T, H, x, gamma, eps, out, r, (hipStream_t)stream), "rmsnorm_fwd");
  return TAW_OK;
}

extern "C" size_t taw_op_rmsnorm_bwd_scratch_floats(int32_t H) { return H > 0 ? (size_t)rmsnorm_bwd_partial_rows() * (size_t)H : 0; }

extern "C" int taw_op_rmsnorm_bwd(int32_t dtype, int64_t T, int32_t H, const void* dout, const void* z, const float* r, const void* gamma,
                                  const void* dres, void* dz, float* dgamma, int32_t accumulate, float* scratch, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || H <= 0) return fail(TAW_ERR_SHAPE, "bad shape T=%lld H=%d", (long long)T, H);
  if (!rmsnorm_supported(dtype, H)) return fail(TAW_ERR_UNSUPPORTED, "H=%d too wide for the RMSNorm kernels", H);
  if (T == 0) return TAW_OK;
  TAW_REQUIRE_PTR(dout); TAW_REQUIRE_PTR(z); TAW_REQUIRE_PTR(r); TAW_REQUIRE_PTR(gamma); TAW_REQUIRE_PTR(dz);
  TAW_REQUIRE_PTR(dgamma); TAW_REQUIRE_PTR(scratch);
  TAW_REQUIRE_ALIGNED(dout); TAW_REQUIRE_ALIGNED(z); TAW_REQUIRE_ALIGNED(gamma); TAW_REQUIRE_ALIGNED(dz); TAW_REQUIRE_ALIGNED(scratch);
  if (dres) TAW_REQUIRE_ALIGNED(dres);
  TAW_LAUNCH(launch_rmsnorm_bwd(dtype, T, H, dout, z, r, gamma, dres, dz, dgamma, accumulate, scratch, (hipStream_t)stream), "rmsnorm_bwd");
  return TAW_OK;
}

// ---- the same operation for callers that cannot allocate: the partial-sum scratch lives in a static device array.
// The array's name is only a host-side handle; its device address is looked up once per device (with that device
// current) and kept, and that address is what the launcher and its kernels get.
static constexpr int kStaticNormMaxH = 8192;
static __device__ __align__(256) float g_norm_scratch[(size_t)512 * kStaticNormMaxH];      // 16 MiB on every GPU the library runs on
static constexpr int kMaxDevices = 64;
static float* g_norm_scratch_ptr[kMaxDevices];
static std::mutex g_norm_scratch_mu;

static int norm_scratch_for_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_fail((int)e, "hipGetDevice");
  if (dev < 0 || dev >= kMaxDevices) return fail(TAW_ERR_UNSUPPORTED, "device ordinal %d is beyond the %d this entry point keeps a scratch address for", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_norm_scratch_mu);
  if (!g_norm_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_norm_scratch));
    if (e != hipSuccess) return hip_fail((int)e, "hipGetSymbolAddress(static RMSNorm scratch)");
    if (!p) return fail(TAW_ERR_HIP, "hipGetSymbolAddress returned a null address for the static RMSNorm scratch");
    g_norm_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_norm_scratch_ptr[dev];
  return TAW_OK;
}

extern "C" int taw_op_rmsnorm_bwd_static(int32_t dtype, int64_t T, int32_t H, const void* dout, const void* z, const float* r,
                                         const void* gamma, const void* dres, void* dz, float* dgamma, int32_t accumulate, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || H <= 0) return fail(TAW_ERR_SHAPE, "bad shape T=%lld H=%d", (long long)T, H);
  if (H > kStaticNormMaxH)
    return fail(TAW_ERR_WORKSPACE, "H=%d exceeds the %d columns the static scratch of taw_op_rmsnorm_bwd_static holds; use taw_op_rmsnorm_bwd with a caller-owned scratch",
                H, kStaticNormMaxH);
  if (!rmsnorm_supported(dtype, H)) return fail(TAW_ERR_UNSUPPORTED, "H=%d too wide for the RMSNorm kernels", H);
  static_assert((size_t)512 * kStaticNormMaxH * sizeof(float) == sizeof(g_norm_scratch), "scratch size");
  if ((size_t)rmsnorm_bwd_partial_rows() * (size_t)H * sizeof(float) > sizeof(g_norm_scratch))
    return fail(TAW_ERR_WORKSPACE, "static scratch too small for H=%d", H);
  if (T == 0) return TAW_OK;
  TAW_REQUIRE_PTR(dout); TAW_REQUIRE_PTR(z); TAW_REQUIRE_PTR(r); TAW_REQUIRE_PTR(gamma); TAW_REQUIRE_PTR(dz); TAW_REQUIRE_PTR(dgamma);
  TAW_REQUIRE_ALIGNED(dout); TAW_REQUIRE_ALIGNED(z); TAW_REQUIRE_ALIGNED(gamma); TAW_REQUIRE_ALIGNED(dz);
  if (dres) TAW_REQUIRE_ALIGNED(dres);
  float* scratch = nullptr;
  rc = norm_scratch_for_current_device(&scratch);
  if (rc) return rc;
  // every partial row the column-sum pass reads is written by this call's first kernel: nothing has to start at zero
  TAW_LAUNCH(launch_rmsnorm_bwd(dtype, T, H, dout, z, r, gamma, dres, dz, dgamma, accumulate, scratch, (hipStream_t)stream), "rmsnorm_bwd (static scratch)");
  return TAW_OK;
}

extern "C" int taw_op_rope(int32_t dtype, int32_t B, int32_t S, int32_t ncols, int32_t head_dim, void* z, int64_t ld,
                           const float* rope_table, int32_t inverse, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (B < 0 || S < 0 || ncols < 0 || head_dim <= 0 || head_dim % 2 || ncols % head_dim || ld < ncols)
    return fail(TAW_ERR_SHAPE, "bad rope shape (B=%d S=%d ncols=%d head_dim=%d ld=%lld)", B, S, ncols, head_dim, (long long)ld);
  if (B == 0 || S == 0 || ncols == 0) return TAW_OK;
  TAW_REQUIRE_PTR(z); TAW_REQUIRE_PTR(rope_table); TAW_REQUIRE_ALIGNED(z); TAW_REQUIRE_ALIGNED(rope_table);
  TAW_LAUNCH(launch_rope(dtype, B, S, ncols, head_dim, z, ld, rope_table, inverse, (hipStream_t)stream), "rope");
  return TAW_OK;
}

extern "C" int taw_op_swiglu_fwd(int32_t dtype, int64_t T, int32_t I, const void* gu, void* a, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || I < 0) return fail(TAW_ERR_SHAPE, "negative dimension");
  if (T == 0 || I == 0) return TAW_OK;
  TAW_REQUIRE_PTR(gu); TAW_REQUIRE_PTR(a); TAW_REQUIRE_ALIGNED(gu); TAW_REQUIRE_ALIGNED(a);
  TAW_LAUNCH(launch_swiglu_fwd(dtype, T, I, gu, a, (hipStream_t)stream), "swiglu_fwd");
  return TAW_OK;
}

extern "C" int taw_op_swiglu_bwd(int32_t dtype, int64_t T, int32_t I, const void* da, const void* gu, void* dgu, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || I < 0) return fail(TAW_ERR_SHAPE, "negative dimension");
  if (T == 0 || I == 0) return TAW_OK;
  TAW_REQUIRE_PTR(da); TAW_REQUIRE_PTR(gu); TAW_REQUIRE_PTR(dgu);
  TAW_REQUIRE_ALIGNED(da); TAW_REQUIRE_ALIGNED(gu); TAW_REQUIRE_ALIGNED(dgu);
  TAW_LAUNCH(launch_swiglu_bwd(dtype, T, I, da, gu, dgu, (hipStream_t)stream), "swiglu_bwd");
  return TAW_OK;
}

static int check_attn(int32_t dtype, int32_t B, int32_t S, int32_t nh, int32_t d, int32_t impl, bool* use_mfma) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (B <= 0 || S <= 0 || nh <= 0 || d <= 0 || d % 2) return fail(TAW_ERR_SHAPE, "bad attention shape (B=%d S=%d n_heads=%d head_dim=%d)", B, S, nh, d);
  if (impl < TAW_IMPL_AUTO || impl > TAW_IMPL_MFMA_STORED) return fail(TAW_ERR_SHAPE, "unknown impl %d", impl);
  const bool can = attn_mfma_supported(dtype, S, nh, d);
  if (impl >= TAW_IMPL_MFMA && !can) return fail(TAW_ERR_UNSUPPORTED, "MFMA attention needs bf16 and head_dim 128");
  *use_mfma = can && impl != TAW_IMPL_GENERIC;
  if (!*use_mfma && !attn_generic_supported(S, d)) return fail(TAW_ERR_UNSUPPORTED, "generic attention kernel takes S <= 4096");
  return TAW_OK;
}

extern "C" int taw_op_attn_fwd(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* qkv, void* o,
                               float* lse, int32_t impl, void* stream) {
  bool mf;
  int rc = check_attn(dtype, B, S, n_heads, head_dim, impl, &mf);
  if (rc) return rc;
  if (impl > TAW_IMPL_MFMA) return fail(TAW_ERR_SHAPE, "impl %d selects a form of the attention backward", impl);
  TAW_REQUIRE_PTR(qkv); TAW_REQUIRE_PTR(o); TAW_REQUIRE_PTR(lse);
  TAW_REQUIRE_ALIGNED(qkv); TAW_REQUIRE_ALIGNED(o); TAW_REQUIRE_ALIGNED(lse);
  if (mf) TAW_LAUNCH(launch_attn_fwd_mfma(B, S, n_heads, qkv, o, lse, (hipStream_t)stream), "attention fwd (mfma)");
  else TAW_LAUNCH(launch_attn_fwd_generic(dtype, B, S, n_heads, head_dim, qkv, o, lse, (hipStream_t)stream), "attention fwd (generic)");
  return TAW_OK;
}

extern "C" size_t taw_op_attn_bwd_scratch_floats(int32_t B, int32_t S, int32_t n_heads) {
  if (B <= 0 || S <= 0 || n_heads <= 0) return 0;
  return attn_bwd_mfma_scratch_floats(B, S, n_heads, ATTN_BWD_ANY);
}

extern "C" int taw_op_attn_bwd(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* qkv, const void* o,
                               const void* dO, const float* lse, void* dqkv, float* scratch, const float* rope_table, int32_t impl,
                               void* stream) {
  bool mf;
  int rc = check_attn(dtype, B, S, n_heads, head_dim, impl, &mf);
  if (rc) return rc;
  TAW_REQUIRE_PTR(qkv); TAW_REQUIRE_PTR(o); TAW_REQUIRE_PTR(dO); TAW_REQUIRE_PTR(lse); TAW_REQUIRE_PTR(dqkv); TAW_REQUIRE_PTR(scratch);
  TAW_REQUIRE_ALIGNED(qkv); TAW_REQUIRE_ALIGNED(o); TAW_REQUIRE_ALIGNED(dO); TAW_REQUIRE_ALIGNED(lse); TAW_REQUIRE_ALIGNED(dqkv);
  TAW_REQUIRE_ALIGNED(scratch); TAW_REQUIRE_ALIGNED(rope_table);
  const hipStream_t st = (hipStream_t)stream;
  const int64_t H = (int64_t)n_heads * head_dim;
  if (mf) {
    const int form = impl == TAW_IMPL_MFMA_FUSED ? ATTN_BWD_FUSED : impl == TAW_IMPL_MFMA_ATOMIC ? ATTN_BWD_FUSED_ATOMIC : impl == TAW_IMPL_MFMA ? ATTN_BWD_SPLIT : ATTN_BWD_STORED;
    TAW_LAUNCH(launch_attn_bwd_mfma(B, S, n_heads, qkv, o, dO, lse, scratch, dqkv, rope_table, form, st), "attention bwd (mfma)");
  } else {
    TAW_LAUNCH(launch_attn_rowdot(dtype, B, S, n_heads, head_dim, o, H, dO, H, scratch, st), "attention row dot");
    TAW_LAUNCH(launch_attn_bwd_generic(dtype, B, S, n_heads, head_dim, qkv, dO, lse, scratch, dqkv, st), "attention bwd (generic)");
    if (rope_table) TAW_LAUNCH(launch_rope(dtype, B, S, (int)(2 * H), head_dim, dqkv, 3 * H, rope_table, 1, st), "rope bwd");
  }
  return TAW_OK;
}

extern "C" int taw_op_qkv_rope(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* xn, const void* w_qkv,
                               void* qkv, const float* rope_table, int32_t impl, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (B <= 0 || S <= 0 || n_heads <= 0 || head_dim <= 0 || head_dim % 2) return fail(TAW_ERR_SHAPE, "bad shape (B=%d S=%d n_heads=%d head_dim=%d)", B, S, n_heads, head_dim);
  if ((int64_t)B * S > (int64_t)1 << 24) return fail(TAW_ERR_SHAPE, "B*S exceeds 2^24 tokens");
  TAW_REQUIRE_PTR(xn); TAW_REQUIRE_PTR(w_qkv); TAW_REQUIRE_PTR(qkv); TAW_REQUIRE_PTR(rope_table);
  TAW_REQUIRE_ALIGNED(xn); TAW_REQUIRE_ALIGNED(w_qkv); TAW_REQUIRE_ALIGNED(qkv); TAW_REQUIRE_ALIGNED(rope_table);
  const hipStream_t st = (hipStream_t)stream;
  const int64_t T = (int64_t)B * S, H = (int64_t)n_heads * head_dim;
  const bool can = gemm_mfma_supported(dtype, GEMM_NT, T, 3 * H, H, H, H, 3 * H, dtype, 0);
  if (impl == TAW_IMPL_MFMA && !can) return fail(TAW_ERR_UNSUPPORTED, "MFMA GEMM needs bf16 and H a multiple of 8");
  if (impl != TAW_IMPL_GENERIC && can) {
    if (head_dim == 128 && gemm_mfma_rope_supported(T, 3 * H, H, 2 * H, S)) {
      TAW_LAUNCH(launch_gemm_mfma_nt_rope(T, 3 * H, H, xn, H, w_qkv, H, qkv, 3 * H, rope_table, S, 2 * H, st), "gemm qkv + rope");
      return TAW_OK;
    }
    TAW_LAUNCH(launch_gemm_mfma(GEMM_NT, T, 3 * H, H, xn, H, w_qkv, H, qkv, 3 * H, dtype, 0, nullptr, 0, st), "gemm qkv (mfma)");
  } else {
    TAW_LAUNCH(launch_gemm_generic(dtype, GEMM_NT, T, 3 * H, H, xn, H, w_qkv, H, qkv, 3 * H, dtype, 0, nullptr, 0, st), "gemm qkv (generic)");
  }
  TAW_LAUNCH(launch_rope(dtype, B, S, (int)(2 * H), head_dim, qkv, 3 * H, rope_table, 0, st), "rope");
  return TAW_OK;
}

extern "C" size_t taw_op_linear_bwd_scratch_floats(int64_t T, int64_t N, int64_t K) { return linear_bwd_scratch_floats(T, N, K); }

extern "C" int taw_op_linear_bwd(int32_t dtype, int64_t T, int64_t N, int64_t K, const void* dy, const void* W, const void* x, void* dx,
                                 float* G, int32_t accumulate, float* scratch, int32_t impl, void* stream) {
  int rc = check_dtype(dtype);
  if (rc) return rc;
  if (T < 0 || N < 0 || K < 0) return fail(TAW_ERR_SHAPE, "negative dimension");
  if (impl < TAW_IMPL_AUTO || impl > TAW_IMPL_MFMA) return fail(TAW_ERR_SHAPE, "unknown impl %d", impl);
  if (T == 0 || N == 0 || K == 0) return TAW_OK;
  TAW_REQUIRE_PTR(dy); TAW_REQUIRE_PTR(W); TAW_REQUIRE_PTR(x); TAW_REQUIRE_PTR(dx); TAW_REQUIRE_PTR(G);
  TAW_REQUIRE_ALIGNED(dy); TAW_REQUIRE_ALIGNED(W); TAW_REQUIRE_ALIGNED(x); TAW_REQUIRE_ALIGNED(dx); TAW_REQUIRE_ALIGNED(G);
  const hipStream_t st = (hipStream_t)stream;
  const bool can = gemm_mfma_supported(dtype, GEMM_NN, T, K, N, N, K, K, dtype, 0) &&
                   gemm_mfma_supported(dtype, GEMM_TN, N, K, T, N, K, K, DT_F32, 0);
  if (impl == TAW_IMPL_MFMA && !can) return fail(TAW_ERR_UNSUPPORTED, "MFMA GEMMs need bf16 and N, K multiples of 8");
  Plan p;
  p.mfma_gemm = can && impl != TAW_IMPL_GENERIC;
  p.mfma_attn = false;
  if (scratch) TAW_REQUIRE_ALIGNED(scratch);
  TAW_LAUNCH(linear_bwd(p, dtype, T, N, K, dy, W, x, dx, G, accumulate ? 1 : 0, scratch, st), "linear backward");
  return TAW_OK;
}
