/* taw_ops.h -- kernel-level entry points of the decoder-layer library.
 *
 * taw_layer_fwd / taw_layer_bwd (taw.h) are sequences of the operations below; these entry
 * points launch one of them on its own so that each kernel can be checked against the matching
 * step of the layer definition and timed against its roofline.  Same rules as taw.h: device
 * pointers, 16-byte aligned, caller-owned, enqueued on `stream`, int status returned, all
 * validation on the host before the launch.  `dtype` is a taw_dtype (storage of activations and
 * weights); arithmetic is fp32 with fp32 accumulation (bf16 MFMA products accumulate in fp32).
 *
 * `impl` selects the kernel family: TAW_IMPL_AUTO picks the MFMA kernel when the shape allows it
 * (bf16, dimensions multiples of 8; attention: head_dim 128) and the shape-generic kernel
 * otherwise; TAW_IMPL_GENERIC / TAW_IMPL_MFMA force one and return TAW_ERR_UNSUPPORTED when it
 * cannot take the shape.
 */
#ifndef TAW_OPS_H
#define TAW_OPS_H

#include "taw.h"

#ifdef __cplusplus
extern "C" {
#endif

enum { TAW_IMPL_AUTO = 0, TAW_IMPL_GENERIC = 1, TAW_IMPL_MFMA = 2,
       /* taw_op_attn_bwd only: the forms of the MFMA backward.  TAW_IMPL_MFMA is the pair of kernels (dK/dV, then dQ) that
          each recompute the scores: 7 matrix products per tile pair, nothing but the row statistics in the scratch.
          TAW_IMPL_AUTO takes TAW_IMPL_MFMA_STORED where the MFMA kernels apply, as taw_layer_bwd does by default. */
       TAW_IMPL_MFMA_FUSED = 3,   /* one kernel, 5 products; dQ partial sums in private fp32 slots, one per worker, summed by a last pass: no atomics, reproducible */
       TAW_IMPL_MFMA_ATOMIC = 4,  /* one kernel, 5 products; dQ added with fp32 atomics into one buffer (not bit-reproducible) */
       TAW_IMPL_MFMA_STORED = 5   /* two kernels, 5 products: the dK/dV kernel also writes dS (bf16) to the scratch and the dQ kernel reads it
                                     back instead of recomputing it; no atomics, same bits as TAW_IMPL_MFMA; the fastest on this part */ };
enum { TAW_GEMM_NT = 0, TAW_GEMM_NN = 1, TAW_GEMM_TN = 2 };

/* The three products of a linear layer y = x W^T (W is [out, in]):
 *   TAW_GEMM_NT  C[M,N] = A[M,K] B[N,K]^T     forward,          y  = x W^T
 *   TAW_GEMM_NN  C[M,N] = A[M,K] B[K,N]       input gradient,   dx = dy W
 *   TAW_GEMM_TN  C[M,N] = A[K,M]^T B[K,N]     weight gradient,  dW = dy^T x  (contraction over tokens)
 * lda/ldb/ldc/ldr are row strides in elements.  C has storage type c_dtype (dtype or TAW_F32);
 * accumulate != 0 adds the product into C (the fp32 gradient-shard update G += dW).
 * R (may be NULL) is a residual of C's type and shape added to the product (h = x + o Wo^T). */
int taw_op_gemm(int32_t dtype, int32_t mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                const void* B, int64_t ldb, void* C, int64_t ldc, int32_t c_dtype, int32_t accumulate,
                const void* R, int64_t ldr, int32_t impl, void* stream);

/* r[t] = 1/sqrt(mean_i x[t,i]^2 + eps);  out[t,i] = x[t,i] r[t] gamma[i].   x,out [T,H]; r fp32 [T]. */
int taw_op_rmsnorm_fwd(int32_t dtype, int64_t T, int32_t H, const void* x, const void* gamma, float eps,
                       void* out, float* r, void* stream);

/* Gradient of the above through z (the forward input), plus an optional residual gradient:
 *   c = dout*gamma;  dz = r c - z r^3 mean_j(c_j z_j) + (dres ? dres : 0)
 *   dgamma[i] (=|+=) sum_t dout[t,i] z[t,i] r[t]      (fp32 [H]; += when accumulate != 0)
 * scratch: fp32, taw_op_rmsnorm_bwd_scratch_floats(H) elements. */
size_t taw_op_rmsnorm_bwd_scratch_floats(int32_t H);
int taw_op_rmsnorm_bwd(int32_t dtype, int64_t T, int32_t H, const void* dout, const void* z, const float* r,
                       const void* gamma, const void* dres, void* dz, float* dgamma, int32_t accumulate,
                       float* scratch, void* stream);

/* taw_op_rmsnorm_bwd for callers that cannot allocate device memory or pass a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with the partial-sum scratch
 * in a static device array inside the library (16 MiB, held on every GPU the library runs on until the process
 * ends).  Same arguments as taw_op_rmsnorm_bwd without `scratch`; same results, bit for bit.
 *   limit       H <= 8192 (TAW_ERR_WORKSPACE beyond it: use taw_op_rmsnorm_bwd with a caller-owned scratch)
 *   allocation  none: no hipMalloc / hipFree, no allocating library call
 *   sharing     every call on a GPU uses that GPU's one array; the call clears nothing because every scratch row it
 *               reads it has written first; two calls that overlap in time on one GPU (different streams) race on
 *               the array and must be ordered by the caller */
int taw_op_rmsnorm_bwd_static(int32_t dtype, int64_t T, int32_t H, const void* dout, const void* z, const float* r,
                              const void* gamma, const void* dres, void* dz, float* dgamma, int32_t accumulate,
                              void* stream);

/* Rotary embedding in place on columns [0, ncols) of z [B*S, ld]; ncols a multiple of head_dim.
 * Pair (2i, 2i+1) of each head at position p turns by p*theta^(-2i/d); inverse != 0 turns back
 * (the backward map). */
int taw_op_rope(int32_t dtype, int32_t B, int32_t S, int32_t ncols, int32_t head_dim, void* z, int64_t ld,
                const float* rope_table, int32_t inverse, void* stream);

/* gu = [gate | up] [T, 2I];  a [T, I] = gate*sigmoid(gate)*up.  Backward: dgu [T, 2I] from da [T, I]. */
int taw_op_swiglu_fwd(int32_t dtype, int64_t T, int32_t I, const void* gu, void* a, void* stream);
int taw_op_swiglu_bwd(int32_t dtype, int64_t T, int32_t I, const void* da, const void* gu, void* dgu, void* stream);

/* Causal softmax attention on qkv [B*S, 3H] (q | k | v; head h = columns h*d..h*d+d-1 of each
 * part; q and k already rotated), scale 1/sqrt(d), keys u <= t.  Writes o [B*S, H] and
 * lse [B, n_heads, S] (fp32, natural log of the row's sum of exponentials of scaled scores). */
int taw_op_attn_fwd(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* qkv,
                    void* o, float* lse, int32_t impl, void* stream);

/* Its gradient: dqkv [B*S, 3H] from dO [B*S, H], recomputing the probabilities from qkv and lse.
 * rope_table (may be NULL): when given (fp32 [S, head_dim/2, 2] from taw_rope_table_init), q and k
 * are taken to be rotated and dq, dk come out as the gradients of the unrotated q, k (the rotary
 * backward, a rotation by the opposite angle, applied before the store); NULL leaves them as the
 * gradients of the q, k passed in.
 * scratch: fp32, taw_op_attn_bwd_scratch_floats(B, S, n_heads) elements, enough for every form: the row statistics
 * D[t] = dO[t].o[t] and a rescaled copy of lse, then either (fused forms) the fp32 partial sums of dq, one [B*S, H] slot
 * per worker of a (batch, head), the count chosen from the shape, or (TAW_IMPL_MFMA_STORED) dS in bf16, about S*S bytes
 * per (batch, head).  Contents are overwritten; the caller clears nothing. */
size_t taw_op_attn_bwd_scratch_floats(int32_t B, int32_t S, int32_t n_heads);
int taw_op_attn_bwd(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* qkv,
                    const void* o, const void* dO, const float* lse, void* dqkv, float* scratch,
                    const float* rope_table, int32_t impl, void* stream);

/* The fused qkv projection with the rotary embedding, as taw_layer_fwd runs it:
 *   qkv [B*S, 3H] = xn [B*S, H] w_qkv[3H, H]^T, then q and k (columns 0 .. 2H-1) rotated by position.
 * On the MFMA path the rotation happens in the GEMM's epilogue when B*S and H allow it (otherwise,
 * and on the generic path, a rotary pass follows the GEMM: same result up to one more rounding). */
int taw_op_qkv_rope(int32_t dtype, int32_t B, int32_t S, int32_t n_heads, int32_t head_dim, const void* xn,
                    const void* w_qkv, void* qkv, const float* rope_table, int32_t impl, void* stream);

/* Backward of a linear y [T, N] = x [T, K] W[N, K]^T given dy, as taw_layer_bwd runs it:
 *   dx [T, K] = dy W              (storage type dtype)
 *   G  [N, K] (=|+=) dy^T x       (fp32; += when accumulate != 0)
 * On the MFMA path the two products share one grid when T and N are multiples of 32.
 * scratch: device, fp32, taw_op_linear_bwd_scratch_floats(T, N, K) elements, or NULL.  A narrow layer's weight gradient
 * has few 256 x 256 tiles, each contracting over all T tokens; with scratch given (and that count not 0) the contraction
 * is cut into ranges of tokens whose partial products land in scratch and are summed into G in a fixed order by a
 * second kernel: deterministic, equal to the uncut result up to the order of fp32 additions.  NULL, or a count of 0:
 * one kernel, no second pass.  Contents are overwritten; the caller clears nothing.
 * A dimension of 0 makes the call a no-op (G is left as it is). */
size_t taw_op_linear_bwd_scratch_floats(int64_t T, int64_t N, int64_t K);
int taw_op_linear_bwd(int32_t dtype, int64_t T, int64_t N, int64_t K, const void* dy, const void* W, const void* x,
                      void* dx, float* G, int32_t accumulate, float* scratch, int32_t impl, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* TAW_OPS_H */
