/* taw.h -- C ABI of the MI355X (gfx950) decoder-layer hot path for weight-pipeline training.
 *
 * What the calls stand for (TawPipe, arXiv 2511.09741).  In weight-passing pipeline parallelism
 * every device keeps its own micro-batch and the layer weights travel: when the weights W_j of
 * layer j arrive, each device applies the layer to its cached activations A_j (forward) or
 * back-propagates through it, producing the gradients G_j of W_j (Methodology, "Group-Based
 * Weight Pipeline Scheduler"; Table 1 for the symbols A, W, G, B, S, H).  The owner of a layer
 * keeps one fixed weight shard and one fixed gradient shard ("Device-Bound Storage") and adds
 * incoming gradient contributions into it; the weights for the next step are prefetched into a
 * dedicated buffer while the current step computes ("Communication-Computation Overlap").
 * This library is the single-GPU part of that: the layer itself (taw_layer_fwd, taw_layer_bwd),
 * the owner-side aggregation (taw_grad_accum) and the prefetch into a staging buffer
 * (taw_weight_stage).  The layer is the LLaMA-2 block the paper trains ("Experimental Setup";
 * "Theoretical Analysis": about 12 H^2 parameters per layer): RMSNorm, fused QKV projection,
 * rotary embedding on adjacent pairs, causal softmax attention, output projection + residual,
 * RMSNorm, SwiGLU MLP + residual.
 *
 * General rules
 *  - Every function returns an int status: TAW_OK (0) or a negative TAW_ERR_* code.  Nothing
 *    throws across the ABI.  taw_status_string() names a code; taw_last_error() gives detail.
 *  - All data pointers are DEVICE pointers unless a parameter says "host".  Descriptor and
 *    layout structs are host memory.
 *  - The library allocates and frees nothing.  The caller owns every buffer and keeps it alive
 *    until the work enqueued on the stream has completed.
 *  - All work is enqueued on the stream passed in (a hipStream_t cast to void*; NULL = the
 *    default stream).  No call synchronises with the host.
 *  - All argument validation happens on the host before the first launch.
 *  - Device pointers must be 16-byte aligned.  Tensors are dense row-major.
 *  - Buffers must not alias unless a parameter says so.
 */
#ifndef TAW_H
#define TAW_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  TAW_OK = 0,
  TAW_ERR_NULL = -1,        /* a required pointer is NULL */
  TAW_ERR_SHAPE = -2,       /* non-positive dimension, H != n_heads*head_dim, odd head_dim, ... */
  TAW_ERR_DTYPE = -3,       /* dtype is neither TAW_F32 nor TAW_BF16 */
  TAW_ERR_ALIGN = -4,       /* a device pointer is not 16-byte aligned */
  TAW_ERR_WORKSPACE = -5,   /* workspace_bytes smaller than taw_layer_workspace_bytes() */
  TAW_ERR_UNSUPPORTED = -6, /* valid request this build has no kernel for */
  TAW_ERR_HIP = -7          /* a HIP runtime call or kernel launch failed */
};

typedef enum { TAW_F32 = 0, TAW_BF16 = 1 } taw_dtype;

/* flags of taw_layer_desc */
#define TAW_ACCUMULATE 1u /* taw_layer_bwd adds the weight gradients into G_shard (G += dW);
                             without it the call overwrites the shard (G = dW) */
#define TAW_RECOMPUTE 2u  /* activation checkpointing, the mode the paper trains in ("Experimental
                             Setup"): the forward keeps nothing but its input x (ctx is unused and may
                             be NULL, taw_layer_ctx_bytes() is 0); the backward first rebuilds the
                             layer's intermediates from x inside the workspace, which is larger by
                             what ctx would have held.  Same results, about 4/3 of the arithmetic. */

/* Forms of the attention backward on the matrix-core path.  Default: a dK/dV kernel that forms the scores once and also
   writes dS (bf16) to the workspace, and a dQ kernel that reads it back: five matrix products per tile pair, no atomics,
   reproducible; the workspace holds about S*S bytes per (batch, head) for it (35 GB at S = 32768 with 32 heads). */
#define TAW_ATTN_BWD_FUSED 4u /* one kernel that forms the scores once and keeps dQ partial sums in private fp32 slots
                                 (the workspace holds those slots instead of dS) */
#define TAW_ATTN_BWD_RECOMPUTE 8u /* the pair of kernels with a dQ kernel that recomputes the scores (seven products):
                                     needs neither dS nor slots in the workspace; about 12 % slower at S = 32768 */

/* One decoder layer and the micro-batch it is applied to (B, S, H as in the paper's Table 1). */
typedef struct {
  int32_t dtype;      /* taw_dtype of activations and weights; the gradient shard is always fp32 */
  int32_t B;          /* micro-batch size */
  int32_t S;          /* sequence length; positions are 0..S-1 in every batch element */
  int32_t H;          /* hidden size, == n_heads * head_dim (multi-head attention, no GQA) */
  int32_t n_heads;
  int32_t head_dim;   /* even */
  int32_t I;          /* SwiGLU intermediate width */
  float rope_theta;   /* rotary base, 10000 for LLaMA-2 */
  float rms_eps;      /* added to the mean of squares inside the square root */
  uint32_t flags;     /* TAW_ACCUMULATE | TAW_RECOMPUTE | TAW_ATTN_BWD_FUSED | TAW_ATTN_BWD_RECOMPUTE */
} taw_layer_desc;

/* Element offsets of the sub-tensors inside the flat weight chunk W_j (the unit that is moved
 * between devices, "Device-Bound Storage").  The fp32 gradient shard G_j uses the same element
 * offsets.  Every offset is a multiple of 128 elements.  Matrices are [out, in] row-major
 * (y = x W^T): w_qkv [3H, H] with rows [Q; K; V] (head-major inside each), w_o [H, H],
 * w_gate_up [2I, H] with rows [gate; up], w_down [H, I]; the two RMSNorm gains are [H]. */
typedef struct {
  size_t gamma_attn, w_qkv, w_o, gamma_mlp, w_gate_up, w_down, total_elems;
} taw_weight_layout;

/* Fills *out (host) for the layer described by *desc (host).  TAW_ERR_NULL / _SHAPE / _DTYPE. */
int taw_layer_weight_layout(const taw_layer_desc* desc, taw_weight_layout* out);

/* Bytes of the activation cache that taw_layer_fwd writes and taw_layer_bwd reads (the cached
 * A_j of the forward phase), and of the scratch workspace either call needs.  Both return 0 for
 * an invalid descriptor.  The workspace holds nothing between calls and may be shared by layers. */
size_t taw_layer_ctx_bytes(const taw_layer_desc* desc);
size_t taw_layer_workspace_bytes(const taw_layer_desc* desc);

/* Writes the rotary table for positions 0..S-1: table[p][i] = (cos, sin)(p * theta^(-2i/d)),
 * fp32 [S, head_dim/2, 2], angles evaluated in fp64 on the device.  One table serves every layer
 * with the same S, head_dim and theta. */
int taw_rope_table_init(const taw_layer_desc* desc, float* rope_table, void* stream);

/* Forward: y = layer(W_chunk, x).
 *   W_chunk     weight chunk, desc->dtype, laid out per taw_layer_weight_layout (read only)
 *   rope_table  from taw_rope_table_init (read only)
 *   x, y        [B, S, H] desc->dtype; y must not alias x
 *   ctx         taw_layer_ctx_bytes() bytes, written here, to be passed unchanged to taw_layer_bwd
 *   workspace   >= taw_layer_workspace_bytes() bytes of scratch (TAW_ERR_WORKSPACE otherwise)
 * bf16 layers compute with fp32 accumulation and store activations in bf16. */
int taw_layer_fwd(const taw_layer_desc* desc, const void* W_chunk, const float* rope_table,
                  const void* x, void* y, void* ctx, void* workspace, size_t workspace_bytes,
                  void* stream);

/* Backward: dx = dL/dx and the weight gradients of the layer for upstream gradient dy = dL/dy.
 *   x, ctx      exactly what the matching taw_layer_fwd call read and wrote (read only)
 *   dy, dx      [B, S, H] desc->dtype; dx must not alias dy or x
 *   G_shard     fp32 gradient shard, total_elems floats at the chunk's element offsets; the
 *               padding between sub-tensors is left untouched.  Overwritten, or accumulated into
 *               when desc->flags has TAW_ACCUMULATE (the caller zeroes it at mini-batch start).
 * No 1/N micro-batch scaling is applied. */
int taw_layer_bwd(const taw_layer_desc* desc, const void* W_chunk, const float* rope_table,
                  const void* x, const void* dy, const void* ctx, void* dx, float* G_shard,
                  void* workspace, size_t workspace_bytes, void* stream);

/* Owner-side aggregation of a gradient contribution into the fixed fp32 gradient shard:
 * G_dst[i] += scale * g_src[i] for i < n_elems.  g_src is fp32 (src_dtype TAW_F32) or bf16
 * (TAW_BF16).  n_elems == 0 is a no-op.  G_dst and g_src must not overlap. */
int taw_grad_accum(float* G_dst, const void* g_src, int32_t src_dtype, size_t n_elems, float scale,
                   void* stream);

/* Prefetch of the next step's weights into a dedicated buffer while the current step computes:
 * copies `bytes` bytes (a multiple of 16) from src_shard to dst_buf on copy_stream.
 *   wait_event   hipEvent_t or NULL: the copy waits for it first (the event the compute stream
 *                recorded after its last read of dst_buf's previous contents)
 *   ready_event  hipEvent_t or NULL: recorded on copy_stream after the copy; the compute stream
 *                waits for it before the layer that consumes dst_buf
 * bytes == 0 only handles the events. */
int taw_weight_stage(void* dst_buf, const void* src_shard, size_t bytes, void* copy_stream,
                     void* wait_event, void* ready_event);

/* Owner-side update of a weight shard from its aggregated gradient shard: the owner keeps the
 * optimizer state next to its shard and updates in place, with no further communication
 * (Methodology, Group-Based Weight Pipeline Scheduler).  The paper does not name the optimizer; this is AdamW (decoupled weight decay), one pass over the
 * shard, for step number `step` (1-based):
 *   g = grad_scale * G[i];  m = beta1 m + (1-beta1) g;  v = beta2 v + (1-beta2) g^2;
 *   w = w - lr * ( (m / (1-beta1^step)) / (sqrt(v / (1-beta2^step)) + eps) + weight_decay * w )
 * master, m, v, G_shard are fp32 arrays of n_elems (the optimizer state colocated with the shard);
 * W_chunk (chunk_dtype, n_elems) receives w rounded to the storage type, ready to be passed on.
 * grad_scale carries the 1/N of micro-batch averaging.  zero_grad != 0 leaves G_shard zeroed for the
 * next mini-batch.  n_elems == 0 is a no-op.  The arrays must not overlap. */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay, grad_scale;
  int32_t step;       /* >= 1 */
  int32_t zero_grad;
} taw_adamw_desc;
int taw_optimizer_step(const taw_adamw_desc* opt, void* W_chunk, int32_t chunk_dtype, float* master, float* m,
                       float* v, float* G_shard, size_t n_elems, void* stream);

/* Name of a status code (static string), and a description of the most recent error on the
 * calling thread (valid until the next failing call on that thread). */
const char* taw_status_string(int status);
const char* taw_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* TAW_H */
