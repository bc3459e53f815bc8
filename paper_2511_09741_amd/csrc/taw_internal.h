// Internal launch interface between the C-ABI front end (taw_api.cpp) and the kernel files.
// Every launcher validates nothing (the front end did), enqueues on `st`, and returns the
// hipError_t of its last launch as an int (0 = success).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace taw {

enum { DT_F32 = 0, DT_BF16 = 1 };
enum { GEMM_NT = 0, GEMM_NN = 1, GEMM_TN = 2 };

inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

// Raises a kernel's dynamic-LDS limit to `bytes` the first time the enclosing function (or template
// instantiation) runs, and returns from it with the HIP error code if that failed.  The limit is a
// property of the kernel, not of a launch: a function-local static is initialised exactly once, and
// thread-safely.  `bytes` must be the largest size that launcher ever asks for.
#define TAW_SET_LDS_LIMIT_ONCE(kernel, bytes)                                                                                  \
  do {                                                                                                                       \
    static const int taw_lds_rc_ = (int)hipFuncSetAttribute((const void*)(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)(bytes)); \
    if (taw_lds_rc_) return taw_lds_rc_;                                                                                     \
  } while (0)

// ---- bandwidth-bound kernels (kernels_bw.hip) ------------------------------------------------
// Largest H the RMSNorm kernels hold in registers: H * sizeof(elem) <= 16 KiB when H is a multiple
// of the 16-byte vector width, else H <= 1024.
bool rmsnorm_supported(int dtype, int H);
int launch_rmsnorm_fwd(int dtype, int64_t T, int H, const void* x, const void* gamma, float eps,
                       void* out, float* r, hipStream_t st);
// number of fp32 partial-sum rows (each H wide) the backward needs as scratch
int rmsnorm_bwd_partial_rows();
// dz = (dres ? dres : 0) + rmsnorm_bwd(dout);  dgamma (=|+=) column sums
int launch_rmsnorm_bwd(int dtype, int64_t T, int H, const void* dout, const void* z, const float* r,
                       const void* gamma, const void* dres, void* dz, float* dgamma, int accumulate,
                       float* partials, hipStream_t st);
int launch_rope_table(int S, int head_dim, double theta, float* table, hipStream_t st);
// rotates columns [0, ncols) of the [B*S, ld] matrix z in place; column j belongs to pair (j % d)/2
int launch_rope(int dtype, int B, int S, int ncols, int head_dim, void* z, int64_t ld,
                const float* table, int inverse, hipStream_t st);
int launch_swiglu_fwd(int dtype, int64_t T, int I, const void* gu, void* a, hipStream_t st);
int launch_swiglu_bwd(int dtype, int64_t T, int I, const void* da, const void* gu, void* dgu,
                      hipStream_t st);
int launch_grad_accum(float* G, const void* g, int src_dtype, size_t n, float scale, hipStream_t st);
int launch_stage_copy(void* dst, const void* src, size_t bytes, hipStream_t st);
// AdamW over n elements; chunk in w_dtype, everything else fp32; b1c = 1 - beta1^t, b2c = 1 - beta2^t
int launch_adamw(int w_dtype, void* chunk, float* master, float* m, float* v, float* G, size_t n, float lr, float beta1, float beta2,
                 float eps, float wd, float b1c, float b2c, float gscale, int zero_grad, hipStream_t st);
// D[b, h, t] = sum_i do[t, h*d + i] * o[t, h*d + i]   (o, do are [B*S, ld_o] / [B*S, ld_do])
int launch_attn_rowdot(int dtype, int B, int S, int nh, int d, const void* o, int64_t ld_o,
                       const void* dO, int64_t ld_do, float* D, hipStream_t st);

// ---- generic (any shape, fp32 or bf16 storage, fp32 arithmetic) kernels (kernels_generic.hip) --
// C[M,N] (=|+=) op(A) op(B) (+ R).  mode NT: A[M,K], B[N,K];  NN: A[M,K], B[K,N];  TN: A[K,M], B[K,N].
// c_dtype is the storage type of C and R (in dtype or fp32); accumulate adds into C.
int launch_gemm_generic(int dtype, int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                        const void* B, int64_t ldb, void* C, int64_t ldc, int c_dtype, int accumulate,
                        const void* R, int64_t ldr, hipStream_t st);
// qkv: [B*S, 3H] (q | k | v, head-major);  o: [B*S, H];  lse: [B, nh, S] natural-log-sum-exp of the scaled scores
bool attn_generic_supported(int S, int d);
int launch_attn_fwd_generic(int dtype, int B, int S, int nh, int d, const void* qkv, void* o, float* lse,
                            hipStream_t st);
int launch_attn_bwd_generic(int dtype, int B, int S, int nh, int d, const void* qkv, const void* dO,
                            const float* lse, const float* D, void* dqkv, hipStream_t st);

// ---- order in which a GEMM grid walks its 256 x 256 output tiles ------------------------------
// Workgroup ids are dealt round-robin to the 8 XCDs (32 compute units and one 4 MiB L2 each), and each XCD
// starts its ids in order, so the ids [256 r, 256 r + 256) run at about the same time ("round" r) and id b
// of a round runs on XCD b % 8.  Tiles are laid along one locality-preserving sequence: super-tiles of
// 16 x 16 tiles (tile rows outer, the super-tiles of 16 rows side by side inner), each made of two halves of
// 8 rows, each half walked in groups of 4 columns, rows fastest.  Position p of that sequence goes to
// round p / 256, XCD (p / 32) % 8: a round then covers about one super-tile, so the whole chip streams 16 + 16
// operand panels per 256 tiles through the memory-side cache (a band of tile rows per XCD streams 64 + 4),
// and an XCD's 32 concurrent tiles are still an 8 x 4 block that shares panels in its own L2.
// The map is a bijection from [0, tiles_m * tiles_n) onto the tiles for every grid shape; ragged edges only
// shift where the blocks fall.  Host code can evaluate it too (the tests do).
__host__ __device__ inline void gemm_tile_of_block(int block, int tiles_m, int tiles_n, int* tm, int* tn) {
  const int ntiles = tiles_m * tiles_n;
  const int n256 = ntiles & ~255;
  int p = block;
  if (block < n256) {
    p = (block & ~255) + (block & 7) * 32 + ((block >> 3) & 31);
  } else {                                      // last, partial round: every XCD takes one run of the sequence
    const int t = block - n256, n8 = (ntiles - n256) & ~7;
    if (t < n8) p = n256 + (t & 7) * (n8 >> 3) + (t >> 3);
  }
  const int per_sr = 16 * tiles_n;              // tiles in a full super-row
  const int R = p / per_sr, p1 = p - R * per_sr;
  const int hR = tiles_m - 16 * R < 16 ? tiles_m - 16 * R : 16;
  const int C = p1 / (hR * 16), p2 = p1 - C * (hR * 16);
  const int wC = tiles_n - 16 * C < 16 ? tiles_n - 16 * C : 16;
  const int ht = hR < 8 ? hR : 8, top = ht * wC;
  const bool lower = p2 >= top;
  const int h = lower ? hR - 8 : ht, q = lower ? p2 - top : p2;
  const int cg = q / (4 * h), q2 = q - cg * (4 * h);
  *tm = 16 * R + (lower ? 8 : 0) + q2 % h;
  *tn = 16 * C + 4 * cg + q2 / h;
}

// ---- MFMA bf16 kernels (gemm_mfma.hip, attn_mfma.hip) -----------------------------------------
bool gemm_mfma_supported(int dtype, int mode, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb,
                         int64_t ldc, int c_dtype, int64_t ldr);
int launch_gemm_mfma(int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B,
                     int64_t ldb, void* C, int64_t ldc, int c_dtype, int accumulate, const void* R,
                     int64_t ldr, hipStream_t st);
// A weight gradient C0[M0,N0] (fp32, TN form, optionally accumulated) and an input gradient C1[M1,N1] (bf16, NN form) in one
// grid: the pair every linear of the backward has.  Needs both K % 32 == 0 on top of gemm_mfma_supported for each.
bool gemm_mfma_dual_supported(int64_t K_tn, int64_t K_nn);
// part / splits / k_chunk: the weight gradient cut into `splits` ranges of k_chunk contraction rows (gemm_dual_splits), their
// partial products in part[splits][M0][N0] fp32, summed into C0 by a second kernel in a fixed order; splits <= 1 or part ==
// nullptr: not cut
int launch_gemm_mfma_dual(int64_t M0, int64_t N0, int64_t K0, const void* A0, int64_t lda0, const void* B0, int64_t ldb0, float* C0,
                          int64_t ldc0, int accumulate0, int64_t M1, int64_t N1, int64_t K1, const void* A1, int64_t lda1,
                          const void* B1, int64_t ldb1, void* C1, int64_t ldc1, float* part, int splits, int64_t k_chunk, hipStream_t st);
// ranges (and rows per range) for the weight gradient of the linear y[T, N] = x[T, K] W^T; 1 = not cut
int gemm_dual_splits(int64_t T, int64_t N, int64_t K, int64_t* k_chunk);
// C[M,N] = A[M,K] B[N,K]^T (bf16) with the rotary embedding applied in the epilogue to the columns below rot_cols (heads of
// 128, adjacent pairs, row r at position r % S; table [S, 64, 2] fp32).  Needs M % 256 == 0, N % 256 == 0, K % 64 == 0,
// rot_cols % 256 == 0, S >= 32.
bool gemm_mfma_rope_supported(int64_t M, int64_t N, int64_t K, int64_t rot_cols, int S);
int launch_gemm_mfma_nt_rope(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                             const float* rope_table, int S, int64_t rot_cols, hipStream_t st);
// bf16, head_dim 128, and S * 3 * n_heads * head_dim * 2 bytes below 4 GiB (32-bit row offsets inside one batch element)
bool attn_mfma_supported(int dtype, int S, int nh, int d);
int launch_attn_fwd_mfma(int B, int S, int nh, const void* qkv, void* o, float* lse, hipStream_t st);
// The MFMA backward exists in four forms.  STORED (the layer's default): a dK/dV kernel that forms S, dP and dS once and
// also writes dS (bf16) to the scratch, and a dQ kernel that reads it back: 5 matrix products per tile pair, no atomics,
// reproducible, about S * S bytes of scratch per (batch, head).  SPLIT: the same pair with a dQ kernel that recomputes
// S and dP instead (7 products), same bits, no dS in the scratch.  FUSED: one key-stationary kernel forms S and dP
// once and produces dK, dV and dQ (5 products); dQ partial sums go to private fp32 slots, one per worker, and a last
// pass sums them: no atomics, reproducible.  FUSED_ATOMIC: the fused kernel adding dQ with fp32 atomics into one buffer.
// S = 32768, 32 heads: 23.7 / 25.8 / 30.9 / 27.6 ms: the atomic units take 25.4 ms for the adds alone, the slots are 78 GB
// of read-modify-write inside the MFMA loop, the recomputation is two more products; dS streamed once each way costs least.
// ANY: only for sizing the scratch (enough for every form).
enum { ATTN_BWD_SPLIT = 0, ATTN_BWD_FUSED = 1, ATTN_BWD_FUSED_ATOMIC = 2, ATTN_BWD_STORED = 3, ATTN_BWD_ANY = -1 };
// ---- layout of the stored dS (ATTN_BWD_STORED), shared by the kernel that writes it, the kernel that reads it and the host
// Per (batch, head): block ib of 256 query rows holds 256 (ib + 1) keys x 256 rows bf16, blocks one after the other; inside a
// block, per 32-row group s, the 2 KiB units dS[32 rows][32 keys] of the key groups g = 0 .. 8 (ib + 1) - 1 one after the
// other.  Inside a unit, 128 slots of 16 bytes: lane (key kk, lane half hh) of the writing wavefront puts its piece tt
// (8 bf16 = accumulator registers 8 tt .. 8 tt + 7) at slot ds_slot(kk, hh, tt); position p = 16 hh + 8 tt + e of a
// key's 32 values is query row ds_row_of_slot(p) of the group.
constexpr int64_t kDsBlockBytes = 256 * 256 * 2;       // one (256 keys, 256 query rows) block
__host__ __device__ inline int64_t ds_block_offset(int ib) { return (int64_t)ib * (ib + 1) / 2 * kDsBlockBytes; }
__host__ __device__ inline int64_t ds_unit_offset(int ib, int s, int g) { return ds_block_offset(ib) + ((int64_t)s * 8 * (ib + 1) + g) * 2048; }
__host__ __device__ inline unsigned ds_slot(int kk, int hh, int tt) { return (unsigned)(tt * 64 + ((((kk >> 2) * 8) + (kk & 3) * 2 + hh) ^ (tt * 8))); }
__host__ __device__ inline int ds_row_of_slot(int p) { return 16 * ((p >> 3) & 1) + 4 * (p >> 4) + (p & 3) + 8 * ((p >> 2) & 1); }
// workers (and fp32 dQ slots) per (batch, head) the fused form uses for this shape
int attn_bwd_slots(int B, int S, int nh);
// fp32 scratch of the MFMA backward in the given form: scaled lse and D, each padded to a multiple of 64 rows per
// (batch, head), followed by the dQ slots (fused forms) or the stored dS (STORED)
size_t attn_bwd_mfma_scratch_floats(int B, int S, int nh, int form);
// computes its own row statistics (scratch) from o, dO and lse.  rope_table != nullptr: q and k were rotated
// (table [S, 64, 2] fp32 of cos, sin) and dq, dk come out as gradients of the unrotated q, k
int launch_attn_bwd_mfma(int B, int S, int nh, const void* qkv, const void* o, const void* dO, const float* lse,
                         float* scratch, void* dqkv, const float* rope_table, int form, hipStream_t st);

}  // namespace taw
