// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   NT  C[M,N] = A[M,K] B[N,K]^T      both operands K-contiguous        (forward linears)
//   NN  C[M,N] = A[M,K] B[K,N]        B is N-contiguous                 (input gradients)
//   TN  C[M,N] = A[K,M]^T B[K,N]      both operands contiguous along the output dim (weight gradients)
//
// One 256-thread workgroup (4 wavefronts, one per SIMD) owns a 256x256 output tile; each
// wavefront owns 128x128 of it as 4x4 MFMA tiles (256 fp32 accumulators per lane).  K advances in
// steps of 64 through a double-buffered LDS tile pair (2 x 64 KiB), filled through registers so the
// next step's global loads are in flight while the current step multiplies.
//
// LDS layouts.  A K-contiguous operand is stored [row][64] with its 16-byte chunks XOR-swizzled by
// (row>>1)&7: every MFMA operand (8 consecutive k of one row) is one ds_read_b128 and 16
// consecutive lanes touch 16 distinct bank groups.  An operand that is contiguous along the output
// dimension is stored as it comes, [k][256], chunks swizzled by (k&3)<<2, and read with
// ds_read_b64_tr_b16, which hands each lane 4 consecutive k of one column: the transposition the
// MFMA operand layout needs happens in the LDS read, not in a separate pass over HBM.
//
// Workgroup ids are remapped so that the 8 XCDs (ids are dealt round-robin to them) each work on a
// contiguous band of tiles and, inside a band, on groups of 8 tile rows: tiles that share an
// operand panel then share one XCD's L2.
#include "dev_common.h"
#include "taw_internal.h"

namespace taw {

namespace {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kTileElems = 256 * BK;               // one operand tile, either layout
constexpr int kStageElems = 2 * kTileElems;        // A tile + B tile
constexpr size_t kLdsBytes = 2 * (size_t)kStageElems * sizeof(bf16_t);  // 128 KiB

typedef bf16_t __attribute__((address_space(3))) lds_bf16_t;

__device__ __forceinline__ s16x4_t lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
}

// ---- global -> registers: 8 chunks of 16 bytes per thread and operand ------------------------
// KC (K-contiguous): tile = 256 rows x 64 k.  thread -> chunk c = tid&7, rows (tid>>3) + 32 i.
// NC (contiguous along the output dim): tile = 64 k x 256 cols.  thread -> chunk c = tid&31, k rows (tid>>5) + 8 i.
template <bool KC>
struct TileLoader {
  const bf16_t* base;   // tile origin at k = 0
  int off[8];           // per-chunk element offsets from base (rows/cols clamped into the matrix)
  int64_t kstep;        // elements to advance per K step
  int kfirst;           // KC: this thread's k offset inside a step; NC: first k row of this thread
  __device__ __forceinline__ void init(const bf16_t* mat, int64_t ld, int64_t origin, int64_t extent, int tid) {
    if (KC) {
      const int c = tid & 7, r0 = tid >> 3;
      base = mat + origin * ld;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        int64_t r = r0 + 32 * i;
        if (origin + r >= extent) r = extent - 1 - origin;
        off[i] = (int)(r * ld) + c * 8;
      }
      kstep = BK;
      kfirst = c * 8;
    } else {
      const int c = tid & 31, k0 = tid >> 5;
      int64_t col = origin + c * 8;
      if (col >= extent) col = 0;
      base = mat + col;
#pragma unroll
      for (int i = 0; i < 8; ++i) off[i] = (int)((k0 + 8 * i) * ld);
      kstep = BK * ld;
      kfirst = k0;
    }
  }
  // issues the loads of the step starting at k0 (addresses of chunks at or beyond K are redirected
  // to a valid place); nothing here touches the loaded registers, so the loads stay in flight
  // while the caller multiplies the previous step
  __device__ __forceinline__ void load(u32x4_t (&regs)[8], int64_t k0, int64_t K) const {
    const bf16_t* p = base + (k0 / BK) * kstep;
    if (KC) {
      const int adj = (k0 + kfirst < K) ? 0 : kfirst;
#pragma unroll
      for (int i = 0; i < 8; ++i) regs[i] = *reinterpret_cast<const u32x4_t*>(p + (off[i] - adj));
    } else {
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const bool valid = k0 + kfirst + 8 * i < K;
        regs[i] = *reinterpret_cast<const u32x4_t*>(valid ? p + off[i] : base);
      }
    }
  }
  // registers -> LDS tile of the step that started at k0; chunks at or beyond K are written as zeros
  __device__ __forceinline__ void store(bf16_t* tile, const u32x4_t (&regs)[8], int tid, int64_t k0, int64_t K) const {
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    if (KC) {
      const int c = tid & 7, r0 = tid >> 3;
      const bool valid = k0 + kfirst < K;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int r = r0 + 32 * i;
        *reinterpret_cast<u32x4_t*>(tile + r * BK + ((c ^ ((r >> 1) & 7)) << 3)) = valid ? regs[i] : zero;
      }
    } else {
      const int c = tid & 31, kr = tid >> 5;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = kr + 8 * i;
        const bool valid = k0 + k < K;
        *reinterpret_cast<u32x4_t*>(tile + k * 256 + ((c ^ ((k & 3) << 2)) << 3)) = valid ? regs[i] : zero;
      }
    }
  }
};

// ---- LDS -> MFMA operand: 8 bf16 of k = 16 ks + 8 (lane>>5) + 0..7 for row/col x0 + (lane&31) ---
template <bool KC>
__device__ __forceinline__ bf16x8_t read_frag(const bf16_t* tile, int x0, int ks, int lane) {
  if (KC) {
    const int r = x0 + (lane & 31);
    const int c = 2 * ks + (lane >> 5);
    return *reinterpret_cast<const bf16x8_t*>(tile + r * BK + ((c ^ ((r >> 1) & 7)) << 3));
  } else {
    const int blk = lane >> 4, i = lane & 15;
    const int n = x0 + 16 * (blk & 1) + 4 * (i & 3);
    const int kb = 16 * ks + 8 * (blk >> 1) + (i >> 2);
    union { s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
      const int k = kb + 4 * r;
      u.h[r] = lds_read_tr(tile + k * 256 + (((n >> 3) ^ ((k & 3) << 2)) << 3) + (n & 7));
    }
    return u.v;
  }
}

template <int MODE, bool C_F32>
__global__ void __launch_bounds__(kThreads, 1)
gemm_mfma_kernel(int64_t M, int64_t N, int64_t K, const bf16_t* __restrict__ A, int64_t lda, const bf16_t* __restrict__ B,
                 int64_t ldb, void* __restrict__ Cv, int64_t ldc, int accumulate, const void* __restrict__ Rv, int64_t ldr,
                 int tiles_m, int tiles_n) {
  constexpr bool A_KC = (MODE != GEMM_TN);
  constexpr bool B_KC = (MODE == GEMM_NT);
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  bf16_t* lds = reinterpret_cast<bf16_t*>(lds_raw);

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // ---- XCD-aware tile id
  const int ntiles = tiles_m * tiles_n;
  int pid = blockIdx.x;
  const int n8 = ntiles & ~7;
  if (pid < n8) pid = (pid & 7) * (n8 >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int per_group = GROUP * tiles_n;
  const int g = pid / per_group;
  const int gm0 = g * GROUP;
  const int gsize = (tiles_m - gm0) < GROUP ? (tiles_m - gm0) : GROUP;
  const int tm = gm0 + (pid % per_group) % gsize;
  const int tn = (pid % per_group) / gsize;
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  TileLoader<A_KC> la;
  TileLoader<B_KC> lb;
  la.init(A, lda, m0, M, tid);
  lb.init(B, ldb, n0, N, tid);

  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4_t ra[8], rb[8];
  la.load(ra, 0, K);
  lb.load(rb, 0, K);
  la.store(lds, ra, tid, 0, K);
  lb.store(lds + kTileElems, rb, tid, 0, K);
  __syncthreads();

  const int64_t nk = (K + BK - 1) / BK;
  for (int64_t kt = 0; kt < nk; ++kt) {
    const bf16_t* sa = lds + (kt & 1) * kStageElems;
    const bf16_t* sb = sa + kTileElems;
    const bool more = kt + 1 < nk;
    if (more) {
      la.load(ra, (kt + 1) * BK, K);
      lb.load(rb, (kt + 1) * BK, K);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t fa[4], fb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fa[i] = read_frag<A_KC>(sa, wm + 32 * i, ks, lane);
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[j] = read_frag<B_KC>(sb, wn + 32 * j, ks, lane);
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      bf16_t* da = lds + ((kt + 1) & 1) * kStageElems;
      la.store(da, ra, tid, (kt + 1) * BK, K);
      lb.store(da + kTileElems, rb, tid, (kt + 1) * BK, K);
    }
    __syncthreads();
  }

  // ---- epilogue: accumulator register r of lane l is C[row0 + 8 (r/4) + 4 (l>>5) + r%4][col0 + (l&31)]
  const int lcol = lane & 31, lrow = 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int64_t col = n0 + wn + 32 * j + lcol;
      if (col >= N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t row = m0 + wm + 32 * i + 8 * (r >> 2) + lrow + (r & 3);
        if (row >= M) continue;
        float v = acc[i][j][r];
        if (C_F32) {
          float* C = static_cast<float*>(Cv);
          if (Rv) v += static_cast<const float*>(Rv)[row * ldr + col];
          if (accumulate) v += C[row * ldc + col];
          C[row * ldc + col] = v;
        } else {
          bf16_t* C = static_cast<bf16_t*>(Cv);
          if (Rv) v += (float)static_cast<const bf16_t*>(Rv)[row * ldr + col];
          if (accumulate) v += (float)C[row * ldc + col];
          C[row * ldc + col] = (bf16_t)v;
        }
      }
    }
  }
}

template <int MODE, bool C_F32>
int launch_t(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
             int accumulate, const void* R, int64_t ldr, hipStream_t st) {
  static bool attr_set = false;   // per instantiation; setting it again is harmless
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void*)gemm_mfma_kernel<MODE, C_F32>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes);
    if (e != hipSuccess) return (int)e;
    attr_set = true;
  }
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
  hipLaunchKernelGGL((gemm_mfma_kernel<MODE, C_F32>), dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), kLdsBytes, st, M, N, K,
                     (const bf16_t*)A, lda, (const bf16_t*)B, ldb, C, ldc, accumulate, R, ldr, tiles_m, tiles_n);
  return (int)hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(int dtype, int mode, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc,
                         int c_dtype, int64_t ldr) {
  (void)ldc; (void)ldr; (void)c_dtype;
  if (dtype != DT_BF16) return false;
  if (M <= 0 || N <= 0 || K <= 0) return false;
  if (lda % 8 || ldb % 8) return false;                     // 16-byte global loads
  if (mode == GEMM_NT) { if (K % 8) return false; }
  else if (mode == GEMM_NN) { if (K % 8 || N % 8) return false; }
  else if (mode == GEMM_TN) { if (M % 8 || N % 8) return false; }
  else return false;
  // per-thread offsets inside a tile are 32-bit
  if (lda > ((int64_t)1 << 22) || ldb > ((int64_t)1 << 22)) return false;
  if ((M + BM - 1) / BM * ((N + BN - 1) / BN) > ((int64_t)1 << 30)) return false;
  return true;
}

int launch_gemm_mfma(int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb,
                     void* C, int64_t ldc, int c_dtype, int accumulate, const void* R, int64_t ldr, hipStream_t st) {
  const bool f32 = c_dtype == DT_F32;
  switch (mode) {
    case GEMM_NT: return f32 ? launch_t<GEMM_NT, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                             : launch_t<GEMM_NT, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
    case GEMM_NN: return f32 ? launch_t<GEMM_NN, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                             : launch_t<GEMM_NN, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
    default: return f32 ? launch_t<GEMM_TN, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                        : launch_t<GEMM_TN, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
  }
}

}  // namespace taw
