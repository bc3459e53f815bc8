// bf16 GEMM on the gfx950 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulation.
//
//   NT  C[M,N] = A[M,K] B[N,K]^T      both operands K-contiguous        (forward linears)
//   NN  C[M,N] = A[M,K] B[K,N]        B is N-contiguous                 (input gradients)
//   TN  C[M,N] = A[K,M]^T B[K,N]      both operands contiguous along the output dim (weight gradients)
//
// One 256-thread workgroup (4 wavefronts, one per SIMD) owns a 256x256 output tile; each
// wavefront owns 128x128 of it as 4x4 MFMA tiles (256 fp32 accumulators per lane).  K advances in
// steps of 64 through a double-buffered LDS tile pair (2 x 64 KiB), filled through registers so the
// next step's global loads are in flight while the current step multiplies.  That is the general
// kernel (any K % 8 == 0).  Two pipelined kernels with direct global->LDS loads take the shapes the
// layer has: 64-deep steps for the NT and NN forms when K % 64 == 0, 32-deep steps for TN and for
// K % 32 == 0 (namespace v2 below).
//
// LDS layouts.  A K-contiguous operand is stored [row][64] with its 16-byte chunks XOR-swizzled by
// (row>>1)&7: every MFMA operand (8 consecutive k of one row) is one ds_read_b128 and 16
// consecutive lanes touch 16 distinct bank groups.  An operand that is contiguous along the output
// dimension is stored as it comes, [k][256], chunks swizzled by (k&3)<<2, and read with
// ds_read_b64_tr_b16, which hands each lane 4 consecutive k of one column: the transposition the
// MFMA operand layout needs happens in the LDS read, not in a separate pass over HBM.
//
// Workgroup ids are remapped (gemm_tile_of_block) so that the 32 tiles an XCD works on at a time are an 8 x 4
// block sharing operand panels in that XCD's L2, and the 256 tiles of the whole chip about a 16 x 16 block
// sharing them in the memory-side cache.
#include <type_traits>

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
  int tm, tn;
  gemm_tile_of_block((int)blockIdx.x, tiles_m, tiles_n, &tm, &tn);
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
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);     // block (i, j) transposed, see stage_rows
    }
    if (more) {
      bf16_t* da = lds + ((kt + 1) & 1) * kStageElems;
      la.store(da, ra, tid, (kt + 1) * BK, K);
      lb.store(da + kTileElems, rb, tid, (kt + 1) * BK, K);
    }
    __syncthreads();
  }

  // ---- epilogue: the blocks are transposed (see stage_rows): accumulator register r of lane l is
  // C[row0 + (l&31)][col0 + 8 (r/4) + 4 (l>>5) + r%4]
  const int lrow = lane & 31, lcol = 4 * (lane >> 5);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int64_t row = m0 + wm + 32 * i + lrow;
    if (row >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int64_t col = n0 + wn + 32 * j + 8 * (r >> 2) + lcol + (r & 3);
        if (col >= N) continue;
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

// =============================================================================== pipelined kernel
// Same tile shape and operand layouts, different data movement: K advances in steps of 32 through
// a 4-stage ring of LDS tiles (4 x 32 KiB) filled by direct global->LDS loads
// (global_load_lds_dwordx4: no staging registers, no LDS store instructions).  Each lane picks
// the global chunk whose swizzled home is the LDS slot its lane number writes, so the swizzle
// costs nothing.  Per K step a wavefront issues its 8 loads for the tile three steps ahead, waits
// (vmcnt) until the tile two steps ahead has landed, and meets the other wavefronts at one raw
// s_barrier.  The first operand fragments of the next tile are read before that barrier (the tile
// became visible at the previous one), so no LDS latency is exposed after it.
//
// The instruction stream of a step is laid out by hand as 16 groups of {2 MFMA, 1 operand
// fragment read, 1 direct load}, each closed by a scheduling barrier: one wavefront per SIMD
// issues in order, so the matrix pipe only stays busy if the LDS reads, the loads and their few
// scalar instructions sit in the shadow of the MFMAs instead of in front of them.
// Needs K % 32 == 0 (the launcher sends other K to the kernel above).
namespace v2 {

constexpr int BK2 = 32;
constexpr int kStages = 4;
constexpr int kOpBytes = 256 * BK2 * 2;          // one operand tile: 16 KiB
constexpr int kStageBytes = 2 * kOpBytes;        // 32 KiB
constexpr size_t kLds2 = (size_t)kStages * kStageBytes;   // 128 KiB

typedef __attribute__((address_space(3))) unsigned char lds_u8_t;

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// 16 bytes per lane from global memory (64-bit scalar base + 32-bit per-lane byte offset) straight
// into LDS at lds_addr + 16 * lane (lds_addr wavefront-uniform).
// Written as inline assembly on purpose: the compiler's wait-count insertion treats every LDS
// read whose address it cannot disambiguate (the transposing reads are such) as depending on all
// outstanding LDS-DMA loads and puts s_waitcnt vmcnt(0) in front of it, which would serialise
// the ring.  Here the loads are invisible to it and the kernel orders them itself: vmcnt waits
// plus a workgroup barrier before a stage is read, a barrier after its last read before it is
// refilled.  m0 is not allocatable: the compiler sets it immediately before each use of its own.
__device__ __forceinline__ void lds_dma16(uint64_t base, unsigned off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_addr));
}

// workgroup barrier that also tells the compiler LDS contents changed (the DMA writes are not
// visible to it): no LDS access may be moved across
__device__ __forceinline__ void stage_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// One operand of the tile: where its direct loads come from and where its MFMA fragments sit in LDS.
//   KC tile [256 rows][32 k] (64-byte rows): load instruction j = 4 i + wave covers rows 16 j .. 16 j + 15;
//      lane l writes slot (l & 3) of row 16 j + (l >> 2); slot s of row r holds chunk s ^ ((r >> 2) & 3).
//   NC tile [32 k][256 cols] (512-byte rows): load instruction j covers k rows 2 j, 2 j + 1;
//      lane l writes position (l & 31) of k row 2 j + (l >> 5); position p of row k holds chunk p ^ ((k & 3) << 2).
// Rows (KC) / column chunks (NC) outside the matrix are clamped to the last valid one: they feed
// output rows / columns that the epilogue does not store.
template <bool KC>
struct Operand {
  uint64_t base;          // tile origin at the current K position (bytes); wavefront-uniform
  uint64_t kstep;         // bytes per K step
  unsigned goff[4];       // per-lane byte offsets of the 4 loads of a step
  // LDS byte offsets (inside an operand tile) of this lane's fragment reads.
  //   KC: rd[ks] for MFMA k-step ks; fragment i is 2048 i bytes further (32 rows)
  //   NC: rd[i] for fragment i; MFMA k-step ks adds 8192, the second transposing read of a fragment 2048
  unsigned rd[KC ? 2 : 4];

  __device__ __forceinline__ void init(const bf16_t* mat, int64_t ld, int64_t origin, int64_t extent, int w0, int lane, int wave) {
    if (KC) {
      base = (uint64_t)(mat + origin * ld);
      kstep = BK2 * 2;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        int64_t r = 16 * (4 * i + wave) + (lane >> 2);
        if (origin + r >= extent) r = extent - 1 - origin;
        const int c = (lane & 3) ^ ((lane >> 4) & 3);
        goff[i] = (unsigned)(r * ld * 2 + c * 16);
      }
      const int r = w0 + (lane & 31);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) rd[ks] = r * 64 + (((2 * ks + (lane >> 5)) ^ ((r >> 2) & 3)) << 4);
    } else {
      base = (uint64_t)(mat + origin);
      kstep = (uint64_t)ld * (BK2 * 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k = 2 * (4 * i + wave) + (lane >> 5);
        int64_t col = ((lane & 31) ^ ((k & 3) << 2)) * 8;
        if (origin + col >= extent) col = extent - 8 - origin;
        goff[i] = (unsigned)((k * ld + col) * 2);
      }
      const int blk = lane >> 4, l16 = lane & 15;
      const int k = 8 * (blk >> 1) + (l16 >> 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = w0 + 32 * i + 16 * (blk & 1) + 4 * (l16 & 3);
        rd[i] = k * 512 + (((n >> 3) ^ ((k & 3) << 2)) << 4) + (n & 7) * 2;
      }
    }
  }
  // direct load number i (0..3) of the current K step into the operand tile at LDS address lds_op
  __device__ __forceinline__ void dma(int i, unsigned lds_op, int wave) const { lds_dma16(base, goff[i], lds_op + (4 * i + wave) * 1024); }
  __device__ __forceinline__ void advance() { base += kstep; }
  // fragment i (32 rows / columns starting at w0 + 32 i) of MFMA k-step ks from the operand tile at op
  __device__ __forceinline__ bf16x8_t frag(const lds_u8_t* op, int i, int ks) const {
    if (KC) {
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(op + rd[ks] + 2048 * i);
    } else {
      union { s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
      for (int r = 0; r < 2; ++r)
        u.h[r] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(op + rd[i] + 8192 * ks + 2048 * r));
      return u.v;
    }
  }
};

// order in which a half step multiplies its 4 x 4 fragment pairs, two per group, and the fragment
// each group reads for the following half step (0..3 = A fragment, 4..7 = B fragment): every
// fragment is read at least five groups before the first MFMA that needs it
__device__ constexpr int kMfmaI[16] = {0, 0, 1, 1, 0, 1, 2, 2, 2, 0, 1, 2, 3, 3, 3, 3};
__device__ constexpr int kMfmaJ[16] = {0, 1, 0, 1, 2, 2, 0, 1, 2, 3, 3, 3, 0, 1, 2, 3};
__device__ constexpr int kReadOrder[8] = {0, 4, 5, 1, 6, 2, 7, 3};

// ---- accumulator block -> staging rows.  The MFMAs multiply (B fragment) x (A fragment)^T, so a 32 x 32 block of
// the result sits transposed in the accumulator registers: lane l holds ROW l & 31 of the block and, in registers
// 4 g .. 4 g + 3, the four consecutive COLUMNS 8 g + 4 (l >> 5) + 0..3.  Four consecutive floats of a row are one
// 16-byte LDS write: a block goes to the fp32 staging rows ([32][SLD], SLD * 4 a multiple of 16) in 4 writes per lane
// instead of the 16 single-float writes the untransposed layout (a lane = a column) needs.
template <int SLD>
__device__ __forceinline__ void stage_rows(const f32x16_t& blk, float* stg_blk, int lane) {
  float* row = stg_blk + (lane & 31) * SLD + 4 * (lane >> 5);
#pragma unroll
  for (int g = 0; g < 4; ++g)
    *reinterpret_cast<f32x4_t*>(row + 8 * g) = f32x4_t{blk[4 * g], blk[4 * g + 1], blk[4 * g + 2], blk[4 * g + 3]};
}

// ---- the same for a tile that lies wholly inside C with 16-byte aligned row segments (all tiles of
// the layer's shapes): no per-element checks, 32-bit lane offsets from the wavefront's corner of C
// The result is stored non-temporally: a round of tiles writes more than an L2 holds, and ordinary stores
// push the operand panels out of it (1-3 % per GEMM).
//
// EPI = kEpiRope (bf16 output only): the rotary embedding applied to the result before it is stored.
// Columns below rot_cols are heads of 128 whose adjacent pairs (2i, 2i+1) are rotated by the angle of
// (row % S, i); table [S][64][2] fp32 of (cos, sin).  A lane holds 8 consecutive columns of a row here,
// i.e. 4 whole pairs, in fp32: the fused qkv projection then needs no rotary pass of its own, and q, k
// are rounded to bf16 once.  rot_cols is a multiple of the tile width, so a tile rotates wholly or not.
constexpr int kEpiNone = 0, kEpiRope = 1;
struct EpiArgs {
  const float* table;
  int S;
  int64_t rot_cols;
};
template <bool C_F32, int EPI = kEpiNone>
__device__ __forceinline__ void store_tile_full(const f32x16_t (&acc)[4][4], unsigned char* lds2, int wave, int lane, int64_t m0, int64_t n0,
                                                int wm, int wn, void* __restrict__ Cv, int64_t ldc, int accumulate,
                                                const void* __restrict__ Rv, int64_t ldr, EpiArgs ea = EpiArgs{nullptr, 1, 0}) {
  constexpr int SLD = 132;
  constexpr int ES = C_F32 ? 4 : 2;                       // bytes per element of C (and R)
  float* stg = reinterpret_cast<float*>(lds2) + wave * (32 * SLD);
  char* cw = static_cast<char*>(Cv) + ((m0 + wm) * ldc + n0 + wn) * ES;
  const char* rw = Rv ? static_cast<const char*>(Rv) + ((m0 + wm) * ldr + n0 + wn) * ES : nullptr;
  // read-back: a lane takes 16 bytes of a row; C_F32: 32 lanes per row (2 rows per pass), else 16 lanes per row (4 rows per pass)
  constexpr int LPR = C_F32 ? 32 : 16, RPP = 64 / LPR, NPASS = 32 / RPP;
  const int rr0 = lane / LPR, ch = lane % LPR;
  const unsigned coff0 = (unsigned)(rr0 * ldc) * ES + ch * 16, roff0 = (unsigned)(rr0 * ldr) * ES + ch * 16;
  const unsigned cstep = (unsigned)(RPP * ldc) * ES, rstep = (unsigned)(RPP * ldr) * ES;
  const float* srow = stg + rr0 * SLD + ch * (16 / ES);
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) stage_rows<SLD>(acc[i][j], stg + 32 * j, lane);
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
    char* ci = cw + (int64_t)(32 * i) * ldc * ES;
    const char* ri = rw ? rw + (int64_t)(32 * i) * ldr * ES : nullptr;
    const bool rotate = EPI == kEpiRope && n0 < ea.rot_cols;                                   // workgroup-uniform
    const int pos0 = EPI == kEpiRope ? (int)((m0 + wm + 32 * i + rr0) % ea.S) : 0;             // this lane's row in pass 0
    const int pair0 = ((wn + ch * 8) & 127) >> 1;                                              // first of its 4 pairs inside the head
#pragma unroll
    for (int it = 0; it < NPASS; ++it) {
      const float* sp = srow + it * RPP * SLD;
      if (C_F32) {
        f32x4_t v = *reinterpret_cast<const f32x4_t*>(sp);
        if (ri) v += *reinterpret_cast<const f32x4_t*>(ri + roff0 + it * rstep);
        if (accumulate) v += *reinterpret_cast<const f32x4_t*>(ci + coff0 + it * cstep);
        __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(ci + coff0 + it * cstep));
      } else {
        const f32x4_t v0 = *reinterpret_cast<const f32x4_t*>(sp), v1 = *reinterpret_cast<const f32x4_t*>(sp + 4);
        float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
        if constexpr (EPI == kEpiRope) {
          if (rotate) {
            int pos = pos0 + it * RPP;
            pos = pos >= ea.S ? pos - ea.S : pos;      // rows of a pass-group never span more than one sequence boundary (S >= 32)
            const float* tb = ea.table + ((int64_t)pos * 64 + pair0) * 2;
            const f32x4_t cs0 = *reinterpret_cast<const f32x4_t*>(tb), cs1 = *reinterpret_cast<const f32x4_t*>(tb + 4);
            const float cc[4] = {cs0[0], cs0[2], cs1[0], cs1[2]}, sn[4] = {cs0[1], cs0[3], cs1[1], cs1[3]};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const float a = v[2 * e], b2 = v[2 * e + 1];
              v[2 * e] = a * cc[e] - b2 * sn[e];
              v[2 * e + 1] = a * sn[e] + b2 * cc[e];
            }
          }
        }
        if (ri) {
          const bf16x8_t rv = *reinterpret_cast<const bf16x8_t*>(ri + roff0 + it * rstep);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += (float)rv[e];
        }
        if (accumulate) {
          const bf16x8_t cv = *reinterpret_cast<const bf16x8_t*>(ci + coff0 + it * cstep);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += (float)cv[e];
        }
        bf16x8_t o;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
        __builtin_nontemporal_store(o, reinterpret_cast<bf16x8_t*>(ci + coff0 + it * cstep));
      }
    }
    __builtin_amdgcn_s_waitcnt(0xc07f);
    __builtin_amdgcn_wave_barrier();
  }
}

// ---- epilogue shared by the pipelined kernels: 32 x 128 accumulator blocks -> fp32 staging in LDS
// ([32 rows][132] per wavefront, in the ring, which every wavefront has finished reading) ->
// 16-byte accesses that cover whole row segments of C
template <bool C_F32, int EPI = kEpiNone>
__device__ __forceinline__ void store_tile(const f32x16_t (&acc)[4][4], unsigned char* lds2, int wave, int lane, int64_t m0, int64_t n0,
                                           int wm, int wn, int64_t M, int64_t N, void* __restrict__ Cv, int64_t ldc, int accumulate,
                                           const void* __restrict__ Rv, int64_t ldr, EpiArgs ea = EpiArgs{nullptr, 1, 0}) {
  if constexpr (EPI != kEpiNone) {      // the host only asks for a fused epilogue when every tile lies inside the matrix
    store_tile_full<C_F32, EPI>(acc, lds2, wave, lane, m0, n0, wm, wn, Cv, ldc, accumulate, Rv, ldr, ea);
    return;
  }
  {
    constexpr int V = C_F32 ? 3 : 7;                      // elements per 16 bytes, minus one
    const bool full = m0 + BM <= M && n0 + BN <= N && (ldc & V) == 0 && (!Rv || (ldr & V) == 0);    // workgroup-uniform
    if (full) {
      store_tile_full<C_F32>(acc, lds2, wave, lane, m0, n0, wm, wn, Cv, ldc, accumulate, Rv, ldr);
      return;
    }
  }
  if (C_F32) {
    float* C = static_cast<float*>(Cv);
    const float* R = static_cast<const float*>(Rv);
    constexpr int SLD = 132;
    float* stg = reinterpret_cast<float*>(lds2) + wave * (32 * SLD);
    const bool vec_ok = (ldc & 3) == 0 && (!R || (ldr & 3) == 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) stage_rows<SLD>(acc[i][j], stg + 32 * j, lane);
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
      // 32 rows x 128 cols = 1024 chunks of 4 columns; lane -> (row = idx >> 5, chunk = idx & 31): half a
      // wavefront covers 512 contiguous bytes of a row
#pragma unroll
      for (int it = 0; it < 16; ++it) {
        const int idx = it * 64 + lane, rr = idx >> 5, ch = idx & 31;
        const int64_t row = m0 + wm + 32 * i + rr, col = n0 + wn + ch * 4;
        if (row < M && col < N) {
          f32x4_t v = *reinterpret_cast<const f32x4_t*>(stg + rr * SLD + ch * 4);
          float* cp = C + row * ldc + col;
          if (col + 4 <= N && vec_ok) {
            if (R) v += *reinterpret_cast<const f32x4_t*>(R + row * ldr + col);
            if (accumulate) v += *reinterpret_cast<const f32x4_t*>(cp);
            *reinterpret_cast<f32x4_t*>(cp) = v;
          } else {
            for (int e = 0; e < 4 && col + e < N; ++e) {
              float x = v[e];
              if (R) x += R[row * ldr + col + e];
              if (accumulate) x += cp[e];
              cp[e] = x;
            }
          }
        }
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
    }
  } else {
    // fp32 staging in LDS ([32 rows][132] per wavefront), then 16-byte coalesced bf16 rows
    bf16_t* C = static_cast<bf16_t*>(Cv);
    const bf16_t* R = static_cast<const bf16_t*>(Rv);
    constexpr int SLD = 132;
    float* stg = reinterpret_cast<float*>(lds2) + wave * (32 * SLD);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int j = 0; j < 4; ++j) stage_rows<SLD>(acc[i][j], stg + 32 * j, lane);
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
      // 32 rows x 128 cols = 512 chunks of 8 columns; lane -> (row = idx >> 4, chunk = idx & 15)
#pragma unroll
      for (int it = 0; it < 8; ++it) {
        const int idx = it * 64 + lane, rr = idx >> 4, ch = idx & 15;
        const int64_t row = m0 + wm + 32 * i + rr, col = n0 + wn + ch * 8;
        if (row < M && col < N) {
          const f32x4_t v0 = *reinterpret_cast<const f32x4_t*>(stg + rr * SLD + ch * 8);
          const f32x4_t v1 = *reinterpret_cast<const f32x4_t*>(stg + rr * SLD + ch * 8 + 4);
          float v[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
          if (col + 8 <= N && (ldc & 7) == 0 && (!R || (ldr & 7) == 0)) {
            if (R) {
              const bf16x8_t rv = *reinterpret_cast<const bf16x8_t*>(R + row * ldr + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += (float)rv[e];
            }
            if (accumulate) {
              const bf16x8_t cv = *reinterpret_cast<const bf16x8_t*>(C + row * ldc + col);
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] += (float)cv[e];
            }
            bf16x8_t o;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] = (bf16_t)v[e];
            *reinterpret_cast<bf16x8_t*>(C + row * ldc + col) = o;
          } else {
            for (int e = 0; e < 8 && col + e < N; ++e) {
              float x = v[e];
              if (R) x += (float)R[row * ldr + col + e];
              if (accumulate) x += (float)C[row * ldc + col + e];
              C[row * ldc + col + e] = (bf16_t)x;
            }
          }
        }
      }
      __builtin_amdgcn_s_waitcnt(0xc07f);
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// one GEMM as the pipelined kernels take it
struct GemmArgs {
  int64_t M, N, K;
  const bf16_t* A;
  int64_t lda;
  const bf16_t* B;
  int64_t ldb;
  void* C;
  int64_t ldc;
  int accumulate;
  const void* R;
  int64_t ldr;
  int tiles_m, tiles_n;
  EpiArgs epi;            // fused epilogues only
  // TN only: the contraction cut into `splits` ranges of k_chunk rows, one workgroup per (range, tile); range s writes its
  // partial product, dense [M][N] fp32, to part + s * M * N, and a second kernel sums the ranges into C in a fixed order
  int splits;
  int64_t k_chunk;
  float* part;
};

template <int MODE, bool C_F32>
__device__ __forceinline__ void gemm_dlds_body(const GemmArgs& ga, int block) {
  const int64_t M = ga.M, N = ga.N, lda = ga.lda, ldb = ga.ldb, ldr = ga.ldr;
  int64_t K = ga.K, ldc = ga.ldc;
  const bf16_t* __restrict__ A = ga.A;
  const bf16_t* __restrict__ B = ga.B;
  void* __restrict__ Cv = ga.C;
  const void* __restrict__ Rv = ga.R;
  int accumulate = ga.accumulate;
  const int tiles_m = ga.tiles_m, tiles_n = ga.tiles_n;
  if (MODE == GEMM_TN && C_F32 && ga.splits > 1) {      // workgroup-uniform: this workgroup's range of the contraction
    const int ntl = tiles_m * tiles_n, sp = block / ntl;
    block -= sp * ntl;
    const int64_t k0 = (int64_t)sp * ga.k_chunk;
    A += k0 * lda;
    B += k0 * ldb;
    K = K - k0 < ga.k_chunk ? K - k0 : ga.k_chunk;
    Cv = ga.part + (int64_t)sp * M * N;
    ldc = N;
    accumulate = 0;
  }
  constexpr bool A_KC = (MODE != GEMM_TN);
  constexpr bool B_KC = (MODE == GEMM_NT);
  extern __shared__ __attribute__((aligned(16))) unsigned char lds2[];
  const lds_u8_t* lds = (const lds_u8_t*)lds2;
  const unsigned lds0 = (unsigned)(size_t)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ---- XCD-aware tile id
  int tm, tn;
  gemm_tile_of_block(block, tiles_m, tiles_n, &tm, &tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  Operand<A_KC> oa;
  Operand<B_KC> ob;
  oa.init(A, lda, m0, M, wm, lane, wave);
  ob.init(B, ldb, n0, N, wn, lane, wave);

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (int)(K / BK2);
  // ---- prologue: tiles 0, 1, 2 in flight; tiles 0 and 1 landed and visible before the loop
  for (int t = 0; t < 3 && t < nk; ++t) {
    const unsigned st = lds0 + t * kStageBytes;
#pragma unroll
    for (int i = 0; i < 4; ++i) oa.dma(i, st, wave);
#pragma unroll
    for (int i = 0; i < 4; ++i) ob.dma(i, st + kOpBytes, wave);
    oa.advance();
    ob.advance();
  }
  if (nk >= 3) wait_vmcnt<8>(); else wait_vmcnt<0>();
  stage_barrier();
  __builtin_amdgcn_sched_barrier(0);

  bf16x8_t fa[2][4], fb[2][4];     // [MFMA k-step of the tile][fragment]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fa[0][i] = oa.frag(lds, i, 0);
    fb[0][i] = ob.frag(lds + kOpBytes, i, 0);
  }

  // one K step.  First half: MFMAs of k-step 0 (fragments already in registers) with the loads
  // of tile kt + 3 (its stage held tile kt - 1, which every wavefront finished before the barrier
  // that ended the previous step) and the fragment reads of k-step 1.  Second half: MFMAs of
  // k-step 1 with the first fragments of tile kt + 1 (visible since the previous barrier).
  auto constexpr_mfma = [&](int e, int h) {
    acc[kMfmaI[e]][kMfmaJ[e]] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[h][kMfmaJ[e]], fa[h][kMfmaI[e]], acc[kMfmaI[e]][kMfmaJ[e]], 0, 0, 0);
  };
  auto step = [&](int kt, auto load_c) {
    constexpr bool LOAD = decltype(load_c)::value;
    const lds_u8_t* cur = lds + (kt & (kStages - 1)) * kStageBytes;
    const lds_u8_t* nxt = lds + ((kt + 1) & (kStages - 1)) * kStageBytes;
    const unsigned dst = lds0 + ((kt + 3) & (kStages - 1)) * kStageBytes;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const lds_u8_t* src = h == 0 ? cur : nxt;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        constexpr_mfma(2 * q, h);
        const int f = kReadOrder[q];
        if (f < 4) fa[1 - h][f] = oa.frag(src, f, 1 - h);
        else fb[1 - h][f - 4] = ob.frag(src + kOpBytes, f - 4, 1 - h);
        __builtin_amdgcn_sched_barrier(0);
        constexpr_mfma(2 * q + 1, h);
        if (LOAD && h == 0) {
          if (q < 4) oa.dma(q, dst, wave);
          else ob.dma(q - 4, dst + kOpBytes, wave);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (LOAD) {
      oa.advance();
      ob.advance();
      wait_vmcnt<8>();      // tile kt + 2 has landed: only tile kt + 3's 8 loads may still be in flight
    } else {
      wait_vmcnt<0>();
    }
    stage_barrier();
    __builtin_amdgcn_sched_barrier(0);
  };
  // the prologue's fragment reads have returned; with nothing outstanding at loop entry the
  // compiler's lgkmcnt bookkeeping inside the loop only has the loop's own LDS reads to consider
  __builtin_amdgcn_s_waitcnt(0xc07f);
  int kt = 0;
  for (; kt + 3 < nk; ++kt) step(kt, std::true_type{});
  for (; kt < nk; ++kt) step(kt, std::false_type{});

  store_tile<C_F32>(acc, lds2, wave, lane, m0, n0, wm, wn, M, N, Cv, ldc, accumulate, Rv, ldr);
}

// =============================================================================== 64-deep K steps
// The same pipeline with K advancing 64 at a time through a ring of two 64 KiB stages.  What it buys:
// a K-contiguous operand row is 128 bytes per step, one full cache line fetched by 8 adjacent lanes,
// instead of two 64-byte halves fetched in two different steps (the L2 serves either as one request,
// and a layer's forward and input-gradient GEMMs were bound by that request rate).
//
// A step is four MFMA k-steps q0..q3 of 16 MFMAs.  Its workgroup barrier sits after q2, not at the
// end: the fragments of k-step 3 are read during q2, so at that barrier the stage is no longer read
// and the next stage (loaded during q3 of the previous step and q0 of this one) has landed.  q3 then
// already reads the first fragments of the next stage and starts refilling the stage just finished.
//   KC tile [256 rows][64 k] (128-byte rows): load instruction j = 4 i + wave covers rows 8 j .. 8 j + 7;
//      lane l writes slot (l & 7) of row 8 j + (l >> 3); slot s of row r holds chunk s ^ ((r >> 1) & 7)
//      (16 consecutive rows of one chunk column then sit in 16 different bank groups).
//   NC tile [64 k][256 cols]: as above with twice the k rows.
constexpr int BK64 = 64;
constexpr int kOp64 = 256 * BK64 * 2;            // one operand tile: 32 KiB
constexpr int kStage64 = 2 * kOp64;              // 64 KiB
constexpr size_t kLds64 = 2 * (size_t)kStage64;  // 128 KiB

template <bool KC>
struct Operand64 {
  uint64_t base;          // tile origin at the current K position (bytes); wavefront-uniform
  uint64_t kstep;         // bytes per K step
  unsigned goff[8];       // per-lane byte offsets of the 8 loads of a step
  // KC: rd[ks] for MFMA k-step ks, fragment i is 4096 i bytes further (32 rows)
  // NC: rd[i] for fragment i; MFMA k-step ks adds 8192, the second transposing read of a fragment 2048
  unsigned rd[4];

  __device__ __forceinline__ void init(const bf16_t* mat, int64_t ld, int64_t origin, int64_t extent, int w0, int lane, int wave) {
    if (KC) {
      base = (uint64_t)(mat + origin * ld);
      kstep = BK64 * 2;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int rt = 8 * (4 * i + wave) + (lane >> 3);      // row of the tile this lane's 16 bytes land in
        int64_t r = rt;
        if (origin + r >= extent) r = extent - 1 - origin;
        const int c = (lane & 7) ^ ((rt >> 1) & 7);
        goff[i] = (unsigned)(r * ld * 2 + c * 16);
      }
      const int r = w0 + (lane & 31);
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) rd[ks] = r * 128 + (((2 * ks + (lane >> 5)) ^ ((r >> 1) & 7)) << 4);
    } else {
      base = (uint64_t)(mat + origin);
      kstep = (uint64_t)ld * (BK64 * 2);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int k = 2 * (4 * i + wave) + (lane >> 5);
        int64_t col = ((lane & 31) ^ ((k & 3) << 2)) * 8;
        if (origin + col >= extent) col = extent - 8 - origin;
        goff[i] = (unsigned)((k * ld + col) * 2);
      }
      const int blk = lane >> 4, l16 = lane & 15;
      const int k = 8 * (blk >> 1) + (l16 >> 2);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int n = w0 + 32 * i + 16 * (blk & 1) + 4 * (l16 & 3);
        rd[i] = k * 512 + (((n >> 3) ^ ((k & 3) << 2)) << 4) + (n & 7) * 2;
      }
    }
  }
  __device__ __forceinline__ void dma(int i, unsigned lds_op, int wave) const { lds_dma16(base, goff[i], lds_op + (4 * i + wave) * 1024); }
  __device__ __forceinline__ void advance() { base += kstep; }
  __device__ __forceinline__ bf16x8_t frag(const lds_u8_t* op, int i, int ks) const {
    if (KC) {
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(op + rd[ks] + 4096 * i);
    } else {
      union { s16x4_t h[2]; bf16x8_t v; } u;
#pragma unroll
      for (int r = 0; r < 2; ++r)
        u.h[r] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(op + rd[i] + 8192 * ks + 2048 * r));
      return u.v;
    }
  }
};

template <int MODE, bool C_F32, int EPI = kEpiNone>
__device__ __forceinline__ void gemm_dlds64_body(const GemmArgs& ga, int block) {
  const int64_t M = ga.M, N = ga.N, K = ga.K, lda = ga.lda, ldb = ga.ldb, ldc = ga.ldc, ldr = ga.ldr;
  const bf16_t* __restrict__ A = ga.A;
  const bf16_t* __restrict__ B = ga.B;
  void* __restrict__ Cv = ga.C;
  const void* __restrict__ Rv = ga.R;
  const int accumulate = ga.accumulate, tiles_m = ga.tiles_m, tiles_n = ga.tiles_n;
  constexpr bool A_KC = (MODE != GEMM_TN);
  constexpr bool B_KC = (MODE == GEMM_NT);
  extern __shared__ __attribute__((aligned(16))) unsigned char lds2[];
  const lds_u8_t* lds = (const lds_u8_t*)lds2;
  const unsigned lds0 = (unsigned)(size_t)lds;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // ---- XCD-aware tile id
  int tm, tn;
  gemm_tile_of_block(block, tiles_m, tiles_n, &tm, &tn);
  const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

  const int wm = (wave >> 1) * 128, wn = (wave & 1) * 128;
  Operand64<A_KC> oa;
  Operand64<B_KC> ob;
  oa.init(A, lda, m0, M, wm, lane, wave);
  ob.init(B, ldb, n0, N, wn, lane, wave);

  f32x16_t acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (int)(K / BK64);
  // ---- prologue: stage 0 whole and the A half of stage 1 in flight; stage 0 landed and visible
#pragma unroll
  for (int i = 0; i < 8; ++i) oa.dma(i, lds0, wave);
#pragma unroll
  for (int i = 0; i < 8; ++i) ob.dma(i, lds0 + kOp64, wave);
  oa.advance();
  ob.advance();
  if (nk > 1) {
#pragma unroll
    for (int i = 0; i < 8; ++i) oa.dma(i, lds0 + kStage64, wave);
    oa.advance();
    wait_vmcnt<8>();
  } else {
    wait_vmcnt<0>();
  }
  stage_barrier();
  __builtin_amdgcn_sched_barrier(0);

  bf16x8_t fa[2][4], fb[2][4];     // [parity of the MFMA k-step][fragment]
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    fa[0][i] = oa.frag(lds, i, 0);
    fb[0][i] = ob.frag(lds + kOp64, i, 0);
  }
  auto constexpr_mfma = [&](int e, int h) {
    acc[kMfmaI[e]][kMfmaJ[e]] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[h][kMfmaJ[e]], fa[h][kMfmaI[e]], acc[kMfmaI[e]][kMfmaJ[e]], 0, 0, 0);
  };
  // one K step of 64.  LB: the B half of stage kt + 1 is still to be loaded (during q0); LA: stage
  // kt + 2 exists, its A half is loaded during q3 into the stage this step has finished with;
  // NEXT: stage kt + 1 exists, q3 reads its first fragments.
  auto step = [&](int kt, auto lb_c, auto la_c, auto next_c) {
    constexpr bool LB = decltype(lb_c)::value, LA = decltype(la_c)::value, NEXT = decltype(next_c)::value;
    const lds_u8_t* cur = lds + (kt & 1) * kStage64;
    const lds_u8_t* nxt = lds + ((kt + 1) & 1) * kStage64;
    const unsigned dst_b = lds0 + ((kt + 1) & 1) * kStage64 + kOp64;
    const unsigned dst_a = lds0 + (kt & 1) * kStage64;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int h = q & 1;
      const lds_u8_t* src = q < 3 ? cur : nxt;
      const int ks = (q + 1) & 3;
      auto read = [&](int f) {
        if (f < 4) fa[1 - h][f] = oa.frag(src, f, ks);
        else fb[1 - h][f - 4] = ob.frag(src + kOp64, f - 4, ks);
      };
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        constexpr_mfma(2 * e, h);
        if (q == 2) {                    // all of k-step 3's fragments early: the barrier after q2 waits for them
          if (e < 4) { read(kReadOrder[2 * e]); read(kReadOrder[2 * e + 1]); }
        } else if (q < 3 || NEXT) {
          read(kReadOrder[e]);
        }
        __builtin_amdgcn_sched_barrier(0);
        constexpr_mfma(2 * e + 1, h);
        if (LB && q == 0) ob.dma(e, dst_b, wave);
        if (LA && q == 3) oa.dma(e, dst_a, wave);
        __builtin_amdgcn_sched_barrier(0);
      }
      if (LB && q == 0) ob.advance();
      if (LA && q == 3) oa.advance();
      if (q == 2) {
        __builtin_amdgcn_s_waitcnt(0xc07f);   // this wavefront's last reads of the stage have returned
        wait_vmcnt<0>();                      // and its share of the next stage has landed
        stage_barrier();
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  __builtin_amdgcn_s_waitcnt(0xc07f);
  int kt = 0;
  for (; kt + 2 < nk; ++kt) step(kt, std::true_type{}, std::true_type{}, std::true_type{});
  if (kt + 1 < nk) { step(kt, std::true_type{}, std::false_type{}, std::true_type{}); ++kt; }
  step(kt, std::false_type{}, std::false_type{}, std::false_type{});

  store_tile<C_F32, EPI>(acc, lds2, wave, lane, m0, n0, wm, wn, M, N, Cv, ldc, accumulate, Rv, ldr, ga.epi);
}

// ---- kernels: one GEMM, or two independent ones in one grid (the first's tiles, then the second's)
template <int MODE, bool C_F32, bool K64, int EPI = kEpiNone>
__global__ void __launch_bounds__(kThreads, 1) gemm_pipe_kernel(GemmArgs g) {
  static_assert(EPI == kEpiNone || K64, "fused epilogues exist for the 64-deep loop only");
  if constexpr (K64) gemm_dlds64_body<MODE, C_F32, EPI>(g, (int)blockIdx.x);
  else gemm_dlds_body<MODE, C_F32>(g, (int)blockIdx.x);
}
// The layer's backward has such pairs at every linear: the input gradient and the weight gradient
// read the same incoming gradient and write different outputs.  Neither tile count is a multiple
// of the 256 compute units for every width, so two launches leave two partly filled last rounds;
// one grid leaves one.  The weight-gradient tiles (longer: they contract over all tokens) go first.
template <int MODE0, bool F32_0, bool K64_0, int MODE1, bool F32_1, bool K64_1>
__global__ void __launch_bounds__(kThreads, 1) gemm_dual_kernel(GemmArgs g0, GemmArgs g1, int n0) {
  if ((int)blockIdx.x < n0) {
    if (K64_0) gemm_dlds64_body<MODE0, F32_0>(g0, (int)blockIdx.x);
    else gemm_dlds_body<MODE0, F32_0>(g0, (int)blockIdx.x);
  } else {
    if (K64_1) gemm_dlds64_body<MODE1, F32_1>(g1, (int)blockIdx.x - n0);
    else gemm_dlds_body<MODE1, F32_1>(g1, (int)blockIdx.x - n0);
  }
}

inline GemmArgs make_args(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                          int accumulate, const void* R, int64_t ldr) {
  GemmArgs g;
  g.M = M; g.N = N; g.K = K;
  g.A = (const bf16_t*)A; g.lda = lda;
  g.B = (const bf16_t*)B; g.ldb = ldb;
  g.C = C; g.ldc = ldc;
  g.accumulate = accumulate;
  g.R = R; g.ldr = ldr;
  g.tiles_m = (int)((M + BM - 1) / BM);
  g.tiles_n = (int)((N + BN - 1) / BN);
  g.epi = EpiArgs{nullptr, 1, 0};
  g.splits = 1;
  g.k_chunk = K;
  g.part = nullptr;
  return g;
}

static_assert(kLds64 == kLds2, "the two pipelined kernels share one LDS size");

template <int MODE, bool C_F32, bool K64, int EPI = kEpiNone>
int launch_pipe(const GemmArgs& g, hipStream_t st) {
  TAW_SET_LDS_LIMIT_ONCE((gemm_pipe_kernel<MODE, C_F32, K64, EPI>), kLds2);
  hipLaunchKernelGGL((gemm_pipe_kernel<MODE, C_F32, K64, EPI>), dim3((unsigned)(g.tiles_m * g.tiles_n)), dim3(kThreads), kLds2, st, g);
  return (int)hipGetLastError();
}

template <int MODE0, bool F32_0, bool K64_0, int MODE1, bool F32_1, bool K64_1>
int launch_dual(const GemmArgs& g0, const GemmArgs& g1, hipStream_t st) {
  TAW_SET_LDS_LIMIT_ONCE((gemm_dual_kernel<MODE0, F32_0, K64_0, MODE1, F32_1, K64_1>), kLds2);
  const int n0 = g0.tiles_m * g0.tiles_n * g0.splits, n1 = g1.tiles_m * g1.tiles_n;
  hipLaunchKernelGGL((gemm_dual_kernel<MODE0, F32_0, K64_0, MODE1, F32_1, K64_1>), dim3((unsigned)(n0 + n1)), dim3(kThreads), kLds2, st, g0, g1, n0);
  return (int)hipGetLastError();
}

}  // namespace v2

template <int MODE, bool C_F32>
int launch_t(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
             int accumulate, const void* R, int64_t ldr, hipStream_t st) {
  TAW_SET_LDS_LIMIT_ONCE((gemm_mfma_kernel<MODE, C_F32>), kLdsBytes);
  const int tiles_m = (int)((M + BM - 1) / BM), tiles_n = (int)((N + BN - 1) / BN);
  hipLaunchKernelGGL((gemm_mfma_kernel<MODE, C_F32>), dim3((unsigned)(tiles_m * tiles_n)), dim3(kThreads), kLdsBytes, st, M, N, K,
                     (const bf16_t*)A, lda, (const bf16_t*)B, ldb, C, ldc, accumulate, R, ldr, tiles_m, tiles_n);
  return (int)hipGetLastError();
}

}  // namespace

bool gemm_mfma_supported(int dtype, int mode, int64_t M, int64_t N, int64_t K, int64_t lda, int64_t ldb, int64_t ldc,
                         int c_dtype, int64_t ldr) {
  (void)c_dtype;
  if (dtype != DT_BF16) return false;
  if (M <= 0 || N <= 0 || K <= 0) return false;
  if (lda % 8 || ldb % 8) return false;                     // 16-byte global loads
  if (mode == GEMM_NT) { if (K % 8) return false; }
  else if (mode == GEMM_NN) { if (K % 8 || N % 8) return false; }
  else if (mode == GEMM_TN) { if (M % 8 || N % 8) return false; }
  else return false;
  // per-thread offsets inside a tile are 32-bit (operand loads, and the result / residual rows of the epilogue)
  if (lda > ((int64_t)1 << 22) || ldb > ((int64_t)1 << 22) || ldc > ((int64_t)1 << 22) || ldr > ((int64_t)1 << 22)) return false;
  if ((M + BM - 1) / BM * ((N + BN - 1) / BN) > ((int64_t)1 << 30)) return false;
  return true;
}

int launch_gemm_mfma(int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb,
                     void* C, int64_t ldc, int c_dtype, int accumulate, const void* R, int64_t ldr, hipStream_t st) {
  const bool f32 = c_dtype == DT_F32;
  if (K % v2::BK2 != 0 || K < v2::BK2) {     // the pipelined kernel has no K tail
    switch (mode) {
      case GEMM_NT: return f32 ? launch_t<GEMM_NT, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                               : launch_t<GEMM_NT, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
      case GEMM_NN: return f32 ? launch_t<GEMM_NN, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                               : launch_t<GEMM_NN, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
      default: return f32 ? launch_t<GEMM_TN, true>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st)
                          : launch_t<GEMM_TN, false>(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr, st);
    }
  }
  // K-contiguous operands gain from 64-deep steps (whole cache lines per row); the weight-gradient form has none
  const v2::GemmArgs g = v2::make_args(M, N, K, A, lda, B, ldb, C, ldc, accumulate, R, ldr);
  const bool k64 = K % v2::BK64 == 0 && mode != GEMM_TN;
  switch (mode) {
    case GEMM_NT:
      if (k64) return f32 ? v2::launch_pipe<GEMM_NT, true, true>(g, st) : v2::launch_pipe<GEMM_NT, false, true>(g, st);
      return f32 ? v2::launch_pipe<GEMM_NT, true, false>(g, st) : v2::launch_pipe<GEMM_NT, false, false>(g, st);
    case GEMM_NN:
      if (k64) return f32 ? v2::launch_pipe<GEMM_NN, true, true>(g, st) : v2::launch_pipe<GEMM_NN, false, true>(g, st);
      return f32 ? v2::launch_pipe<GEMM_NN, true, false>(g, st) : v2::launch_pipe<GEMM_NN, false, false>(g, st);
    default:
      return f32 ? v2::launch_pipe<GEMM_TN, true, false>(g, st) : v2::launch_pipe<GEMM_TN, false, false>(g, st);
  }
}

// C[M][N] (row stride ldc) = (accumulate ? C : 0) + part[0] + part[1] + ... + part[splits - 1], in that order; N % 4 == 0
__global__ void __launch_bounds__(256) splitk_reduce_kernel(float* __restrict__ C, int64_t ldc, const float* __restrict__ part, int splits,
                                                            int64_t M, int64_t N, int accumulate) {
  const int64_t n4 = N / 4, total = M * n4;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
    const int64_t r = i / n4, c4 = i - r * n4;
    float* cp = C + r * ldc + c4 * 4;
    f32x4_t v = accumulate ? *reinterpret_cast<const f32x4_t*>(cp) : f32x4_t{0.f, 0.f, 0.f, 0.f};
    const float* pp = part + r * N + c4 * 4;
    for (int sidx = 0; sidx < splits; ++sidx) v += __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(pp + (int64_t)sidx * M * N));
    *reinterpret_cast<f32x4_t*>(cp) = v;
  }
}

// Into how many ranges the weight gradient of the linear y[T, N] = x[T, K] W^T is cut (1 = not at all), and the rows per
// range.  Its tiles contract over all T tokens: with few of them (narrow layers) a tile runs long after everything else
// in the grid is done, most compute units idle.  The ranges are sized so that one takes at most about half of what a
// compute unit's fair share of the whole grid (both GEMMs) takes; never shorter than 512 rows, never more than 32 ranges.
int gemm_dual_splits(int64_t T, int64_t N, int64_t K, int64_t* k_chunk) {
  const int64_t tn_tiles = ((N + BM - 1) / BM) * ((K + BN - 1) / BN), nn_tiles = ((T + BM - 1) / BM) * ((K + BN - 1) / BN);
  const double fair = ((double)tn_tiles * (double)T + (double)nn_tiles * (double)N) / 256.0;     // contraction rows per compute unit
  int64_t sp = fair > 0 ? (int64_t)(2.0 * (double)T / fair + 0.999) : 1;
  if (sp > 32) sp = 32;
  if (sp > T / 512) sp = T / 512;
  if (sp < 2) { *k_chunk = T; return 1; }
  int64_t chunk = ((T + sp - 1) / sp + 63) / 64 * 64;
  sp = (T + chunk - 1) / chunk;
  *k_chunk = chunk;
  return (int)sp;
}

bool gemm_mfma_dual_supported(int64_t K_tn, int64_t K_nn) { return K_tn >= v2::BK2 && K_tn % v2::BK2 == 0 && K_nn >= v2::BK2 && K_nn % v2::BK2 == 0; }

int launch_gemm_mfma_dual(int64_t M0, int64_t N0, int64_t K0, const void* A0, int64_t lda0, const void* B0, int64_t ldb0, float* C0,
                          int64_t ldc0, int accumulate0, int64_t M1, int64_t N1, int64_t K1, const void* A1, int64_t lda1,
                          const void* B1, int64_t ldb1, void* C1, int64_t ldc1, float* part, int splits, int64_t k_chunk, hipStream_t st) {
  v2::GemmArgs g0 = v2::make_args(M0, N0, K0, A0, lda0, B0, ldb0, C0, ldc0, accumulate0, nullptr, 0);
  const v2::GemmArgs g1 = v2::make_args(M1, N1, K1, A1, lda1, B1, ldb1, C1, ldc1, 0, nullptr, 0);
  if (part && splits > 1) {
    g0.splits = splits;
    g0.k_chunk = k_chunk;
    g0.part = part;
  }
  const int rc = K1 % v2::BK64 == 0 ? v2::launch_dual<GEMM_TN, true, false, GEMM_NN, false, true>(g0, g1, st)
                                    : v2::launch_dual<GEMM_TN, true, false, GEMM_NN, false, false>(g0, g1, st);
  if (rc || g0.splits == 1) return rc;
  const int64_t total = M0 * (N0 / 4);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 2048 ? (total + 255) / 256 : 2048);
  hipLaunchKernelGGL(splitk_reduce_kernel, dim3(blocks), dim3(256), 0, st, C0, ldc0, part, g0.splits, M0, N0, accumulate0);
  return (int)hipGetLastError();
}

bool gemm_mfma_rope_supported(int64_t M, int64_t N, int64_t K, int64_t rot_cols, int S) {
  return M % BM == 0 && N % BN == 0 && K % v2::BK64 == 0 && rot_cols % BN == 0 && rot_cols % 128 == 0 && S >= 32;
}

int launch_gemm_mfma_nt_rope(int64_t M, int64_t N, int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C, int64_t ldc,
                             const float* rope_table, int S, int64_t rot_cols, hipStream_t st) {
  v2::GemmArgs g = v2::make_args(M, N, K, A, lda, B, ldb, C, ldc, 0, nullptr, 0);
  g.epi = v2::EpiArgs{rope_table, S, rot_cols};
  return v2::launch_pipe<GEMM_NT, false, true, v2::kEpiRope>(g, st);
}

}  // namespace taw
