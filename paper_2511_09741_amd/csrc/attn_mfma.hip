// Causal softmax attention for head_dim 128 on the gfx950 matrix cores: tiled, online softmax, no
// S x S matrix in memory.  bf16 operands, fp32 accumulation, fp32 softmax statistics.
//
// Layout of the operands: qkv [B*S, 3H] row-major, q | k | v, head h at columns h*128 of each part.
//
// All three kernels use v_mfma_f32_32x32x16_bf16.  Its accumulator layout gives lane l column
// (l & 31) and rows 8(r/4) + 4(l>>5) + r%4 for register r; its operand layout gives lane l row or
// column (l & 31) and k = 8(l>>5) + 0..7.  The kernels are arranged so that the accumulator of the
// first product can be fed, converted to bf16 and nothing else, into the operand of the second:
//
//   forward / dQ kernel:  S^T[kv][q] = K Q^T  -> lane owns one query column: the softmax row
//     statistics (max, sum, lse, D) are per-lane scalars; P^T (or dS^T) is then the B operand of
//     O^T[d][q] += V^T[d][kv] P^T[kv][q]   (dQ^T += K^T dS^T).
//   dK/dV kernel:  S[q][kv] = Q K^T  -> lane owns one key column; P (dS) is the B operand of
//     dV^T[d][kv] += dO^T[d][q] P[q][kv]   (dK^T += Q^T dS).
//
// The A operands V^T, K^T, dO^T, Q^T are "transposed" tiles: they are read from the row-major LDS
// tile with ds_read_b64_tr_b16, which returns 4 consecutive rows of one column per lane: exactly
// the 4-row groups of the accumulator layout.  Nothing is transposed through memory.
#include "dev_common.h"
#include "taw_internal.h"

namespace taw {

namespace {

constexpr int D = 128;             // head_dim
constexpr int kThreads = 256;      // 4 wavefronts
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ s16x4_t lds_read_tr(const bf16_t* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
}
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ f32x16_t mfma(bf16x8_t a, bf16x8_t b, f32x16_t c) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// ---- row-major [rows][128] bf16 tile in LDS, 16-byte chunks XOR-swizzled ------------------------
// A row is 256 bytes = one pass over all 64 banks, so the chunk index is the bank group.  One
// swizzle serves both access patterns:  chunk ^= ((row & 3) << 2) | ((row >> 2) & 3).
//   natural reads (8 consecutive d of one row per lane, ds_read_b128): 16 consecutive lanes read 16
//     consecutive rows of one chunk -> 16 distinct bank groups;
//   transposing reads (4 consecutive rows of one d per lane, ds_read_b64_tr_b16): 32 lanes read
//     4 rows x 4 chunks -> 16 distinct bank groups.
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ (((row & 3) << 2) | ((row >> 2) & 3)); }

// global -> registers -> LDS for a [ROWS][128] tile: ROWS*16/256 chunks of 16 bytes per thread.
// src points at (row 0, column 0 of this head); rows at or beyond `limit` are clamped to limit-1.
template <int N>
__device__ __forceinline__ void tile_load(u32x4_t (&regs)[N], const bf16_t* src, int64_t ld, int row0, int limit, int tid) {
  const int c = tid & 15, r0 = tid >> 4;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    int r = row0 + r0 + 16 * i;
    if (r >= limit) r = limit - 1;
    regs[i] = *reinterpret_cast<const u32x4_t*>(src + (int64_t)r * ld + c * 8);
  }
}
template <int N>
__device__ __forceinline__ void tile_store(bf16_t* tile, const u32x4_t (&regs)[N], int tid) {
  const int c = tid & 15, r0 = tid >> 4;
#pragma unroll
  for (int i = 0; i < N; ++i) {
    const int r = r0 + 16 * i;
    *reinterpret_cast<u32x4_t*>(tile + r * D + (swz(r, c) << 3)) = regs[i];
  }
}

// natural operand: rows row0 + (lane&31), d = 16 ks + 8 (lane>>5) + 0..7
__device__ __forceinline__ bf16x8_t frag_nat(const bf16_t* tile, int row0, int ks, int lane) {
  const int r = row0 + (lane & 31), c = 2 * ks + (lane >> 5);
  return *reinterpret_cast<const bf16x8_t*>(tile + r * D + (swz(r, c) << 3));
}

// transposed operand for the second product: lane gets column d = d0 + (lane&31) and the 8 rows
//   row0 + 16 t + {4h..4h+3, 8+4h..8+4h+3},  h = lane>>5,
// which are the rows that accumulator registers 8t..8t+7 of the first product hold.
__device__ __forceinline__ bf16x8_t frag_tr(const bf16_t* tile, int row0, int t, int d0, int lane) {
  const int blk = lane >> 4, i = lane & 15, h = blk >> 1;
  const int d = d0 + 16 * (blk & 1) + 4 * (i & 3);
  union { s16x4_t h2[2]; bf16x8_t v; } u;
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const int r = row0 + 16 * t + 8 * rr + 4 * h + (i >> 2);
    u.h2[rr] = lds_read_tr(tile + r * D + (swz(r, d >> 3) << 3) + (d & 7));
  }
  return u.v;
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& x, int t) {
  bf16x8_t p;
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = (bf16_t)x[8 * t + j];
  return p;
}

// ---- direct global -> LDS tile loads ----------------------------------------------------------------
typedef __attribute__((address_space(3))) unsigned char lds_u8_t;

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding: vmcnt[3:0] | expcnt<<4 | lgkmcnt<<8 | vmcnt[5:4]<<14)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// 16 bytes per lane from global memory (64-bit scalar base + 32-bit per-lane byte offset) straight
// into LDS at lds_addr + 16 * lane (lds_addr wavefront-uniform).  Inline assembly so that the
// compiler's wait-count insertion does not see the load: it would put s_waitcnt vmcnt(0) in front
// of every transposing LDS read that follows.  The kernels order these loads themselves (vmcnt
// wait + workgroup barrier before a stage is read, barrier after its last read before a refill).
__device__ __forceinline__ void lds_dma16(uint64_t base, unsigned off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_addr));
}
// 4 bytes per lane, same addressing (LDS destination lds_addr + 4 * lane)
__device__ __forceinline__ void lds_dma4(uint64_t base, unsigned off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_addr));
}
// workgroup barrier that also tells the compiler that LDS changed behind its back
__device__ __forceinline__ void stage_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

constexpr int kWaves8 = 8, kThreads8 = 512;
constexpr int kTileBytes = 64 * D * 2;      // a [64][128] bf16 tile: 16 KiB

// This wavefront's share (2 of the 16 one-KiB pieces) of a [64][128] tile load: rows row0 .. row0+63
// of a row-major matrix (row stride ld_bytes, rows clamped to limit-1) into the swizzled LDS tile at
// lds_tile.  Piece j holds rows 4j..4j+3; lane l writes slot l&15 of row 4j + (l>>4), and slot s of
// row r holds chunk s ^ swizzle(r): the lane fetches the chunk that belongs where it writes.
__device__ __forceinline__ void tile_dma(uint64_t base, unsigned ld_bytes, int row0, int limit, unsigned lds_tile, int lane, int wave) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int j = wave + 8 * i;
    const int r = 4 * j + (lane >> 4);
    const int c = swz(r, lane & 15);
    int rg = row0 + r;
    rg = rg < limit ? rg : limit - 1;
    lds_dma16(base, (unsigned)rg * ld_bytes + c * 16, lds_tile + j * 1024);
  }
}

// =============================================================================== forward
// Workgroup: 8 wavefronts (two per SIMD, so one's softmax arithmetic overlaps the other's MFMAs),
// one (batch, head, 256 query rows); wavefront w owns rows 32w .. 32w+31.  Keys/values stream
// through a 4-stage LDS ring of 64-key tiles filled by direct global->LDS loads issued three
// tiles ahead; one workgroup barrier per tile.
//
// Online softmax in the exp2 domain.  The running maximum of a row is only raised when a tile
// exceeds it by more than kMaxSlack (in log2 units): until then the probabilities of the tile are
// taken relative to the stale maximum (they stay below 2^kMaxSlack, harmless in fp32 / bf16) and
// the 64 accumulator registers need no rescaling.  The final division by the row sum makes the
// result independent of which maximum was used.
constexpr float kMaxSlack = 8.0f;

__global__ void __launch_bounds__(kThreads8, 1)
attn_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ o, float* __restrict__ lse, int B, int S, int nh, float scale) {
  constexpr int BQ = 256, WQ = 32, BKV = 64, NS = 4;
  constexpr int kStage = 2 * kTileBytes;   // K tile | V tile
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(size_t)(const lds_u8_t*)lds_raw;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqt = (S + BQ - 1) / BQ;
  const int bh = blockIdx.x % (B * nh);
  const int qt = nqt - 1 - blockIdx.x / (B * nh);      // longest rows first
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const uint64_t kbase = (uint64_t)(qbase + H), vbase = (uint64_t)(qbase + 2 * H);
  const unsigned ldb = (unsigned)(ld * 2);
  const int q0 = qt * BQ, q0w = q0 + wave * WQ;
  const float c = scale * kLog2e;

  const int kv_end = (q0 + BQ < S) ? q0 + BQ : S;
  const int nkv = (kv_end + BKV - 1) / BKV;
  auto issue = [&](int t) {
    const unsigned st = lds0 + (t & (NS - 1)) * kStage;
    tile_dma(kbase, ldb, t * BKV, S, st, lane, wave);
    tile_dma(vbase, ldb, t * BKV, S, st + kTileBytes, lane, wave);
  };
  for (int t = 0; t < NS - 1 && t < nkv; ++t) issue(t);

  // Q as B operands, straight from global memory
  bf16x8_t qf[8];
  {
    int row = q0w + (lane & 31);
    if (row >= S) row = S - 1;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) qf[ks] = *reinterpret_cast<const bf16x8_t*>(qbase + (int64_t)row * ld + 16 * ks + 8 * hh);
  }
  f32x16_t oacc[4];
  float m = -INFINITY, l = 0.f;      // running maximum (scaled, log2 domain) and sum of this lane's half of the keys
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[dt][r] = 0.f;
  const int qidx = q0w + (lane & 31);

  for (int j = 0; j < nkv; ++j) {
    // tile j has landed (each wavefront waits for its own pieces, the barrier collects them); the
    // barrier also says every wavefront is done with tile j-1, whose stage tile j+3 goes into
    const int ahead = nkv - 1 - j;
    if (ahead >= 2) wait_vmcnt<8>(); else if (ahead == 1) wait_vmcnt<4>(); else wait_vmcnt<0>();
    stage_barrier();
    if (j + NS - 1 < nkv) issue(j + NS - 1);
    const int kv0 = j * BKV;
    if (kv0 > q0w + WQ - 1) continue;                  // no key of the tile is visible to this wavefront
    const bf16_t* sk = reinterpret_cast<const bf16_t*>(lds_raw + (j & (NS - 1)) * kStage);
    const bf16_t* sv = sk + 64 * D;

    f32x16_t s[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int r = 0; r < 16; ++r) s[kb][r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) s[kb] = mfma(frag_nat(sk, kb * 32, ks, lane), qf[ks], s[kb]);
    }
    if (kv0 + BKV - 1 > q0w) {                         // tile crosses the diagonal (or the end of the sequence)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          s[kb][r] = kv > qidx ? -INFINITY : s[kb][r];
        }
    }
    float mx = fmaxf(s[0][0], s[1][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, fmaxf(s[0][r], s[1][r]));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c;
    if (__builtin_amdgcn_ballot_w64(mx > m + kMaxSlack) != 0) {    // wavefront-uniform: some row's maximum moved far
      const float m_new = fmaxf(m, mx);
      const float alpha = fast_exp2(m - m_new);        // m = -inf on the first tile: alpha = 0, the accumulators are 0
      m = m_new;
      l *= alpha;
#pragma unroll
      for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[dt][r] *= alpha;
    }
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(__builtin_fmaf(s[kb][r], c, -m));
        s[kb][r] = p;
        rs += p;
      }
    l += rs;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8_t pf = pack8(s[kb], t);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) oacc[dt] = mfma(frag_tr(sv, kb * 32, t, dt * 32, lane), pf, oacc[dt]);
      }
  }
  __syncthreads();          // every wavefront is done with the ring: it becomes the output staging area

  // ---- epilogue: O^T accumulators -> [q][136] bf16 staging in LDS -> coalesced rows of o
  constexpr int OLD = 136;
  bf16_t* ob = reinterpret_cast<bf16_t*>(lds_raw) + wave * (WQ * OLD);
  {
    const float lsum = l + __shfl_xor(l, 32, 64);
    const float inv = 1.0f / lsum;
    const int qrow = lane & 31;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4_t pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (bf16_t)(oacc[dt][4 * r4 + e] * inv);
        *reinterpret_cast<bf16x4_t*>(ob + qrow * OLD + dt * 32 + 8 * r4 + 4 * hh) = pk;
      }
    if (hh == 0 && qidx < S) lse[((int64_t)b * nh + h) * S + qidx] = m * kLn2 + logf(lsum);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0): this wavefront's LDS writes are done
  __builtin_amdgcn_wave_barrier();
  bf16_t* obase = o + (int64_t)b * S * H + (int64_t)h * D;
#pragma unroll
  for (int it = 0; it < WQ * 16 / 64; ++it) {
    const int idx = it * 64 + lane, row = idx >> 4, ch = idx & 15;
    if (q0w + row < S)
      *reinterpret_cast<u32x4_t*>(obase + (int64_t)(q0w + row) * H + ch * 8) = *reinterpret_cast<const u32x4_t*>(ob + row * OLD + ch * 8);
  }
}

// ---- shared epilogue: a wavefront's transposed accumulators X^T[128 d][32 rows] (lane = row,
// registers = d) -> [32][136] bf16 staging in LDS -> coalesced 16-byte stores of rows of `out`
// (row stride ld_out elements).  Rows at or beyond `limit` are dropped.
__device__ __forceinline__ void store_rows_T(const f32x16_t (&acc)[4], float mul, bf16_t* stage, bf16_t* out,
                                             int64_t ld_out, int row0, int limit, int lane) {
  constexpr int OLD = 136;
  const int hh = lane >> 5, lrow = lane & 31;
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      bf16x4_t pk;
#pragma unroll
      for (int e = 0; e < 4; ++e) pk[e] = (bf16_t)(acc[dt][4 * r4 + e] * mul);
      *reinterpret_cast<bf16x4_t*>(stage + lrow * OLD + dt * 32 + 8 * r4 + 4 * hh) = pk;
    }
  __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int it = 0; it < 8; ++it) {
    const int idx = it * 64 + lane, row = idx >> 4, ch = idx & 15;
    if (row0 + row < limit)
      *reinterpret_cast<u32x4_t*>(out + (int64_t)(row0 + row) * ld_out + ch * 8) = *reinterpret_cast<const u32x4_t*>(stage + row * OLD + ch * 8);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_wave_barrier();
}

// =============================================================================== backward: dK, dV
// Workgroup: 8 wavefronts, one (batch, head, 256 keys); wavefront w owns keys 32w..32w+31 and keeps
// their K and V rows in registers as B operands.  Query rows stream through a 4-stage LDS ring in
// blocks of 64 (Q and dO tiles plus the rows' lse and D), from the diagonal to the end of the
// sequence, filled by direct global->LDS loads three blocks ahead.
//   S = Q K^T;  P = exp(S/sqrt(d) - lse);  dP = dO V^T;  dS = P (dP - D)
//   dV^T += dO^T P;   dK^T += Q^T dS  (scaled by 1/sqrt(d) at the end)
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
                    const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv, int B, int S, int nh, float scale) {
  constexpr int BKVW = 256, BQ = 64, NS = 4;
  constexpr int kStage = 2 * kTileBytes + 2 * BQ * 4;   // Q tile | dO tile | lse[64] | D[64]
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(size_t)(const lds_u8_t*)lds_raw;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int bh = blockIdx.x % (B * nh);
  const int kt = blockIdx.x / (B * nh);                 // early key tiles see the most queries: they go first
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const bf16_t* kbase = qbase + H;
  const bf16_t* vbase = qbase + 2 * H;
  const uint64_t qb64 = (uint64_t)qbase, do64 = (uint64_t)(dO + (int64_t)b * S * H + (int64_t)h * D);
  const uint64_t l64 = (uint64_t)(lse + ((int64_t)b * nh + h) * S), d64 = (uint64_t)(Dsum + ((int64_t)b * nh + h) * S);
  const unsigned ldb = (unsigned)(ld * 2), ldob = (unsigned)(H * 2);
  const int kv0 = kt * BKVW, kv0w = kv0 + wave * 32;
  const float c = scale * kLog2e;

  const int jb = kv0 / BQ, je = (S + BQ - 1) / BQ;      // query blocks jb .. je-1
  const int nblk = je - jb;
  auto issue = [&](int t) {
    const unsigned st = lds0 + (t & (NS - 1)) * kStage;
    const int row0 = (jb + t) * BQ;
    tile_dma(qb64, ldb, row0, S, st, lane, wave);
    tile_dma(do64, ldob, row0, S, st + kTileBytes, lane, wave);
    if (wave < 2) {                                     // wavefront 0: the block's lse; wavefront 1: its D
      int row = row0 + lane;
      row = row < S ? row : S - 1;
      lds_dma4(wave == 0 ? l64 : d64, (unsigned)row * 4u, st + 2 * kTileBytes + wave * (BQ * 4));
    }
  };
  for (int t = 0; t < NS - 1 && t < nblk; ++t) issue(t);

  bf16x8_t kf[8], vf[8];
  {
    int row = kv0w + (lane & 31);
    if (row >= S) row = S - 1;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      kf[ks] = *reinterpret_cast<const bf16x8_t*>(kbase + (int64_t)row * ld + 16 * ks + 8 * hh);
      vf[ks] = *reinterpret_cast<const bf16x8_t*>(vbase + (int64_t)row * ld + 16 * ks + 8 * hh);
    }
  }
  f32x16_t dk[4], dv[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }
  const int kvi = kv0w + (lane & 31);

  for (int t = 0; t < nblk; ++t) {
    const int ahead = nblk - 1 - t;
    if (wave < 2) { if (ahead >= 2) wait_vmcnt<10>(); else if (ahead == 1) wait_vmcnt<5>(); else wait_vmcnt<0>(); }
    else { if (ahead >= 2) wait_vmcnt<8>(); else if (ahead == 1) wait_vmcnt<4>(); else wait_vmcnt<0>(); }
    stage_barrier();
    if (t + NS - 1 < nblk) issue(t + NS - 1);
    const int qb0 = (jb + t) * BQ;
    if (qb0 + BQ - 1 < kv0w) continue;                   // no query of the block sees this wavefront's keys
    const unsigned char* stg = lds_raw + (t & (NS - 1)) * kStage;
    const bf16_t* sq = reinterpret_cast<const bf16_t*>(stg);
    const bf16_t* sdo = sq + 64 * D;
    const float* sl = reinterpret_cast<const float*>(stg + 2 * kTileBytes);
    const float* sd = sl + BQ;
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qrow0 = qb0 + qb * 32;
      if (qrow0 + 31 < kv0w) continue;                   // wavefront-uniform
      f32x16_t sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        sacc = mfma(frag_nat(sq, qb * 32, ks, lane), kf[ks], sacc);
        pacc = mfma(frag_nat(sdo, qb * 32, ks, lane), vf[ks], pacc);
      }
      const bool need_mask = (qrow0 < kv0w + 31) || (qrow0 + 31 >= S);
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int rbase = qb * 32 + 8 * r4 + 4 * hh;
        const f32x4_t l4 = *reinterpret_cast<const f32x4_t*>(sl + rbase);
        const f32x4_t d4 = *reinterpret_cast<const f32x4_t*>(sd + rbase);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * r4 + e;
          float p = fast_exp2(__builtin_fmaf(sacc[r], c, -l4[e] * kLog2e));
          if (need_mask) {
            const int qi = qb0 + rbase + e;
            p = (kvi > qi || qi >= S) ? 0.f : p;
          }
          sacc[r] = p;
          pacc[r] = p * (pacc[r] - d4[e]);
        }
      }
#pragma unroll
      for (int tt = 0; tt < 2; ++tt) {
        const bf16x8_t pb = pack8(sacc, tt), dsb = pack8(pacc, tt);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) {
          dv[dt] = mfma(frag_tr(sdo, qb * 32, tt, dt * 32, lane), pb, dv[dt]);
          dk[dt] = mfma(frag_tr(sq, qb * 32, tt, dt * 32, lane), dsb, dk[dt]);
        }
      }
    }
  }
  __syncthreads();          // the ring becomes the output staging area

  bf16_t* stage = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
  bf16_t* dkout = dqkv + (int64_t)b * S * ld + H + (int64_t)h * D;
  bf16_t* dvout = dkout + H;
  store_rows_T(dk, scale, stage, dkout, ld, kv0w, S, lane);
  store_rows_T(dv, 1.0f, stage, dvout, ld, kv0w, S, lane);
}

// =============================================================================== backward: dQ
// Same workgroup shape and K/V ring as the forward: 8 wavefronts, 256 query rows, wavefront w owns
// rows 32w..32w+31 and keeps their Q and dO rows in registers as B operands.
//   S^T = K Q^T;  P^T = exp(S^T/sqrt(d) - lse);  dP^T = V dO^T;  dS^T = P^T (dP^T - D);
//   dQ^T += K^T dS^T  (scaled by 1/sqrt(d) at the end)
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, const float* __restrict__ lse,
                   const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv, int B, int S, int nh, float scale) {
  constexpr int BQ = 256, WQ = 32, BKV = 64, NS = 4;
  constexpr int kStage = 2 * kTileBytes;   // K tile | V tile
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(size_t)(const lds_u8_t*)lds_raw;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nqt = (S + BQ - 1) / BQ;
  const int bh = blockIdx.x % (B * nh);
  const int qt = nqt - 1 - blockIdx.x / (B * nh);
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const uint64_t kbase = (uint64_t)(qbase + H), vbase = (uint64_t)(qbase + 2 * H);
  const bf16_t* dobase = dO + (int64_t)b * S * H + (int64_t)h * D;
  const unsigned ldb = (unsigned)(ld * 2);
  const int q0 = qt * BQ, q0w = q0 + wave * WQ;
  const float c = scale * kLog2e;

  const int kv_end = (q0 + BQ < S) ? q0 + BQ : S;
  const int nkv = (kv_end + BKV - 1) / BKV;
  auto issue = [&](int t) {
    const unsigned st = lds0 + (t & (NS - 1)) * kStage;
    tile_dma(kbase, ldb, t * BKV, S, st, lane, wave);
    tile_dma(vbase, ldb, t * BKV, S, st + kTileBytes, lane, wave);
  };
  for (int t = 0; t < NS - 1 && t < nkv; ++t) issue(t);

  bf16x8_t qf[8], dof[8];
  float l2, dsum;
  f32x16_t dq[4];
  {
    int row = q0w + (lane & 31);
    if (row >= S) row = S - 1;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      qf[ks] = *reinterpret_cast<const bf16x8_t*>(qbase + (int64_t)row * ld + 16 * ks + 8 * hh);
      dof[ks] = *reinterpret_cast<const bf16x8_t*>(dobase + (int64_t)row * H + 16 * ks + 8 * hh);
    }
    l2 = lse[((int64_t)b * nh + h) * S + row] * kLog2e;
    dsum = Dsum[((int64_t)b * nh + h) * S + row];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  }
  const int qidx = q0w + (lane & 31);

  for (int j = 0; j < nkv; ++j) {
    const int ahead = nkv - 1 - j;
    if (ahead >= 2) wait_vmcnt<8>(); else if (ahead == 1) wait_vmcnt<4>(); else wait_vmcnt<0>();
    stage_barrier();
    if (j + NS - 1 < nkv) issue(j + NS - 1);
    const int kv0 = j * BKV;
    if (kv0 > q0w + WQ - 1) continue;
    const bf16_t* sk = reinterpret_cast<const bf16_t*>(lds_raw + (j & (NS - 1)) * kStage);
    const bf16_t* sv = sk + 64 * D;
    const bool need_mask = kv0 + BKV - 1 > q0w;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16_t sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        sacc = mfma(frag_nat(sk, kb * 32, ks, lane), qf[ks], sacc);
        pacc = mfma(frag_nat(sv, kb * 32, ks, lane), dof[ks], pacc);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = fast_exp2(__builtin_fmaf(sacc[r], c, -l2));
        if (need_mask) {
          const int kv = kv0 + kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          p = kv > qidx ? 0.f : p;
        }
        pacc[r] = p * (pacc[r] - dsum);
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const bf16x8_t dsb = pack8(pacc, t);
#pragma unroll
        for (int dt = 0; dt < 4; ++dt) dq[dt] = mfma(frag_tr(sk, kb * 32, t, dt * 32, lane), dsb, dq[dt]);
      }
    }
  }
  __syncthreads();          // the ring becomes the output staging area

  bf16_t* stage = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
  bf16_t* dqout = dqkv + (int64_t)b * S * ld + (int64_t)h * D;
  store_rows_T(dq, scale, stage, dqout, ld, q0w, S, lane);
}

int launch_fwd(int B, int S, int nh, const void* qkv, void* o, float* lse, hipStream_t st) {
  constexpr int BQ = 256;
  constexpr size_t lds = 4 * 2 * kTileBytes;      // the ring; the output staging (8 x 32 x 136 bf16) fits inside
  static_assert(lds >= 8 * 32 * 136 * sizeof(bf16_t), "staging area");
  hipError_t e = hipFuncSetAttribute((const void*)attn_fwd_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return (int)e;
  const int nqt = (S + BQ - 1) / BQ;
  const float scale = 1.0f / sqrtf((float)D);
  hipLaunchKernelGGL(attn_fwd_kernel, dim3((unsigned)(nqt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (bf16_t*)o, lse, B, S, nh, scale);
  return (int)hipGetLastError();
}

}  // namespace

bool attn_mfma_supported(int dtype, int S, int nh, int d) {
  return dtype == DT_BF16 && d == D && S >= 1 && nh >= 1 && (int64_t)S * 3 * nh * D * 2 < ((int64_t)1 << 32);
}

int launch_attn_fwd_mfma(int B, int S, int nh, const void* qkv, void* o, float* lse, hipStream_t st) {
  return launch_fwd(B, S, nh, qkv, o, lse, st);
}

int launch_attn_bwd_mfma(int B, int S, int nh, const void* qkv, const void* dO, const float* lse, const float* Dv, void* dqkv, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)D);
  {
    constexpr size_t lds = 4 * (2 * kTileBytes + 2 * 64 * sizeof(float));
    static_assert(lds >= 8 * 32 * 136 * sizeof(bf16_t), "staging area");
    hipError_t e = hipFuncSetAttribute((const void*)attn_bwd_dkv_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    const int nkt = (S + 255) / 256;
    hipLaunchKernelGGL(attn_bwd_dkv_kernel, dim3((unsigned)(nkt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (const bf16_t*)dO, lse, Dv,
                       (bf16_t*)dqkv, B, S, nh, scale);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
  }
  {
    constexpr size_t lds = 4 * 2 * kTileBytes;
    hipError_t e = hipFuncSetAttribute((const void*)attn_bwd_dq_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return (int)e;
    const int nqt = (S + 255) / 256;
    hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3((unsigned)(nqt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (const bf16_t*)dO, lse, Dv,
                       (bf16_t*)dqkv, B, S, nh, scale);
    return (int)hipGetLastError();
  }
}

}  // namespace taw
