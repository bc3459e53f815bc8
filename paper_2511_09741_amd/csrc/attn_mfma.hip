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
#include <type_traits>
#include <utility>

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

typedef __attribute__((address_space(3))) unsigned char lds_u8_t;

// compile-time loop: f(std::integral_constant<int, 0>{}), ..., f(std::integral_constant<int, N - 1>{})
template <class F, int... I> __device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
  (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) { static_for_impl(f, std::make_integer_sequence<int, N>{}); }
#define TAW_CONST(name, c) constexpr int name = decltype(c)::value

// ---- the same two fragment reads with hand-made LDS byte addresses --------------------------------
// Both swizzled addresses are "per-lane constant XOR small immediate": one register per pattern
// (plus the stage offset, a multiple of 256 bytes, added per tile) instead of one per fragment.
//   natural:    (nat ^ (ks << 5)) + 256 * row0            nat = (l&31)*256 + chunk bits of ks = 0
//   transposed: (tr ^ ((dt << 6) | (rr << 5))) + 256 * (row0 + 16 t + 8 rr)
struct LaneAddr {
  unsigned nat, tr;
  __device__ __forceinline__ void init(int lane) {
    const int r = lane & 31, hh = lane >> 5;
    nat = r * 256 + (swz(r, hh) << 4);
    const int blk = lane >> 4, i = lane & 15, h = blk >> 1;
    const int rl = 4 * h + (i >> 2), d = 16 * (blk & 1) + 4 * (i & 3);
    tr = rl * 256 + (swz(rl, d >> 3) << 4) + (d & 7) * 2;
  }
};
// x ^ k.  OPAQUE: computed where it is written; as an opaque instruction the compiler can neither hoist the
// eight variants of an address out of the loop nor keep them all alive (that costs the registers
// that decide between two wavefronts per SIMD with or without spills in the dK/dV kernel)
template <int K, bool OPAQUE> __device__ __forceinline__ unsigned xor_here(unsigned x) {
  if (K == 0) return x;
  if (!OPAQUE) return x ^ (unsigned)K;
  unsigned r;
  asm volatile("v_xor_b32 %0, %1, %2" : "=v"(r) : "i"(K), "v"(x));
  return r;
}
// nat_t / tr_t: the lane constant plus the LDS byte address of the stage (a multiple of 256);
// OFF: byte offset of the tile inside the stage plus 256 * row0
template <int KS, int OFF, bool OPAQUE = false> __device__ __forceinline__ bf16x8_t frag_nat2(unsigned nat_t) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(xor_here<(KS << 5), OPAQUE>(nat_t) + OFF);
}
// both transposing reads of fragment (t, dt) at tile offsets OFF0 and OFF1 (two tiles of one stage share the address)
template <int T, int DT, int OFF0, int OFF1, bool OPAQUE = false>
__device__ __forceinline__ void frag_tr2x2(unsigned tr_t, bf16x8_t& f0, bf16x8_t& f1) {
  union { s16x4_t h2[2]; bf16x8_t v; } u0, u1;
#pragma unroll
  for (int rr = 0; rr < 2; ++rr) {
    const unsigned a = (rr == 0 ? xor_here<(DT << 6), OPAQUE>(tr_t) : xor_here<((DT << 6) | 32), OPAQUE>(tr_t)) + (16 * T + 8 * rr) * 256;
    u0.h2[rr] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4_t __attribute__((address_space(3)))*>(a + OFF0));
    if (OFF1 >= 0) u1.h2[rr] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4_t __attribute__((address_space(3)))*>(a + OFF1));
  }
  f0 = u0.v;
  if (OFF1 >= 0) f1 = u1.v;
}

__device__ __forceinline__ bf16x8_t pack8(const f32x16_t& x, int t) {
  bf16x8_t p;
#pragma unroll
  for (int j = 0; j < 8; ++j) p[j] = (bf16_t)x[8 * t + j];
  return p;
}

// ---- direct global -> LDS tile loads ----------------------------------------------------------------
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
// the same with the non-temporal hint: for data read exactly once (it is not worth a place in the caches that the
// re-read K / V / Q / dO tiles live in)
__device__ __forceinline__ void lds_dma16_nt(uint64_t base, unsigned off, unsigned lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1 nt" ::"v"(off), "s"(base), "s"(lds_addr));
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

// Which (batch, head) pair and which of its nt tiles a workgroup id takes; rank 0 is the tile with the most work.
// Ids are dealt round-robin to the 8 XCDs and each XCD starts its ids in order.  XCD x owns the pairs x, x + 8, ...
// and walks them in bands of `band` consecutive ranks: band 0 of its first pair, band 0 of its second, ..., then
// band 1 of each, and so on.  With 32 compute units per XCD, 32 / band pairs are in flight on an XCD at a time, each
// with `band` neighbouring tiles that stream the same operands (one fill of that L2 serves them), and 8 * 32 / band
// pairs on the chip, whose operands (17 MB per pair at S = 32768) then fit the 256 MiB memory-side cache together;
// all pairs side by side do not.  Long tiles still start before short ones (bands are walked in rank order), which
// is what keeps the last round of workgroups short.  Pairs beyond the last multiple of 8 are dealt out tile by tile.
// Measured: the forward gains 2 - 5 % from bands at S >= 16384 and loses 3 % at S = 8192 (few tiles per pair: the finer
// longest-first order of band = 1 matters more there); the two backward kernels lose 0.5 - 2 % at every size and keep
// band = 1, every pair of the XCD side by side, rank by rank.
__device__ __forceinline__ int pair_band(int nt) { return nt >= 128 ? 32 : nt >= 64 ? 16 : 1; }
template <bool BANDS = true>
__device__ __forceinline__ void pair_tile_of_block(int blk, int npairs, int nt, int& bh, int& rank) {
  const int p8 = npairs & ~7;
  if (blk < p8 * nt) {
    const int P = p8 >> 3, band = BANDS ? pair_band(nt) : 1;
    const int i = blk >> 3;
    const int full = (nt / band) * band;               // ranks covered by whole bands
    int pair, r;
    if (i < P * full) {
      const int bnd = i / (P * band), j = i - bnd * (P * band);
      pair = j / band;
      r = bnd * band + j % band;
    } else {
      const int last = nt - full, j = i - P * full;
      pair = j / last;
      r = full + j % last;
    }
    bh = (blk & 7) + 8 * pair;
    rank = r;
  } else {
    const int r = blk - p8 * nt, pr = npairs - p8;
    bh = p8 + r % pr;
    rank = r / pr;
  }
}

// max of three without the canonicalising self-maximum the compiler puts in front of fmaxf on MFMA results
__device__ __forceinline__ float max3(float a, float b, float c) {
  float d;
  asm("v_max3_f32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "v"(b), "v"(c));
  return d;
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
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  const lds_u8_t* L = (const lds_u8_t*)lds_raw;
  const unsigned lds0 = (unsigned)(size_t)L;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LaneAddr la;
  la.init(lane);
  const int nqt = (S + BQ - 1) / BQ;
  int bh, rank;
  pair_tile_of_block((int)blockIdx.x, B * nh, nqt, bh, rank);
  const int qt = nqt - 1 - rank;                       // longest rows first
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
  for (int t = 0; t < NS - 2 && t < nkv; ++t) issue(t);

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

  // The two wavefronts of a SIMD (w and w + 4) run the three phases of a tile in different orders, so
  // that one's softmax arithmetic meets the other's MFMAs instead of both doing the same thing after
  // every barrier: wavefronts 0..3 do S = K Q^T, softmax, O += V^T P within the tile's period; the
  // late ones 4..7 start a period with the O += V^T P of the previous tile (its P waits in registers,
  // its V stays in the ring one period longer, which is why tiles are issued two ahead, not three).
  const bool late = wave >= kWaves8 / 2;
  bf16x8_t pf[2][2];
  bool pend = false;
  unsigned pend_tr = 0;
  // O^T += V^T P^T: 16 MFMAs, fragment i = (kb, t, dt) = (i / 8, (i / 4) % 2, i % 4).  The fragment reads run kAhead MFMAs
  // ahead of their use, in registers of their own: an LDS read takes several MFMA issue slots to return, and a read placed
  // right in front of its MFMA leaves the matrix pipe idle for that long, sixteen times per tile.  The scheduling barriers
  // keep the compiler from moving the reads back next to their use.
  constexpr int kAhead = 4;
  auto pv = [&](unsigned tr_t) {
    bf16x8_t vfr[16];
    auto rd = [&](auto i_c) {
      TAW_CONST(i, i_c);
      bf16x8_t unused;
      frag_tr2x2<(i / 4) % 2, i % 4, kTileBytes + (i / 8) * 8192, -1>(tr_t, vfr[i], unused);
    };
    static_for<kAhead>(rd);
    __builtin_amdgcn_s_setprio(1);
    static_for<16>([&](auto i_c) {
      TAW_CONST(i, i_c);
      if constexpr (i + kAhead < 16) rd(std::integral_constant<int, i + kAhead>{});
      __builtin_amdgcn_sched_barrier(0);
      oacc[i % 4] = mfma(vfr[i], pf[i / 8][(i / 4) % 2], oacc[i % 4]);
      __builtin_amdgcn_sched_barrier(0);
    });
    __builtin_amdgcn_s_setprio(0);
  };

  // The register-resident operands loaded above have arrived: said here, once, so that the compiler
  // does not wait for them (and with them for every tile load in flight) at their first use inside the loop.
  wait_vmcnt<0>();
  for (int j = 0; j < nkv; ++j) {
    // tile j has landed (each wavefront waits for its own pieces, the barrier collects them); the
    // barrier also says every wavefront is done with tile j-2, whose stage tile j+2 goes into
    if (j + 1 < nkv) wait_vmcnt<4>(); else wait_vmcnt<0>();
    stage_barrier();
    if (j + NS - 2 < nkv) issue(j + NS - 2);
    if (pend) {                                        // late wavefronts: the previous tile's O += V^T P
      pv(pend_tr);
      pend = false;
    }
    const int kv0 = j * BKV;
    if (kv0 > q0w + WQ - 1) continue;                  // no key of the tile is visible to this wavefront
    const unsigned so = lds0 + (j & (NS - 1)) * kStage;
    const unsigned nat_t = la.nat + so, tr_t = la.tr + so;

    // S^T = K Q^T: 16 MFMAs in two independent accumulation chains (the two 32-key halves of the tile), issued alternately;
    // fragment reads kAhead MFMAs ahead, as in pv
    f32x16_t s[2];
    {
#pragma unroll
      for (int r = 0; r < 16; ++r) { s[0][r] = 0.f; s[1][r] = 0.f; }      // (folded into the first MFMA of each chain as the constant 0)
      bf16x8_t kfr[16];
      auto rd = [&](auto i_c) {
        TAW_CONST(i, i_c);
        kfr[i] = frag_nat2<i / 2, (i % 2) * 8192>(nat_t);
      };
      static_for<kAhead>(rd);
      __builtin_amdgcn_s_setprio(1);
      static_for<16>([&](auto i_c) {
        TAW_CONST(i, i_c);
        if constexpr (i + kAhead < 16) rd(std::integral_constant<int, i + kAhead>{});
        __builtin_amdgcn_sched_barrier(0);
        s[i % 2] = mfma(kfr[i], qf[i / 2], s[i % 2]);
        __builtin_amdgcn_sched_barrier(0);
      });
      __builtin_amdgcn_s_setprio(0);
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
    // v_max3_f32 by name: fmaxf on MFMA results makes the compiler quiet possible signalling NaNs first, one extra
    // instruction per score, and pair the maxima up with two-operand instructions (58 instructions for 32 scores instead of 16)
    float mx = max3(s[0][0], s[1][0], s[0][0]);
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = max3(mx, s[0][r], s[1][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64)) * c;      // (v_permlane32_swap instead of this LDS round trip measured 3 % slower)
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
    // probabilities, packed to bf16 in pairs; the row sum is taken from the packed pairs (one dot
    // product instruction per pair): the sum of exactly what the second product multiplies by
    float rs = 0.f;
    const bf16x2_t ones = {(bf16_t)1.0f, (bf16_t)1.0f};
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        u32x4_t w;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const float p0 = fast_exp2(__builtin_fmaf(s[kb][8 * t + 2 * j], c, -m));
          const float p1 = fast_exp2(__builtin_fmaf(s[kb][8 * t + 2 * j + 1], c, -m));
          const bf16x2_t pk = {(bf16_t)p0, (bf16_t)p1};
          rs = __builtin_amdgcn_fdot2_f32_bf16(pk, ones, rs, false);
          w[j] = __builtin_bit_cast(unsigned, pk);
        }
        pf[kb][t] = __builtin_bit_cast(bf16x8_t, w);
      }
    l += rs;
    if (late) {
      pend = true;
      pend_tr = tr_t;
    } else {
      pv(tr_t);
    }
  }
  if (pend) pv(pend_tr);
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
// lrow: which of the 32 rows this lane's accumulators belong to (lane & 31 unless the producer permuted them)
__device__ __forceinline__ void store_rows_T(const f32x16_t (&acc)[4], float mul, bf16_t* stage, bf16_t* out,
                                             int64_t ld_out, int row0, int limit, int lane, int lrow) {
  constexpr int OLD = 136;
  const int hh = lane >> 5;
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

__device__ __forceinline__ void store_rows_T(const f32x16_t (&acc)[4], float mul, bf16_t* stage, bf16_t* out,
                                             int64_t ld_out, int row0, int limit, int lane) {
  store_rows_T(acc, mul, stage, out, ld_out, row0, limit, lane, lane & 31);
}

// Inverse rotary rotation of a wavefront's transposed accumulators X^T[128 d][32 rows] in place, for
// the gradients of rotated q and k (the rotation's transpose is the rotation by the opposite
// angle).  Lane = sequence position, registers (4g, 4g+1) and (4g+2, 4g+3) of a d block are the
// rotated pairs; table [S][64][2] fp32 (cos, sin).  In registers and in fp32: no extra pass over
// the gradients and one rounding instead of two.
__device__ __forceinline__ void rope_inverse_T(f32x16_t (&acc)[4], const float* __restrict__ table, int pos, int limit, int lane) {
  const int hh = lane >> 5;
  if (pos >= limit) pos = limit - 1;                   // rows beyond the sequence are dropped by the store
  const float* tb = table + (int64_t)pos * D;          // 64 pairs x 2 floats
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      const f32x4_t cs = *reinterpret_cast<const f32x4_t*>(tb + 2 * (dt * 16 + 4 * g + 2 * hh));
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float a = acc[dt][4 * g + 2 * e], bb = acc[dt][4 * g + 2 * e + 1], c = cs[2 * e], sn = cs[2 * e + 1];
        acc[dt][4 * g + 2 * e] = a * c + bb * sn;
        acc[dt][4 * g + 2 * e + 1] = bb * c - a * sn;
      }
    }
}

// =============================================================================== backward: row statistics
// prep [2][B*nh][Sp] fp32, Sp = S rounded up to 64:  prep[0] = lse * log2(e) (what the exp2-domain
// recomputation subtracts), +inf for rows S..Sp-1 so that their probabilities come out as exactly 0;
// prep[1] = D[t] = dO[t] . o[t], 0 for the padding rows.  16 lanes share one (row, head): a wavefront
// reads 1 KiB of contiguous o / dO.
__global__ void __launch_bounds__(256) attn_bwd_prep_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dO,
                                                            const float* __restrict__ lse, float* __restrict__ prep,
                                                            int B, int S, int Sp, int nh) {
  const int64_t gid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int part = (int)(gid & 15);
  const int64_t pair = gid >> 4;                       // (b, s in [0, Sp), h), h fastest
  const int64_t npairs = (int64_t)B * Sp * nh;
  if (pair >= npairs) return;                          // whole 16-lane groups leave together
  const int h = (int)(pair % nh);
  const int64_t bs = pair / nh;
  const int sidx = (int)(bs % Sp), b = (int)(bs / Sp);
  float dot = 0.f, l2 = INFINITY;
  if (sidx < S) {
    const int64_t off = ((int64_t)b * S + sidx) * ((int64_t)nh * D) + (int64_t)h * D + part * 8;
    const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(o + off);
    const bf16x8_t g = *reinterpret_cast<const bf16x8_t*>(dO + off);
#pragma unroll
    for (int j = 0; j < 8; ++j) dot += (float)a[j] * (float)g[j];
    l2 = lse[((int64_t)b * nh + h) * S + sidx] * kLog2e;
  }
#pragma unroll
  for (int m = 8; m > 0; m >>= 1) dot += __shfl_xor(dot, m, 64);
  if (part == 0) {
    const int64_t at = ((int64_t)b * nh + h) * Sp + sidx;
    prep[at] = l2;
    prep[(int64_t)B * nh * Sp + at] = dot;
  }
}

// =============================================================================== backward: dK, dV
// Workgroup: 8 wavefronts, one (batch, head, 256 keys); wavefront w owns keys 32w..32w+31.  Their V rows stay in
// registers as B operands; their K rows are read from a copy of the key tile in LDS (64 KiB), which leaves the
// registers for both score accumulators at once and for reading fragments ahead of the MFMAs.  Query rows stream
// through a 2-stage LDS ring in blocks of 64 (Q and dO tiles plus the rows' lse and D), from the diagonal to the end
// of the sequence, filled by direct global->LDS loads one block ahead (a block takes several microseconds to process,
// more than a load takes to land).
//   S = Q K^T and dP = dO V^T as two alternating accumulation chains;  P = exp(S/sqrt(d) - lse);  dS = P (dP - D)
//   dV^T += dO^T P;   dK^T += Q^T dS  (scaled by 1/sqrt(d) at the end)
constexpr int kKvOffRing = 65536;                                        // key tile [256][128] bf16 in front of the ring
constexpr int kKvStage = 2 * kTileBytes + 2 * 64 * 4;                    // Q tile | dO tile | lse[64] | D[64]
constexpr size_t kKvLds = kKvOffRing + 2 * kKvStage;
//
// STORE_DS: every dS block this kernel forms is also written to memory (bf16, exactly what the dK product multiplies by) for
// a dQ kernel that then needs one matrix product instead of three (attn_bwd_dq_stored_kernel).  Layout of `ds`, per (batch,
// head): for block ib of 256 query rows, and in it for each 32-row group s (the rows of one wavefront of the dQ kernel),
// the units of the key groups g = 0 .. 8 (ib + 1) - 1 one after the other (ds_unit_offset).  A unit is what one wavefront
// here holds after one block: dS[32 rows][32 keys], 2 KiB, as 128 slots of 16 bytes.  Lane (key kk, lane half hh) holds the
// two pieces tt = 0, 1 = accumulator registers 8 tt .. 8 tt + 7 = query rows 16 tt + 4 hh + {0..3, 8..11} of the group
// (ds_row_of_slot gives the row for the position 16 hh + 8 tt + e the dQ kernel sees it at).  Piece tt goes to slot
// ds_slot(kk, hh, tt): the 64 lanes of one store instruction fill one contiguous KiB, and the dQ kernel, which copies
// units into LDS as they are, reads them back by transposing reads without bank conflicts (the 16 slots one half-wavefront
// reads - 4 keys x 2 lane halves x 2 pieces - differ in their low 4 bits).  Units whose 32 queries all lie in front of
// their 32 keys (dS = 0 there) are never written; the dQ kernel copies the ones inside its diagonal block into LDS along
// with the rest of a tile but never feeds them to an MFMA.  Likewise the units of row groups at or beyond S rounded up to
// 64: what is read there only reaches rows of dQ that are not stored.  The caller clears nothing.
// The stores cost this kernel 13 % (16.3 instead of 14.4 ms at S = 32768, 32 heads) wherever in the loop they are issued,
// whether the next iteration's wait for loads also waits for them or not, and whether they go to 35 GB of memory or
// over and over to the same few KiB: it is the issue of the store instructions that costs, not the traffic.
// (ds_block_offset, ds_unit_offset, ds_slot, ds_row_of_slot: taw_internal.h, where host code can check them)

template <bool STORE_DS>
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, const float* __restrict__ lse2,
                    const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv, int B, int S, int Sp, int nh, float scale,
                    const float* __restrict__ rope, unsigned char* __restrict__ ds, int64_t ds_pair_bytes) {
  constexpr int BKVW = 256, BQ = 64, NS = 2;
  constexpr int kStage = kKvStage;
  constexpr int kA = 1;                                // fragment reads run this many MFMA steps ahead of their use (deeper costs registers this kernel does not have)
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  const lds_u8_t* L = (const lds_u8_t*)lds_raw;
  const unsigned lds0 = (unsigned)(size_t)L;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LaneAddr la;
  la.init(lane);
  int bh, kt;                                          // key tile 0 meets every query block: longest first
  pair_tile_of_block<false>((int)blockIdx.x, B * nh, (S + BKVW - 1) / BKVW, bh, kt);
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const bf16_t* kbase = qbase + H;
  const bf16_t* vbase = qbase + 2 * H;
  const uint64_t qb64 = (uint64_t)qbase, k64 = (uint64_t)kbase, do64 = (uint64_t)(dO + (int64_t)b * S * H + (int64_t)h * D);
  const uint64_t l64 = (uint64_t)(lse2 + ((int64_t)b * nh + h) * Sp), d64 = (uint64_t)(Dsum + ((int64_t)b * nh + h) * Sp);
  const unsigned ldb = (unsigned)(ld * 2), ldob = (unsigned)(H * 2);
  const int kv0 = kt * BKVW, kv0w = kv0 + wave * 32;
  const float c = scale * kLog2e;

  const int jb = kv0 / BQ, je = (S + BQ - 1) / BQ;
  const int nblk = je - jb;
  // key tile -> LDS (8 pieces of 4 rows per wavefront)
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int j = wave + 8 * i;
    const int r = 4 * j + (lane >> 4);
    const int cc = swz(r, lane & 15);
    int rg = kv0 + r;
    rg = rg < S ? rg : S - 1;
    lds_dma16(k64, (unsigned)rg * ldb + cc * 16, lds0 + j * 1024);
  }
  auto issue = [&](int t) {
    const unsigned st = lds0 + kKvOffRing + (t & (NS - 1)) * kStage;
    const int row0 = (jb + t) * BQ;
    tile_dma(qb64, ldb, row0, S, st, lane, wave);
    tile_dma(do64, ldob, row0, S, st + kTileBytes, lane, wave);
    if (wave < 2)
      lds_dma4(wave == 0 ? l64 : d64, (unsigned)(row0 + lane) * 4u, st + 2 * kTileBytes + wave * (BQ * 4));
  };
  issue(0);

  bf16x8_t vf[8];
  {
    int row = kv0w + (lane & 31);
    if (row >= S) row = S - 1;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) vf[ks] = *reinterpret_cast<const bf16x8_t*>(vbase + (int64_t)row * ld + 16 * ks + 8 * hh);
  }
  f32x16_t dk[4], dv[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }
  const int kvi = kv0w + (lane & 31);
  const unsigned knat_t = la.nat + lds0 + wave * 8192;
  unsigned char* const ds_pair = STORE_DS ? ds + (int64_t)bh * ds_pair_bytes : nullptr;
  for (int t = 0; t < nblk; ++t) {
    wait_vmcnt<0>();                                     // block t (issued one iteration ago) has landed
    stage_barrier();
    if (t + 1 < nblk) issue(t + 1);                      // into the stage every wavefront finished reading before this barrier
    const int qb0 = (jb + t) * BQ;
    if (qb0 + BQ - 1 < kv0w) continue;
    const unsigned so = lds0 + kKvOffRing + (t & (NS - 1)) * kStage;
    const unsigned nat_t = la.nat + so, tr_t = la.tr + so;
    const unsigned sl = so + 2 * kTileBytes + 16 * hh;
    static_for<2>([&](auto qb_c) {
      TAW_CONST(qb, qb_c);
      const int qrow0 = qb0 + qb * 32;
      if (qrow0 + 31 < kv0w) return;
      typedef const __attribute__((address_space(3))) f32x4_t* lds_f4_t;
      bf16x8_t pb[2], dsb[2];
      {
        f32x16_t sacc, pacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
        // step i: S MFMA needs Q(i) and K(i) from LDS, dP MFMA needs dO(i)
        bf16x8_t fq[8], fk[8], fo[8];
        auto rd = [&](auto i_c) {
          TAW_CONST(i, i_c);
          // Q and dO fragments sit at the same place of their tiles: one address for both
          const unsigned a = xor_here<(i << 5), true>(nat_t);
          fq[i] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(a + qb * 8192);
          fk[i] = frag_nat2<i, 0, true>(knat_t);
          fo[i] = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8_t*>(a + kTileBytes + qb * 8192);
        };
        static_for<kA>(rd);
        __builtin_amdgcn_s_setprio(1);
        static_for<8>([&](auto i_c) {
          TAW_CONST(i, i_c);
          if constexpr (i + kA < 8) rd(std::integral_constant<int, i + kA>{});
          __builtin_amdgcn_sched_barrier(0);
          sacc = mfma(fq[i], fk[i], sacc);
          pacc = mfma(fo[i], vf[i], pacc);
          __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_s_setprio(0);
        if (qrow0 < kv0w + 31) {
          asm volatile("" ::: "memory");
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int qi = qrow0 + 8 * (r >> 2) + 4 * hh + (r & 3);
            sacc[r] = kvi > qi ? -INFINITY : sacc[r];
          }
        }
#pragma unroll
        for (int r4 = 0; r4 < 4; ++r4) {
          const f32x4_t l4 = *reinterpret_cast<lds_f4_t>(sl + (qb * 32 + 8 * r4) * 4);
          const f32x4_t d4 = *reinterpret_cast<lds_f4_t>(sl + (BQ + qb * 32 + 8 * r4) * 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * r4 + e;
            const float pr = fast_exp2(__builtin_fmaf(sacc[r], c, -l4[e]));
            sacc[r] = pr;
            pacc[r] = pr * (pacc[r] - d4[e]);
          }
        }
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) { pb[tt] = pack8(sacc, tt); dsb[tt] = pack8(pacc, tt); }
        if constexpr (STORE_DS) {
          unsigned char* unit = ds_pair + ds_unit_offset(qrow0 >> 8, (qrow0 >> 5) & 7, kv0w >> 5);      // wavefront-uniform
          int ln = lane;
          asm volatile("" : "+v"(ln));                     // the slot numbers are made here, from the lane id, not kept in registers through the loop
          // non-temporal: written once, read once by the next kernel, and 35 GB of it at S = 32768: nothing to keep in a cache
          __builtin_nontemporal_store(dsb[0], reinterpret_cast<bf16x8_t*>(unit + ds_slot(ln & 31, ln >> 5, 0) * 16u));
          __builtin_nontemporal_store(dsb[1], reinterpret_cast<bf16x8_t*>(unit + ds_slot(ln & 31, ln >> 5, 1) * 16u));
        }
      }
      {
        bf16x8_t fq[8], fdo[8];
        auto rd = [&](auto i_c) {
          TAW_CONST(i, i_c);
          frag_tr2x2<i % 2, i / 2, qb * 8192, kTileBytes + qb * 8192, true>(tr_t, fq[i], fdo[i]);
        };
        static_for<kA>(rd);
        __builtin_amdgcn_s_setprio(1);
        static_for<8>([&](auto i_c) {
          TAW_CONST(i, i_c);
          if constexpr (i + kA < 8) rd(std::integral_constant<int, i + kA>{});
          __builtin_amdgcn_sched_barrier(0);
          dv[i / 2] = mfma(fdo[i], pb[i % 2], dv[i / 2]);
          dk[i / 2] = mfma(fq[i], dsb[i % 2], dk[i / 2]);
          __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_s_setprio(0);
      }
    });
  }
  __syncthreads();

  bf16_t* stage = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
  bf16_t* dkout = dqkv + (int64_t)b * S * ld + H + (int64_t)h * D;
  bf16_t* dvout = dkout + H;
  if (rope) {
    int ln = lane;
    asm volatile("" : "+v"(ln));
    rope_inverse_T(dk, rope, kv0w + (ln & 31), S, ln);
  }
  store_rows_T(dk, scale, stage, dkout, ld, kv0w, S, lane);
  store_rows_T(dv, 1.0f, stage, dvout, ld, kv0w, S, lane);
}

// =============================================================================== backward: dQ
// Same workgroup shape and K/V ring as the forward: 8 wavefronts, 256 query rows, wavefront w owns
// rows 32w..32w+31 and keeps their Q and dO rows in registers as B operands.
//   S^T = K Q^T;  P^T = exp(S^T/sqrt(d) - lse);  dP^T = V dO^T;  dS^T = P^T (dP^T - D);
//   dQ^T += K^T dS^T  (scaled by 1/sqrt(d) at the end)
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, const float* __restrict__ lse2,
                   const float* __restrict__ Dsum, bf16_t* __restrict__ dqkv, int B, int S, int Sp, int nh, float scale,
                   const float* __restrict__ rope) {
  constexpr int BQ = 256, WQ = 32, BKV = 64, NS = 4;
  constexpr int kStage = 2 * kTileBytes;   // K tile | V tile
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  const lds_u8_t* L = (const lds_u8_t*)lds_raw;
  const unsigned lds0 = (unsigned)(size_t)L;

  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LaneAddr la;
  la.init(lane);
  const int nqt = (S + BQ - 1) / BQ;
  int bh, rank;
  pair_tile_of_block<false>((int)blockIdx.x, B * nh, nqt, bh, rank);
  const int qt = nqt - 1 - rank;
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
    l2 = lse2[((int64_t)b * nh + h) * Sp + row];
    dsum = Dsum[((int64_t)b * nh + h) * Sp + row];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  }
  const int qidx = q0w + (lane & 31);

  // The register-resident operands loaded above have arrived: said here, once, so that the compiler
  // does not wait for them (and with them for every tile load in flight) at their first use inside the loop.
  wait_vmcnt<0>();
  for (int j = 0; j < nkv; ++j) {
    const int ahead = nkv - 1 - j;
    if (ahead >= 2) wait_vmcnt<8>(); else if (ahead == 1) wait_vmcnt<4>(); else wait_vmcnt<0>();
    stage_barrier();
    if (j + NS - 1 < nkv) issue(j + NS - 1);
    const int kv0 = j * BKV;
    if (kv0 > q0w + WQ - 1) continue;
    const unsigned so = lds0 + (j & (NS - 1)) * kStage;
    const unsigned nat_t = la.nat + so, tr_t = la.tr + so;
    const bool need_mask = kv0 + BKV - 1 > q0w;
    static_for<2>([&](auto kb_c) {
      TAW_CONST(kb, kb_c);
      f32x16_t sacc, pacc;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
      {
        // 16 MFMAs, the S^T and dP^T chains alternating; fragment i = (K or V, ks) = (i % 2, i / 2), read kAheadDq MFMAs ahead
        // of its use into registers of its own (a read placed right in front of its MFMA idles the matrix pipe for the
        // read's latency); the scheduling barriers keep the compiler from moving the reads back
        constexpr int kAheadDq = 4;
        bf16x8_t fr[16];
        auto rd = [&](auto i_c) {
          TAW_CONST(i, i_c);
          fr[i] = frag_nat2<i / 2, (i % 2) * kTileBytes + kb * 8192>(nat_t);
        };
        static_for<kAheadDq>(rd);
        __builtin_amdgcn_s_setprio(1);
        static_for<16>([&](auto i_c) {
          TAW_CONST(i, i_c);
          if constexpr (i + kAheadDq < 16) rd(std::integral_constant<int, i + kAheadDq>{});
          __builtin_amdgcn_sched_barrier(0);
          if constexpr (i % 2 == 0) sacc = mfma(fr[i], qf[i / 2], sacc);
          else pacc = mfma(fr[i], dof[i / 2], pacc);
          __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_s_setprio(0);
      }
      if (need_mask) {                                   // wavefront-uniform
        asm volatile("" ::: "memory");                   // keeps this a branch: most tiles skip the compares
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int kv = kv0 + kb * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          sacc[r] = kv > qidx ? -INFINITY : sacc[r];
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(__builtin_fmaf(sacc[r], c, -l2));
        pacc[r] = p * (pacc[r] - dsum);
      }
      {
        // dQ^T += K^T dS^T: 8 MFMAs, fragment i = (t, dt) = (i / 4, i % 4), read ahead in the same way
        constexpr int kAheadDq2 = 3;
        const bf16x8_t dsb[2] = {pack8(pacc, 0), pack8(pacc, 1)};
        bf16x8_t fk[8];
        auto rd = [&](auto i_c) {
          TAW_CONST(i, i_c);
          bf16x8_t unused;
          frag_tr2x2<i / 4, i % 4, kb * 8192, -1>(tr_t, fk[i], unused);
        };
        static_for<kAheadDq2>(rd);
        __builtin_amdgcn_s_setprio(1);
        static_for<8>([&](auto i_c) {
          TAW_CONST(i, i_c);
          if constexpr (i + kAheadDq2 < 8) rd(std::integral_constant<int, i + kAheadDq2>{});
          __builtin_amdgcn_sched_barrier(0);
          dq[i % 4] = mfma(fk[i], dsb[i / 4], dq[i % 4]);
          __builtin_amdgcn_sched_barrier(0);
        });
        __builtin_amdgcn_s_setprio(0);
      }
    });
  }
  __syncthreads();          // the ring becomes the output staging area

  bf16_t* stage = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
  bf16_t* dqout = dqkv + (int64_t)b * S * ld + (int64_t)h * D;
  if (rope) {
    int ln = lane;
    asm volatile("" : "+v"(ln));                       // table addresses are made here, not kept in registers through the loop
    rope_inverse_T(dq, rope, q0w + (ln & 31), S, ln);
  }
  store_rows_T(dq, scale, stage, dqout, ld, q0w, S, lane);
}

// =============================================================================== backward: dQ from stored dS
// dQ^T[d][q] += K^T[d][kv] dS^T[kv][q] with dS read back from what attn_bwd_dkv_kernel<true> wrote: one product per (query
// block, key block) pair instead of three, paid for with S^2 bytes per (batch, head) written once and read once.  Same
// workgroup shape as the kernel above (256 query rows, wavefront w owns the 32-row group w), keys in tiles of 64 through a
// 3-stage ring filled by direct global->LDS loads two tiles ahead: the K tile [64][128], shared, and per wavefront the two
// dS units (32 keys each) of its own row group, 4 KiB copied as they lie in memory (consecutive tiles are consecutive
// there: eight sequential streams per workgroup).  Both operands are transposing reads: K^T as in the kernel above, dS^T
// from the wavefront's units at the slots ds_slot() gave them.  The 32 rows of a group come in the order the dK/dV kernel's
// accumulators had them (ds_row_of_slot); only the epilogue needs to know.  With 16 MFMAs per wavefront and 48 KiB per
// tile the kernel is bound by the rate the dS matrix streams in from memory.
constexpr int kDqsStage = kTileBytes + 8 * 4096;       // K tile | 8 wavefronts x (2 units of 2 KiB)
constexpr int kDqsStages = 3;
constexpr size_t kDqsLds = (size_t)kDqsStages * kDqsStage;       // 144 KiB
static_assert(kDqsLds <= 160 * 1024, "LDS budget");
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_dq_stored_kernel(const bf16_t* __restrict__ qkv, const unsigned char* __restrict__ ds, int64_t ds_pair_bytes,
                          bf16_t* __restrict__ dqkv, int B, int S, int nh, float scale, const float* __restrict__ rope) {
  constexpr int BQ = 256, WQ = 32, BKV = 64, NS = kDqsStages;
  constexpr int kStage = kDqsStage;
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  const lds_u8_t* L = (const lds_u8_t*)lds_raw;
  const unsigned lds0 = (unsigned)(size_t)L;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LaneAddr la;
  la.init(lane);
  const int nqt = (S + BQ - 1) / BQ;
  int bh, rank;
  pair_tile_of_block<false>((int)blockIdx.x, B * nh, nqt, bh, rank);
  const int qt = nqt - 1 - rank;
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const uint64_t kbase = (uint64_t)(qbase + H);
  // this wavefront's units of block qt, key group 0 first: 2 KiB per key group, 8 (qt + 1) of them
  const uint64_t dsbase = (uint64_t)(ds + (int64_t)bh * ds_pair_bytes + ds_unit_offset(qt, wave, 0));
  const unsigned ldb = (unsigned)(ld * 2);
  const int q0 = qt * BQ, q0w = q0 + wave * WQ;

  const int kv_end = (q0 + BQ < S) ? q0 + BQ : S;
  const int nkv = (kv_end + BKV - 1) / BKV;               // key groups 0 .. 2 nkv - 1 <= 8 (qt + 1) - 1: every unit read exists
  auto issue = [&](int t, int stage) {
    const unsigned st = lds0 + stage * kStage;
    tile_dma(kbase, ldb, t * BKV, S, st, lane, wave);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      lds_dma16_nt(dsbase, (unsigned)(t * 4096 + i * 1024 + lane * 16), st + kTileBytes + wave * 4096 + i * 1024);      // (6.0 instead of 6.8 ms at S = 32768)
  };
  for (int t = 0; t < NS - 1 && t < nkv; ++t) issue(t, t);

  f32x16_t dq[4];
#pragma unroll
  for (int dt = 0; dt < 4; ++dt)
#pragma unroll
    for (int r = 0; r < 16; ++r) dq[dt][r] = 0.f;
  // Transposing read of fragment T (keys 16 T + 8 rr + 4 h + (i >> 2), rr = 0, 1) of a unit: lane (blk = lane >> 4,
  // i = lane & 15) reads 8 bytes = 4 consecutive positions 16 (blk & 1) + 4 (i & 3) .. of its key, which lie in piece
  // tt = (i >> 1) & 1 of lane half blk & 1, at bytes 8 (i & 1) of the slot; T and rr add 512 T + 256 rr (they move the
  // key by whole groups of four: bits 4, 5 of the slot number, clear of the XOR).
  unsigned trd;
  {
    const int blk = lane >> 4, i = lane & 15;
    trd = ds_slot(4 * (blk >> 1) + (i >> 2), blk & 1, (i >> 1) & 1) * 16u + 8u * (i & 1) + (unsigned)kTileBytes + (unsigned)wave * 4096u;
  }

  int stage = 0, stage_in = NS - 1;                     // stage of tile j; stage the next issue goes into
  for (int j = 0; j < nkv; ++j) {
    // 6 loads per tile and wavefront; tiles j and j + 1 are in flight here (issued two ahead)
    if (j + 1 < nkv) wait_vmcnt<6>(); else wait_vmcnt<0>();
    stage_barrier();                                    // the K tile j is visible; everybody is done with tile j - 1, whose stage tile j + 2 takes
    if (j + NS - 1 < nkv) issue(j + NS - 1, stage_in);
    const unsigned so = lds0 + stage * kStage;
    stage = stage + 1 == NS ? 0 : stage + 1;
    stage_in = stage_in + 1 == NS ? 0 : stage_in + 1;
    const int kv0 = j * BKV;
    if (kv0 > q0w + WQ - 1) continue;                   // every key of the tile lies behind this wavefront's rows: dS = 0, never written
    const unsigned tr_t = la.tr + so, trd_t = trd + so;
    static_for<2>([&](auto kb_c) {
      TAW_CONST(kb, kb_c);
      if (kv0 + kb * 32 > q0w + WQ - 1) return;         // wavefront-uniform; same for this half of the tile
      constexpr int kAheadK = 3;
      typedef s16x4_t __attribute__((address_space(3)))* lds_tr_t;
      bf16x8_t fk[8];
      union { s16x4_t h2[2]; bf16x8_t v; } dsb[2];
#pragma unroll
      for (int T = 0; T < 2; ++T)
#pragma unroll
        for (int rr = 0; rr < 2; ++rr)
          dsb[T].h2[rr] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_tr_t>(trd_t + kb * 2048 + 512 * T + 256 * rr));
      auto rd = [&](auto i_c) {
        TAW_CONST(i, i_c);
        bf16x8_t un2;
        frag_tr2x2<i / 4, i % 4, kb * 8192, -1>(tr_t, fk[i], un2);
      };
      static_for<kAheadK>(rd);
      __builtin_amdgcn_s_setprio(1);
      static_for<8>([&](auto i_c) {
        TAW_CONST(i, i_c);
        if constexpr (i + kAheadK < 8) rd(std::integral_constant<int, i + kAheadK>{});
        __builtin_amdgcn_sched_barrier(0);
        dq[i % 4] = mfma(fk[i], dsb[i / 4].v, dq[i % 4]);
        __builtin_amdgcn_sched_barrier(0);
      });
      __builtin_amdgcn_s_setprio(0);
    });
  }
  __syncthreads();          // the ring becomes the output staging area

  bf16_t* stage_out = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
  bf16_t* dqout = dqkv + (int64_t)b * S * ld + (int64_t)h * D;
  const int lrow = ds_row_of_slot(lane & 31);           // the query row (of the wavefront's 32) this lane's column of dQ^T is
  if (rope) rope_inverse_T(dq, rope, q0w + lrow, S, lane);
  store_rows_T(dq, scale, stage_out, dqout, ld, q0w, S, lane, lrow);
}

// =============================================================================== backward: dK, dV and dQ in one kernel
// Five matrix products per (query block, key block) pair, like the pair of kernels with stored dS above, in one kernel: S and dP are formed
// once, by the key-stationary side, and dQ is produced from the same dS.  The obstacle is the register layout: the
// accumulators of S and dP give a lane one KEY column, and the matrix cores contract over registers, never over lanes, so
// dQ[q][d] = sum_kv dS[q][kv] K[kv][d] cannot be fed from them.  Here dS crosses the workgroup through LDS:
//   phase 1 (every wavefront, its own 32 keys, one block of 32 query rows): S, P, dP, dS as in the dK/dV kernel above;
//           dV^T += dO^T P, dK^T += Q^T dS; dS (bf16) is written to an exchange tile Ex^T[256 keys][32 rows];
//   phase 2 (one block later, after the workgroup barrier that publishes Ex^T): dQ[32 rows][128] = dS[32][256] K[256][128],
//           split by OUTPUT: four wavefronts take one 32-column tile each and contract over all 256 keys (operands: dS from
//           Ex^T and K from a copy of the key tile in LDS, both by transposing reads); the two wavefronts of a SIMD take
//           turns, so every SIMD sees 80 MFMAs per block.
// Where the dQ tile goes decides the kernel's speed, and on this part neither way beats the pairs of kernels above, which
// is why one of those is the default (S = 32768, 32 heads: 23.7 ms with stored dS, 25.8 ms recomputing; this kernel
// 24.1 ms when it drops the dQ tiles, 27.6 ms with atomics, 30.9 ms with slots):
//   kDqAtomic  fp32 atomic adds into one dQ buffer.  The atomic units retire 0.34 T adds/s, and a 256-key workgroup
//              issues S^2/4 adds per head: 25.4 ms for the adds alone at that size.
//   kDqSlots   a deterministic two-level split over key blocks without atomics: the key blocks of a (batch, head) are dealt
//              to Ns WORKERS (one workgroup each, processing its key blocks one after the other); worker s owns a private
//              fp32 copy ("slot") of dQ and adds each tile into it with plain loads and stores (nobody else touches that
//              slot, and one workgroup's own accesses are ordered); a last pass sums the slots, scales, rotates back and
//              rounds to bf16.  A worker's first key block stores instead of adding, and slot s is never read above the
//              first row it wrote, so nothing has to be cleared.  Every tile pair moves 32 KB through HBM this way
//              (69 GB at that size), which costs more than recomputing the scores does.
constexpr int kDqSlots = 0, kDqAtomic = 1;
constexpr int kFBQ = 32;                               // query rows per block
constexpr int kFStage = 2 * 8192 + 256;                // Q tile [32][128] | dO tile | lse[32] | D[32]
constexpr int kFStages = 3;
constexpr int kFOffK = 0;                              // key tile [256][128] bf16
constexpr int kFOffEx = 65536;                         // two exchange tiles [256][32] bf16
constexpr int kFOffRing = kFOffEx + 2 * 16384;
constexpr size_t kFusedLds = kFOffRing + kFStages * kFStage;     // 148224 bytes
static_assert(kFusedLds <= 160 * 1024, "LDS budget");
static_assert(kFusedLds >= 8 * 32 * 136 * sizeof(bf16_t), "output staging area");

// one-KiB piece `wave` (rows 4 wave .. 4 wave + 3) of a [32][128] tile, as tile_dma does for [64][128]
__device__ __forceinline__ void tile32_dma(uint64_t base, unsigned ld_bytes, int row0, int limit, unsigned lds_tile, int lane, int wave) {
  const int r = 4 * wave + (lane >> 4);
  const int c = swz(r, lane & 15);
  int rg = row0 + r;
  rg = rg < limit ? rg : limit - 1;
  lds_dma16(base, (unsigned)rg * ld_bytes + c * 16, lds_tile + wave * 1024);
}

// Key blocks of one (batch, head) dealt to Ns workers in snake order: round r gives worker s the block r Ns + s (r even)
// or r Ns + Ns - 1 - s (r odd), so every worker gets the same number of (query block, key block) pairs when the
// number of rounds is even.  Worker s starts at block s.
__device__ __forceinline__ int worker_block(int r, int s, int Ns) { return r * Ns + ((r & 1) ? Ns - 1 - s : s); }

template <int DQ>
__global__ void __launch_bounds__(kThreads8, 1)
attn_bwd_fused_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dO, const float* __restrict__ prep,
                      bf16_t* __restrict__ dqkv, float* __restrict__ dq_slots, int B, int S, int Sp, int nh, float scale,
                      const float* __restrict__ rope, int Ns, int nworkers) {
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  const lds_u8_t* L = (const lds_u8_t*)lds_raw;
  const unsigned lds0 = (unsigned)(size_t)L;
  const int tid = threadIdx.x, lane = tid & 63, hh = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  LaneAddr la;
  la.init(lane);
  const int dtile = wave & 3;                            // phase 2: this wavefront's 32 columns of dQ

  // ---- which (batch, head) and which key blocks
  int wid = blockIdx.x;
  if ((nworkers & 7) == 0) wid = (wid & 7) * (nworkers >> 3) + (wid >> 3);       // workers of one head share an XCD's L2
  const int nkt = (S + 255) / 256;
  int bh, slot;
  if (DQ == kDqSlots) { bh = wid / Ns; slot = wid % Ns; }
  else { bh = blockIdx.x % (B * nh); slot = 0; }
  const int b = bh / nh, h = bh % nh;
  const int64_t H = (int64_t)nh * D, ld = 3 * H;
  const bf16_t* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * D;
  const bf16_t* kbase = qbase + H;
  const bf16_t* vbase = qbase + 2 * H;
  const uint64_t qb64 = (uint64_t)qbase, k64 = (uint64_t)kbase, do64 = (uint64_t)(dO + (int64_t)b * S * H + (int64_t)h * D);
  const uint64_t l64 = (uint64_t)(prep + ((int64_t)b * nh + h) * Sp);
  const unsigned d_off = (unsigned)((int64_t)B * nh * Sp * 4);                   // D follows the scaled lse in prep
  const unsigned ldb = (unsigned)(ld * 2), ldob = (unsigned)(H * 2);
  const float c = scale * kLog2e;
  // dQ tile of this wavefront in its slot (or in the one atomic buffer), row 0 of the (batch, head): wavefront-uniform
  float* dq_tile = dq_slots + (int64_t)slot * ((int64_t)B * S * H) + (int64_t)b * S * H + (int64_t)h * D + dtile * 32;
  const unsigned Hb = (unsigned)(H * 4);

  for (int round = 0;; ++round) {
    int kt;
    if (DQ == kDqSlots) { kt = worker_block(round, slot, Ns); if (kt >= nkt) break; }
    else { if (round) break; kt = blockIdx.x / (B * nh); }
    const bool first = DQ == kDqSlots && round == 0;     // store, do not add: the slot holds nothing yet
    const int kv0 = kt * 256, kv0w = kv0 + wave * 32;
    const int jb = kv0 / kFBQ, je = (S + kFBQ - 1) / kFBQ, nblk = je - jb;

    __syncthreads();                                     // everybody is done with the previous key block's LDS
    // key tile -> LDS (8 pieces of 4 rows per wavefront), then the first two query blocks
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int j = wave + 8 * i;
      const int r = 4 * j + (lane >> 4);
      const int cc = swz(r, lane & 15);
      int rg = kv0 + r;
      rg = rg < S ? rg : S - 1;
      lds_dma16(k64, (unsigned)rg * ldb + cc * 16, lds0 + kFOffK + j * 1024);
    }
    auto issue = [&](int t) {
      const unsigned st = lds0 + kFOffRing + (t % kFStages) * kFStage;
      const int row0 = (jb + t) * kFBQ;
      tile32_dma(qb64, ldb, row0, S, st, lane, wave);
      tile32_dma(do64, ldob, row0, S, st + 8192, lane, wave);
      if (wave == 0) lds_dma4(l64, (lane < 32 ? 0u : d_off) + (unsigned)(row0 + (lane & 31)) * 4u, st + 16384);
    };
    for (int t = 0; t < 2 && t < nblk; ++t) issue(t);

    // V rows of this wavefront's keys stay in registers as B operands; its K rows are read from the key tile in LDS
    // (which phase 2 needs there anyway): the registers they would take are what phase 2 accumulates in
    bf16x8_t vf[8];
    {
      int row = kv0w + (lane & 31);
      if (row >= S) row = S - 1;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) vf[ks] = *reinterpret_cast<const bf16x8_t*>(vbase + (int64_t)row * ld + 16 * ks + 8 * hh);
    }
    f32x16_t dk[4], dv[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dk[dt][r] = 0.f; dv[dt][r] = 0.f; }
    const int kvi = kv0w + (lane & 31);
    const unsigned knat_t = la.nat + lds0 + kFOffK + wave * 8192;

    // ---- phase 2 in three parts, so that the slot values a wavefront adds to are requested a whole phase 1 before they are
    // needed (they come from HBM).  Lane constants are made from an opaque copy of the lane number where they are used, so
    // that none of them stays in a register through phase 1.
    // accumulator register r of a lane is dQ[qrow0 + 8 (r / 4) + 4 (lane >> 5) + r % 4][lane & 31]: a wavefront-uniform row
    // base (scalar arithmetic) plus one 32-bit lane offset
    auto dq_at = [&](int tq, int ln, int r) {
      char* tile = reinterpret_cast<char*>(dq_tile + (int64_t)((jb + tq) * kFBQ) * H);
      const unsigned voff = (unsigned)(4 * (ln >> 5)) * Hb + (unsigned)(ln & 31) * 4u;
      return reinterpret_cast<float*>(tile + (size_t)(8 * (r >> 2) + (r & 3)) * Hb + (size_t)voff);
    };
    // (a) what the slot holds for query block tq (zeros where there is nothing to add to)
    auto dq_fetch = [&](int tq, f32x16_t& acc) {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int qrow0 = (jb + tq) * kFBQ;
      if (DQ != kDqSlots || first) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
      } else if (qrow0 + kFBQ <= S) {
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = __hip_atomic_load(dq_at(tq, ln, r), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      } else {                                           // the last block of a sequence that is no multiple of 32
        const int qlane = qrow0 + 4 * (ln >> 5);
#pragma unroll
        for (int r = 0; r < 16; ++r)
          acc[r] = qlane + 8 * (r >> 2) + (r & 3) < S ? __hip_atomic_load(dq_at(tq, ln, r), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : 0.f;
      }
    };
    // (b) acc += dS K over the keys up to the block's last row: two independent accumulation chains (even and odd key steps)
    auto dq_mfma = [&](int tq, f32x16_t& acc) {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      unsigned ex_tr, k_tr;
      {
        const int blk = ln >> 4, i = ln & 15, hb = blk >> 1;
        const int rl = 4 * hb + (i >> 2), q = 16 * (blk & 1) + 4 * (i & 3);
        ex_tr = rl * 64 + (((q >> 3) ^ ((rl >> 2) & 3)) << 4) + (q & 7) * 2;                 // exchange tile: 64-byte rows, chunks swizzled by (row >> 2) & 3
        k_tr = (rl * 256 + (swz(rl, q >> 3) << 4) + (q & 7) * 2) ^ ((unsigned)dtile << 6);   // key tile: as LaneAddr::tr, at this wavefront's 32 columns
      }
      const int qrow0 = (jb + tq) * kFBQ;
      int nks = (qrow0 + kFBQ - kv0 + 15) >> 4;          // 16-key steps that hold a visible key: even, wavefront-uniform
      nks = nks < 16 ? nks : 16;
      const unsigned exa = lds0 + kFOffEx + (tq & 1) * 16384 + ex_tr;
      const unsigned ka = lds0 + kFOffK + k_tr;
      f32x16_t acc1;
#pragma unroll
      for (int r = 0; r < 16; ++r) acc1[r] = 0.f;
      auto kstep = [&](int ks, f32x16_t& a_) {
        union { s16x4_t h2[2]; bf16x8_t v; } fa, fb;
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
          const unsigned a = (exa ^ (rr ? 32u : 0u)) + (unsigned)(ks * 1024 + rr * 512);
          const unsigned kk = (ka ^ (rr ? 32u : 0u)) + (unsigned)(ks * 4096 + rr * 2048);
          fa.h2[rr] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4_t __attribute__((address_space(3)))*>(a));
          fb.h2[rr] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<s16x4_t __attribute__((address_space(3)))*>(kk));
        }
        a_ = mfma(fa.v, fb.v, a_);
      };
      __builtin_amdgcn_s_setprio(1);
      int ks0 = 0;
#pragma nounroll
      for (; ks0 + 4 <= nks; ks0 += 4) {                 // four key steps at a time: their fragment reads go out ahead of the MFMAs
        kstep(ks0, acc); kstep(ks0 + 1, acc1); kstep(ks0 + 2, acc); kstep(ks0 + 3, acc1);
      }
      if (ks0 < nks) { kstep(ks0, acc); kstep(ks0 + 1, acc1); }
      __builtin_amdgcn_s_setprio(0);
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[r] += acc1[r];
    };
    // (c) the tile goes out
    auto dq_put = [&](int tq, const f32x16_t& acc) {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      const int qrow0 = (jb + tq) * kFBQ;
      // Everything older than the tile loads this iteration issued has to be complete BEFORE the stores below go out:
      // loads and stores retire out of order with respect to each other, so once stores are in flight the counter no
      // longer tells whether the next block's tile has landed (the next iteration does not wait for it again).
      if (wave == 0) wait_vmcnt<3>(); else wait_vmcnt<2>();
      auto put = [&](int r) {
        if (DQ == kDqAtomic) __builtin_amdgcn_global_atomic_fadd_f32((__attribute__((address_space(1))) float*)dq_at(tq, ln, r), acc[r]);
        else __hip_atomic_store(dq_at(tq, ln, r), acc[r], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      };
      if (qrow0 + kFBQ <= S) {
#pragma unroll
        for (int r = 0; r < 16; ++r) put(r);
      } else {
        const int qlane = qrow0 + 4 * (ln >> 5);
#pragma unroll
        for (int r = 0; r < 16; ++r)
          if (qlane + 8 * (r >> 2) + (r & 3) < S) put(r);
      }
    };

    wait_vmcnt<0>();                                     // V rows in registers; the key tile and the first blocks too (once per key block)
    for (int t = 0; t < nblk; ++t) {
      // Block t has landed and block t - 1's dS is complete in its exchange tile after this barrier.  A wavefront that
      // did phase 2 in the previous iteration has waited for all of its loads there (before its stores went out), so it
      // must not wait here for those stores.
      const bool had_turn = t > 1 && (wave >> 2) == ((t - 1) & 1);
      if (!had_turn) {
        if (t + 1 < nblk) { if (wave == 0) wait_vmcnt<3>(); else wait_vmcnt<2>(); }
        else wait_vmcnt<0>();
      }
      stage_barrier();
      if (t + 2 < nblk) issue(t + 2);
      const bool turn = t > 0 && (wave >> 2) == (t & 1);  // this wavefront produces the dQ tile of block t - 1 in this iteration
      f32x16_t dqacc;
      if (turn) dq_fetch(t - 1, dqacc);
      const int qb0 = (jb + t) * kFBQ;
      if (qb0 + kFBQ - 1 >= kv0w) {                       // else no query of the block sees this wavefront's keys: its rows of Ex^T are not read
        const unsigned so = lds0 + kFOffRing + (t % kFStages) * kFStage;
        const unsigned nat_t = la.nat + so, tr_t = la.tr + so;
        const unsigned sl = so + 16384 + 16 * hh;          // lse, then D, of the block's rows 4 hh ..
        typedef const __attribute__((address_space(3))) f32x4_t* lds_f4_t;
        bf16x8_t pb[2], dsb[2];
        {
          // S = Q K^T and dP = dO V^T: two independent accumulation chains, issued alternately
          f32x16_t sacc, pacc;
#pragma unroll
          for (int r = 0; r < 16; ++r) { sacc[r] = 0.f; pacc[r] = 0.f; }
          __builtin_amdgcn_s_setprio(1);
          static_for<8>([&](auto ks_c) {
            TAW_CONST(ks, ks_c);
            sacc = mfma(frag_nat2<ks, 0, true>(nat_t), frag_nat2<ks, 0, true>(knat_t), sacc);
            pacc = mfma(frag_nat2<ks, 8192, true>(nat_t), vf[ks], pacc);
          });
          __builtin_amdgcn_s_setprio(0);
          if (qb0 < kv0w + 31) {                           // block crosses the diagonal (wavefront-uniform)
            asm volatile("" ::: "memory");
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int qi = qb0 + 8 * (r >> 2) + 4 * hh + (r & 3);
              sacc[r] = kvi > qi ? -INFINITY : sacc[r];
            }
          }
#pragma unroll
          for (int r4 = 0; r4 < 4; ++r4) {
            const f32x4_t l4 = *reinterpret_cast<lds_f4_t>(sl + (8 * r4) * 4);     // +inf for rows beyond S: p = 0
            const f32x4_t d4 = *reinterpret_cast<lds_f4_t>(sl + (32 + 8 * r4) * 4);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              const int r = 4 * r4 + e;
              const float pr = fast_exp2(__builtin_fmaf(sacc[r], c, -l4[e]));
              sacc[r] = pr;
              pacc[r] = pr * (pacc[r] - d4[e]);
            }
          }
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) { pb[tt] = pack8(sacc, tt); dsb[tt] = pack8(pacc, tt); }
        }
        // dS -> exchange tile t & 1: rows = this wavefront's keys, four 8-byte pieces (4 consecutive query rows each) per lane
        {
          int ln = lane;
          asm volatile("" : "+v"(ln));
          const unsigned row = (unsigned)(32 * wave + (ln & 31));
          const unsigned exw = lds0 + kFOffEx + (t & 1) * 16384 + row * 64u + 8u * (unsigned)(ln >> 5);
          const unsigned sw = (row >> 2) & 3;
#pragma unroll
          for (int tt = 0; tt < 2; ++tt) {
            const u32x4_t w = __builtin_bit_cast(u32x4_t, dsb[tt]);
#pragma unroll
            for (int half = 0; half < 2; ++half) {
              const unsigned a = exw + (((unsigned)(2 * tt + half) ^ sw) << 4);
              typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
              *reinterpret_cast<__attribute__((address_space(3))) u32x2_t*>(a) = u32x2_t{w[2 * half], w[2 * half + 1]};
            }
          }
        }
        __builtin_amdgcn_s_setprio(1);
        static_for<4>([&](auto dt_c) {
          TAW_CONST(dt, dt_c);
          static_for<2>([&](auto tt_c) {
            TAW_CONST(tt, tt_c);
            bf16x8_t fq, fdo;
            frag_tr2x2<tt, dt, 0, 8192, true>(tr_t, fq, fdo);
            dv[dt] = mfma(fdo, pb[tt], dv[dt]);
            dk[dt] = mfma(fq, dsb[tt], dk[dt]);
          });
        });
        __builtin_amdgcn_s_setprio(0);
      }
      if (turn) {
        dq_mfma(t - 1, dqacc);
        dq_put(t - 1, dqacc);
      }
    }
    wait_vmcnt<0>();
    stage_barrier();                                     // the last block's dS is complete
    if ((wave >> 2) == (nblk & 1)) {
      f32x16_t dqacc;
      dq_fetch(nblk - 1, dqacc);
      dq_mfma(nblk - 1, dqacc);
      dq_put(nblk - 1, dqacc);
    }
    __syncthreads();                                     // LDS becomes the output staging area

    bf16_t* stage = reinterpret_cast<bf16_t*>(lds_raw) + wave * (32 * 136);
    bf16_t* dkout = dqkv + (int64_t)b * S * ld + H + (int64_t)h * D;
    bf16_t* dvout = dkout + H;
    if (rope) {
      int ln = lane;
      asm volatile("" : "+v"(ln));
      rope_inverse_T(dk, rope, kv0w + (ln & 31), S, ln);
    }
    store_rows_T(dk, scale, stage, dkout, ld, kv0w, S, lane);
    store_rows_T(dv, 1.0f, stage, dvout, ld, kv0w, S, lane);
  }
}

// dq = bf16( rotate_back( scale * sum of the slots that hold row t ) ): slot s holds the rows from 256 s on (the first key
// block of its worker), so row t at position p reads slots 0 .. min(Ns - 1, p / 256).  One thread per 8 columns.
__global__ void __launch_bounds__(256) attn_bwd_dq_reduce_kernel(const float* __restrict__ slots, int Ns, int64_t slot_stride,
                                                                 bf16_t* __restrict__ dqkv, int64_t rows, int S, int H, float scale,
                                                                 const float* __restrict__ rope) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int cpr = H / 8;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int col = (int)(idx % cpr) * 8;
  const int pos = (int)(row % S);
  int ns = pos / 256 + 1;
  ns = ns < Ns ? ns : Ns;
  float v[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const float* p = slots + row * (int64_t)H + col;
  for (int s = 0; s < ns; ++s) {
    const f32x4_t a = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p + s * slot_stride));
    const f32x4_t b2 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p + s * slot_stride + 4));
#pragma unroll
    for (int e = 0; e < 4; ++e) { v[e] += a[e]; v[4 + e] += b2[e]; }
  }
  if (rope) {
    const float* tb = rope + ((int64_t)pos * (D / 2) + (col % D) / 2) * 2;
    const f32x4_t cs0 = *reinterpret_cast<const f32x4_t*>(tb), cs1 = *reinterpret_cast<const f32x4_t*>(tb + 4);
    const float cc[4] = {cs0[0], cs0[2], cs1[0], cs1[2]}, sn[4] = {cs0[1], cs0[3], cs1[1], cs1[3]};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float a = v[2 * e], b2 = v[2 * e + 1];
      v[2 * e] = a * cc[e] + b2 * sn[e];
      v[2 * e + 1] = b2 * cc[e] - a * sn[e];
    }
  }
  bf16x8_t o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16_t)(v[e] * scale);
  *reinterpret_cast<bf16x8_t*>(dqkv + row * (int64_t)(3 * H) + col) = o;
}

__global__ void __launch_bounds__(256) zero_f32_kernel(f32x4_t* __restrict__ p, size_t nvec) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) p[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
}

int launch_fwd(int B, int S, int nh, const void* qkv, void* o, float* lse, hipStream_t st) {
  constexpr int BQ = 256;
  constexpr size_t lds = 4 * 2 * kTileBytes;      // the ring; the output staging (8 x 32 x 136 bf16) fits inside
  static_assert(lds >= 8 * 32 * 136 * sizeof(bf16_t), "staging area");
  TAW_SET_LDS_LIMIT_ONCE(attn_fwd_kernel, lds);
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

// Workers per (batch, head) for the slot form: as many as fill the 256 compute units in whole rounds, preferring few (every
// slot is one more fp32 copy of dQ to write and to sum).  At most one worker per key block.
int attn_bwd_slots(int B, int S, int nh) {
  constexpr int kCUs = 256;
  const int nkt = (S + 255) / 256;
  int best = 1;
  double best_score = -1.0;
  for (int ns = 1; ns <= 16 && ns <= nkt; ++ns) {
    const int64_t w = (int64_t)B * nh * ns;
    const double eff = (double)w / (double)((w + kCUs - 1) / kCUs * kCUs);
    const int rounds = (nkt + ns - 1) / ns;
    const double balance = (rounds & 1) && rounds < 8 ? 1.0 - 0.5 / rounds : 1.0;     // an odd, small number of snake rounds leaves the workers uneven
    const double score = eff * balance - 0.004 * ns;
    if (score > best_score) { best_score = score; best = ns; }
  }
  return best;
}

// bytes of stored dS per (batch, head): block ib of 256 query rows holds 256 (ib + 1) keys x 256 rows bf16
static int64_t attn_bwd_ds_pair_bytes(int S) { return ds_block_offset((S + 255) / 256); }

size_t attn_bwd_mfma_scratch_floats(int B, int S, int nh, int form) {
  const size_t prep = 2 * (size_t)B * nh * ((S + 63) / 64 * 64);
  const size_t slots = (size_t)attn_bwd_slots(B, S, nh) * (size_t)B * S * nh * D;      // one slot suffices for the atomic form
  const size_t stored = (size_t)B * nh * (size_t)attn_bwd_ds_pair_bytes(S) / 4;
  switch (form) {
    case ATTN_BWD_SPLIT: return prep;
    case ATTN_BWD_FUSED: case ATTN_BWD_FUSED_ATOMIC: return prep + slots;
    case ATTN_BWD_STORED: return prep + stored;
    default: return prep + (slots > stored ? slots : stored);                           // enough for every form
  }
}

int launch_attn_bwd_mfma(int B, int S, int nh, const void* qkv, const void* o, const void* dO, const float* lse, float* prep,
                         void* dqkv, const float* rope_table, int form, hipStream_t st) {
  const float scale = 1.0f / sqrtf((float)D);
  const int Sp = (S + 63) / 64 * 64;
  const float* lse2 = prep;
  const float* Dv = prep + (size_t)B * nh * Sp;
  float* slots = prep + 2 * (size_t)B * nh * Sp;
  {
    const int64_t threads = (int64_t)B * Sp * nh * 16;
    hipLaunchKernelGGL(attn_bwd_prep_kernel, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, st, (const bf16_t*)o, (const bf16_t*)dO, lse, prep,
                       B, S, Sp, nh);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
  }
  if (form == ATTN_BWD_FUSED || form == ATTN_BWD_FUSED_ATOMIC) {
    const int64_t H = (int64_t)nh * D, rows = (int64_t)B * S;
    const int nkt = (S + 255) / 256;
    int ns = 1;
    if (form == ATTN_BWD_FUSED) {
      ns = attn_bwd_slots(B, S, nh);
      const int nworkers = B * nh * ns;
      TAW_SET_LDS_LIMIT_ONCE((attn_bwd_fused_kernel<kDqSlots>), kFusedLds);
      hipLaunchKernelGGL((attn_bwd_fused_kernel<kDqSlots>), dim3((unsigned)nworkers), dim3(kThreads8), kFusedLds, st, (const bf16_t*)qkv,
                         (const bf16_t*)dO, prep, (bf16_t*)dqkv, slots, B, S, Sp, nh, scale, rope_table, ns, nworkers);
    } else {
      const size_t nvec = (size_t)rows * H / 4;
      hipLaunchKernelGGL(zero_f32_kernel, dim3(2048), dim3(256), 0, st, reinterpret_cast<f32x4_t*>(slots), nvec);
      int rc = (int)hipGetLastError();
      if (rc) return rc;
      TAW_SET_LDS_LIMIT_ONCE((attn_bwd_fused_kernel<kDqAtomic>), kFusedLds);
      hipLaunchKernelGGL((attn_bwd_fused_kernel<kDqAtomic>), dim3((unsigned)(nkt * B * nh)), dim3(kThreads8), kFusedLds, st, (const bf16_t*)qkv,
                         (const bf16_t*)dO, prep, (bf16_t*)dqkv, slots, B, S, Sp, nh, scale, rope_table, 1, nkt * B * nh);
    }
    int rc = (int)hipGetLastError();
    if (rc) return rc;
    const int64_t n = rows * (H / 8);
    hipLaunchKernelGGL(attn_bwd_dq_reduce_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, slots, ns, rows * H, (bf16_t*)dqkv, rows, S,
                       (int)H, scale, rope_table);
    return (int)hipGetLastError();
  }
  if (form == ATTN_BWD_STORED) {
    // the stored dS follows the row statistics (a multiple of 512 bytes in front of it)
    unsigned char* ds = reinterpret_cast<unsigned char*>(slots);
    const int64_t pair_bytes = attn_bwd_ds_pair_bytes(S);
    constexpr size_t lds = kKvLds;
    TAW_SET_LDS_LIMIT_ONCE(attn_bwd_dkv_kernel<true>, lds);
    const int nkt = (S + 255) / 256;
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<true>, dim3((unsigned)(nkt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (const bf16_t*)dO, lse2,
                       Dv, (bf16_t*)dqkv, B, S, Sp, nh, scale, rope_table, ds, pair_bytes);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
    static_assert(kDqsLds >= 8 * 32 * 136 * sizeof(bf16_t), "staging area");
    TAW_SET_LDS_LIMIT_ONCE(attn_bwd_dq_stored_kernel, kDqsLds);
    hipLaunchKernelGGL(attn_bwd_dq_stored_kernel, dim3((unsigned)(nkt * B * nh)), dim3(kThreads8), kDqsLds, st, (const bf16_t*)qkv, ds, pair_bytes,
                       (bf16_t*)dqkv, B, S, nh, scale, rope_table);
    return (int)hipGetLastError();
  }
  {
    constexpr size_t lds = kKvLds;
    static_assert(lds >= 8 * 32 * 136 * sizeof(bf16_t), "staging area");
    TAW_SET_LDS_LIMIT_ONCE(attn_bwd_dkv_kernel<false>, lds);
    const int nkt = (S + 255) / 256;
    hipLaunchKernelGGL(attn_bwd_dkv_kernel<false>, dim3((unsigned)(nkt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (const bf16_t*)dO, lse2, Dv,
                       (bf16_t*)dqkv, B, S, Sp, nh, scale, rope_table, nullptr, (int64_t)0);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
  }
  {
    constexpr size_t lds = 4 * 2 * kTileBytes;
    TAW_SET_LDS_LIMIT_ONCE(attn_bwd_dq_kernel, lds);
    const int nqt = (S + 255) / 256;
    hipLaunchKernelGGL(attn_bwd_dq_kernel, dim3((unsigned)(nqt * B * nh)), dim3(kThreads8), lds, st, (const bf16_t*)qkv, (const bf16_t*)dO, lse2, Dv,
                       (bf16_t*)dqkv, B, S, Sp, nh, scale, rope_table);
    return (int)hipGetLastError();
  }
}

}  // namespace taw
