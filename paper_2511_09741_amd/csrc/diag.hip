// Measurement probes (include/taw_diag.h): short synthetic kernels that record what the part sustains.
// Each entry point launches on the default stream, waits, and returns the figures in host memory.
#include <hip/hip_runtime.h>

#include "../../include/taw_diag.h"
#include "dev_common.h"
#include "taw_internal.h"

namespace taw {
namespace {

typedef __attribute__((address_space(3))) unsigned char lds_u8_t;

__device__ __forceinline__ unsigned mix(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
  return x;
}
// a random bf16 in +-[2^-4, 1): sign, one of four exponents, seven mantissa bits
__device__ __forceinline__ unsigned rnd_bf16(unsigned x) { return ((x >> 31) << 15) | ((123u + (x >> 8) % 4u) << 7) | (x & 0x7fu); }

// per-workgroup (wall-clock ticks, core-clock ticks) of the measured loop
__device__ long long g_clk[2 * 256];

template <int KIND>
__global__ void __launch_bounds__(256, 1) mfma_loop_kernel(int iters, const unsigned char* __restrict__ src, unsigned src_mask, float* sink) {
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  unsigned* lds = reinterpret_cast<unsigned*>(lds_raw);
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (KIND >= TAW_DIAG_MFMA_LDS) {
    for (int i = tid; i < 16384; i += 256) {                     // 64 KiB of random bf16 pairs
      const unsigned x = mix(i * 2654435761u + blockIdx.x), y = mix(x);
      lds[i] = rnd_bf16(x) | (rnd_bf16(y) << 16);
    }
    __syncthreads();
  }
  const unsigned lds0 = (unsigned)(size_t)(const lds_u8_t*)lds_raw;
  const unsigned rd = lds0 + wave * 16384 + lane * 16;            // conflict-free: consecutive lanes, consecutive 16 bytes
  union { unsigned u[4]; bf16x8_t v; } fa[2], fb[2];
#pragma unroll
  for (int j = 0; j < 2; ++j)
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const unsigned x = mix(tid * 8 + j * 4 + e + 1), y = mix(x);
      fa[j].u[e] = KIND == TAW_DIAG_MFMA_ZERO ? 0u : rnd_bf16(x) | (rnd_bf16(y) << 16);
      fb[j].u[e] = KIND == TAW_DIAG_MFMA_ZERO ? 0u : rnd_bf16(y ^ 0x9e3779b9u) | (rnd_bf16(x ^ 0x85ebca6bu) << 16);
    }
  f32x16_t acc[8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  // loads of kind 3 land in the second half of LDS (this wavefront's 16 KiB), a different KiB per load of a step
  const unsigned dma_dst = lds0 + 65536 + wave * 16384;
  unsigned goff = (unsigned)((blockIdx.x * 4 + wave) * 65536u + lane * 16u);
  u32x4_t pend[2];
  if (KIND >= TAW_DIAG_MFMA_LDS) {
    asm volatile("ds_read_b128 %0, %1" : "=v"(pend[0]) : "v"(rd));
    asm volatile("ds_read_b128 %0, %1" : "=v"(pend[1]) : "v"(rd + 1024));
  }
  const long long w0 = wall_clock64(), c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      if (KIND >= TAW_DIAG_MFMA_LDS && (u & 1) == 0) {             // one fragment read per two MFMAs, consumed four MFMAs after it was issued
        const int slot = (u >> 1) & 1;
        asm volatile("s_waitcnt lgkmcnt(1)" ::: "memory");         // all but the newest read have returned: pend[slot] is the older of the two
        if ((u >> 1) & 2) fa[slot].v = __builtin_bit_cast(bf16x8_t, pend[slot]);
        else fb[slot].v = __builtin_bit_cast(bf16x8_t, pend[slot]);
        asm volatile("ds_read_b128 %0, %1" : "=v"(pend[slot]) : "v"(rd + ((u >> 1) & 7) * 1024 + ((it & 1) ? 8192 : 0)));
      }
      if (KIND == TAW_DIAG_MFMA_LDS_LOADS && (u & 3) == 0) {       // one direct load per four MFMAs
        asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(goff & src_mask), "s"((unsigned long long)src), "s"(dma_dst + (u >> 2) * 1024));
        goff += 1024u;
      }
      acc[u & 7] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[u & 1].v, fb[(u >> 1) & 1].v, acc[u & 7], 0, 0, 0);
    }
    if (KIND == TAW_DIAG_MFMA_LDS_LOADS) {
      __builtin_amdgcn_s_waitcnt((4 & 15) | (7 << 4) | (15 << 8));  // vmcnt(4): the previous trip's loads have landed
      goff += 65536u * 1024u - 4096u;                               // next trip: 64 MiB further (wraps inside the buffer)
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  const long long w1 = wall_clock64(), c1 = clock64();
  if (tid == 0) { g_clk[2 * blockIdx.x] = w1 - w0; g_clk[2 * blockIdx.x + 1] = c1 - c0; }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[i][r];
  if (s == 12345.678f) sink[0] = s;                                 // keeps the accumulators alive; never true in practice
}

template <int INSTR, int WAVES>
__global__ void __launch_bounds__(WAVES * 64, 1) lds_rate_kernel(int iters, unsigned* sink) {
  extern __shared__ __attribute__((aligned(256))) unsigned char lds_raw[];
  for (int i = threadIdx.x; i < 65536 / 4; i += blockDim.x) reinterpret_cast<unsigned*>(lds_raw)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned lds0 = (unsigned)(size_t)(const lds_u8_t*)lds_raw;
  const unsigned a = lds0 + (INSTR == 0 ? lane * 16 : lane * 8) + (wave & 3) * 4096;
  u32x4_t acc4 = {0, 0, 0, 0};
  typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
  u32x2_t acc2 = {0, 0};
  const long long w0 = wall_clock64(), c0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      const unsigned ad = a + (u % 4) * 1024 + (u / 4) * 16384;
      if (INSTR == 0) { u32x4_t v; asm volatile("ds_read_b128 %0, %1" : "=v"(v) : "v"(ad)); acc4 += v; }
      else if (INSTR == 1) { u32x2_t v; asm volatile("ds_read_b64 %0, %1" : "=v"(v) : "v"(ad)); acc2 += v; }
      else { u32x2_t v; asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(v) : "v"(ad)); acc2 += v; }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  }
  const long long w1 = wall_clock64(), c1 = clock64();
  if (threadIdx.x == 0) { g_clk[2 * blockIdx.x] = w1 - w0; g_clk[2 * blockIdx.x + 1] = c1 - c0; }
  if ((acc4[0] ^ acc4[1] ^ acc4[2] ^ acc4[3] ^ acc2[0] ^ acc2[1]) == 0x12345679u) sink[0] = 1;
}

// workgroup (head, key block): from row 256 * key block down, 32 rows per step; wavefront w takes rows 4 w .. 4 w + 3 of the step,
// two rows per instruction (one per half wavefront), the 128 columns of the head in four instructions
template <int MODE>
__global__ void __launch_bounds__(512) dq_update_kernel(float* buf, int S, int LD, int nheads) {
  const int head = blockIdx.x % nheads, kvb = blockIdx.x / nheads;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* base = buf + (size_t)head * 128;
  for (int r0 = kvb * 256; r0 + 32 <= S; r0 += 32) {
#pragma unroll
    for (int rr = 0; rr < 4; rr += 2) {
      const int row = r0 + wave * 4 + rr + (lane >> 5);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float* p = base + (size_t)row * LD + c * 32 + (lane & 31);
        if (MODE == 0) __builtin_amdgcn_global_atomic_fadd_f32((__attribute__((address_space(1))) float*)p, 1.0f);
        else if (MODE == 1) *p = 1.0f;
        else *p = *p + 1.0f;
      }
    }
  }
}

__global__ void fill_zero_kernel(float* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

// ---- how vector instructions issue beside MFMAs.  Every wavefront runs `iters` trips of 4 slots; a slot is one MFMA
// (MODE 0, 1: in every wavefront; MODE 2: in wavefronts 0..3 only) followed by NV vector instructions (MODE 0, 1: in the same
// wavefront; MODE 2: in wavefronts 4..7, which issue no MFMA).  MODE 0 runs one wavefront per SIMD, MODE 1 and 2 two.
// KIND 0: v_fma_f32, 1: v_exp_f32.  Core-clock ticks of the loop, per wavefront of workgroup 0, go to g_clk[wave].
template <int KIND> __device__ __forceinline__ void issue_valu(float& x, float c) {
  if constexpr (KIND == 0) asm volatile("v_fma_f32 %0, %0, %1, %0" : "+v"(x) : "v"(c));
  else asm volatile("v_exp_f32 %0, %0" : "+v"(x));
}
template <int MODE, int KIND, int NV>
__global__ void __launch_bounds__(512, 1) issue_kernel(int iters, float* sink) {
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  union { unsigned u[4]; bf16x8_t v; } fa, fb;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const unsigned x = mix(threadIdx.x * 4 + e + 1), y = mix(x);
    fa.u[e] = rnd_bf16(x) | (rnd_bf16(y) << 16);
    fb.u[e] = rnd_bf16(y ^ 0x9e3779b9u) | (rnd_bf16(x ^ 0x85ebca6bu) << 16);
  }
  f32x16_t acc[4];
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[a][r] = 0.f;
  float v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = 1e-3f * (float)(i + 1);
  const float c = 1e-6f;
  const bool do_mfma = MODE != 2 || wave < 4;                    // wavefront-uniform
  __syncthreads();
  const long long t0 = __builtin_readcyclecounter();
  if (MODE != 2) {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[a]) : "v"(fa.v), "v"(fb.v));
#pragma unroll
        for (int j = 0; j < NV; ++j) issue_valu<KIND>(v[(a * NV + j) & 7], c);
      }
    }
  } else if (do_mfma) {                                          // two loops, so that neither carries the other's branches
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int a = 0; a < 4; ++a) asm volatile("v_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(acc[a]) : "v"(fa.v), "v"(fb.v));
    }
  } else {
    for (int it = 0; it < iters; ++it) {
#pragma unroll
      for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int j = 0; j < NV; ++j) issue_valu<KIND>(v[(a * NV + j) & 7], c);
    }
  }
  const long long t1 = __builtin_readcyclecounter();
  float sum = 0.f;
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int r = 0; r < 16; ++r) sum += acc[a][r];
#pragma unroll
  for (int i = 0; i < 8; ++i) sum += v[i];
  if (sum == 123.456f) sink[threadIdx.x] = sum;                  // keeps the arithmetic alive
  if (blockIdx.x == 0 && (threadIdx.x & 63) == 0) g_clk[wave] = t1 - t0;
}

int read_clocks(int nblocks, double* wall, double* core) {
  static long long h[2 * 256];
  hipError_t e = hipMemcpyFromSymbol(h, HIP_SYMBOL(g_clk), sizeof(long long) * 2 * nblocks);
  if (e != hipSuccess) return (int)e;
  *wall = 0; *core = 0;
  for (int b = 0; b < nblocks; ++b) { *wall += (double)h[2 * b]; *core += (double)h[2 * b + 1]; }
  return 0;
}

template <typename F> int timed(F&& launch, float* ms) {
  hipEvent_t e0, e1;
  hipError_t e = hipEventCreate(&e0);
  if (e != hipSuccess) return (int)e;
  e = hipEventCreate(&e1);
  if (e != hipSuccess) { (void)hipEventDestroy(e0); return (int)e; }
  int rc = 0;
  for (int rep = 0; rep < 3 && !rc; ++rep) {                      // the last of three launches is the one reported
    (void)hipEventRecord(e0, 0);
    launch();
    rc = (int)hipGetLastError();
    (void)hipEventRecord(e1, 0);
    if (!rc) rc = (int)hipEventSynchronize(e1);
    if (!rc) rc = (int)hipEventElapsedTime(ms, e0, e1);
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  return rc;
}

}  // namespace
}  // namespace taw

using namespace taw;

extern "C" int taw_diag_mfma_loop(int32_t kind, int32_t iters, const void* src, size_t src_bytes, taw_diag_rate* out) {
  if (!out) return TAW_ERR_NULL;
  if (kind < TAW_DIAG_MFMA_RANDOM || kind > TAW_DIAG_MFMA_LDS_LOADS || iters < 1) return TAW_ERR_SHAPE;
  unsigned mask = 0;
  if (kind == TAW_DIAG_MFMA_LDS_LOADS) {
    if (!src) return TAW_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) != 0) return TAW_ERR_ALIGN;
    if (src_bytes < ((size_t)1 << 20)) return TAW_ERR_SHAPE;
    size_t pow2 = (size_t)1 << 20;                                  // loads wrap inside the largest power of two that fits (at most 2 GiB)
    while (pow2 * 2 <= src_bytes && pow2 < ((size_t)1 << 31)) pow2 *= 2;
    mask = (unsigned)(pow2 - 1) & ~15u;
  }
  static float* sink = nullptr;                                     // never written in practice; the static device array doubles as the sink
  if (!sink) {
    void* p = nullptr;
    hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(g_clk));
    if (e != hipSuccess) return TAW_ERR_HIP;
    sink = reinterpret_cast<float*>(p);
  }
  const size_t lds = kind >= TAW_DIAG_MFMA_LDS ? 131072 : 0;
  float ms = 0.f;
  int rc;
  const unsigned char* s8 = static_cast<const unsigned char*>(src);
#define TAW_DIAG_RUN(K)                                                                                                        \
  do {                                                                                                                       \
    hipError_t e_ = hipFuncSetAttribute((const void*)mfma_loop_kernel<K>, hipFuncAttributeMaxDynamicSharedMemorySize, 131072); \
    if (e_ != hipSuccess) return TAW_ERR_HIP;                                                                                \
    rc = timed([&] { hipLaunchKernelGGL((mfma_loop_kernel<K>), dim3(256), dim3(256), lds, 0, iters, s8, mask, sink); }, &ms);  \
  } while (0)
  switch (kind) {
    case TAW_DIAG_MFMA_RANDOM: TAW_DIAG_RUN(TAW_DIAG_MFMA_RANDOM); break;
    case TAW_DIAG_MFMA_ZERO: TAW_DIAG_RUN(TAW_DIAG_MFMA_ZERO); break;
    case TAW_DIAG_MFMA_LDS: TAW_DIAG_RUN(TAW_DIAG_MFMA_LDS); break;
    default: TAW_DIAG_RUN(TAW_DIAG_MFMA_LDS_LOADS); break;
  }
#undef TAW_DIAG_RUN
  if (rc) return TAW_ERR_HIP;
  double wall, core;
  if (read_clocks(256, &wall, &core)) return TAW_ERR_HIP;
  out->ms = ms;
  out->tflops = 256.0 * 4 * (double)iters * 16 * 32768.0 / ((double)ms * 1e9);
  out->clock_ghz = core / wall / 10.0;                              // wall clock: 100 MHz
  out->mfma_busy = (double)iters * 16 * 32 / (core / 256.0);
  return TAW_OK;
}

extern "C" int taw_diag_lds_read_rate(int32_t instr, int32_t waves, double* bytes_per_clock_per_cu, double* clock_ghz) {
  if (!bytes_per_clock_per_cu || !clock_ghz) return TAW_ERR_NULL;
  if (instr < 0 || instr > 2 || (waves != 4 && waves != 8)) return TAW_ERR_SHAPE;
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_clk)) != hipSuccess) return TAW_ERR_HIP;
  unsigned* sink = reinterpret_cast<unsigned*>(p);
  const int iters = 20000;
  float ms = 0.f;
  int rc = 0;
#define TAW_DIAG_LDS(I, W)                                                                                                    \
  do {                                                                                                                       \
    if (hipFuncSetAttribute((const void*)lds_rate_kernel<I, W>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess) return TAW_ERR_HIP; \
    rc = timed([&] { hipLaunchKernelGGL((lds_rate_kernel<I, W>), dim3(256), dim3(W * 64), 65536, 0, iters, sink); }, &ms);     \
  } while (0)
  if (waves == 4) { if (instr == 0) TAW_DIAG_LDS(0, 4); else if (instr == 1) TAW_DIAG_LDS(1, 4); else TAW_DIAG_LDS(2, 4); }
  else { if (instr == 0) TAW_DIAG_LDS(0, 8); else if (instr == 1) TAW_DIAG_LDS(1, 8); else TAW_DIAG_LDS(2, 8); }
#undef TAW_DIAG_LDS
  if (rc) return TAW_ERR_HIP;
  double wall, core;
  if (read_clocks(256, &wall, &core)) return TAW_ERR_HIP;
  const double bytes_per_cu = (double)waves * iters * 16 * 64 * (instr == 0 ? 16 : 8);
  *bytes_per_clock_per_cu = bytes_per_cu / (core / 256.0);
  *clock_ghz = core / wall / 10.0;
  return TAW_OK;
}

extern "C" int taw_diag_dq_update_rate(float* buf, int32_t S, int32_t n_heads, int32_t mode, double* updates_per_s, double* ms_out) {
  if (!buf || !updates_per_s || !ms_out) return TAW_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return TAW_ERR_ALIGN;
  if (S < 256 || S % 256 || n_heads < 1 || mode < 0 || mode > 2) return TAW_ERR_SHAPE;
  const int LD = n_heads * 128, nkvb = S / 256;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(2048), dim3(256), 0, 0, buf, (size_t)S * LD);
  float ms = 0.f;
  int rc;
  if (mode == 0) rc = timed([&] { hipLaunchKernelGGL((dq_update_kernel<0>), dim3(n_heads * nkvb), dim3(512), 0, 0, buf, S, LD, n_heads); }, &ms);
  else if (mode == 1) rc = timed([&] { hipLaunchKernelGGL((dq_update_kernel<1>), dim3(n_heads * nkvb), dim3(512), 0, 0, buf, S, LD, n_heads); }, &ms);
  else rc = timed([&] { hipLaunchKernelGGL((dq_update_kernel<2>), dim3(n_heads * nkvb), dim3(512), 0, 0, buf, S, LD, n_heads); }, &ms);
  if (rc) return TAW_ERR_HIP;
  double elems = 0;
  for (int kvb = 0; kvb < nkvb; ++kvb) elems += (double)(S - kvb * 256) * 128;
  elems *= n_heads;
  *updates_per_s = elems / ((double)ms * 1e-3);
  *ms_out = ms;
  return TAW_OK;
}

// ---- what a vector store costs a SIMD that is otherwise issuing MFMAs -------------------------------------------------
// Every wavefront: `iters` trips of NM MFMAs (four independent accumulators) followed by NS non-temporal stores of one
// contiguous KiB (16 bytes per lane) into a 64 KiB window of its own, walked KiB by KiB.
template <int NM, int NS>
__global__ void __launch_bounds__(512, 1) store_cost_kernel(unsigned char* __restrict__ buf, int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  unsigned char* win = buf + ((size_t)blockIdx.x * nw + wave) * 65536;
  bf16x8_t a, b;
  unsigned x = (threadIdx.x + blockIdx.x * 977u) * 2654435761u;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    x = x * 1664525u + 1013904223u;
    a[i] = (bf16_t)(((x >> 9) & 255) / 256.0f + 0.06f);
    x = x * 1664525u + 1013904223u;
    b[i] = (bf16_t)(((x >> 9) & 255) / 256.0f - 0.5f);
  }
  f32x16_t acc[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  u32x4_t v = {x, x + 1, x + 2, x + 3};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int m = 0; m < NM; ++m) acc[m & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[m & 3], 0, 0, 0);
#pragma unroll
    for (int st = 0; st < NS; ++st) {
      unsigned char* p = win + ((((it & 63) * 1024) + st * 16384) & 65535) + lane * 16;      // at most 64512 + 1008 + 16 bytes into the window
      __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
    }
    v[0] += 1;
    __builtin_amdgcn_sched_barrier(0);
  }
  float t = 0.f;
#pragma unroll
  for (int j = 0; j < 4; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) t += acc[j][r];
  if (t == 12345.678f) sink[0] = t;
}

extern "C" size_t taw_diag_store_cost_bytes(void) { return (size_t)256 * 8 * 65536; }

extern "C" int taw_diag_store_cost(void* buf, size_t buf_bytes, int32_t waves, int32_t mfmas, int32_t stores, double* ns_per_trip) {
  if (!buf || !ns_per_trip) return TAW_ERR_NULL;
  if ((reinterpret_cast<uintptr_t>(buf) & 15u) != 0) return TAW_ERR_ALIGN;
  if (buf_bytes < taw_diag_store_cost_bytes()) return TAW_ERR_WORKSPACE;       // 256 workgroups x 8 wavefronts x 64 KiB, whatever `waves` is
  if ((waves != 4 && waves != 8) || (mfmas != 16 && mfmas != 64) || (stores != 0 && stores != 1 && stores != 2 && stores != 4)) return TAW_ERR_SHAPE;
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_clk)) != hipSuccess) return TAW_ERR_HIP;
  float* sink = reinterpret_cast<float*>(p) + 64;
  const int iters = 20000;
  float ms = 0.f;
  int rc = -1;
#define TAW_DIAG_STORE(M, N)                                                                                                 \
  if (mfmas == M && stores == N)                                                                                             \
    rc = timed([&] { hipLaunchKernelGGL((store_cost_kernel<M, N>), dim3(256), dim3(waves * 64), 0, 0, static_cast<unsigned char*>(buf), iters, sink); }, &ms);
  TAW_DIAG_STORE(16, 0) TAW_DIAG_STORE(16, 1) TAW_DIAG_STORE(16, 2) TAW_DIAG_STORE(16, 4)
  TAW_DIAG_STORE(64, 0) TAW_DIAG_STORE(64, 1) TAW_DIAG_STORE(64, 2) TAW_DIAG_STORE(64, 4)
#undef TAW_DIAG_STORE
  if (rc) return TAW_ERR_HIP;
  *ns_per_trip = (double)ms * 1e6 / iters;
  return TAW_OK;
}

extern "C" int taw_diag_gemm_tile_order(int32_t tiles_m, int32_t tiles_n, int32_t* tile_rows, int32_t* tile_cols) {
  if (tiles_m < 1 || tiles_n < 1 || (int64_t)tiles_m * tiles_n > (1 << 24)) return TAW_ERR_SHAPE;
  if (!tile_rows || !tile_cols) return TAW_ERR_NULL;
  for (int b = 0; b < tiles_m * tiles_n; ++b) {
    int tm, tn;
    taw::gemm_tile_of_block(b, tiles_m, tiles_n, &tm, &tn);
    tile_rows[b] = tm;
    tile_cols[b] = tn;
  }
  return TAW_OK;
}

extern "C" int taw_diag_attn_ds_layout(int32_t S, int64_t* pair_bytes, int64_t* unit_offsets, int32_t* slots, int32_t* rows) {
  if (S < 1 || S > (1 << 20)) return TAW_ERR_SHAPE;
  if (!pair_bytes || !unit_offsets || !slots || !rows) return TAW_ERR_NULL;
  const int nqt = (S + 255) / 256;
  *pair_bytes = taw::ds_block_offset(nqt);
  size_t n = 0;
  for (int ib = 0; ib < nqt; ++ib)
    for (int s8 = 0; s8 < 8; ++s8)
      for (int g = 0; g < 8 * (ib + 1); ++g) unit_offsets[n++] = taw::ds_unit_offset(ib, s8, g);
  for (int tt = 0; tt < 2; ++tt)
    for (int hh = 0; hh < 2; ++hh)
      for (int kk = 0; kk < 32; ++kk) slots[(tt * 2 + hh) * 32 + kk] = (int32_t)taw::ds_slot(kk, hh, tt);
  for (int p = 0; p < 32; ++p) rows[p] = taw::ds_row_of_slot(p);
  return TAW_OK;
}

extern "C" int taw_diag_issue_rate(int32_t mode, int32_t kind, int32_t nvalu, double* cycles_mfma_wave, double* cycles_valu_wave) {
  if (!cycles_mfma_wave || !cycles_valu_wave) return TAW_ERR_NULL;
  if (mode < 0 || mode > 2 || kind < 0 || kind > 1 || (nvalu != 0 && nvalu != 2 && nvalu != 4 && nvalu != 8)) return TAW_ERR_SHAPE;
  void* p = nullptr;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_clk)) != hipSuccess) return TAW_ERR_HIP;
  float* sink = reinterpret_cast<float*>(p) + 64;                 // 512 floats inside g_clk, behind the per-wavefront results
  const int iters = 20000;
  const int threads = mode == 0 ? 256 : 512;
  float ms = 0.f;
  int rc = -1;
#define TAW_DIAG_ISSUE(M, K, N)                                                                                              \
  if (mode == M && kind == K && nvalu == N) rc = timed([&] { hipLaunchKernelGGL((issue_kernel<M, K, N>), dim3(256), dim3(threads), 0, 0, iters, sink); }, &ms);
#define TAW_DIAG_ISSUE_N(M, K) TAW_DIAG_ISSUE(M, K, 0) TAW_DIAG_ISSUE(M, K, 2) TAW_DIAG_ISSUE(M, K, 4) TAW_DIAG_ISSUE(M, K, 8)
  TAW_DIAG_ISSUE_N(0, 0) TAW_DIAG_ISSUE_N(0, 1) TAW_DIAG_ISSUE_N(1, 0) TAW_DIAG_ISSUE_N(1, 1) TAW_DIAG_ISSUE_N(2, 0) TAW_DIAG_ISSUE_N(2, 1)
#undef TAW_DIAG_ISSUE_N
#undef TAW_DIAG_ISSUE
  if (rc) return TAW_ERR_HIP;
  long long h[8];
  if (hipMemcpyFromSymbol(h, HIP_SYMBOL(g_clk), sizeof(h)) != hipSuccess) return TAW_ERR_HIP;
  const double slots = (double)iters * 4;
  *cycles_mfma_wave = (double)h[0] / slots;                         // wavefront 0 issues MFMAs in every mode
  *cycles_valu_wave = (double)h[mode == 0 ? 3 : 7] / slots;         // the last wavefront: the vector-only one in mode 2
  return TAW_OK;
}
