// Shape-generic kernels: fp32 arithmetic on fp32 or bf16 storage, any dimensions.  They carry the
// fp32 configuration (head_dim 16, widths that fit no MFMA tile) and every bf16 shape the MFMA
// kernels do not take.  Simple LDS-tiled GEMM and one-wavefront-per-row attention.
#include "dev_common.h"
#include "taw_internal.h"

namespace taw {

// =============================================================================== GEMM
// C[m,n] (=|+=) sum_k A(m,k) B(k,n) (+ R[m,n]);  A(m,k) = A[m*a_rs + k*a_cs], B(k,n) = B[k*b_rs + n*b_cs].
// 32x32 output tile per 256-thread workgroup, 2x2 outputs per thread, k ascending in steps of 16.
template <typename TI, typename TC>
__global__ void __launch_bounds__(256) gemm_generic_kernel(int64_t M, int64_t N, int64_t K, const TI* __restrict__ A,
                                                           int64_t a_rs, int64_t a_cs, const TI* __restrict__ B,
                                                           int64_t b_rs, int64_t b_cs, TC* __restrict__ C, int64_t ldc,
                                                           int accumulate, const TC* __restrict__ R, int64_t ldr) {
  __shared__ float As[16][33];  // [k][m]
  __shared__ float Bs[16][33];  // [k][n]
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int64_t m0 = (int64_t)blockIdx.y * 32, n0 = (int64_t)blockIdx.x * 32;
  float acc[2][2] = {{0.f, 0.f}, {0.f, 0.f}};
  for (int64_t k0 = 0; k0 < K; k0 += 16) {
    for (int e = threadIdx.x; e < 512; e += 256) {
      const int kk = e & 15, mm = e >> 4;
      const int64_t gm = m0 + mm, gn = n0 + mm, gk = k0 + kk;
      As[kk][mm] = (gm < M && gk < K) ? (float)A[gm * a_rs + gk * a_cs] : 0.f;
      Bs[kk][mm] = (gn < N && gk < K) ? (float)B[gk * b_rs + gn * b_cs] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      const float a0 = As[kk][ty], a1 = As[kk][ty + 16];
      const float b0 = Bs[kk][tx], b1 = Bs[kk][tx + 16];
      acc[0][0] += a0 * b0; acc[0][1] += a0 * b1;
      acc[1][0] += a1 * b0; acc[1][1] += a1 * b1;
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t gm = m0 + ty + 16 * i, gn = n0 + tx + 16 * j;
      if (gm < M && gn < N) {
        float v = acc[i][j];
        if (R) v += (float)R[gm * ldr + gn];
        if (accumulate) v += (float)C[gm * ldc + gn];
        C[gm * ldc + gn] = (TC)v;
      }
    }
}

int launch_gemm_generic(int dtype, int mode, int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                        const void* B, int64_t ldb, void* C, int64_t ldc, int c_dtype, int accumulate,
                        const void* R, int64_t ldr, hipStream_t st) {
  if (M == 0 || N == 0) return 0;
  int64_t a_rs, a_cs, b_rs, b_cs;
  if (mode == GEMM_NT) { a_rs = lda; a_cs = 1; b_rs = 1; b_cs = ldb; }
  else if (mode == GEMM_NN) { a_rs = lda; a_cs = 1; b_rs = ldb; b_cs = 1; }
  else { a_rs = 1; a_cs = lda; b_rs = ldb; b_cs = 1; }
  const dim3 grid((unsigned)((N + 31) / 32), (unsigned)((M + 31) / 32));
  if (dtype == DT_BF16) {
    if (c_dtype == DT_BF16)
      hipLaunchKernelGGL((gemm_generic_kernel<bf16_t, bf16_t>), grid, dim3(256), 0, st, M, N, K, (const bf16_t*)A, a_rs, a_cs,
                         (const bf16_t*)B, b_rs, b_cs, (bf16_t*)C, ldc, accumulate, (const bf16_t*)R, ldr);
    else
      hipLaunchKernelGGL((gemm_generic_kernel<bf16_t, float>), grid, dim3(256), 0, st, M, N, K, (const bf16_t*)A, a_rs, a_cs,
                         (const bf16_t*)B, b_rs, b_cs, (float*)C, ldc, accumulate, (const float*)R, ldr);
  } else {
    hipLaunchKernelGGL((gemm_generic_kernel<float, float>), grid, dim3(256), 0, st, M, N, K, (const float*)A, a_rs, a_cs,
                       (const float*)B, b_rs, b_cs, (float*)C, ldc, accumulate, (const float*)R, ldr);
  }
  return (int)hipGetLastError();
}

// =============================================================================== attention
// One wavefront per (batch, head, row).  Scores of the row live in LDS (S floats per wavefront).
constexpr int kGenAttnMaxS = 4096;  // backward: 4 wavefronts x 2 arrays x 4096 x 4 B = 128 KiB of LDS
bool attn_generic_supported(int S, int d) { return S >= 1 && S <= kGenAttnMaxS && d >= 2; }

template <typename T>
__device__ __forceinline__ float dot_d(const T* a, const T* b, int d) {
  float s = 0.f;
  for (int i = 0; i < d; ++i) s += (float)a[i] * (float)b[i];
  return s;
}

// o[t] = sum_{u<=t} softmax_u(q[t].k[u]/sqrt(d)) v[u];  lse[t] = log sum_u exp(score)
template <typename T>
__global__ void __launch_bounds__(256) attn_fwd_generic_kernel(const T* __restrict__ qkv, T* __restrict__ o,
                                                               float* __restrict__ lse, int B, int S, int nh, int d) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* p = lds + (size_t)wave * S;
  const int64_t gid = (int64_t)blockIdx.x * 4 + wave;  // (b, h, t)
  const int64_t total = (int64_t)B * nh * S;
  if (gid >= total) return;
  const int t = (int)(gid % S);
  const int h = (int)((gid / S) % nh);
  const int b = (int)(gid / ((int64_t)S * nh));
  const int64_t H = (int64_t)nh * d, ld = 3 * H;
  const T* qrow = qkv + ((int64_t)b * S + t) * ld + (int64_t)h * d;
  const T* kbase = qkv + (int64_t)b * S * ld + H + (int64_t)h * d;
  const T* vbase = kbase + H;
  const float scale = 1.0f / sqrtf((float)d);
  float m = -INFINITY;
  for (int u = lane; u <= t; u += 64) {
    const float s = dot_d(qrow, kbase + (int64_t)u * ld, d) * scale;
    p[u] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float z = 0.f;
  for (int u = lane; u <= t; u += 64) {
    const float e = expf(p[u] - m);
    p[u] = e;
    z += e;
  }
  z = wave_sum(z);
  if (lane == 0) lse[((int64_t)b * nh + h) * S + t] = m + logf(z);
  const float inv = 1.0f / z;
  // LDS writes above are read by other lanes of the same wavefront below
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0)
  __builtin_amdgcn_wave_barrier();
  T* orow = o + ((int64_t)b * S + t) * H + (int64_t)h * d;
  for (int i = lane; i < d; i += 64) {
    float acc = 0.f;
    for (int u = 0; u <= t; ++u) acc += p[u] * (float)vbase[(int64_t)u * ld + i];
    orow[i] = (T)(acc * inv);
  }
}

// dq[t] = (1/sqrt d) sum_{u<=t} dS[t,u] k[u],  dS = P (dP - D),  P = exp(score - lse),  dP = do[t].v[u]
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dq_generic_kernel(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                                  const float* __restrict__ lse, const float* __restrict__ D,
                                                                  T* __restrict__ dqkv, int B, int S, int nh, int d) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* ds = lds + (size_t)wave * S;
  const int64_t gid = (int64_t)blockIdx.x * 4 + wave;
  const int64_t total = (int64_t)B * nh * S;
  if (gid >= total) return;
  const int t = (int)(gid % S);
  const int h = (int)((gid / S) % nh);
  const int b = (int)(gid / ((int64_t)S * nh));
  const int64_t H = (int64_t)nh * d, ld = 3 * H;
  const T* qrow = qkv + ((int64_t)b * S + t) * ld + (int64_t)h * d;
  const T* kbase = qkv + (int64_t)b * S * ld + H + (int64_t)h * d;
  const T* vbase = kbase + H;
  const T* dorow = dO + ((int64_t)b * S + t) * H + (int64_t)h * d;
  const float scale = 1.0f / sqrtf((float)d);
  const float L = lse[((int64_t)b * nh + h) * S + t];
  const float Dt = D[((int64_t)b * nh + h) * S + t];
  for (int u = lane; u <= t; u += 64) {
    const float s = dot_d(qrow, kbase + (int64_t)u * ld, d) * scale;
    const float pr = expf(s - L);
    const float dP = dot_d(dorow, vbase + (int64_t)u * ld, d);
    ds[u] = pr * (dP - Dt);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_wave_barrier();
  T* dqrow = dqkv + ((int64_t)b * S + t) * ld + (int64_t)h * d;
  for (int i = lane; i < d; i += 64) {
    float acc = 0.f;
    for (int u = 0; u <= t; ++u) acc += ds[u] * (float)kbase[(int64_t)u * ld + i];
    dqrow[i] = (T)(acc * scale);
  }
}

// dv[u] = sum_{t>=u} P[t,u] do[t];  dk[u] = (1/sqrt d) sum_{t>=u} dS[t,u] q[t]
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_dkv_generic_kernel(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                                   const float* __restrict__ lse, const float* __restrict__ D,
                                                                   T* __restrict__ dqkv, int B, int S, int nh, int d) {
  extern __shared__ float lds[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* pp = lds + (size_t)wave * 2 * S;
  float* ds = pp + S;
  const int64_t gid = (int64_t)blockIdx.x * 4 + wave;
  const int64_t total = (int64_t)B * nh * S;
  if (gid >= total) return;
  const int u = (int)(gid % S);
  const int h = (int)((gid / S) % nh);
  const int b = (int)(gid / ((int64_t)S * nh));
  const int64_t H = (int64_t)nh * d, ld = 3 * H;
  const T* qbase = qkv + (int64_t)b * S * ld + (int64_t)h * d;
  const T* krow = qbase + H + (int64_t)u * ld;
  const T* vrow = krow + H;
  const T* dobase = dO + (int64_t)b * S * H + (int64_t)h * d;
  const float* Lb = lse + ((int64_t)b * nh + h) * S;
  const float* Db = D + ((int64_t)b * nh + h) * S;
  const float scale = 1.0f / sqrtf((float)d);
  for (int t = u + lane; t < S; t += 64) {
    const float s = dot_d(qbase + (int64_t)t * ld, krow, d) * scale;
    const float pr = expf(s - Lb[t]);
    const float dP = dot_d(dobase + (int64_t)t * H, vrow, d);
    pp[t - u] = pr;
    ds[t - u] = pr * (dP - Db[t]);
  }
  __builtin_amdgcn_s_waitcnt(0xc07f);
  __builtin_amdgcn_wave_barrier();
  T* dkrow = dqkv + ((int64_t)b * S + u) * ld + H + (int64_t)h * d;
  T* dvrow = dkrow + H;
  for (int i = lane; i < d; i += 64) {
    float ak = 0.f, av = 0.f;
    for (int t = u; t < S; ++t) {
      ak += ds[t - u] * (float)qbase[(int64_t)t * ld + i];
      av += pp[t - u] * (float)dobase[(int64_t)t * H + i];
    }
    dkrow[i] = (T)(ak * scale);
    dvrow[i] = (T)av;
  }
}

template <typename T>
static int attn_fwd_generic_t(int B, int S, int nh, int d, const T* qkv, T* o, float* lse, hipStream_t st) {
  const int64_t total = (int64_t)B * nh * S;
  if (total == 0) return 0;
  const size_t lds = (size_t)4 * S * sizeof(float);
  TAW_SET_LDS_LIMIT_ONCE((attn_fwd_generic_kernel<T>), (size_t)4 * kGenAttnMaxS * sizeof(float));
  hipLaunchKernelGGL((attn_fwd_generic_kernel<T>), dim3((unsigned)((total + 3) / 4)), dim3(256), lds, st, qkv, o, lse, B, S, nh, d);
  return (int)hipGetLastError();
}

int launch_attn_fwd_generic(int dtype, int B, int S, int nh, int d, const void* qkv, void* o, float* lse, hipStream_t st) {
  if (dtype == DT_BF16) return attn_fwd_generic_t<bf16_t>(B, S, nh, d, (const bf16_t*)qkv, (bf16_t*)o, lse, st);
  return attn_fwd_generic_t<float>(B, S, nh, d, (const float*)qkv, (float*)o, lse, st);
}

template <typename T>
static int attn_bwd_generic_t(int B, int S, int nh, int d, const T* qkv, const T* dO, const float* lse, const float* D,
                              T* dqkv, hipStream_t st) {
  const int64_t total = (int64_t)B * nh * S;
  if (total == 0) return 0;
  const unsigned grid = (unsigned)((total + 3) / 4);
  size_t lds = (size_t)4 * S * sizeof(float);
  TAW_SET_LDS_LIMIT_ONCE((attn_bwd_dq_generic_kernel<T>), (size_t)4 * kGenAttnMaxS * sizeof(float));
  hipLaunchKernelGGL((attn_bwd_dq_generic_kernel<T>), dim3(grid), dim3(256), lds, st, qkv, dO, lse, D, dqkv, B, S, nh, d);
  int rc = (int)hipGetLastError();
  if (rc) return rc;
  lds *= 2;
  TAW_SET_LDS_LIMIT_ONCE((attn_bwd_dkv_generic_kernel<T>), (size_t)8 * kGenAttnMaxS * sizeof(float));
  hipLaunchKernelGGL((attn_bwd_dkv_generic_kernel<T>), dim3(grid), dim3(256), lds, st, qkv, dO, lse, D, dqkv, B, S, nh, d);
  return (int)hipGetLastError();
}

int launch_attn_bwd_generic(int dtype, int B, int S, int nh, int d, const void* qkv, const void* dO,
                            const float* lse, const float* D, void* dqkv, hipStream_t st) {
  if (dtype == DT_BF16) return attn_bwd_generic_t<bf16_t>(B, S, nh, d, (const bf16_t*)qkv, (const bf16_t*)dO, lse, D, (bf16_t*)dqkv, st);
  return attn_bwd_generic_t<float>(B, S, nh, d, (const float*)qkv, (const float*)dO, lse, D, (float*)dqkv, st);
}

}  // namespace taw
