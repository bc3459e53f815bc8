// Bandwidth-bound kernels of the decoder layer: RMSNorm forward/backward, rotary embedding,
// SwiGLU forward/backward, gradient-shard accumulation, the staging copy, the rotary table and
// the attention-backward row dot product.  Each one streams its operands once with 16-byte
// accesses per lane; reductions stay inside one wavefront (64 lanes) wherever a row fits.
#include "dev_common.h"
#include "taw_internal.h"

namespace taw {

// =============================================================================== RMSNorm forward
// One wavefront per token row; the row stays packed in registers between the sum of squares
// and the scaling, so x is read from HBM exactly once.
template <typename T, int V, int MAXC>
__global__ void __launch_bounds__(256) rmsnorm_fwd_kernel(const T* __restrict__ x, const T* __restrict__ gamma,
                                                          T* __restrict__ out, float* __restrict__ r,
                                                          int64_t rows, int H, float eps) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  const int nch = H / V;
  const T* xr = x + row * (int64_t)H;
  Vec<T, V> c[MAXC];
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int ci = i * 64 + lane;
    if (ci < nch) {
      c[i].load(xr + ci * V);
#pragma unroll
      for (int j = 0; j < V; ++j) { float v = c[i].get(j); ss += v * v; }
    }
  }
  ss = wave_sum(ss);
  const float rr = 1.0f / sqrtf(ss / (float)H + eps);
  if (lane == 0) r[row] = rr;
  T* orow = out + row * (int64_t)H;
#pragma unroll
  for (int i = 0; i < MAXC; ++i) {
    const int ci = i * 64 + lane;
    if (ci < nch) {
      Vec<T, V> g, o;
      g.load(gamma + ci * V);
#pragma unroll
      for (int j = 0; j < V; ++j) o.set(j, c[i].get(j) * rr * g.get(j));
      o.store(orow + ci * V);
    }
  }
}

// =============================================================================== RMSNorm backward
// c = dout*gamma;  dz = r c - z r^3 mean(c z) (+ dres);  dgamma_i = sum_t dout[t,i] z[t,i] r_t.
// A wavefront walks rows with a grid stride; a row's z and dout stay packed in registers between
// the dot product and the write of dz.  The wavefront's share of the dgamma column sums lives in
// its own LDS array (registers would not hold H/64 more floats per lane for wide rows), gamma is
// read from LDS too.  The four arrays of a workgroup are then summed in a fixed order and written
// as one partial row, which colsum_kernel reduces.  No atomics: results are reproducible.
//
// REG = true (rows whose sums and packed z, dout take at most 128 registers per lane): the wavefront's column sums stay in registers
// instead (no LDS read-modify-write per element, and LDS holds only gamma and one row of floats); the
// wavefronts then add their sums to that row one after the other, in the same fixed order.
template <typename T, int V, int MAXC, bool REG>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(REG ? 2 : 1))) rmsnorm_bwd_kernel(const T* __restrict__ dout, const T* __restrict__ z,
                                                          const float* __restrict__ r, const T* __restrict__ gamma,
                                                          const T* __restrict__ dres, T* __restrict__ dz,
                                                          float* __restrict__ partials, int64_t rows, int H) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds_norm[];
  constexpr int NACC = REG ? 1 : 4;
  float* lds_acc = reinterpret_cast<float*>(lds_norm);               // [NACC][H]
  T* lds_g = reinterpret_cast<T*>(lds_acc + NACC * (size_t)H);       // [H]
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int nch = H / V;
  float* my_acc = lds_acc + (REG ? 0 : (size_t)wave * H);
  float racc[REG ? MAXC * V : 1];
  for (int c = threadIdx.x; c < H; c += 256) lds_g[c] = gamma[c];
  if (REG) {
#pragma unroll
    for (int i = 0; i < (REG ? MAXC * V : 1); ++i) racc[i] = 0.f;
  } else {
    for (int c = lane; c < H; c += 64) my_acc[c] = 0.f;
  }
  __syncthreads();
  const float invH = 1.0f / (float)H;
  for (int64_t row = (int64_t)blockIdx.x * 4 + wave; row < rows; row += (int64_t)gridDim.x * 4) {
    const int64_t base = row * (int64_t)H;
    Vec<T, V> zc[MAXC], dc[MAXC], rs[MAXC];      // the residual gradient is fetched with the row: one memory round trip per row
    float dot = 0.f;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int ci = i * 64 + lane;
      if (ci < nch) {
        zc[i].load_nt(z + base + ci * V);              // each operand is streamed through once
        dc[i].load_nt(dout + base + ci * V);
        if (dres) rs[i].load_nt(dres + base + ci * V);
      }
    }
    const float rr = r[row];
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int ci = i * 64 + lane;
      if (ci < nch) {
        Vec<T, V> g;
        g.load(lds_g + ci * V);
        float* ap = my_acc + ci * V;
#pragma unroll
        for (int j = 0; j < V; ++j) {
          const float zz = zc[i].get(j), dd = dc[i].get(j);
          dot += dd * g.get(j) * zz;
          if (REG) racc[REG ? i * V + j : 0] += dd * zz * rr;
          else ap[j] += dd * zz * rr;
        }
      }
    }
    // only the packed row crosses the reduction
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      zc[i].pin();
      dc[i].pin();
    }
    dot = wave_sum(dot);
    const float coef = rr * rr * rr * dot * invH;
#pragma unroll
    for (int i = 0; i < MAXC; ++i) {
      const int ci = i * 64 + lane;
      if (ci < nch) {
        Vec<T, V> o, g;
        g.load(lds_g + ci * V);
#pragma unroll
        for (int j = 0; j < V; ++j) {
          float v = rr * dc[i].get(j) * g.get(j) - zc[i].get(j) * coef;
          if (dres) v += rs[i].get(j);
          o.set(j, v);
        }
        o.store_nt(dz + base + ci * V);
      }
    }
  }
  float* prow = partials + (int64_t)blockIdx.x * H;
  if (REG) {
    // ((w0 + w1) + w2) + w3, each wavefront adding its registers to the shared row in turn
    for (int w = 0; w < 4; ++w) {
      if (wave == w) {
#pragma unroll
        for (int i = 0; i < MAXC; ++i) {
          const int ci = i * 64 + lane;
          if (ci < nch) {
#pragma unroll
            for (int j = 0; j < V; ++j) {
              const float a = racc[REG ? i * V + j : 0];
              my_acc[ci * V + j] = w == 0 ? a : my_acc[ci * V + j] + a;
            }
          }
        }
      }
      __syncthreads();
    }
    for (int c = threadIdx.x; c < H; c += 256) prow[c] = lds_acc[c];
    return;
  }
  __syncthreads();
  // fixed-order sum of the four wavefronts' column sums
  for (int c = threadIdx.x; c < H; c += 256)
    prow[c] = ((lds_acc[c] + lds_acc[(size_t)H + c]) + lds_acc[2 * (size_t)H + c]) + lds_acc[3 * (size_t)H + c];
}

// out[c] (=|+=) sum_p partials[p][c].  A workgroup owns 64 columns: thread (q = tid & 15, g = tid >> 4)
// sums rows g, g + 16, ... of columns 4q .. 4q + 3 (16-byte loads, a 256-byte row segment per 16
// threads), then the 16 row groups are added in a fixed order through LDS: reproducible, no atomics.
__global__ void __launch_bounds__(256) colsum_kernel(const float* __restrict__ partials, int np, int H,
                                                     float* __restrict__ out, int accumulate) {
  __shared__ float red[16][64];
  const int q = threadIdx.x & 15, g = threadIdx.x >> 4;
  const int c0 = blockIdx.x * 64 + 4 * q;
  float s[4] = {0.f, 0.f, 0.f, 0.f};
  if (c0 + 3 < H && (H & 3) == 0) {
    for (int p = g; p < np; p += 16) {
      const f32x4_t v = *reinterpret_cast<const f32x4_t*>(partials + (int64_t)p * H + c0);
#pragma unroll
      for (int j = 0; j < 4; ++j) s[j] += v[j];
    }
  } else {
    for (int p = g; p < np; p += 16)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (c0 + j < H) s[j] += partials[(int64_t)p * H + c0 + j];
  }
#pragma unroll
  for (int j = 0; j < 4; ++j) red[g][4 * q + j] = s[j];
  __syncthreads();
  if (threadIdx.x < 64) {
    const int c = blockIdx.x * 64 + threadIdx.x;
    if (c < H) {
      float t = 0.f;
#pragma unroll
      for (int gg = 0; gg < 16; ++gg) t += red[gg][threadIdx.x];
      out[c] = accumulate ? out[c] + t : t;
    }
  }
}

// =============================================================================== rotary table
// table[p][i] = (cos, sin)(p * theta^(-2i/d)), evaluated in fp64 (fp32 sin/cos lose accuracy at
// arguments of order 3e4), stored fp32.
__global__ void __launch_bounds__(256) rope_table_kernel(float* __restrict__ table, int S, int half, double theta, int d) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)S * half) return;
  const int p = (int)(idx / half), i = (int)(idx % half);
  const double inv_freq = exp(-(2.0 * (double)i / (double)d) * log(theta));
  const double ang = (double)p * inv_freq;
  table[2 * idx] = (float)cos(ang);
  table[2 * idx + 1] = (float)sin(ang);
}

// =============================================================================== rotary embedding
// In place on columns [0, ncols) of z[B*S, ld].  Adjacent pairs (2i, 2i+1) of every head:
// (a, b) -> (a cos - b sin, a sin + b cos); inverse rotates by the negative angle.
template <typename T, int V>
__global__ void __launch_bounds__(256) rope_kernel(T* __restrict__ z, int64_t ld, int64_t rows, int S, int ncols,
                                                   int d, const float* __restrict__ table, int inverse) {
  const int cpr = ncols / V;  // chunks per row
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int col = (int)(idx % cpr) * V;
  const int p = (int)(row % S);
  T* ptr = z + row * ld + col;
  Vec<T, V> v;
  v.load(ptr);
  const int half = d / 2;
  const float* tb = table + ((int64_t)p * half + (col % d) / 2) * 2;
  Vec<T, V> o;
#pragma unroll
  for (int j = 0; j < V; j += 2) {
    const float c = tb[j], s = inverse ? -tb[j + 1] : tb[j + 1];
    const float a = v.get(j), b = v.get(j + 1);
    o.set(j, a * c - b * s);
    o.set(j + 1, a * s + b * c);
  }
  o.store(ptr);
}

// scalar-pair variant for head dims that are not a multiple of the vector width
template <typename T>
__global__ void __launch_bounds__(256) rope_pair_kernel(T* __restrict__ z, int64_t ld, int64_t rows, int S, int ncols,
                                                        int d, const float* __restrict__ table, int inverse) {
  const int ppr = ncols / 2;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * ppr) return;
  const int64_t row = idx / ppr;
  const int col = (int)(idx % ppr) * 2;
  const int p = (int)(row % S);
  const float* tb = table + ((int64_t)p * (d / 2) + (col % d) / 2) * 2;
  const float c = tb[0], s = inverse ? -tb[1] : tb[1];
  T* ptr = z + row * ld + col;
  const float a = (float)ptr[0], b = (float)ptr[1];
  ptr[0] = (T)(a * c - b * s);
  ptr[1] = (T)(a * s + b * c);
}

// =============================================================================== SwiGLU
// gu = [gate | up] per row ([T, 2I]);  a = gate * sigmoid(gate) * up.
template <typename T, int V>
__global__ void __launch_bounds__(256) swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ a, int64_t rows, int I) {
  const int cpr = I / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int col = (int)(idx % cpr) * V;
  Vec<T, V> g, u, o;
  g.load_nt(gu + row * 2 * (int64_t)I + col);
  u.load_nt(gu + row * 2 * (int64_t)I + I + col);
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const float gg = g.get(j);
    const float sig = 1.0f / (1.0f + __expf(-gg));
    o.set(j, gg * sig * u.get(j));
  }
  o.store_nt(a + row * (int64_t)I + col);
}

// dg = da u sig (1 + g (1 - sig));  du = da g sig
template <typename T, int V>
__global__ void __launch_bounds__(256) swiglu_bwd_kernel(const T* __restrict__ da, const T* __restrict__ gu,
                                                         T* __restrict__ dgu, int64_t rows, int I) {
  const int cpr = I / V;
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * cpr) return;
  const int64_t row = idx / cpr;
  const int col = (int)(idx % cpr) * V;
  Vec<T, V> g, u, d, og, ou;
  g.load_nt(gu + row * 2 * (int64_t)I + col);
  u.load_nt(gu + row * 2 * (int64_t)I + I + col);
  d.load_nt(da + row * (int64_t)I + col);
#pragma unroll
  for (int j = 0; j < V; ++j) {
    const float gg = g.get(j), dd = d.get(j);
    const float sig = 1.0f / (1.0f + __expf(-gg));
    og.set(j, dd * u.get(j) * sig * (1.0f + gg * (1.0f - sig)));
    ou.set(j, dd * gg * sig);
  }
  og.store_nt(dgu + row * 2 * (int64_t)I + col);
  ou.store_nt(dgu + row * 2 * (int64_t)I + I + col);
}

// =============================================================================== gradient accumulation
// G[i] += scale * g[i].  A workgroup takes kAccumRows consecutive rows of 256 x 16 bytes of G, once: all of
// its loads are issued before the first store, and a workgroup's traffic stays inside a few DRAM pages
// (a grid-stride loop over the same data, one vector per lane per trip, reaches two thirds of this rate).
// Streamed once: non-temporal accesses (12 % faster than leaving the lines in the caches).
constexpr int kAccumRows = 4;
template <typename TS>
__global__ void __launch_bounds__(256) grad_accum_kernel(float* __restrict__ G, const TS* __restrict__ g, size_t n, float scale) {
  const size_t nvec = n / 4;
  const size_t i0 = (size_t)blockIdx.x * (kAccumRows * 256) + threadIdx.x;
  auto src = [&](size_t i) -> f32x4_t {
    if constexpr (sizeof(TS) == 4) {
      return __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(g + 4 * i));
    } else {
      const bf16x4_t s = __builtin_nontemporal_load(reinterpret_cast<const bf16x4_t*>(g + 4 * i));
      return f32x4_t{(float)s[0], (float)s[1], (float)s[2], (float)s[3]};
    }
  };
  if (i0 + (kAccumRows - 1) * 256 < nvec) {
    f32x4_t acc[kAccumRows], s[kAccumRows];
#pragma unroll
    for (int u = 0; u < kAccumRows; ++u) {
      acc[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(G + 4 * (i0 + u * 256)));
      s[u] = src(i0 + u * 256);
    }
#pragma unroll
    for (int u = 0; u < kAccumRows; ++u) {
      acc[u] += s[u] * scale;
      __builtin_nontemporal_store(acc[u], reinterpret_cast<f32x4_t*>(G + 4 * (i0 + u * 256)));
    }
  } else {
    for (int u = 0; u < kAccumRows; ++u) {
      const size_t i = i0 + u * 256;
      if (i < nvec) {
        f32x4_t acc = *reinterpret_cast<const f32x4_t*>(G + 4 * i);
        acc += src(i) * scale;
        *reinterpret_cast<f32x4_t*>(G + 4 * i) = acc;
      }
    }
  }
  // tail (n not a multiple of 4)
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const size_t i = nvec * 4 + threadIdx.x;
    G[i] += (float)g[i] * scale;
  }
}

// =============================================================================== owner-side optimizer step
// AdamW with decoupled weight decay over a whole shard, one pass: reads G, m, v and the fp32 master
// weights, writes m, v, the master weights and the weight chunk in its storage type; optionally
// leaves G zeroed for the next mini-batch.  b1c = 1 - beta1^t, b2c = 1 - beta2^t come from the host.
constexpr int kAdamRows = 2;
template <typename TW>
__global__ void __launch_bounds__(256) adamw_kernel(TW* __restrict__ chunk, float* __restrict__ master, float* __restrict__ m,
                                                     float* __restrict__ v, float* __restrict__ G, size_t n, float lr, float beta1,
                                                     float beta2, float eps, float wd, float b1c, float b2c, float gscale,
                                                     int zero_grad) {
  const size_t nvec = n / 4;
  auto upd = [&](float g, float& mm, float& vv, float& w) {
    g *= gscale;
    mm = beta1 * mm + (1.f - beta1) * g;
    vv = beta2 * vv + (1.f - beta2) * g * g;
    const float mh = mm / b1c, vh = vv / b2c;
    w = w - lr * (mh / (sqrtf(vh) + eps) + wd * w);
  };
  // a workgroup takes kAdamRows consecutive rows of 256 x 16 bytes of each array, once (as grad_accum_kernel does)
  const size_t i0 = (size_t)blockIdx.x * (kAdamRows * 256) + threadIdx.x;
  f32x4_t g4[kAdamRows], m4[kAdamRows], v4[kAdamRows], w4[kAdamRows];
  bool live[kAdamRows];
#pragma unroll
  for (int u = 0; u < kAdamRows; ++u) {
    const size_t i = i0 + u * 256;
    live[u] = i < nvec;
    if (live[u]) {
      g4[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(G + 4 * i));
      m4[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(m + 4 * i));
      v4[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(v + 4 * i));
      w4[u] = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(master + 4 * i));
    }
  }
#pragma unroll
  for (int u = 0; u < kAdamRows; ++u) {
    const size_t i = i0 + u * 256;
    if (!live[u]) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float mm = m4[u][j], vv = v4[u][j], w = w4[u][j];
      upd(g4[u][j], mm, vv, w);
      m4[u][j] = mm; v4[u][j] = vv; w4[u][j] = w;
    }
    __builtin_nontemporal_store(m4[u], reinterpret_cast<f32x4_t*>(m + 4 * i));
    __builtin_nontemporal_store(v4[u], reinterpret_cast<f32x4_t*>(v + 4 * i));
    __builtin_nontemporal_store(w4[u], reinterpret_cast<f32x4_t*>(master + 4 * i));
    if constexpr (sizeof(TW) == 4) {
      *reinterpret_cast<f32x4_t*>(chunk + 4 * i) = w4[u];       // the chunk is what the next forward reads: ordinary store
    } else {
      bf16x4_t o;
#pragma unroll
      for (int j = 0; j < 4; ++j) o[j] = (bf16_t)w4[u][j];
      *reinterpret_cast<bf16x4_t*>(chunk + 4 * i) = o;
    }
    if (zero_grad) __builtin_nontemporal_store(f32x4_t{0.f, 0.f, 0.f, 0.f}, reinterpret_cast<f32x4_t*>(G + 4 * i));
  }
  if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
    const size_t i = nvec * 4 + threadIdx.x;
    float mm = m[i], vv = v[i], w = master[i];
    upd(G[i], mm, vv, w);
    m[i] = mm; v[i] = vv; master[i] = w;
    chunk[i] = (TW)w;
    if (zero_grad) G[i] = 0.f;
  }
}

// =============================================================================== staging copy
// HBM-to-HBM copy of a weight chunk.  A modest grid on purpose: it runs beside the layer's
// compute kernels on another stream and should take few compute units away from them.
__global__ void __launch_bounds__(256) stage_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t nvec) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < nvec; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a; dst[i + stride] = b; dst[i + 2 * stride] = c; dst[i + 3 * stride] = d;
  }
  for (; i < nvec; i += stride) dst[i] = src[i];
}

// =============================================================================== attention row dot
// D[b,h,t] = sum_i do[t, h*d+i] * o[t, h*d+i]; one thread group of d/V lanes per (t, h).
template <typename T, int V>
__global__ void __launch_bounds__(256) attn_rowdot_kernel(const T* __restrict__ o, int64_t ld_o, const T* __restrict__ dO,
                                                          int64_t ld_do, float* __restrict__ D, int B, int S, int nh, int d) {
  // one thread per (row, head): small d/V (16 lanes x 8 for d=128) would need a segmented
  // reduction; a single thread reading d contiguous elements keeps 16-byte accesses instead.
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t rows = (int64_t)B * S;
  if (idx >= rows * nh) return;
  // consecutive threads take consecutive rows of one head so the D stores are coalesced
  const int64_t t = idx % rows;
  const int h = (int)(idx / rows);
  const T* po = o + t * ld_o + (int64_t)h * d;
  const T* pd = dO + t * ld_do + (int64_t)h * d;
  float s = 0.f;
  for (int c = 0; c < d; c += V) {
    Vec<T, V> a, b;
    a.load(po + c);
    b.load(pd + c);
#pragma unroll
    for (int j = 0; j < V; ++j) s += a.get(j) * b.get(j);
  }
  const int b_ = (int)(t / S), p = (int)(t % S);
  D[((int64_t)b_ * nh + h) * S + p] = s;
}

// =============================================================================== launchers
static inline int last_err() { return (int)hipGetLastError(); }

template <typename T> static constexpr int vw() { return VecWidth<T>::value; }

bool rmsnorm_supported(int dtype, int H) {
  const int V = dtype == DT_BF16 ? 8 : 4;
  if (H <= 0) return false;
  if (H % V == 0) return H / V <= 64 * 16;
  return H <= 64 * 16;
}

template <typename T, int V>
static int rmsnorm_fwd_dispatch(int64_t T_, int H, const T* x, const T* g, float eps, T* out, float* r, hipStream_t st) {
  const int nch = H / V;
  const unsigned grid = (unsigned)((T_ + 3) / 4);
#define TAW_RN_FWD(MAXC) hipLaunchKernelGGL((rmsnorm_fwd_kernel<T, V, MAXC>), dim3(grid), dim3(256), 0, st, x, g, out, r, T_, H, eps)
  if (nch <= 64) TAW_RN_FWD(1);
  else if (nch <= 128) TAW_RN_FWD(2);
  else if (nch <= 256) TAW_RN_FWD(4);
  else if (nch <= 512) TAW_RN_FWD(8);
  else TAW_RN_FWD(16);
#undef TAW_RN_FWD
  return last_err();
}

int launch_rmsnorm_fwd(int dtype, int64_t T_, int H, const void* x, const void* gamma, float eps, void* out,
                       float* r, hipStream_t st) {
  if (T_ == 0) return 0;
  if (dtype == DT_BF16) {
    if (H % 8 == 0) return rmsnorm_fwd_dispatch<bf16_t, 8>(T_, H, (const bf16_t*)x, (const bf16_t*)gamma, eps, (bf16_t*)out, r, st);
    return rmsnorm_fwd_dispatch<bf16_t, 1>(T_, H, (const bf16_t*)x, (const bf16_t*)gamma, eps, (bf16_t*)out, r, st);
  }
  if (H % 4 == 0) return rmsnorm_fwd_dispatch<float, 4>(T_, H, (const float*)x, (const float*)gamma, eps, (float*)out, r, st);
  return rmsnorm_fwd_dispatch<float, 1>(T_, H, (const float*)x, (const float*)gamma, eps, (float*)out, r, st);
}

static constexpr int kNormBwdGrid = 512;      // two workgroups per CU: all resident at once where the register variant runs
int rmsnorm_bwd_partial_rows() { return kNormBwdGrid; }

template <typename T, int V>
static int rmsnorm_bwd_dispatch(int64_t T_, int H, const T* dout, const T* z, const float* r, const T* g,
                                const T* dres, T* dz, float* dgamma, int accumulate, float* partials, hipStream_t st) {
  const int nch = H / V;
  int grid = (int)((T_ + 3) / 4);
  if (grid > kNormBwdGrid) grid = kNormBwdGrid;
  // column sums in registers for rows up to 4096 bf16 / 2048 fp32 elements, in LDS (<= 144 KiB for the widest supported row) beyond
#define TAW_RN_BWD(MAXC, REG)                                                                                                \
  do {                                                                                                                     \
    const size_t lds = ((REG) ? 1 : 4) * (size_t)H * sizeof(float) + (size_t)H * sizeof(T);                                  \
    /* the widest row this instantiation takes is MAXC * 64 * V elements */                                                  \
    TAW_SET_LDS_LIMIT_ONCE((rmsnorm_bwd_kernel<T, V, MAXC, REG>), (((REG) ? 1 : 4) * sizeof(float) + sizeof(T)) * (size_t)(MAXC) * 64 * V); \
    hipLaunchKernelGGL((rmsnorm_bwd_kernel<T, V, MAXC, REG>), dim3(grid), dim3(256), lds, st, dout, z, r, g, dres, dz, partials, T_, H); \
  } while (0)
  // registers per lane: the sums (one per element) and the packed z and dout rows
#define TAW_RN_REG(MAXC) ((MAXC) * V * (4 + 2 * (int)sizeof(T)) <= 512)
  if (nch <= 64) TAW_RN_BWD(1, TAW_RN_REG(1));
  else if (nch <= 128) TAW_RN_BWD(2, TAW_RN_REG(2));
  else if (nch <= 256) TAW_RN_BWD(4, TAW_RN_REG(4));
  else if (nch <= 512) TAW_RN_BWD(8, TAW_RN_REG(8));
  else TAW_RN_BWD(16, TAW_RN_REG(16));
#undef TAW_RN_REG
#undef TAW_RN_BWD
  int e = last_err();
  if (e) return e;
  hipLaunchKernelGGL(colsum_kernel, dim3((H + 63) / 64), dim3(256), 0, st, partials, grid, H, dgamma, accumulate);
  return last_err();
}

int launch_rmsnorm_bwd(int dtype, int64_t T_, int H, const void* dout, const void* z, const float* r,
                       const void* gamma, const void* dres, void* dz, float* dgamma, int accumulate,
                       float* partials, hipStream_t st) {
  if (T_ == 0) return 0;
  if (dtype == DT_BF16) {
    if (H % 8 == 0)
      return rmsnorm_bwd_dispatch<bf16_t, 8>(T_, H, (const bf16_t*)dout, (const bf16_t*)z, r, (const bf16_t*)gamma,
                                             (const bf16_t*)dres, (bf16_t*)dz, dgamma, accumulate, partials, st);
    return rmsnorm_bwd_dispatch<bf16_t, 1>(T_, H, (const bf16_t*)dout, (const bf16_t*)z, r, (const bf16_t*)gamma,
                                           (const bf16_t*)dres, (bf16_t*)dz, dgamma, accumulate, partials, st);
  }
  if (H % 4 == 0)
    return rmsnorm_bwd_dispatch<float, 4>(T_, H, (const float*)dout, (const float*)z, r, (const float*)gamma,
                                          (const float*)dres, (float*)dz, dgamma, accumulate, partials, st);
  return rmsnorm_bwd_dispatch<float, 1>(T_, H, (const float*)dout, (const float*)z, r, (const float*)gamma,
                                        (const float*)dres, (float*)dz, dgamma, accumulate, partials, st);
}

int launch_rope_table(int S, int head_dim, double theta, float* table, hipStream_t st) {
  const int half = head_dim / 2;
  const int64_t n = (int64_t)S * half;
  if (n == 0) return 0;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, table, S, half, theta, head_dim);
  return last_err();
}

template <typename T>
static int rope_dispatch(int B, int S, int ncols, int d, T* z, int64_t ld, const float* table, int inverse, hipStream_t st) {
  constexpr int V = VecWidth<T>::value;
  const int64_t rows = (int64_t)B * S;
  if (rows == 0 || ncols == 0) return 0;
  if (d % V == 0 && ld % V == 0) {
    const int64_t n = rows * (ncols / V);
    hipLaunchKernelGGL((rope_kernel<T, V>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, z, ld, rows, S, ncols, d, table, inverse);
  } else {
    const int64_t n = rows * (ncols / 2);
    hipLaunchKernelGGL((rope_pair_kernel<T>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, z, ld, rows, S, ncols, d, table, inverse);
  }
  return last_err();
}

int launch_rope(int dtype, int B, int S, int ncols, int head_dim, void* z, int64_t ld, const float* table,
                int inverse, hipStream_t st) {
  if (dtype == DT_BF16) return rope_dispatch<bf16_t>(B, S, ncols, head_dim, (bf16_t*)z, ld, table, inverse, st);
  return rope_dispatch<float>(B, S, ncols, head_dim, (float*)z, ld, table, inverse, st);
}

template <typename T>
static int swiglu_dispatch(bool bwd, int64_t T_, int I, const T* da, const T* gu, T* out, hipStream_t st) {
  constexpr int VW = VecWidth<T>::value;
  if (T_ == 0 || I == 0) return 0;
  if (I % VW == 0) {
    const int64_t n = T_ * (I / VW);
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (bwd) hipLaunchKernelGGL((swiglu_bwd_kernel<T, VW>), dim3(grid), dim3(256), 0, st, da, gu, out, T_, I);
    else hipLaunchKernelGGL((swiglu_fwd_kernel<T, VW>), dim3(grid), dim3(256), 0, st, gu, out, T_, I);
  } else {
    const int64_t n = T_ * I;
    const unsigned grid = (unsigned)((n + 255) / 256);
    if (bwd) hipLaunchKernelGGL((swiglu_bwd_kernel<T, 1>), dim3(grid), dim3(256), 0, st, da, gu, out, T_, I);
    else hipLaunchKernelGGL((swiglu_fwd_kernel<T, 1>), dim3(grid), dim3(256), 0, st, gu, out, T_, I);
  }
  return last_err();
}

int launch_swiglu_fwd(int dtype, int64_t T_, int I, const void* gu, void* a, hipStream_t st) {
  if (dtype == DT_BF16) return swiglu_dispatch<bf16_t>(false, T_, I, nullptr, (const bf16_t*)gu, (bf16_t*)a, st);
  return swiglu_dispatch<float>(false, T_, I, nullptr, (const float*)gu, (float*)a, st);
}
int launch_swiglu_bwd(int dtype, int64_t T_, int I, const void* da, const void* gu, void* dgu, hipStream_t st) {
  if (dtype == DT_BF16) return swiglu_dispatch<bf16_t>(true, T_, I, (const bf16_t*)da, (const bf16_t*)gu, (bf16_t*)dgu, st);
  return swiglu_dispatch<float>(true, T_, I, (const float*)da, (const float*)gu, (float*)dgu, st);
}

int launch_grad_accum(float* G, const void* g, int src_dtype, size_t n, float scale, hipStream_t st) {
  if (n == 0) return 0;
  size_t want = (n / 4 + kAccumRows * 256 - 1) / (kAccumRows * 256);
  if (want == 0) want = 1;      // fewer than 4 elements: the tail lanes of one workgroup
  if (want > 0x7fffffffu) return (int)hipErrorInvalidValue;
  const unsigned grid = (unsigned)want;
  if (src_dtype == DT_BF16) hipLaunchKernelGGL((grad_accum_kernel<bf16_t>), dim3(grid), dim3(256), 0, st, G, (const bf16_t*)g, n, scale);
  else hipLaunchKernelGGL((grad_accum_kernel<float>), dim3(grid), dim3(256), 0, st, G, (const float*)g, n, scale);
  return last_err();
}

int launch_adamw(int w_dtype, void* chunk, float* master, float* m, float* v, float* G, size_t n, float lr, float beta1, float beta2,
                 float eps, float wd, float b1c, float b2c, float gscale, int zero_grad, hipStream_t st) {
  if (n == 0) return 0;
  size_t want = (n / 4 + kAdamRows * 256 - 1) / (kAdamRows * 256);
  if (want == 0) want = 1;
  if (want > 0x7fffffffu) return (int)hipErrorInvalidValue;
  const unsigned grid = (unsigned)want;
  if (w_dtype == DT_BF16)
    hipLaunchKernelGGL((adamw_kernel<bf16_t>), dim3(grid), dim3(256), 0, st, (bf16_t*)chunk, master, m, v, G, n, lr, beta1, beta2, eps, wd, b1c, b2c, gscale, zero_grad);
  else
    hipLaunchKernelGGL((adamw_kernel<float>), dim3(grid), dim3(256), 0, st, (float*)chunk, master, m, v, G, n, lr, beta1, beta2, eps, wd, b1c, b2c, gscale, zero_grad);
  return last_err();
}

int launch_stage_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
  const size_t nvec = bytes / 16;
  if (nvec == 0) return 0;
  size_t want = (nvec + 255) / 256;
  const unsigned grid = (unsigned)(want > 256 ? 256 : want);
  hipLaunchKernelGGL(stage_copy_kernel, dim3(grid), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, nvec);
  return last_err();
}

int launch_attn_rowdot(int dtype, int B, int S, int nh, int d, const void* o, int64_t ld_o, const void* dO,
                       int64_t ld_do, float* D, hipStream_t st) {
  const int64_t n = (int64_t)B * S * nh;
  if (n == 0) return 0;
  const unsigned grid = (unsigned)((n + 255) / 256);
  if (dtype == DT_BF16) {
    if (d % 8 == 0 && ld_o % 8 == 0 && ld_do % 8 == 0)
      hipLaunchKernelGGL((attn_rowdot_kernel<bf16_t, 8>), dim3(grid), dim3(256), 0, st, (const bf16_t*)o, ld_o, (const bf16_t*)dO, ld_do, D, B, S, nh, d);
    else
      hipLaunchKernelGGL((attn_rowdot_kernel<bf16_t, 1>), dim3(grid), dim3(256), 0, st, (const bf16_t*)o, ld_o, (const bf16_t*)dO, ld_do, D, B, S, nh, d);
  } else {
    if (d % 4 == 0 && ld_o % 4 == 0 && ld_do % 4 == 0)
      hipLaunchKernelGGL((attn_rowdot_kernel<float, 4>), dim3(grid), dim3(256), 0, st, (const float*)o, ld_o, (const float*)dO, ld_do, D, B, S, nh, d);
    else
      hipLaunchKernelGGL((attn_rowdot_kernel<float, 1>), dim3(grid), dim3(256), 0, st, (const float*)o, ld_o, (const float*)dO, ld_do, D, B, S, nh, d);
  }
  return last_err();
}

}  // namespace taw
