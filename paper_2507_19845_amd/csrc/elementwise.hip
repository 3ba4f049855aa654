// HBM-bound kernels of the stage: LayerNorm forward/backward (with the residual
// gradient and the bias gradient of the preceding linear layer folded in), column sums
// for the other bias gradients, and the fixed-order reduction of per-workgroup partial
// sums.  One workgroup per token row at a time (256 threads forward, 512 backward),
// 16-byte loads, the row cached in registers, fp32 statistics.
#include "../../include/gpt_stage.h"

#include <mutex>

#include "kernels.hpp"

namespace gpts {

constexpr int kLnThreads = 256;

// 8 consecutive elements <-> fp32 registers (one 16-byte access for bf16, two for fp32)
__device__ __forceinline__ void load8(const float* p, float (&v)[8]) {
  const f32x4 a = *reinterpret_cast<const f32x4*>(p), b = *reinterpret_cast<const f32x4*>(p + 4);
#pragma unroll
  for (int e = 0; e < 4; ++e) { v[e] = a[e]; v[4 + e] = b[e]; }
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8]) {
  const bf16x8 a = *reinterpret_cast<const bf16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
}
__device__ __forceinline__ void load8(const f16* p, float (&v)[8]) {
  const f16x8 a = *reinterpret_cast<const f16x8*>(p);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = (float)a[e];
}
__device__ __forceinline__ void store8(f16* p, const float (&v)[8]) {
  f16x8 a;
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = sat_f16(v[e]);
  *reinterpret_cast<f16x8*>(p) = a;
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8]) {
  f32x4 a, b;
#pragma unroll
  for (int e = 0; e < 4; ++e) { a[e] = v[e]; b[e] = v[4 + e]; }
  *reinterpret_cast<f32x4*>(p) = a;
  *reinterpret_cast<f32x4*>(p + 4) = b;
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8]) {
  bf16x8 a;
#pragma unroll
  for (int e = 0; e < 8; ++e) a[e] = (bf16)v[e];
  *reinterpret_cast<bf16x8*>(p) = a;
}

// ----------------------------------------------------------------- LN fwd ----
// Per token: mu = mean(x), var = mean((x-mu)^2), r = 1/sqrt(var+eps),
// out = (x-mu) r gamma + beta.  TX = type of x (the residual stream, fp32 inside
// bf16 stages), T = type of gamma/beta, TO = type of out (T, or fp16 when the forward
// activations of a bf16 stage are kept in fp16).  NCH = 8-element chunks per thread.
template <typename TX, typename T, typename TO, int NCH>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_kernel(
    const TX* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
    TO* __restrict__ out, float* __restrict__ mean, float* __restrict__ rstd, int H, float eps) {
  __shared__ float red[2][kLnThreads / kWave];
  const int row = blockIdx.x;
  const int nvec = H / 8;
  const TX* xr = x + (size_t)row * H;
  float xv[NCH][8];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
      load8(xr + (size_t)i * 8, xv[c]);
#pragma unroll
      for (int e = 0; e < 8; ++e) s += xv[c][e];
    }
  }
  const float mu = block_sum<kLnThreads / kWave>(s, red[0]) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float d = xv[c][e] - mu;
        q += d * d;
      }
    }
  }
  const float var = block_sum<kLnThreads / kWave>(q, red[1]) / (float)H;
  const float r = 1.f / sqrtf(var + eps);
  TO* orow = out + (size_t)row * H;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
      float g[8], b[8], o[8];
      load8(gamma + (size_t)i * 8, g);
      load8(beta + (size_t)i * 8, b);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = (xv[c][e] - mu) * r * g[e] + b[e];
      store8(orow + (size_t)i * 8, o);
    }
  }
  if (threadIdx.x == 0) {
    mean[row] = mu;
    rstd[row] = r;
  }
}

// ----------------------------------------------------------------- LN bwd ----
// Per token, with xhat = (x-mu) r and g = dout*gamma:
//   dx = dres + r (g - mean(g) - xhat mean(g xhat)).
// Each workgroup walks rows blockIdx.x, +gridDim.x, ... and keeps its share of
// sum_t dout*xhat and sum_t dout in registers; it writes them once to
// partial[blockIdx.x][0][H] / [1][H] for the fixed-order reduction below.  With DXSUM it
// also keeps the column sums of dx as stored (partial[blockIdx.x][2][H]): dx is the
// gradient of the output of the linear layer in front of the residual branch, so these
// are that layer's bias gradient, which then needs no pass of its own over dx.
constexpr int kLnBwdThreads = 512;
// workgroups of the backward kernel (measured at 4096 rows of 4096: 256 -> 42.6 us, 512 -> 39.6,
// 1024 -> 50.2: more workgroups put more rows in flight but each writes its own partial sums)
#ifndef GPTS_LN_BWD_BLOCKS
#define GPTS_LN_BWD_BLOCKS 512
#endif
constexpr int kLnBwdMaxBlocks = GPTS_LN_BWD_BLOCKS;

template <typename TX, typename T, int NCH, bool DXSUM>
__global__ __launch_bounds__(kLnBwdThreads) void ln_bwd_kernel(
    const T* __restrict__ dout, const TX* __restrict__ x, const float* __restrict__ mean,
    const float* __restrict__ rstd, const T* __restrict__ gamma, const T* __restrict__ dres,
    T* __restrict__ dx, float* __restrict__ partial, int T_rows, int H) {
  // One barrier per row: the two row sums are reduced together and the LDS slots alternate
  // between rows, so a row's writes cannot overtake the previous row's reads.  The loads of
  // the next row (when the row fits few registers) and of the residual gradient are issued
  // before the barrier, so that memory latency overlaps the reduction.
  constexpr int NT = kLnBwdThreads, NWV = NT / kWave, NPART = DXSUM ? 3 : 2;
  constexpr bool PREFETCH = NCH <= 2;
  __shared__ float red[2][2][NWV];
  const int nvec = H / 8;
  const int wv = threadIdx.x / kWave;
  float dg[NCH][8], db[NCH][8], dc[DXSUM ? NCH : 1][8], gam[NCH][8];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * NT;
    if (i < nvec) load8(gamma + (size_t)i * 8, gam[c]);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      dg[c][e] = db[c][e] = 0.f;
      if constexpr (DXSUM) dc[c][e] = 0.f;
    }
  }
  float dv[NCH][8], xh[NCH][8], dvn[PREFETCH ? NCH : 1][8], xn[PREFETCH ? NCH : 1][8];
  auto load_row = [&](int row, float (&d)[NCH][8], float (&xx)[NCH][8]) {
    const size_t base = (size_t)row * H;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int i = threadIdx.x + c * NT;
      if (i < nvec) {
        load8(dout + base + (size_t)i * 8, d[c]);
        load8(x + base + (size_t)i * 8, xx[c]);
      }
    }
  };
  if constexpr (PREFETCH) {
    if ((int)blockIdx.x < T_rows) load_row(blockIdx.x, dv, xh);
  }
  int buf = 0;
  for (int row = blockIdx.x; row < T_rows; row += gridDim.x, buf ^= 1) {
    if constexpr (!PREFETCH) load_row(row, dv, xh);
    const float mu = mean[row], r = rstd[row];
    const size_t base = (size_t)row * H;
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int i = threadIdx.x + c * NT;
      if (i < nvec) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float d = dv[c][e];
          xh[c][e] = (xh[c][e] - mu) * r;
          const float g = d * gam[c][e];
          s1 += g;
          s2 += g * xh[c][e];
          dg[c][e] += d * xh[c][e];
          db[c][e] += d;
        }
      }
    }
    s1 = wave_sum(s1);
    s2 = wave_sum(s2);
    if ((threadIdx.x & (kWave - 1)) == 0) {
      red[buf][0][wv] = s1;
      red[buf][1][wv] = s2;
    }
    float rs[NCH][8];
    if (dres) {
#pragma unroll
      for (int c = 0; c < NCH; ++c) {
        const int i = threadIdx.x + c * NT;
        if (i < nvec) load8(dres + base + (size_t)i * 8, rs[c]);
      }
    }
    if constexpr (PREFETCH) {
      const int nxt = row + gridDim.x;
      if (nxt < T_rows) load_row(nxt, dvn, xn);
    }
    __syncthreads();
    float m1 = 0.f, m2 = 0.f;
#pragma unroll
    for (int i = 0; i < NWV; ++i) {
      m1 += red[buf][0][i];
      m2 += red[buf][1][i];
    }
    m1 /= (float)H;
    m2 /= (float)H;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int i = threadIdx.x + c * NT;
      if (i < nvec) {
        float o[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          float v = r * (dv[c][e] * gam[c][e] - m1 - xh[c][e] * m2);
          if (dres) v += rs[c][e];
          o[e] = v;
          if constexpr (DXSUM) dc[c][e] += (float)(T)v;
        }
        store8(dx + base + (size_t)i * 8, o);
      }
    }
    if constexpr (PREFETCH) {
#pragma unroll
      for (int c = 0; c < NCH; ++c)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          dv[c][e] = dvn[c][e];
          xh[c][e] = xn[c][e];
        }
    }
  }
  float* pg = partial + (size_t)blockIdx.x * NPART * H;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * NT;
    if (i < nvec) {
      store8(pg + (size_t)i * 8, dg[c]);
      store8(pg + (size_t)H + (size_t)i * 8, db[c]);
      if constexpr (DXSUM) store8(pg + (size_t)2 * H + (size_t)i * 8, dc[c]);
    }
  }
}

// out[i] = (float) in[i]   (stage input -> fp32 residual stream), 8 elements per thread
__global__ __launch_bounds__(256) void widen_kernel(const bf16* __restrict__ in, float* __restrict__ out,
                                                    size_t n8) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  float v[8];
  load8(in + i * 8, v);
  store8(out + i * 8, v);
}

// out[c] += sum_{g<G} partial[g*stride + c], the columns c < N being split at N0 and N1
// over out0 (c < N0), out1 (N0 <= c < N1) and out2 (N1 <= c).  32 columns x 32 row groups per
// workgroup; the row groups are combined through LDS in fixed order, so the result is
// deterministic.
__global__ __launch_bounds__(1024) void reduce_partials_kernel(const float* __restrict__ partial, int G,
                                                               size_t stride, int N, float* __restrict__ out0,
                                                               int N0, float* __restrict__ out1, int N1,
                                                               float* __restrict__ out2) {
  __shared__ float sm[32][33];
  const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cx;
  float s = 0.f;
  if (c < N)
    for (int g = ry; g < G; g += 32) s += partial[(size_t)g * stride + c];
  sm[ry][cx] = s;
  __syncthreads();
  if (ry == 0 && c < N) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 32; ++i) t += sm[i][cx];
    if (c < N0) out0[c] += t;
    else if (c < N1) out1[c - N0] += t;
    else out2[c - N1] += t;
  }
}

// ----------------------------------------------------------------- colsum ----
// partial[blockIdx.y][n] = sum over this workgroup's rows of A[m][n].
// Lane owns one 16-byte column vector; the 4 waves take interleaved rows and
// are combined through LDS in fixed order.
template <typename T>
__global__ __launch_bounds__(256) void colsum_partial_kernel(const T* __restrict__ A,
                                                             float* __restrict__ partial, int M,
                                                             int N) {
  constexpr int V = Vec16<T>::N;
  __shared__ float sm[4][kWave * V];
  const int lane = threadIdx.x & (kWave - 1), w = threadIdx.x / kWave;
  const int col = (blockIdx.x * kWave + lane) * V;
  float acc[V];
#pragma unroll
  for (int e = 0; e < V; ++e) acc[e] = 0.f;
  if (col < N) {
    for (int m = blockIdx.y * 4 + w; m < M; m += gridDim.y * 4) {
      const Vec16<T> v = load16(A + (size_t)m * N + col);
#pragma unroll
      for (int e = 0; e < V; ++e) acc[e] += v.get(e);
    }
  }
#pragma unroll
  for (int e = 0; e < V; ++e) sm[w][lane * V + e] = acc[e];
  __syncthreads();
  if (w == 0 && col < N) {
#pragma unroll
    for (int e = 0; e < V; ++e) {
      const int i = lane * V + e;
      partial[(size_t)blockIdx.y * N + col + e] = sm[0][i] + sm[1][i] + sm[2][i] + sm[3][i];
    }
  }
}

// --------------------------------------------------------------- launchers ----
template <typename TX, typename T, typename TO>
static hipError_t ln_fwd_t(int T_rows, int H, float eps, const TX* x, const T* gamma, const T* beta,
                           TO* out, float* mean, float* rstd, hipStream_t st) {
  const int nch = (H / 8 + kLnThreads - 1) / kLnThreads;
  dim3 g(T_rows), b(kLnThreads);
#define GPTS_LN_FWD(N)                                                                           \
  hipLaunchKernelGGL((ln_fwd_kernel<TX, T, TO, N>), g, b, 0, st, x, gamma, beta, out, mean, rstd, H, eps)
  if (nch <= 1) GPTS_LN_FWD(1);
  else if (nch <= 2) GPTS_LN_FWD(2);
  else if (nch <= 4) GPTS_LN_FWD(4);
  else GPTS_LN_FWD(8);
#undef GPTS_LN_FWD
  return hipGetLastError();
}

hipError_t ln_fwd(int dtype, bool x_f32, int T_rows, int H, float eps, const void* x,
                  const void* gamma, const void* beta, void* out, float* mean, float* rstd,
                  hipStream_t st, bool out_f16) {
  if (dtype == 0) {
    if (out_f16) return hipErrorInvalidValue;
    return ln_fwd_t<float, float, float>(T_rows, H, eps, (const float*)x, (const float*)gamma,
                                         (const float*)beta, (float*)out, mean, rstd, st);
  }
  if (x_f32) {
    if (out_f16)
      return ln_fwd_t<float, bf16, f16>(T_rows, H, eps, (const float*)x, (const bf16*)gamma,
                                        (const bf16*)beta, (f16*)out, mean, rstd, st);
    return ln_fwd_t<float, bf16, bf16>(T_rows, H, eps, (const float*)x, (const bf16*)gamma,
                                       (const bf16*)beta, (bf16*)out, mean, rstd, st);
  }
  if (out_f16) return hipErrorInvalidValue;
  return ln_fwd_t<bf16, bf16, bf16>(T_rows, H, eps, (const bf16*)x, (const bf16*)gamma, (const bf16*)beta,
                                    (bf16*)out, mean, rstd, st);
}

int ln_bwd_blocks(int T_rows) { return T_rows < kLnBwdMaxBlocks ? T_rows : kLnBwdMaxBlocks; }

template <typename TX, typename T>
static hipError_t ln_bwd_t(int T_rows, int H, const T* dout, const TX* x, const float* mean,
                           const float* rstd, const T* gamma, const T* dres, T* dx, float* dgamma,
                           float* dbeta, float* dxsum, float* partial, hipStream_t st) {
  const int nch = (H / 8 + kLnBwdThreads - 1) / kLnBwdThreads;
  const int G = ln_bwd_blocks(T_rows);
  dim3 g(G), b(kLnBwdThreads);
#define GPTS_LN_BWD(N)                                                                                  \
  do {                                                                                                  \
    if (dxsum)                                                                                          \
      hipLaunchKernelGGL((ln_bwd_kernel<TX, T, N, true>), g, b, 0, st, dout, x, mean, rstd, gamma, dres, \
                         dx, partial, T_rows, H);                                                       \
    else                                                                                                \
      hipLaunchKernelGGL((ln_bwd_kernel<TX, T, N, false>), g, b, 0, st, dout, x, mean, rstd, gamma,     \
                         dres, dx, partial, T_rows, H);                                                 \
  } while (0)
  if (nch <= 1) GPTS_LN_BWD(1);
  else if (nch <= 2) GPTS_LN_BWD(2);
  else if (nch <= 4) GPTS_LN_BWD(4);
  else GPTS_LN_BWD(8);
#undef GPTS_LN_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int np = dxsum ? 3 : 2;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((np * H + 31) / 32), dim3(1024), 0, st, partial, G,
                     (size_t)np * H, np * H, dgamma, H, dbeta, 2 * H, dxsum);
  return hipGetLastError();
}

hipError_t ln_bwd(int dtype, bool x_f32, int T_rows, int H, const void* dout, const void* x,
                  const float* mean, const float* rstd, const void* gamma, const void* dres, void* dx,
                  float* dgamma, float* dbeta, float* dxsum, float* partial, hipStream_t st) {
  if (H > 8 * 8 * kLnBwdThreads) return hipErrorInvalidValue;
  if (dtype == 0)
    return ln_bwd_t<float, float>(T_rows, H, (const float*)dout, (const float*)x, mean, rstd,
                                  (const float*)gamma, (const float*)dres, (float*)dx, dgamma, dbeta,
                                  dxsum, partial, st);
  if (x_f32)
    return ln_bwd_t<float, bf16>(T_rows, H, (const bf16*)dout, (const float*)x, mean, rstd,
                                 (const bf16*)gamma, (const bf16*)dres, (bf16*)dx, dgamma, dbeta,
                                 dxsum, partial, st);
  return ln_bwd_t<bf16, bf16>(T_rows, H, (const bf16*)dout, (const bf16*)x, mean, rstd,
                              (const bf16*)gamma, (const bf16*)dres, (bf16*)dx, dgamma, dbeta, dxsum,
                              partial, st);
}

// g[i] = gelu(u[i]), 8 elements per thread (recomputation of the MLP activation)
template <typename TU, typename T, int KIND>
__global__ __launch_bounds__(256) void gelu_kernel(const TU* __restrict__ u, T* __restrict__ g, size_t n8) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  float v[8];
  load8(u + i * 8, v);
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = gelu_f<KIND>(v[e]);
  store8(g + i * 8, v);
}

hipError_t gelu_fwd(int dtype, int kind, const void* u, void* g, size_t n, hipStream_t st, bool u_f16) {
  const size_t n8 = n / 8;
  dim3 grid((unsigned)((n8 + 255) / 256)), blk(256);
  if (dtype == 0) {
    if (u_f16) return hipErrorInvalidValue;
    if (kind == 0) hipLaunchKernelGGL((gelu_kernel<float, float, 0>), grid, blk, 0, st, (const float*)u, (float*)g, n8);
    else hipLaunchKernelGGL((gelu_kernel<float, float, 1>), grid, blk, 0, st, (const float*)u, (float*)g, n8);
  } else if (u_f16) {
    if (kind == 0) hipLaunchKernelGGL((gelu_kernel<f16, bf16, 0>), grid, blk, 0, st, (const f16*)u, (bf16*)g, n8);
    else hipLaunchKernelGGL((gelu_kernel<f16, bf16, 1>), grid, blk, 0, st, (const f16*)u, (bf16*)g, n8);
  } else {
    if (kind == 0) hipLaunchKernelGGL((gelu_kernel<bf16, bf16, 0>), grid, blk, 0, st, (const bf16*)u, (bf16*)g, n8);
    else hipLaunchKernelGGL((gelu_kernel<bf16, bf16, 1>), grid, blk, 0, st, (const bf16*)u, (bf16*)g, n8);
  }
  return hipGetLastError();
}

// out[i] = bf16(in[i]) for fp16 in: the backward phase's bf16 copies of forward activations
// that were stored in fp16
__global__ __launch_bounds__(256) void f16_to_bf16_kernel(const f16* __restrict__ in, bf16* __restrict__ out,
                                                          size_t n8) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  float v[8];
  load8(in + i * 8, v);
  store8(out + i * 8, v);
}
hipError_t f16_to_bf16(const void* in, void* out, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  hipLaunchKernelGGL(f16_to_bf16_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st, (const f16*)in,
                     (bf16*)out, n8);
  return hipGetLastError();
}

hipError_t widen_to_f32(const void* in, float* out, size_t n, hipStream_t st) {
  const size_t n8 = n / 8;
  hipLaunchKernelGGL(widen_kernel, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, st, (const bf16*)in,
                     out, n8);
  return hipGetLastError();
}

size_t ln_bwd_scratch_bytes(int T_rows, int H) {
  return (size_t)ln_bwd_blocks(T_rows) * 3 * H * sizeof(float);
}

int colsum_splits(int M) { return M < 4 * 64 ? (M + 3) / 4 : 64; }
size_t colsum_scratch_bytes(int M, int N) { return (size_t)colsum_splits(M) * N * sizeof(float); }

hipError_t reduce_colsum_partials(const float* partial, int G, int N, float* out, hipStream_t st) {
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((N + 31) / 32), dim3(1024), 0, st, partial, G, (size_t)N, N,
                     out, N, (float*)nullptr, N, (float*)nullptr);
  return hipGetLastError();
}

hipError_t colsum(int dtype, int M, int N, const void* A, float* out, float* partial,
                  hipStream_t st) {
  const int G = colsum_splits(M);
  const int V = dtype == 0 ? 4 : 8;
  dim3 g((N / V + kWave - 1) / kWave, G), b(256);
  if (dtype == 0)
    hipLaunchKernelGGL(colsum_partial_kernel<float>, g, b, 0, st, (const float*)A, partial, M, N);
  else
    hipLaunchKernelGGL(colsum_partial_kernel<bf16>, g, b, 0, st, (const bf16*)A, partial, M, N);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((N + 31) / 32), dim3(1024), 0, st, partial, G, (size_t)N, N,
                     out, N, (float*)nullptr, N, (float*)nullptr);
  return hipGetLastError();
}

// ---- column sums for callers that cannot allocate ------------------------------------------
// gpt_stage_op_colsum needs a scratch buffer for its per-workgroup partial sums.  This variant
// takes them from a fixed array in device memory instead, so the call allocates nothing: for
// callers under HIP graph capture, in tight serving loops, or in harnesses that forbid
// hipMalloc.  Each GPU the library runs on holds its own copy of the array (4 MiB) until the
// process ends.  In host code the array's name is only a stand-in: its device address is looked
// up once per device and that pointer is what the kernels get.
namespace {
constexpr int kNoAllocMaxN = 16384;   // columns; colsum_splits() never exceeds 64 rows of partials
constexpr int kNoAllocMaxDevices = 64;
static __device__ __align__(256) float scratch[64 * kNoAllocMaxN];
std::mutex g_scratch_mutex;
float* g_scratch_ptr[kNoAllocMaxDevices] = {};

// device address of `scratch` on the current device (looked up on first use per device)
hipError_t scratch_on_current_device(float** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kNoAllocMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = static_cast<float*>(p);
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}
}  // namespace
}  // namespace gpts

extern "C" int gpt_stage_op_colsum_noalloc(int dtype, int M, int N, const void* A, float* colsum_out,
                                           void* stream) {
  using namespace gpts;
  if ((dtype != GPTS_FP32 && dtype != GPTS_BF16) || !A || !colsum_out)
    return set_error(GPTS_EINVAL, "colsum_noalloc: bad argument");
  if (M < 1 || N < 8 || N % 8) return set_error(GPTS_ESHAPE, "colsum_noalloc: N must be a multiple of 8");
  if (N > kNoAllocMaxN || colsum_scratch_bytes(M, N) > sizeof(float) * 64 * (size_t)kNoAllocMaxN)
    return set_error(GPTS_ESHAPE, "colsum_noalloc: N exceeds 16384, the size the built-in scratch array is made for");
  float* partial = nullptr;
  hipError_t e = scratch_on_current_device(&partial);
  if (e == hipSuccess) e = colsum(dtype, M, N, A, colsum_out, partial, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return set_error(GPTS_EHIP, hipGetErrorString(e));
  return GPTS_OK;
}
