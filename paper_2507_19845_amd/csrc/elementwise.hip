// HBM-bound kernels of the stage: LayerNorm forward/backward (with the residual
// gradient folded in), column sums for bias gradients, and the fixed-order
// reduction of per-workgroup partial sums.  One 256-thread workgroup (4 waves)
// per token row, 16-byte loads, the row cached in registers, fp32 statistics.
#include "kernels.hpp"

namespace gpts {

constexpr int kLnThreads = 256;

// ----------------------------------------------------------------- LN fwd ----
// Per token: mu = mean(x), var = mean((x-mu)^2), r = 1/sqrt(var+eps),
// out = (x-mu) r gamma + beta.  NCH = 16-byte chunks cached per thread.
template <typename T, int NCH>
__global__ __launch_bounds__(kLnThreads) void ln_fwd_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
    T* __restrict__ out, float* __restrict__ mean, float* __restrict__ rstd, int H, float eps) {
  constexpr int V = Vec16<T>::N;
  __shared__ float red[2][kLnThreads / kWave];
  const int row = blockIdx.x;
  const int nvec = H / V;
  const T* xr = x + (size_t)row * H;
  Vec16<T> xv[NCH];
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
      xv[c] = load16(xr + (size_t)i * V);
#pragma unroll
      for (int e = 0; e < V; ++e) s += xv[c].get(e);
    }
  }
  const float mu = block_sum<kLnThreads / kWave>(s, red[0]) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        const float d = xv[c].get(e) - mu;
        q += d * d;
      }
    }
  }
  const float var = block_sum<kLnThreads / kWave>(q, red[1]) / (float)H;
  const float r = 1.f / sqrtf(var + eps);
  T* orow = out + (size_t)row * H;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
      const Vec16<T> g = load16(gamma + (size_t)i * V);
      const Vec16<T> b = load16(beta + (size_t)i * V);
      Vec16<T> o;
#pragma unroll
      for (int e = 0; e < V; ++e) o.set(e, (xv[c].get(e) - mu) * r * g.get(e) + b.get(e));
      store16(orow + (size_t)i * V, o);
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
// partial[blockIdx.x][0][H] / [1][H] for the fixed-order reduction below.
template <typename T, int NCH>
__global__ __launch_bounds__(kLnThreads) void ln_bwd_kernel(
    const T* __restrict__ dout, const T* __restrict__ x, const float* __restrict__ mean,
    const float* __restrict__ rstd, const T* __restrict__ gamma, const T* __restrict__ dres,
    T* __restrict__ dx, float* __restrict__ partial, int T_rows, int H) {
  constexpr int V = Vec16<T>::N;
  __shared__ float red[2][kLnThreads / kWave];
  const int nvec = H / V;
  float dg[NCH][V], db[NCH][V];
  Vec16<T> gam[NCH];
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) gam[c] = load16(gamma + (size_t)i * V);
#pragma unroll
    for (int e = 0; e < V; ++e) dg[c][e] = db[c][e] = 0.f;
  }
  for (int row = blockIdx.x; row < T_rows; row += gridDim.x) {
    const float mu = mean[row], r = rstd[row];
    const size_t base = (size_t)row * H;
    Vec16<T> dv[NCH], xv[NCH];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int i = threadIdx.x + c * kLnThreads;
      if (i < nvec) {
        dv[c] = load16(dout + base + (size_t)i * V);
        xv[c] = load16(x + base + (size_t)i * V);
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float d = dv[c].get(e);
          const float xh = (xv[c].get(e) - mu) * r;
          const float g = d * gam[c].get(e);
          s1 += g;
          s2 += g * xh;
          dg[c][e] += d * xh;
          db[c][e] += d;
        }
      }
    }
    const float m1 = block_sum<kLnThreads / kWave>(s1, red[0]) / (float)H;
    const float m2 = block_sum<kLnThreads / kWave>(s2, red[1]) / (float)H;
#pragma unroll
    for (int c = 0; c < NCH; ++c) {
      const int i = threadIdx.x + c * kLnThreads;
      if (i < nvec) {
        Vec16<T> o;
        Vec16<T> rs;
        if (dres) rs = load16(dres + base + (size_t)i * V);
#pragma unroll
        for (int e = 0; e < V; ++e) {
          const float xh = (xv[c].get(e) - mu) * r;
          const float g = dv[c].get(e) * gam[c].get(e);
          float v = r * (g - m1 - xh * m2);
          if (dres) v += rs.get(e);
          o.set(e, v);
        }
        store16(dx + base + (size_t)i * V, o);
      }
    }
  }
  float* pg = partial + (size_t)blockIdx.x * 2 * H;
#pragma unroll
  for (int c = 0; c < NCH; ++c) {
    const int i = threadIdx.x + c * kLnThreads;
    if (i < nvec) {
#pragma unroll
      for (int e = 0; e < V; ++e) {
        pg[(size_t)i * V + e] = dg[c][e];
        pg[(size_t)H + (size_t)i * V + e] = db[c][e];
      }
    }
  }
}

// out[c] += sum_{g<G} partial[g*stride + c] for c < N0 (into out0) and N0 <= c < N
// (into out1[c-N0]).  32 columns x 8 row groups per workgroup; the row groups are
// combined through LDS in fixed order, so the result is deterministic.
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial,
                                                              float* __restrict__ out0,
                                                              float* __restrict__ out1, int G,
                                                              size_t stride, int N0, int N) {
  __shared__ float sm[8][32];
  const int cx = threadIdx.x & 31, ry = threadIdx.x >> 5;
  const int c = blockIdx.x * 32 + cx;
  float s = 0.f;
  if (c < N)
    for (int g = ry; g < G; g += 8) s += partial[(size_t)g * stride + c];
  sm[ry][cx] = s;
  __syncthreads();
  if (ry == 0 && c < N) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) t += sm[i][cx];
    if (c < N0) out0[c] += t;
    else out1[c - N0] += t;
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
template <typename T>
static hipError_t ln_fwd_t(int T_rows, int H, float eps, const T* x, const T* gamma, const T* beta,
                           T* out, float* mean, float* rstd, hipStream_t st) {
  constexpr int V = Vec16<T>::N;
  const int nch = (H / V + kLnThreads - 1) / kLnThreads;
  dim3 g(T_rows), b(kLnThreads);
#define GPTS_LN_FWD(N)                                                                       \
  hipLaunchKernelGGL((ln_fwd_kernel<T, N>), g, b, 0, st, x, gamma, beta, out, mean, rstd, H, eps)
  if (nch <= 1) GPTS_LN_FWD(1);
  else if (nch <= 2) GPTS_LN_FWD(2);
  else if (nch <= 4) GPTS_LN_FWD(4);
  else if (nch <= 8) GPTS_LN_FWD(8);
  else GPTS_LN_FWD(16);
#undef GPTS_LN_FWD
  return hipGetLastError();
}

hipError_t ln_fwd(int dtype, int T_rows, int H, float eps, const void* x, const void* gamma,
                  const void* beta, void* out, float* mean, float* rstd, hipStream_t st) {
  if (dtype == 0)
    return ln_fwd_t<float>(T_rows, H, eps, (const float*)x, (const float*)gamma, (const float*)beta,
                           (float*)out, mean, rstd, st);
  return ln_fwd_t<bf16>(T_rows, H, eps, (const bf16*)x, (const bf16*)gamma, (const bf16*)beta,
                        (bf16*)out, mean, rstd, st);
}

int ln_bwd_blocks(int T_rows) { return T_rows < 256 ? T_rows : 256; }

template <typename T>
static hipError_t ln_bwd_t(int T_rows, int H, const T* dout, const T* x, const float* mean,
                           const float* rstd, const T* gamma, const T* dres, T* dx, float* dgamma,
                           float* dbeta, float* partial, hipStream_t st) {
  constexpr int V = Vec16<T>::N;
  const int nch = (H / V + kLnThreads - 1) / kLnThreads;
  const int G = ln_bwd_blocks(T_rows);
  dim3 g(G), b(kLnThreads);
#define GPTS_LN_BWD(N)                                                                          \
  hipLaunchKernelGGL((ln_bwd_kernel<T, N>), g, b, 0, st, dout, x, mean, rstd, gamma, dres, dx, \
                     partial, T_rows, H)
  if (nch <= 1) GPTS_LN_BWD(1);
  else if (nch <= 2) GPTS_LN_BWD(2);
  else if (nch <= 4) GPTS_LN_BWD(4);
  else if (nch <= 8) GPTS_LN_BWD(8);
  else GPTS_LN_BWD(16);
#undef GPTS_LN_BWD
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((2 * H + 31) / 32), dim3(256), 0, st, partial, dgamma,
                     dbeta, G, (size_t)2 * H, H, 2 * H);
  return hipGetLastError();
}

hipError_t ln_bwd(int dtype, int T_rows, int H, const void* dout, const void* x, const float* mean,
                  const float* rstd, const void* gamma, const void* dres, void* dx, float* dgamma,
                  float* dbeta, float* partial, hipStream_t st) {
  if (dtype == 0)
    return ln_bwd_t<float>(T_rows, H, (const float*)dout, (const float*)x, mean, rstd,
                           (const float*)gamma, (const float*)dres, (float*)dx, dgamma, dbeta,
                           partial, st);
  return ln_bwd_t<bf16>(T_rows, H, (const bf16*)dout, (const bf16*)x, mean, rstd,
                        (const bf16*)gamma, (const bf16*)dres, (bf16*)dx, dgamma, dbeta, partial, st);
}

size_t ln_bwd_scratch_bytes(int T_rows, int H) {
  return (size_t)ln_bwd_blocks(T_rows) * 2 * H * sizeof(float);
}

int colsum_splits(int M) { return M < 4 * 64 ? (M + 3) / 4 : 64; }
size_t colsum_scratch_bytes(int M, int N) { return (size_t)colsum_splits(M) * N * sizeof(float); }

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
  hipLaunchKernelGGL(reduce_partials_kernel, dim3((N + 31) / 32), dim3(256), 0, st, partial, out,
                     (float*)nullptr, G, (size_t)N, N, N);
  return hipGetLastError();
}

}  // namespace gpts
