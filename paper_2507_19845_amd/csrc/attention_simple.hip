// Causal softmax attention in fp32 FMA arithmetic (fp32 stages and head sizes the
// MFMA kernels do not cover).  A query (or key) row is owned by G = D/32
// adjacent lanes, each holding a 32-wide slice of the head dimension; dot
// products are completed with xor-shuffles inside the group.  Tiles of 32
// rows of the other operand are staged in LDS as fp32.  Per head, for row i:
//   s_ij = q_i.k_j / sqrt(D) (j <= i),  p_ij = exp(s_ij - lse_i),  o_i = sum_j p_ij v_j
// and in reverse, with delta_i = do_i.o_i:
//   dv_j = sum_i p_ij do_i,  ds_ij = p_ij (do_i.v_j - delta_i),
//   dq_i = sum_j ds_ij k_j / sqrt(D),  dk_j = sum_i ds_ij q_i / sqrt(D).
#include "kernels.hpp"

namespace gpts {

constexpr int kRows = 64;  // rows per workgroup
constexpr int kTile = 32;  // staged rows of the other operand
constexpr int kSl = 32;    // head-dim slice per lane

template <int G> __device__ __forceinline__ float group_sum(float v) {
  if constexpr (G >= 2) v += __shfl_xor(v, 1, 64);
  if constexpr (G >= 4) v += __shfl_xor(v, 2, 64);
  return v;
}

// Cooperative load of `kTile` rows (row0..) of one head slice [*, D] into fp32 LDS.
template <typename T, int D>
__device__ __forceinline__ void stage_rows(float (*dst)[D], const T* __restrict__ src, size_t ld,
                                           int row0, int S, int nthreads) {
  for (int i = threadIdx.x; i < kTile * D; i += nthreads) {
    const int r = i / D, c = i % D;
    dst[r][c] = (row0 + r < S) ? to_f32(src[(size_t)(row0 + r) * ld + c]) : 0.f;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kRows* D / kSl) void attn_fwd_simple_kernel(
    const T* __restrict__ qkv, T* __restrict__ out, float* __restrict__ lse, int S, int a) {
  constexpr int G = D / kSl;
  __shared__ float Ks[kTile][D];
  __shared__ float Vs[kTile][D];
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const int n = blockIdx.y, b = blockIdx.z;
  const T* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const int r = threadIdx.x / G, part = threadIdx.x % G;
  const int qi = blockIdx.x * kRows + r;
  const float scale = 1.f / sqrtf((float)D);
  float q[kSl], o[kSl];
#pragma unroll
  for (int e = 0; e < kSl; ++e) {
    q[e] = qi < S ? to_f32(base[(size_t)qi * ld + part * kSl + e]) : 0.f;
    o[e] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const int last = min(S, (int)(blockIdx.x + 1) * kRows);  // keys needed by this tile: [0, last)
  for (int k0 = 0; k0 < last; k0 += kTile) {
    __syncthreads();
    stage_rows<T, D>(Ks, base + P, ld, k0, S, blockDim.x);
    stage_rows<T, D>(Vs, base + 2 * P, ld, k0, S, blockDim.x);
    __syncthreads();
    for (int j = 0; j < kTile; ++j) {
      const int kj = k0 + j;
      if (kj > qi || kj >= S || qi >= S) continue;  // uniform inside a lane group
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < kSl; ++e) s = fmaf(q[e], Ks[j][part * kSl + e], s);
      s = group_sum<G>(s) * scale;
      const float mn = fmaxf(m, s);
      const float corr = __expf(m - mn), p = __expf(s - mn);
      l = l * corr + p;
#pragma unroll
      for (int e = 0; e < kSl; ++e) o[e] = o[e] * corr + p * Vs[j][part * kSl + e];
      m = mn;
    }
  }
  if (qi < S) {
    const float inv = 1.f / l;
    T* orow = out + ((size_t)b * S + qi) * P + (size_t)n * D + part * kSl;
#pragma unroll
    for (int e = 0; e < kSl; ++e) orow[e] = from_f32<T>(o[e] * inv);
    if (part == 0) lse[((size_t)b * a + n) * S + qi] = m + logf(l);
  }
}

// dq and delta.  One lane group per query row.
template <typename T, int D>
__global__ __launch_bounds__(kRows* D / kSl) void attn_bwd_dq_simple_kernel(
    const T* __restrict__ qkv, const T* __restrict__ out, const float* __restrict__ lse,
    const T* __restrict__ dout, T* __restrict__ dqkv, float* __restrict__ delta, int S, int a) {
  constexpr int G = D / kSl;
  __shared__ float Ks[kTile][D];
  __shared__ float Vs[kTile][D];
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const int n = blockIdx.y, b = blockIdx.z;
  const T* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const int r = threadIdx.x / G, part = threadIdx.x % G;
  const int qi = blockIdx.x * kRows + r;
  const float scale = 1.f / sqrtf((float)D);
  float q[kSl], dO[kSl], dq[kSl];
  float dl = 0.f;
  const size_t orow = ((size_t)b * S + qi) * P + (size_t)n * D + part * kSl;
#pragma unroll
  for (int e = 0; e < kSl; ++e) {
    q[e] = qi < S ? to_f32(base[(size_t)qi * ld + part * kSl + e]) : 0.f;
    dO[e] = qi < S ? to_f32(dout[orow + e]) : 0.f;
    dl += qi < S ? dO[e] * to_f32(out[orow + e]) : 0.f;
    dq[e] = 0.f;
  }
  dl = group_sum<G>(dl);
  const float L = qi < S ? lse[((size_t)b * a + n) * S + qi] : 0.f;
  if (qi < S && part == 0) delta[((size_t)b * a + n) * S + qi] = dl;
  const int last = min(S, (int)(blockIdx.x + 1) * kRows);
  for (int k0 = 0; k0 < last; k0 += kTile) {
    __syncthreads();
    stage_rows<T, D>(Ks, base + P, ld, k0, S, blockDim.x);
    stage_rows<T, D>(Vs, base + 2 * P, ld, k0, S, blockDim.x);
    __syncthreads();
    for (int j = 0; j < kTile; ++j) {
      const int kj = k0 + j;
      if (kj > qi || kj >= S || qi >= S) continue;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < kSl; ++e) {
        s = fmaf(q[e], Ks[j][part * kSl + e], s);
        dp = fmaf(dO[e], Vs[j][part * kSl + e], dp);
      }
      s = group_sum<G>(s) * scale;
      dp = group_sum<G>(dp);
      const float ds = __expf(s - L) * (dp - dl) * scale;
#pragma unroll
      for (int e = 0; e < kSl; ++e) dq[e] = fmaf(ds, Ks[j][part * kSl + e], dq[e]);
    }
  }
  if (qi < S) {
    T* d = dqkv + ((size_t)b * S + qi) * ld + (size_t)n * D + part * kSl;
#pragma unroll
    for (int e = 0; e < kSl; ++e) d[e] = from_f32<T>(dq[e]);
  }
}

// dk and dv.  One lane group per key row; query rows i >= j are streamed.
template <typename T, int D>
__global__ __launch_bounds__(kRows* D / kSl) void attn_bwd_dkv_simple_kernel(
    const T* __restrict__ qkv, const float* __restrict__ lse, const T* __restrict__ dout,
    const float* __restrict__ delta, T* __restrict__ dqkv, int S, int a) {
  constexpr int G = D / kSl;
  __shared__ float Qs[kTile][D];
  __shared__ float dOs[kTile][D];
  __shared__ float Ls[kTile], Ds[kTile];
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const int n = blockIdx.y, b = blockIdx.z;
  const T* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const T* dobase = dout + (size_t)b * S * P + (size_t)n * D;
  const int r = threadIdx.x / G, part = threadIdx.x % G;
  const int kj = blockIdx.x * kRows + r;
  const float scale = 1.f / sqrtf((float)D);
  float k[kSl], v[kSl], dk[kSl], dv[kSl];
#pragma unroll
  for (int e = 0; e < kSl; ++e) {
    k[e] = kj < S ? to_f32(base[(size_t)kj * ld + P + part * kSl + e]) : 0.f;
    v[e] = kj < S ? to_f32(base[(size_t)kj * ld + 2 * P + part * kSl + e]) : 0.f;
    dk[e] = dv[e] = 0.f;
  }
  const int first = (blockIdx.x * kRows / kTile) * kTile;  // queries needed: [first, S)
  for (int q0 = first; q0 < S; q0 += kTile) {
    __syncthreads();
    stage_rows<T, D>(Qs, base, ld, q0, S, blockDim.x);
    stage_rows<T, D>(dOs, dobase, (size_t)P, q0, S, blockDim.x);
    if (threadIdx.x < kTile) {
      const int qi = q0 + threadIdx.x;
      Ls[threadIdx.x] = qi < S ? lse[((size_t)b * a + n) * S + qi] : 0.f;
      Ds[threadIdx.x] = qi < S ? delta[((size_t)b * a + n) * S + qi] : 0.f;
    }
    __syncthreads();
    for (int i = 0; i < kTile; ++i) {
      const int qi = q0 + i;
      if (qi < kj || qi >= S || kj >= S) continue;
      float s = 0.f, dp = 0.f;
#pragma unroll
      for (int e = 0; e < kSl; ++e) {
        s = fmaf(Qs[i][part * kSl + e], k[e], s);
        dp = fmaf(dOs[i][part * kSl + e], v[e], dp);
      }
      s = group_sum<G>(s) * scale;
      dp = group_sum<G>(dp);
      const float p = __expf(s - Ls[i]);
      const float ds = p * (dp - Ds[i]) * scale;
#pragma unroll
      for (int e = 0; e < kSl; ++e) {
        dv[e] = fmaf(p, dOs[i][part * kSl + e], dv[e]);
        dk[e] = fmaf(ds, Qs[i][part * kSl + e], dk[e]);
      }
    }
  }
  if (kj < S) {
    T* d = dqkv + ((size_t)b * S + kj) * ld + (size_t)n * D + part * kSl;
#pragma unroll
    for (int e = 0; e < kSl; ++e) {
      d[P + e] = from_f32<T>(dk[e]);
      d[2 * P + e] = from_f32<T>(dv[e]);
    }
  }
}

template <typename T, int D>
static hipError_t attn_fwd_td(int B, int S, int a, const T* qkv, T* out, float* lse, hipStream_t st) {
  dim3 g((S + kRows - 1) / kRows, a, B), b(kRows * D / kSl);
  hipLaunchKernelGGL((attn_fwd_simple_kernel<T, D>), g, b, 0, st, qkv, out, lse, S, a);
  return hipGetLastError();
}
template <typename T, int D>
static hipError_t attn_bwd_td(int B, int S, int a, const T* qkv, const T* out, const float* lse,
                              const T* dout, T* dqkv, float* delta, hipStream_t st) {
  dim3 g((S + kRows - 1) / kRows, a, B), b(kRows * D / kSl);
  hipLaunchKernelGGL((attn_bwd_dq_simple_kernel<T, D>), g, b, 0, st, qkv, out, lse, dout, dqkv, delta, S, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkv_simple_kernel<T, D>), g, b, 0, st, qkv, lse, dout, delta, dqkv, S, a);
  return hipGetLastError();
}

template <typename T>
static hipError_t attn_fwd_t(int B, int S, int a, int d, const T* qkv, T* out, float* lse, hipStream_t st) {
  switch (d) {
    case 32: return attn_fwd_td<T, 32>(B, S, a, qkv, out, lse, st);
    case 64: return attn_fwd_td<T, 64>(B, S, a, qkv, out, lse, st);
    case 128: return attn_fwd_td<T, 128>(B, S, a, qkv, out, lse, st);
  }
  return hipErrorInvalidValue;
}
template <typename T>
static hipError_t attn_bwd_t(int B, int S, int a, int d, const T* qkv, const T* out, const float* lse,
                             const T* dout, T* dqkv, float* delta, hipStream_t st) {
  switch (d) {
    case 32: return attn_bwd_td<T, 32>(B, S, a, qkv, out, lse, dout, dqkv, delta, st);
    case 64: return attn_bwd_td<T, 64>(B, S, a, qkv, out, lse, dout, dqkv, delta, st);
    case 128: return attn_bwd_td<T, 128>(B, S, a, qkv, out, lse, dout, dqkv, delta, st);
  }
  return hipErrorInvalidValue;
}

hipError_t attention_fwd_simple(int dtype, int B, int S, int a, int d, const void* qkv, void* out,
                                float* lse, hipStream_t st) {
  if (dtype == 0) return attn_fwd_t<float>(B, S, a, d, (const float*)qkv, (float*)out, lse, st);
  return attn_fwd_t<bf16>(B, S, a, d, (const bf16*)qkv, (bf16*)out, lse, st);
}
hipError_t attention_bwd_simple(int dtype, int B, int S, int a, int d, const void* qkv,
                                const void* out, const float* lse, const void* dout, void* dqkv,
                                float* delta, hipStream_t st) {
  if (dtype == 0)
    return attn_bwd_t<float>(B, S, a, d, (const float*)qkv, (const float*)out, lse,
                             (const float*)dout, (float*)dqkv, delta, st);
  return attn_bwd_t<bf16>(B, S, a, d, (const bf16*)qkv, (const bf16*)out, lse, (const bf16*)dout,
                          (bf16*)dqkv, delta, st);
}

}  // namespace gpts
