// Plain LDS-tiled matrix product with fp32 FMA arithmetic, for fp32 stages and
// for shapes the MFMA kernels do not cover.  64x64 output tile, 16-deep slices,
// 256 threads each owning a 4x4 block.  Operands are addressed through
// (row, col) strides so the three forms of the stage share one kernel:
//   NT (forward)  C = A[M,K] B[N,K]^T      NN (dgrad)  C = A[M,K] B[K,N]
//   TN (wgrad)    Cf32 += A[K,M]^T B[K,N]
#include "kernels.hpp"

namespace gpts {

constexpr int BM = 64, BN = 64, BK = 16;

template <typename T, bool A_KCONTIG, bool B_KCONTIG, bool ACCUM_F32, int GELU>
__global__ __launch_bounds__(256) void gemm_simple_kernel(
    const T* __restrict__ A, const T* __restrict__ B, void* __restrict__ Cv, int M, int N, int K,
    size_t sam, size_t sak, size_t sbk, size_t sbn, const T* __restrict__ bias,
    const void* __restrict__ residual, T* __restrict__ gelu_out, const T* __restrict__ dgelu_u,
    bool res_f32, bool out_f32) {
  __shared__ float As[BK][BM + 4];
  __shared__ float Bs[BK][BN + 4];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int tx = tid % 16, ty = tid / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += BK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // choose the thread->element map so the contiguous dimension runs along lanes
      int am, ak, bn, bk;
      if (A_KCONTIG) { ak = tid % BK; am = tid / BK + i * 16; } else { am = tid % BM; ak = tid / BM + i * 4; }
      if (B_KCONTIG) { bk = tid % BK; bn = tid / BK + i * 16; } else { bn = tid % BN; bk = tid / BN + i * 4; }
      float av = 0.f, bv = 0.f;
      if (m0 + am < M && k0 + ak < K) av = to_f32(A[(size_t)(m0 + am) * sam + (size_t)(k0 + ak) * sak]);
      if (n0 + bn < N && k0 + bk < K) bv = to_f32(B[(size_t)(k0 + bk) * sbk + (size_t)(n0 + bn) * sbn]);
      As[ak][am] = av;
      Bs[bk][bn] = bv;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < BK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n >= N) continue;
      const size_t o = (size_t)m * N + n;
      float v = acc[i][j];
      if constexpr (ACCUM_F32) {
        float* C = static_cast<float*>(Cv);
        C[o] += v;
      } else {
        T* C = static_cast<T*>(Cv);
        if (bias) v += to_f32(bias[n]);
        if constexpr (GELU >= 0) {
          if (gelu_out) {
            C[o] = from_f32<T>(v);
            gelu_out[o] = from_f32<T>(gelu_f<GELU < 0 ? 0 : GELU>(to_f32(C[o])));  // GeLU of u as stored
            continue;
          }
          if (dgelu_u) v *= gelu_grad_f<GELU < 0 ? 0 : GELU>(to_f32(dgelu_u[o]));
        }
        if (residual)
          v += res_f32 ? static_cast<const float*>(residual)[o] : to_f32(static_cast<const T*>(residual)[o]);
        if (out_f32) static_cast<float*>(Cv)[o] = v;
        else C[o] = from_f32<T>(v);
      }
    }
  }
}

template <typename T>
static hipError_t gemm_simple_t(int form, int M, int N, int K, const T* A, const T* B, void* C,
                                const GemmEpilogue& ep, hipStream_t st) {
  dim3 g((N + BN - 1) / BN, (M + BM - 1) / BM), b(256);
  const T* bias = (const T*)ep.bias;
  const void* res = ep.residual;
  const bool r32 = ep.residual_f32, o32 = ep.out_f32;
  T* go = (T*)ep.gelu_out;
  const T* du = (const T*)ep.dgelu_u;
  const bool act = go || du;
#define GPTS_SG(AK, BKC, ACC, G, sam, sak, sbk, sbn)                                           \
  hipLaunchKernelGGL((gemm_simple_kernel<T, AK, BKC, ACC, G>), g, b, 0, st, A, B, C, M, N, K,   \
                     (size_t)(sam), (size_t)(sak), (size_t)(sbk), (size_t)(sbn), bias, res, go, du, r32, o32)
  if (form == 0) {
    if (!act) GPTS_SG(true, true, false, -1, K, 1, 1, K);
    else if (ep.gelu_kind == 0) GPTS_SG(true, true, false, 0, K, 1, 1, K);
    else GPTS_SG(true, true, false, 1, K, 1, 1, K);
  } else if (form == 1) {
    if (!act) GPTS_SG(true, false, false, -1, K, 1, N, 1);
    else if (ep.gelu_kind == 0) GPTS_SG(true, false, false, 0, K, 1, N, 1);
    else GPTS_SG(true, false, false, 1, K, 1, N, 1);
  } else {
    GPTS_SG(false, false, true, -1, 1, M, N, 1);
  }
#undef GPTS_SG
  return hipGetLastError();
}

hipError_t gemm_simple(int dtype, int form, int M, int N, int K, const void* A, const void* B,
                       void* C, const GemmEpilogue& ep, hipStream_t st) {
  if (dtype == 0) return gemm_simple_t<float>(form, M, N, K, (const float*)A, (const float*)B, C, ep, st);
  return gemm_simple_t<bf16>(form, M, N, K, (const bf16*)A, (const bf16*)B, C, ep, st);
}

}  // namespace gpts
