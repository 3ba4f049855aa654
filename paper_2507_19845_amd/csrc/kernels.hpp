// Internal launcher interface between the stage orchestrator and the kernels.
// Every launcher only enqueues on `st` and returns hipGetLastError().
#pragma once
#include "common.hpp"

namespace gpts {

// dtype: 0 = fp32 storage, 1 = bf16 storage (fp32 arithmetic in both).

// x_f32: the normalised tensor x (the residual stream) is fp32 even when dtype is bf16.
// out_f16 (bf16 stages with an fp32 x only): out is written as fp16 instead of bf16.
hipError_t ln_fwd(int dtype, bool x_f32, int T_rows, int H, float eps, const void* x,
                  const void* gamma, const void* beta, void* out, float* mean, float* rstd,
                  hipStream_t st, bool out_f16 = false);
size_t ln_bwd_scratch_bytes(int T_rows, int H);
// dxsum (may be null): += column sums of dx as stored
hipError_t ln_bwd(int dtype, bool x_f32, int T_rows, int H, const void* dout, const void* x,
                  const float* mean, const float* rstd, const void* gamma, const void* dres, void* dx,
                  float* dgamma, float* dbeta, float* dxsum, float* partial, hipStream_t st);
// out[i] = (float) in[i] for n bf16 elements (n a multiple of 8)
hipError_t widen_to_f32(const void* in, float* out, size_t n, hipStream_t st);
// g = gelu(u) elementwise (kind 0 tanh form, 1 erf form); n a multiple of 8
// u_f16 (bf16 stages): u is fp16, g is still written as bf16
hipError_t gelu_fwd(int dtype, int kind, const void* u, void* g, size_t n, hipStream_t st, bool u_f16 = false);
// out[i] = bf16(in[i]) for n fp16 elements (n a multiple of 8)
hipError_t f16_to_bf16(const void* in, void* out, size_t n, hipStream_t st);
size_t colsum_scratch_bytes(int M, int N);
int colsum_splits(int M);   // rows of partial sums that colsum_scratch_bytes() provides for
hipError_t colsum(int dtype, int M, int N, const void* A, float* out, float* partial,
                  hipStream_t st);
// out[n] += sum_{g<G} partial[g*N + n], in fixed order
hipError_t reduce_colsum_partials(const float* partial, int G, int N, float* out, hipStream_t st);

// Epilogue description shared by all GEMM implementations.
struct GemmEpilogue {
  const void* bias = nullptr;      // [N], storage dtype, added to every row
  const void* residual = nullptr;  // [M,N], added; storage dtype unless residual_f32
  bool residual_f32 = false;       // bf16 stages: residual is fp32
  bool out_f32 = false;            // bf16 stages: C is written as fp32 (forms 0 with residual only)
  void* gelu_out = nullptr;        // [M,N]: if set, C keeps the pre-activation and this gets gelu(C)
  const void* dgelu_u = nullptr;   // [M,N]: if set, C *= gelu'(u)
  int gelu_kind = 0;               // 0 tanh, 1 erf
  float* colsum_partial = nullptr; // with dgelu_u, MFMA path only: [gemm_mfma_colsum_rows()][N] fp32,
                                   // written (not added to): column sums of C (fp32, before it is
                                   // rounded for storage), one row per group of tile rows; their sum
                                   // over the rows is sum_m C[m, :]
  const void* b_image = nullptr;   // forms 0/1, bf16: B re-laid-out by gemm_prepare_image() as the
                                   // tiled image of its [N rows, K contiguous] view (optional)
  // form 2, bf16 MFMA path only (gemm_wgrad_segments_supported): the contraction runs over
  // k_segments pieces of K rows each; piece s of A (B) starts seg_stride_a (seg_stride_b)
  // ELEMENTS after piece s-1.  One launch, one read-modify-write of C.
  int k_segments = 1;
  size_t seg_stride_a = 0, seg_stride_b = 0;
};
// form 0: C[M,N] = A[M,K] B[N,K]^T ; form 1: C[M,N] = A[M,K] B[K,N] ;
// form 2: Cf32[M,N] += A[K,M]^T B[K,N].
hipError_t gemm_simple(int dtype, int form, int M, int N, int K, const void* A, const void* B,
                       void* C, const GemmEpilogue& ep, hipStream_t st);
// bf16 MFMA path; returns hipErrorNotSupported if the shape does not fit its tiles.
bool gemm_mfma_supported(int form, int M, int N, int K);
// Tiled image of a B operand for the 256x256x32 kernel: `transposed` = src is [K,N]
// (the dgrad view of a weight [out=K, in=N]); else src is [N,K].  N any, K % 32 == 0.
size_t gemm_image_elems(int N, int K);
// to_f16: the image holds the bf16 source values converted to fp16.
hipError_t gemm_prepare_image(const void* src, void* img, int N, int K, bool transposed, hipStream_t st,
                              bool to_f16 = false);
// Forward product with fp16 operands on the matrix cores' f16 instructions:
// C[M,N] = A[M,K] (fp16) W^T, W given as its fp16 image (gemm_prepare_image(.., to_f16 = true));
// epilogues as form 0: bias; bias + GeLU (C and gelu_out written as fp16); bias + fp32 residual
// (C fp32 or bf16 as ep.out_f32 says).  Without a residual C is written as fp16.  Any M, N % 8 == 0,
// K % 128 == 0.
bool gemm_fwd_f16_supported(int M, int N, int K);
hipError_t gemm_fwd_f16(int M, int N, int K, const void* A, const void* b_image, void* C,
                        const GemmEpilogue& ep, hipStream_t st);
hipError_t gemm_mfma(int form, int M, int N, int K, const void* A, const void* B, void* C,
                     const GemmEpilogue& ep, hipStream_t st);
bool gemm_wgrad_segments_supported(int form, int M, int N, int K);
// rows of GemmEpilogue::colsum_partial that gemm_mfma() writes for an [M,N] product
int gemm_mfma_colsum_rows(int M, int N);

hipError_t attention_fwd_simple(int dtype, int B, int S, int a, int d, const void* qkv, void* out,
                                float* lse, hipStream_t st);
hipError_t attention_bwd_simple(int dtype, int B, int S, int a, int d, const void* qkv,
                                const void* out, const float* lse, const void* dout, void* dqkv,
                                float* delta, hipStream_t st);

// bf16 MFMA attention (head_dim 32, 64 or 128).  scratch: device memory of
// attention_mfma_scratch_bytes(B, S, a, d, phase) bytes (phase 0 forward: the transposed
// image of V; phase 1 backward: delta and the transposed images of Q, K and dO).
bool attention_mfma_supported(int B, int S, int a, int d);   // head_dim 32/64/128 and index ranges
size_t attention_mfma_scratch_bytes(int B, int S, int a, int d, int phase);
// f16: qkv and out are fp16 (forward activations kept in fp16); lse is fp32 either way.
hipError_t attention_fwd_mfma(int B, int S, int a, int d, const void* qkv, void* out, float* lse,
                              void* scratch, hipStream_t st, bool f16 = false);
// qkv_f16 (optional): the fp16 qkv of an fp16 forward pass; the logits are then recomputed from
// its Q and K, `out` is that pass's fp16 output (it only enters delta = rowsum(dO * O)), and
// qkv is the bf16 copy that every other product reads.
hipError_t attention_bwd_mfma(int B, int S, int a, int d, const void* qkv, const void* out,
                              const float* lse, const void* dout, void* dqkv, void* scratch,
                              hipStream_t st, const void* qkv_f16 = nullptr);

// Records the thread's error text and returns `code` (for sources outside stage.hip).
int set_error(int code, const char* msg);

}  // namespace gpts
