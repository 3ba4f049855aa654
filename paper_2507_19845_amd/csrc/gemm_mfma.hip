// bf16 (and, for the forward phase of cfg.fwd_fp16 stages, fp16) matrix products on the gfx950
// matrix cores, fp32 accumulation, for the three forms the stage needs:
//   NT  C[M,N]   = A[M,K] B[N,K]^T     forward linears   (both operands K-contiguous)
//   NN  C[M,N]   = A[M,K] B[K,N]       data gradients    (B is K-major)
//   TN  Cf[M,N] += A[K,M]^T B[K,N]     weight gradients  (both operands K-major)
//
// Two kernels:
//  * gemm_mi16_kernel -- the one that does almost all the work.  256x256 output tile per
//    workgroup of 4 waves (2x2, 128x128 per wave), K in slices of 32 through a ring of FOUR LDS
//    stages (three slices in flight), v_mfma_f32_16x16x32 with the wave's 64 accumulator blocks
//    placed by hand in AGPRs a0..a255 (agpr_ops.hpp).  It serves the forward products (on raw
//    weights or on weight images), the data gradients through weight images, and the weight
//    gradients (both operands K-major, fragments by transposing LDS reads; the contraction may
//    run over several buffers, one per micro-batch).
//  * gemm_mfma_kernel -- v_mfma_f32_32x32x16 with compiler-allocated accumulators, templated
//    on tile and stage count: data gradients on raw weights (256x256x32, five-stage ring with
//    paired fetches), contraction lengths that are not a multiple of 128, and the 128x128x64
//    two-stage tiles for products of fewer than 100 large tiles.
// Common to both:
//  * Slices go global -> LDS by the DMA path (global_load_lds_dwordx4: no registers, no
//    ds_write), issued from inline assembly and waited for with explicit vmcnt counts, spread
//    between the matrix instructions; one barrier per slice.
//  * The DMA writes 16-byte slots in lane order, so bank-conflict avoidance is done by
//    choosing WHICH global chunk a lane fetches (an XOR swizzle of the chunk index), never by
//    padding.  Weight images (prepare_image_kernel) store a weight in exactly that LDS order, so
//    that every DMA instruction copies 1 KiB of contiguous memory.
//  * K-major operands are stored in LDS as they sit in memory ([k][rows]) and fragments are read
//    with the transposing LDS load ds_read_b64_tr_b16, so no operand is ever transposed in HBM.
//  * The two MFMA operands are swapped (D = B-fragment x A-fragment): a lane owns consecutive
//    output columns of one row.  The epilogue stages the wave's block through the (then free)
//    pipeline LDS and reads it back row-major, so that every global access of the fused bias /
//    GeLU / GeLU' / residual / fp32-accumulate epilogues covers whole cache lines.
//  * Workgroup -> tile map: consecutive workgroup ids land on different XCDs, so ids are first
//    regrouped per XCD and then walked in bands of 4 tile rows to keep each XCD's L2 working
//    set to a compact patch of the output.
#include <type_traits>
#include <utility>

#include "agpr_ops.hpp"
#include "kernels.hpp"

namespace gpts {
namespace {

#ifndef GPTS_KC_STAGES
// LDS stages of the 256x256 kernel for raw (not prepared) operands when A is K-contiguous:
// 5 = ring with paired fetches (measured +3 % on the raw forward product), 4 = plain ring.
// With a prepared B image the plain ring is as fast (the image is contiguous anyway).
#define GPTS_KC_STAGES 5
#endif
#ifndef GPTS_BIG_WAVES
#define GPTS_BIG_WAVES 4   // waves per workgroup of the 256x256 kernel
#endif

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(1))) const void* glb_ptr;

// epilogue kinds
// (RES32: the residual is fp32; OUT32: C is written as fp32 -- the residual stream of a bf16 stage)
enum { EPI_BIAS_RES = 0, EPI_GELU_TANH, EPI_GELU_ERF, EPI_PLAIN, EPI_DGELU_TANH, EPI_DGELU_ERF, EPI_ACCUM,
       EPI_BIAS_RES32_OUT32, EPI_BIAS_RES32_OUT16, EPI_BIAS /* bias only: no residual operand */ };

struct MfmaArgs {
  const bf16* A;
  const bf16* B;
  void* C;
  int M, N, K;
  const bf16* bias;
  const void* residual;
  bf16* gelu_out;
  const bf16* dgelu_u;
  float* colsum;   // GeLU' epilogue only, may be null: per-wave-row column sums of C
  // K-major products only (weight gradients): the contraction runs over `k_segments` pieces of
  // K rows each (K is then the length of ONE piece), piece s of A starting seg_stride_a elements
  // after piece s-1, likewise B: the tokens of several micro-batches, each in its own buffer.
  int k_segments = 1;
  size_t seg_stride_a = 0, seg_stride_b = 0;
};

// 16-byte chunk swizzle of a K-contiguous tile row with CPR chunks per row.  Chosen
// so that 16 consecutive rows read at the same logical chunk hit 16 different
// (row parity / quarter, chunk) bank groups, for 64- and for 32-bank layouts.
template <int CPR> __device__ __forceinline__ int swz_kc(int row) {
  if constexpr (CPR == 8) return (row & 7) ^ ((row >> 3) & 1);
  else return ((row >> 1) & 3) ^ ((row >> 3) & 1);
}
// 32-byte unit swizzle of a K-major tile row, as a function of the k-row.
template <bool NAT> __device__ __forceinline__ int swz_km(int k) {
  return ((k & 3) << 1) | ((NAT ? (k >> 3) : (k >> 2)) & 1);
}
// k (within a 16-wide MFMA step) held in element 4t+j of the fragment of k-group kg.
// NAT: the order a K-contiguous 16-byte read gives (8kg + 4t + j); otherwise 8t + 4kg + j.
template <bool NAT> __device__ __forceinline__ int kperm(int kg, int t, int j) {
  return NAT ? 8 * kg + 4 * t + j : 8 * t + 4 * kg + j;
}

// Per-lane state of one operand: global offsets for the DMA and LDS offsets for
// the fragment reads.  R = tile rows (BM or BN), WR = rows per wave, BK = slice depth.
// IMG: the operand was re-laid-out beforehand (prepare_image below) as the exact LDS image
// of its K-contiguous tiles, [tile of R rows][slice of BK][R*BK elements]: every DMA
// instruction then copies 1 KiB of contiguous memory.
template <int R, int WR, int BK, bool KMAJOR, bool NAT, bool IMG = false, int NW = 4> struct Operand {
  static_assert(!(IMG && KMAJOR), "images are K-contiguous");
  static constexpr int NI = R * BK * 2 / 1024 / NW;  // DMA instructions (1 KiB each) per wave and slice
  static constexpr int TILES = WR / 32;     // 32-row MFMA sub-tiles per wave
  static constexpr int KS = BK / 16;        // MFMA steps per slice
  static constexpr int RB = BK * 2;         // bytes per row of a K-contiguous tile
  static constexpr int CPR = BK / 8;        // 16-byte chunks per such row
  static constexpr int ROWB = R * 2;        // bytes per k-row of a K-major tile
  uint32_t goff[NI];                        // byte offset of this lane's chunk, slice 0
  uint32_t rd[KMAJOR ? 2 * TILES : KS];     // LDS read offsets (see frag())
  uint32_t rdbase;

  __device__ __forceinline__ void init(int r0, int rtotal, size_t ld, int wave, int lane, int wr0) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int slot = (wave * NI + i) * 64 + lane;
      if constexpr (IMG) {
        goff[i] = (uint32_t)(((size_t)(r0 / R) * R * ld + (size_t)slot * 8) * 2);
      } else if constexpr (!KMAJOR) {
        const int row = slot / CPR;
        const int chunk = (slot % CPR) ^ swz_kc<CPR>(row);
        int gr = r0 + row;
        gr = gr < rtotal ? gr : rtotal - 1;
        goff[i] = (uint32_t)(((size_t)gr * ld + chunk * 8) * 2);
      } else {
        const int byte = slot * 16;
        const int k = byte / ROWB, wb = byte % ROWB;
        const int u = (wb >> 5) ^ swz_km<NAT>(k);
        const int col = u * 16 + ((wb >> 4) & 1) * 8;
        const int gc = (r0 + col < rtotal) ? r0 + col : 0;
        goff[i] = (uint32_t)(((size_t)k * ld + gc) * 2);
      }
    }
    if constexpr (!KMAJOR) {
      const int row = wr0 + (lane & 31);
      rdbase = row * RB;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) rd[ks] = ((2 * ks + (lane >> 5)) ^ swz_kc<CPR>(row)) << 4;
    } else {
      const int g = lane >> 4, i = lane & 15, mh = g & 1, kg = g >> 1, j = i >> 2, q = i & 3;
      rdbase = q * 8;
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int k = kperm<NAT>(kg, t, j);
#pragma unroll
        for (int rb = 0; rb < TILES; ++rb) {
          const int u = (wr0 >> 4) + rb * 2 + mh;
          rd[t * TILES + rb] = k * ROWB + ((u ^ swz_km<NAT>(k)) << 5);
        }
      }
    }
  }

  // Enqueue DMA instruction i (a compile-time constant after unrolling) of slice `kt`:
  // 64 lanes x 16 bytes from X + goff -> 1 KiB of LDS at byte address lds_tile + i*1024
  // (wave-uniform, passed in M0).  Written as inline assembly on purpose: the compiler
  // then does not track these copies, so it neither drains them (vmcnt(0)) in front of
  // LDS reads it cannot prove independent, nor counts them; completion is waited for
  // explicitly with wait_dma_and_barrier().
  __device__ __forceinline__ void issue_one(const bf16* __restrict__ X, size_t ld, int kt,
                                            uint32_t lds_tile, int wave, int i) const {
    const bf16* base = IMG ? X + (size_t)kt * R * BK : (KMAJOR ? X + (size_t)kt * BK * ld : X + (size_t)kt * BK);
    const uint32_t dst = lds_tile + (wave * NI + i) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 ::"s"(dst), "v"(goff[i]), "s"(base)
                 : "memory");
  }
  // the same with the slice's base address given (X advanced to the slice by the caller)
  __device__ __forceinline__ void issue_at(const bf16* __restrict__ base, uint32_t lds_tile, int wave, int i) const {
    const uint32_t dst = lds_tile + (wave * NI + i) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 ::"s"(dst), "v"(goff[i]), "s"(base)
                 : "memory");
  }
  __device__ __forceinline__ void issue(const bf16* __restrict__ X, size_t ld, int kt, uint32_t lds_tile,
                                        int wave) const {
#pragma unroll
    for (int i = 0; i < NI; ++i) issue_one(X, ld, kt, lds_tile, wave, i);
  }

  // fragment of sub-tile rb for MFMA step ks (16 k): 8 bf16 per lane
  __device__ __forceinline__ bf16x8 frag(const char* tile, int rb, int ks) const {
    if constexpr (!KMAJOR) {
      return *reinterpret_cast<const bf16x8*>(tile + rdbase + rb * 32 * RB + rd[ks]);
    } else {
      const char* p = tile + rdbase + ks * 16 * ROWB;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(p + rd[rb]));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (s16x4 __attribute__((address_space(3)))*)(p + rd[TILES + rb]));
      typedef short s16x8 __attribute__((ext_vector_type(8)));
      const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// eight bf16 from two transposing LDS reads (each delivers 4 consecutive k of the lane's column)
__device__ __forceinline__ bf16x8 tr_pair(const char* p0, const char* p1) {
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p1);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Scheduling hint for one MFMA step: spread the LDS reads that fetch the next
// step's fragments (and, with N_DMA > 0, the DMA instructions of a later slice)
// between the MFMAs of the current step, one read after each of the first MFMAs.
// (mask 0x008 = MFMA, 0x100 = DS read, 0x010 = any VMEM: the DMA both loads and stores)
template <int N_PAIR, int N_DS, int N_MMA, int N_DMA, int I = 0>
__device__ __forceinline__ void sched_pairs() {
  if constexpr (I < N_PAIR) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, ((I + 1) * N_DS) / N_PAIR - (I * N_DS) / N_PAIR, 0);
    if constexpr (((I + 1) * N_DMA) / N_PAIR > (I * N_DMA) / N_PAIR)  // spread evenly
      __builtin_amdgcn_sched_group_barrier(0x010, ((I + 1) * N_DMA) / N_PAIR - (I * N_DMA) / N_PAIR, 0);
    sched_pairs<N_PAIR, N_DS, N_MMA, N_DMA, I + 1>();
  } else if constexpr (N_MMA > N_PAIR) {
    __builtin_amdgcn_sched_group_barrier(0x008, N_MMA - N_PAIR, 0);
  }
}

// Wait until at most VM of this wave's DMA instructions are still in flight and all
// of its LDS reads have returned, then meet the other waves.  (A plain barrier
// intrinsic would make the compiler drain every outstanding DMA first.)
template <int VM> __device__ __forceinline__ void wait_dma_and_barrier() {
  asm volatile("s_waitcnt vmcnt(%0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::"n"(VM) : "memory");
}

// ---- epilogue --------------------------------------------------------------------
// Shared by the kernels below.  acc[i][j]: the wave's 32x32 blocks (block row i, block column j)
// in the accumulator layout of the swapped MFMA (lane owns row lane&31 and four-column groups).
// lds: LDS_BYTES of workgroup LDS that no wave reads any more and no DMA still writes.
// write_pass(pass_constant, stg): stores rows [pass*RP, pass*RP + RP) of the wave's block
// into the staging area, element (row, col) as fp32 at
//   stg + row*WN + ((col/4) ^ (row & (WN/4 - 1)))*4 + col%4     (see stage_slot()).
template <int WN> __device__ __forceinline__ int stage_slot(int row, int chunk) {
  return row * WN + ((chunk ^ (row & (WN / 4 - 1))) * 4);
}
template <int... I, class F> __device__ __forceinline__ void static_for_impl(std::integer_sequence<int, I...>, F&& f) {
  (f(std::integral_constant<int, I>{}), ...);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): a loop whose index is a constant expression
template <int N, class F> __device__ __forceinline__ void static_for(F&& f) {
  static_for_impl(std::make_integer_sequence<int, N>{}, f);
}
// OUT16: the 16-bit outputs (C of the bias-only epilogue; C and the GeLU output of the GeLU
// epilogues) are written as fp16 instead of bf16 (forward activations kept in fp16).
template <int BM, int BN, int EPI, int NW, int LDS_BYTES, bool OUT16 = false, class StageWriter>
__device__ __forceinline__ void gemm_epilogue(StageWriter&& write_pass, const MfmaArgs& a, char* lds,
                                              int m0, int n0, int wm, int wn, int wave, int lane) {
  static_assert(!OUT16 || EPI == EPI_BIAS || EPI == EPI_GELU_TANH || EPI == EPI_GELU_ERF ||
                    EPI == EPI_BIAS_RES32_OUT32 || EPI == EPI_BIAS_RES32_OUT16,
                "fp16 outputs exist for the forward epilogues only");
  constexpr int WGN = NW / 2, WM = BM / 2, WN = BN / WGN;
  // The accumulators hold a lane-per-row layout (lane owns row lane&31 and four-column
  // groups), which would store 16-byte pieces scattered over 32 rows.  Each wave instead
  // transposes its block through the pipeline's LDS (free once every wave has left the
  // main loop) in passes of RP rows, and reads it back row-major: CW lanes cover one row
  // of the wave's WN columns, so every global load and store of the epilogue touches
  // whole cache lines.  The 16-byte chunks of a staged row are XOR-swizzled with the row
  // so that the column-wise writes spread over the banks.
  __builtin_amdgcn_s_barrier();
  constexpr int CW = WN / 4;                                 // 16-byte fp32 chunks per staged row
  constexpr int RP_FIT = LDS_BYTES / NW / (WN * 4);         // rows of the wave's block that fit its LDS share
  constexpr int RP = RP_FIT >= WM ? WM : RP_FIT / 32 * 32;   // rows per pass
  static_assert(RP >= 32 && WM % RP == 0 && 64 % CW == 0, "epilogue staging does not fit");
  constexpr int RPI = 64 / CW;                               // rows per read instruction
  float* stg = reinterpret_cast<float*>(lds + wave * (RP * WN * 4));
  const int rd_chunk = lane % CW, rd_row = lane / CW;
  const int n = n0 + wn * WN + rd_chunk * 4;
  const bool n_ok = n < a.N;
  constexpr bool RES32 = EPI == EPI_BIAS_RES32_OUT32 || EPI == EPI_BIAS_RES32_OUT16;
  constexpr bool GELU = EPI == EPI_GELU_TANH || EPI == EPI_GELU_ERF;
  constexpr bool DGELU = EPI == EPI_DGELU_TANH || EPI == EPI_DGELU_ERF;
  float bias_v[4] = {0.f, 0.f, 0.f, 0.f};
  // GeLU' epilogue: the lane's share of the column sums of C, before rounding to bf16 (the bias
  // gradient of the linear layer whose output gradient this product forms)
  float cs[4] = {0.f, 0.f, 0.f, 0.f};
  if constexpr (EPI == EPI_BIAS_RES || EPI == EPI_BIAS || RES32 || GELU) {
    if (a.bias && n_ok) {
      const bf16x4 b = *reinterpret_cast<const bf16x4*>(a.bias + n);
#pragma unroll
      for (int e = 0; e < 4; ++e) bias_v[e] = (float)b[e];
    }
  }
  // The readback goes in batches of UB row instructions.  The global loads of a batch (the
  // fp32 tile an accumulating product adds to, a residual, u for GeLU') depend on addresses
  // only, so they are issued one batch ahead -- the first before the tile is even staged --
  // and a batch's memory latency overlaps the staging and the arithmetic and stores of the
  // batch before it.
  constexpr int UB = 8, NPASS = WM / RP, BPP = RP / RPI / UB, NBATCH = NPASS * BPP;
  static_assert((RP / RPI) % UB == 0, "row batches");
  constexpr bool HAS_LOADS = EPI == EPI_ACCUM || RES32 || DGELU || EPI == EPI_BIAS_RES;
  struct Batch {
    f32x4 in32[UB];
    bf16x4 in16[UB];
    bool ok[UB];
    size_t o[UB];
  } bt[2];
  auto issue = [&](auto idx_c) {
    constexpr int idx = decltype(idx_c)::value, pass = idx / BPP, it0 = (idx % BPP) * UB;
    Batch& t = bt[idx & 1];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int row = (it0 + u) * RPI + rd_row;
      const int m = m0 + wm * WM + pass * RP + row;
      t.ok[u] = m < a.M && n_ok;
      t.o[u] = t.ok[u] ? (size_t)m * a.N + n : 0;  // element 0 is always a valid address
      if constexpr (EPI == EPI_ACCUM) t.in32[u] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(a.C) + t.o[u]);
      if constexpr (RES32) t.in32[u] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(a.residual) + t.o[u]);
      if constexpr (DGELU) t.in16[u] = *reinterpret_cast<const bf16x4*>(a.dgelu_u + t.o[u]);
      if constexpr (EPI == EPI_BIAS_RES) t.in16[u] = *reinterpret_cast<const bf16x4*>(static_cast<const bf16*>(a.residual) + t.o[u]);
    }
  };
  auto finish = [&](auto idx_c) {
    constexpr int idx = decltype(idx_c)::value, it0 = (idx % BPP) * UB;
    Batch& t = bt[idx & 1];
    f32x4 sv[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int row = (it0 + u) * RPI + rd_row;
      sv[u] = *reinterpret_cast<const f32x4*>(stg + row * WN + ((rd_chunk ^ (row & (CW - 1))) * 4));
    }
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      if (!t.ok[u]) continue;
      float v[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) v[e] = sv[u][e] + bias_v[e];
      if constexpr (EPI == EPI_ACCUM) {
        f32x4 c;
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = t.in32[u][e] + v[e];
        *reinterpret_cast<f32x4*>(static_cast<float*>(a.C) + t.o[u]) = c;
      } else if constexpr (GELU) {
        using T16 = std::conditional_t<OUT16, f16, bf16>;
        typedef T16 t16x4 __attribute__((ext_vector_type(4)));
        t16x4 uq, gq;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          uq[e] = from_f32<T16>(v[e]);
          // g is the GeLU of u AS STORED, so that a backward pass that recomputes g from
          // the stashed u gets the same bits
          gq[e] = from_f32<T16>(gelu_f<EPI == EPI_GELU_TANH ? 0 : 1>((float)uq[e]));
        }
        *reinterpret_cast<t16x4*>(static_cast<T16*>(a.C) + t.o[u]) = uq;
        *reinterpret_cast<t16x4*>(reinterpret_cast<T16*>(a.gelu_out) + t.o[u]) = gq;
      } else {
        if constexpr (DGELU) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] *= gelu_grad_f<EPI == EPI_DGELU_TANH ? 0 : 1>((float)t.in16[u][e]);
        }
        if constexpr (EPI == EPI_BIAS_RES) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += (float)t.in16[u][e];
        }
        if constexpr (RES32) {
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] += t.in32[u][e];
        }
        if constexpr (EPI == EPI_BIAS_RES32_OUT32) {
          f32x4 out;
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = v[e];
          *reinterpret_cast<f32x4*>(static_cast<float*>(a.C) + t.o[u]) = out;
        } else if constexpr (OUT16 && EPI == EPI_BIAS) {
          f16x4 out;
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = sat_f16(v[e]);
          *reinterpret_cast<f16x4*>(static_cast<f16*>(a.C) + t.o[u]) = out;
        } else {
          bf16x4 out;
#pragma unroll
          for (int e = 0; e < 4; ++e) out[e] = (bf16)v[e];
          *reinterpret_cast<bf16x4*>(static_cast<bf16*>(a.C) + t.o[u]) = out;
          if constexpr (DGELU) {
#pragma unroll
            for (int e = 0; e < 4; ++e) cs[e] += v[e];
          }
        }
      }
    }
  };
  if constexpr (HAS_LOADS) issue(std::integral_constant<int, 0>{});
  static_for<NBATCH>([&](auto idx_c) {
    constexpr int idx = decltype(idx_c)::value;
    if constexpr (idx % BPP == 0) {
      write_pass(std::integral_constant<int, idx / BPP>{}, std::integral_constant<int, RP>{}, stg);
      // LDS operations of one wave complete in order: no wait is needed between the
      // writes above and the reads below, only that the compiler keeps their order
      asm volatile("" ::: "memory");
    }
    if constexpr (HAS_LOADS) {
      if constexpr (idx + 1 < NBATCH) issue(std::integral_constant<int, idx + 1>{});
    } else {
      issue(idx_c);
    }
    finish(idx_c);
  });
  if constexpr (DGELU) {
    if (a.colsum) {
      // lanes CW apart hold the same columns of different rows
#pragma unroll
      for (int off = CW; off < 64; off <<= 1)
#pragma unroll
        for (int e = 0; e < 4; ++e) cs[e] += __shfl_xor(cs[e], off);
      if (lane < CW && n_ok) {
        f32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = cs[e];
        *reinterpret_cast<f32x4*>(a.colsum + (size_t)((m0 / BM) * 2 + wm) * a.N + n) = out;
      }
    }
  }
}

template <int BM, int BN, int BK, int NS, bool A_KMAJOR, bool B_KMAJOR, int EPI, bool B_IMG = false, int NW = 4>
__global__ __launch_bounds__(64 * NW) void gemm_mfma_kernel(const MfmaArgs a) {
  // NW waves in a 2 x (NW/2) grid
  constexpr int WGN = NW / 2;
  constexpr int WM = BM / 2, WN = BN / WGN, TM = WM / 32, TN = WN / 32, KS = BK / 16;
  static_assert(((NS & (NS - 1)) == 0 || NS == 5) && KS % 2 == 0, "stages: power of two or 5; even MFMA steps per slice");
  // k order inside fragments: natural unless both operands are K-major
  constexpr bool NAT = !(A_KMAJOR && B_KMAJOR);
  constexpr int A_BYTES = BM * BK * 2, B_BYTES = BN * BK * 2;
  constexpr int STAGE = A_BYTES + B_BYTES;  // one slice of both operands
  __shared__ __attribute__((aligned(1024))) char lds[NS * STAGE];
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)lds;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform (SGPR)
  const int wm = wave / WGN, wn = wave % WGN;

  // ---- workgroup -> tile --------------------------------------------------------
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int nb = tiles_m * tiles_n;
  int id = blockIdx.x;
  if ((nb & 7) == 0) id = (id & 7) * (nb >> 3) + (id >> 3);  // contiguous range per XCD
  constexpr int GROUP = 4;
  const int per_group = GROUP * tiles_n;
  const int grp = id / per_group, first_m = grp * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int tm_i = first_m + (id % per_group) % gsz, tn_i = (id % per_group) / gsz;
  const int m0 = tm_i * BM, n0 = tn_i * BN;

  const size_t lda = A_KMAJOR ? (size_t)a.M : (size_t)a.K;
  const size_t ldb = B_KMAJOR ? (size_t)a.N : (size_t)a.K;
  Operand<BM, WM, BK, A_KMAJOR, NAT, false, NW> opA;
  Operand<BN, WN, BK, B_KMAJOR, NAT, B_IMG, NW> opB;
  opA.init(m0, a.M, lda, wave, lane, wm * WM);
  opB.init(n0, a.N, ldb, wave, lane, wn * WN);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  const int nk = a.K / BK;
  // LDS reads per MFMA step and how many MFMAs to pair with each in the schedule
  constexpr int N_DS = (A_KMAJOR ? 2 : 1) * TM + (B_KMAJOR ? 2 : 1) * TN;
  constexpr int N_MMA = TM * TN;
  constexpr int N_PAIR = N_DS < N_MMA ? N_DS : N_MMA;  // (MFMA, DS read) pairs per step
  constexpr int N_DMA = (BM + BN) * BK * 2 / 1024 / NW;  // DMA instructions per wave and slice

  auto load_frags = [&](bf16x8(&fa)[TM], bf16x8(&fb)[TN], const char* stage, int ks) {
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[i] = opA.frag(stage, i, ks);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[j] = opB.frag(stage + A_BYTES, j, ks);
  };
  auto mma = [&](const bf16x8(&fa)[TM], const bf16x8(&fb)[TN]) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };
  // DMA instructions [part*N/PARTS, (part+1)*N/PARTS) of each operand's slice -> stage;
  // slice indices past the end are clamped: the copy is redundant but keeps the
  // loop body free of branches.
  constexpr int NIA = BM * BK * 2 / 1024 / NW, NIB = BN * BK * 2 / 1024 / NW;
  // MFMAs with linear index i*TN + j in [lo, hi)
  auto mma_range = [&](const bf16x8(&fa)[TM], const bf16x8(&fb)[TN], int lo, int hi) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        if (i * TN + j >= lo && i * TN + j < hi)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
  };
  auto issue_all = [&](int slice, int stage) {
    const int sl = min(slice, nk - 1);
    opA.issue(a.A, lda, sl, lds_base + stage * STAGE, wave);
    opB.issue(a.B, ldb, sl, lds_base + stage * STAGE + A_BYTES, wave);
  };

  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  if constexpr (NS == 5) {
    // Ring of five stages with PAIRED fetches.  A K-contiguous operand row contributes
    // only 64 bytes to a slice of 32, half a cache line; the other half belongs to the next
    // slice.  Fetching the two slices at different times asks the L2 for every line twice.
    // Here the DMA instructions of slices 2q and 2q+1 are issued back to back (same lane
    // addresses, +64 bytes), so the second request finds the line in, or on its way to, the
    // L1; each line is requested from the L2 once.  Slice t lives in stage t % 5; the pair
    // (t+3, t+4) is issued during every ODD iteration t, into the stages that slices t-2
    // and t-1 have left; even iterations issue nothing.  A slice is needed two or three
    // iterations after its issue.
    static_assert(KS == 2, "paired fetch is written for slices of two MFMA steps");
    constexpr int RING = 5 * STAGE;
    auto issue_pair_part = [&](int even_slice, uint32_t st_even, uint32_t st_odd, int j, bool second) {
      // instruction j of the A operand (j < NIA) or of the B operand, for one slice of the pair
      const int sl = min(even_slice + (second ? 1 : 0), nk - 1);
      const uint32_t base = lds_base + (second ? st_odd : st_even);
      if (j < NIA) opA.issue_one(a.A, lda, sl, base, wave, j);
      else opB.issue_one(a.B, ldb, sl, base + A_BYTES, wave, j - NIA);
    };
    // one MFMA step; H = 0: no DMA, H = 1 / 2: first / second half of the pair's instructions
    auto step5 = [&](const bf16x8(&fac)[TM], const bf16x8(&fbc)[TN], bf16x8(&fan)[TM], bf16x8(&fbn)[TN],
                     const char* stage_nxt, int ks_nxt, auto half, int even_slice, uint32_t st_even, uint32_t st_odd) {
      constexpr int H = decltype(half)::value;
      load_frags(fan, fbn, stage_nxt, ks_nxt);
      if constexpr (H == 0) {
        mma(fac, fbc);
        sched_pairs<N_PAIR, N_DS, N_MMA, 0>();
      } else {
        constexpr int ND = N_DMA;              // instructions of this step: N_DMA/2 per slice, two slices
        constexpr int N1 = N_DS < N_MMA - ND ? N_DS : N_MMA - ND;
        constexpr int Q = (N_MMA - N1) / ND;
        static_assert(Q >= 1, "not enough MFMAs to spread the DMA instructions");
        mma_range(fac, fbc, 0, N1);
        sched_pairs<N1, N_DS, N1, 0>();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < ND; ++d) {
          mma_range(fac, fbc, N1 + d * Q, N1 + (d + 1) * Q);
          __builtin_amdgcn_sched_barrier(0);
          issue_pair_part(even_slice, st_even, st_odd, (H - 1) * (N_DMA / 2) + d / 2, (d & 1) != 0);
          __builtin_amdgcn_sched_barrier(0);
        }
        mma_range(fac, fbc, N1 + ND * Q, N_MMA);
      }
    };
    auto next_stage = [&](uint32_t st) { return st + STAGE == RING ? 0u : st + STAGE; };
    std::integral_constant<int, 0> no_dma;
    std::integral_constant<int, 1> first_half;
    std::integral_constant<int, 2> second_half;
    // prologue: pairs (0,1) and (2,3) into stages 0..3
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int j = 0; j < N_DMA; ++j) {
        issue_pair_part(2 * q, (2 * q) * STAGE, (2 * q + 1) * STAGE, j, false);
        issue_pair_part(2 * q, (2 * q) * STAGE, (2 * q + 1) * STAGE, j, true);
      }
    wait_dma_and_barrier<2 * N_DMA>();   // pair 0 has landed
    load_frags(fa0, fb0, lds, 0);
    uint32_t st = 0;                     // stage offset of slice kt
    for (int kt = 0; kt < nk; kt += 2) {
      // even slice kt: nothing to fetch
      const uint32_t st1 = next_stage(st), st2 = next_stage(st1), st3 = next_stage(st2), st4 = next_stage(st3);
      step5(fa0, fb0, fa1, fb1, lds + st, 1, no_dma, 0, 0, 0);
      wait_dma_and_barrier<2 * N_DMA>();            // slice kt+1: every pair but the youngest has landed
      step5(fa1, fb1, fa0, fb0, lds + st1, 0, no_dma, 0, 0, 0);
      // odd slice kt+1: fetch the pair (kt+4, kt+5) into the stages of slices kt-1 and kt
      step5(fa0, fb0, fa1, fb1, lds + st1, 1, first_half, kt + 4, st4, st);
      wait_dma_and_barrier<N_DMA>();                // slice kt+2: only this iteration's first half may be in flight
      step5(fa1, fb1, fa0, fb0, lds + st2, 0, second_half, kt + 4, st4, st);
      st = st2;
    }
  } else if constexpr (NS >= 4) {
    // Deep pipeline: slice t lives in stage t % NS.  At the top of iteration kt slice
    // kt is complete, slices kt+1 .. kt+NS-2 are in flight and the stage of slice
    // kt-1 is free: slice kt+NS-1 is fetched into it during this iteration, its DMA
    // instructions spread evenly between the MFMAs of all steps so that the four
    // waves never queue up behind each other at the address unit (a wave blocked on
    // issuing a DMA cannot issue MFMAs either).
    static_assert(NIA % KS == 0 && NIB % KS == 0, "DMA instructions must split evenly over the steps");
    constexpr int PA = NIA / KS, PB = NIB / KS, PSTEP = PA + PB;
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_all(s, s);
    wait_dma_and_barrier<(NS - 2) * N_DMA>();
    load_frags(fa0, fb0, lds, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const char* st = lds + (kt & (NS - 1)) * STAGE;
      const uint32_t fill = lds_base + ((kt + NS - 1) & (NS - 1)) * STAGE;
      const int sl = min(kt + NS - 1, nk - 1);
      // One MFMA step: the LDS reads of the next step's fragments are paired with the
      // first N1 MFMAs; the step's share of the slice's DMA instructions (part p) is
      // issued one at a time between the remaining MFMAs.  The scheduling fences pin
      // that order: a wave is blocked while the address unit takes its DMA (the four
      // waves of the workgroup contend for it), and a block is only free when it falls
      // in the shadow of an MFMA that is already executing.
      constexpr int N1 = N_DS < N_MMA - PSTEP ? N_DS : N_MMA - PSTEP;
      constexpr int Q = (N_MMA - N1) / PSTEP;
      auto step = [&](const bf16x8(&fac)[TM], const bf16x8(&fbc)[TN], bf16x8(&fan)[TM], bf16x8(&fbn)[TN],
                      const char* stage_nxt, int ks_nxt, int p) {
        load_frags(fan, fbn, stage_nxt, ks_nxt);
        mma_range(fac, fbc, 0, N1);
        sched_pairs<N1, N_DS, N1, 0>();
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int d = 0; d < PSTEP; ++d) {
          mma_range(fac, fbc, N1 + d * Q, N1 + (d + 1) * Q);
          __builtin_amdgcn_sched_barrier(0);
          if (d < PA) opA.issue_one(a.A, lda, sl, fill, wave, p * PA + d);
          else opB.issue_one(a.B, ldb, sl, fill + A_BYTES, wave, p * PB + d - PA);
          __builtin_amdgcn_sched_barrier(0);
        }
        mma_range(fac, fbc, N1 + PSTEP * Q, N_MMA);
      };
      if constexpr (KS == 4) {
        step(fa0, fb0, fa1, fb1, st, 1, 0);
        step(fa1, fb1, fa0, fb0, st, 2, 1);
      }
      step(fa0, fb0, fa1, fb1, st, KS - 1, KS - 2);
      // slice kt+1 must have landed; younger DMAs may stay in flight
      wait_dma_and_barrier<(NS - 3) * N_DMA + (KS - 1) * PSTEP>();
      step(fa1, fb1, fa0, fb0, lds + ((kt + 1) & (NS - 1)) * STAGE, 0, KS - 1);
    }
  } else {
    // Two stages: slice kt+2 can only be fetched once every wave has taken its last
    // fragments of slice kt out of the stage, i.e. after the barrier of iteration kt.
    static_assert(NS == 2, "2 or >= 4 stages");
    issue_all(0, 0);
    issue_all(1, 1);
    wait_dma_and_barrier<N_DMA>();
    load_frags(fa0, fb0, lds, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1;
      const char* st = lds + cur * STAGE;
#pragma unroll
      for (int ks = 0; ks + 2 < KS; ks += 2) {
        load_frags(fa1, fb1, st, ks + 1);
        mma(fa0, fb0);
        sched_pairs<N_PAIR, N_DS, N_MMA, 0>();
        load_frags(fa0, fb0, st, ks + 2);
        mma(fa1, fb1);
        sched_pairs<N_PAIR, N_DS, N_MMA, 0>();
      }
      load_frags(fa1, fb1, st, KS - 1);
      mma(fa0, fb0);
      sched_pairs<N_PAIR, N_DS, N_MMA, 0>();
      wait_dma_and_barrier<0>();
      issue_all(kt + 2, cur);
      load_frags(fa0, fb0, lds + (cur ^ 1) * STAGE, 0);
      mma(fa1, fb1);
      sched_pairs<N_PAIR, N_DS, N_MMA, N_DMA>();
    }
  }
  // no DMA may still be writing LDS when the workgroup retires
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // lane owns row lane&31 of each 32x32 block and, per group g, columns 8g + 4*(lane>>5) .. +3
  auto write_pass = [&](auto pass_c, auto rp_c, float* stg) {
    constexpr int pass = decltype(pass_c)::value, TI = decltype(rp_c)::value / 32;
#pragma unroll
    for (int ii = 0; ii < TI; ++ii)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[pass * TI + ii][j][g * 4 + e];
          *reinterpret_cast<f32x4*>(stg + stage_slot<WN>(ii * 32 + (lane & 31), j * 8 + g * 2 + (lane >> 5))) = v;
        }
  };
  gemm_epilogue<BM, BN, EPI, NW, NS * STAGE>(write_pass, a, lds, m0, n0, wm, wn, wave, lane);
}

// ---- 16x16x32 products with hand-placed accumulators -------------------------------------
// The chip sustains a clearly higher clock on a stream of v_mfma_f32_16x16x32_bf16 than on the
// same flops issued as 32x32x16 (2.05 against 1.80 GHz on matrix instructions alone), so the
// K-contiguous products (forward; dgrad through the weight image) use the smaller shape.  The
// compiler, however, shuffles sixty-four 4-register accumulators between register files in
// every iteration, so here the accumulators are placed by hand: block (ib, jb) of the wave's
// 8 x 8 grid of 16x16 blocks lives in AGPRs a[4*(8*ib+jb) .. +3] for the whole kernel, the
// matrix instructions are inline assembly naming those registers, and the epilogue reads them
// back with v_accvgpr_read.  The compiler never allocates AGPRs in this kernel on its own (it
// has no matrix builtin and needs well under 256 ordinary registers); the clearing block below
// names all 256 as clobbered, which is what makes the kernel's register allocation include them.
// Operands are swapped as in the 32x32 kernel: D'[n][m] = B-fragment x A-fragment, so lane l
// holds, for output row m = l%16 of the block, the four columns n = 4*(l/16) .. +3.
// One workgroup: 256 x 256 tile, 4 waves (2 x 2, 128 x 128 each), K slices of 32 through the
// same four-stage DMA ring and LDS layout as gemm_mfma_kernel; a slice is ONE matrix step
// (k = 32): 8 A and 8 B fragments of 16 rows, 64 matrix instructions.  Fragments are double
// buffered in registers: while slice t is multiplied, the 16 fragments of slice t+1 are read
// from LDS and the 8 DMA instructions of slice t+3 are issued, one LDS read after every 4 and
// one DMA after every 8 matrix instructions.  One barrier per slice, at its start.
// (Staging the slices through registers -- plain loads two slices ahead, ds_write into a
// two-stage ring -- was measured 3-6 % slower than the DMA ring in this kernel.)
// KM: both operands K-major (wgrad: A is [K, M], B is [K, N]); their slices sit in LDS as they
// sit in memory (32 k-rows of 512 bytes, 32-byte units swizzled with the k-row) and a fragment
// is two transposing reads: lane group lane>>4 is the k-octet, lane&15 the column.
// F16: both operands hold fp16 values (A an activation stored in fp16, B the fp16 image of a
// weight); the f16 form of the matrix instruction is used and the 16-bit outputs are fp16.
// BKM: only B is K-major (data gradient on the raw weight: A = dOut [M, K] K-contiguous, B = W
// [K, N]); A fragments are plain 16-byte reads, B fragments transposing reads -- both hand a
// lane the same eight k values, so the two kinds mix freely.
template <int EPI, bool B_IMG, bool KM = false, bool F16 = false, bool BKM = false>
__global__ __launch_bounds__(256) void gemm_mi16_kernel(const MfmaArgs a) {
  static_assert(!(KM && B_IMG) && !(BKM && (KM || B_IMG)), "images are K-contiguous; BKM is the mixed form");
  constexpr bool B_KM = KM || BKM;
  static_assert(!F16 || B_IMG, "fp16 products read the weight through its fp16 image");
  constexpr int BM = 256, BN = 256, BK = 32, NS = 4, NW = 4, WGN = 2;
  constexpr int WM = BM / 2, WN = BN / WGN, NB = WM / 16;   // 8 x 8 blocks of 16 x 16 per wave
  constexpr int A_BYTES = BM * BK * 2, STAGE = A_BYTES + BN * BK * 2, RB = BK * 2;
  __shared__ __attribute__((aligned(1024))) char lds[NS * STAGE];
  const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)lds;

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int nb = tiles_m * tiles_n;
  int id = blockIdx.x;
  if ((nb & 7) == 0) id = (id & 7) * (nb >> 3) + (id >> 3);  // contiguous range per XCD
  constexpr int GROUP = 4;
  const int per_group = GROUP * tiles_n;
  const int grp = id / per_group, first_m = grp * GROUP;
  const int gsz = min(tiles_m - first_m, GROUP);
  const int tm_i = first_m + (id % per_group) % gsz, tn_i = (id % per_group) / gsz;
  const int m0 = tm_i * BM, n0 = tn_i * BN;
  const int sps = a.K / BK;                     // slices per K segment: a multiple of 4 (checked by the dispatcher)
  const int nk = sps * a.k_segments;

  const size_t lda = KM ? (size_t)a.M : (size_t)a.K, ldb = B_KM ? (size_t)a.N : (size_t)a.K;
  Operand<BM, WM, BK, KM, true, false, NW> opA;
  Operand<BN, WN, BK, B_KM, true, B_IMG, NW> opB;
  opA.init(m0, a.M, lda, wave, lane, wm * WM);
  opB.init(n0, a.N, ldb, wave, lane, wn * WN);
  constexpr int NIA = BM * BK * 2 / 1024 / NW, NIB = BN * BK * 2 / 1024 / NW, N_DMA = NIA + NIB;
  static_assert(N_DMA == 8 && NB == 8, "the slice schedule below is written for 8 DMA instructions and 8 x 8 blocks");

  // K-contiguous: fragment of 16 rows x 32 k: lane reads chunk lane>>4 of row lane&15 (the
  // swizzle has period 16 rows)
  const int frag_off = (lane & 15) * RB + (((lane >> 4) ^ swz_kc<BK / 8>(lane & 15)) << 4);
  const char* fragA = lds + (KM ? 0 : wm * WM * RB + frag_off);
  const char* fragB = lds + A_BYTES + (B_KM ? 0 : wn * WN * RB + frag_off);
  // K-major: transposing read t (0, 1) of block rb fetches k-rows 8*(lane>>4) + 4t + 0..3 of the
  // block's 16 columns; the lane supplies the address of k-row +(lane&15)>>2, 8-byte piece lane&3
  int rdA[KM ? 2 : 1][KM ? NB : 1], rdB[B_KM ? 2 : 1][B_KM ? NB : 1];
  if constexpr (B_KM) {
    constexpr int ROWB = BM * 2;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int k = 8 * (lane >> 4) + 4 * t + ((lane & 15) >> 2), sw = swz_km<true>(k);
#pragma unroll
      for (int rb = 0; rb < NB; ++rb) {
        if constexpr (KM) rdA[t][rb] = k * ROWB + (((((wm * WM) >> 4) + rb) ^ sw) << 5) + (lane & 3) * 8;
        rdB[t][rb] = k * ROWB + (((((wn * WN) >> 4) + rb) ^ sw) << 5) + (lane & 3) * 8;
      }
    }
  }
  auto frag_a = [&](int stage, int rb) -> bf16x8 {
    if constexpr (!KM) return *reinterpret_cast<const bf16x8*>(fragA + stage * STAGE + rb * 16 * RB);
    else return tr_pair(fragA + stage * STAGE + rdA[0][rb], fragA + stage * STAGE + rdA[1][rb]);
  };
  auto frag_b = [&](int stage, int rb) -> bf16x8 {
    if constexpr (!B_KM) return *reinterpret_cast<const bf16x8*>(fragB + stage * STAGE + rb * 16 * RB);
    else return tr_pair(fragB + stage * STAGE + rdB[0][rb], fragB + stage * STAGE + rdB[1][rb]);
  };
  bf16x8 fa[2][NB], fb[2][NB];

  agpr_clear_all();

  // K-major operands may come in segments (see MfmaArgs): the slice being fetched is tracked by
  // its base addresses, advanced once per slice with wave-uniform arithmetic -- one slice down
  // inside a segment, to the next segment's start at its end.  The first NS-1 slices lie in the
  // first segment (a segment has at least 4 slices).
  const bf16* fillA = a.A;
  const bf16* fillB = a.B;
  int fill_slice = 0, fill_in_seg = 0;
  auto advance_fill = [&]() {
    if constexpr (KM) {
      if (fill_slice < nk - 1) {     // past the end the last slice is fetched again (redundant, branch-free loop)
        ++fill_slice;
        if (++fill_in_seg == sps) {
          fill_in_seg = 0;
          fillA += a.seg_stride_a - (size_t)(sps - 1) * BK * lda;
          fillB += a.seg_stride_b - (size_t)(sps - 1) * BK * ldb;
        } else {
          fillA += (size_t)BK * lda;
          fillB += (size_t)BK * ldb;
        }
      }
    }
  };
  auto dma = [&](int slice, int stage, int i) {   // DMA instruction i of a slice: A first, then B
    if constexpr (KM) {
      if (i < NIA) opA.issue_at(fillA, lds_base + stage * STAGE, wave, i);
      else opB.issue_at(fillB, lds_base + stage * STAGE + A_BYTES, wave, i - NIA);
    } else {
      const int sl = min(slice, nk - 1);
      if (i < NIA) opA.issue_one(a.A, lda, sl, lds_base + stage * STAGE, wave, i);
      else opB.issue_one(a.B, ldb, sl, lds_base + stage * STAGE + A_BYTES, wave, i - NIA);
    }
  };
#pragma unroll
  for (int s0 = 0; s0 < NS - 1; ++s0) {
#pragma unroll
    for (int i = 0; i < N_DMA; ++i) dma(s0, s0, i);
    advance_fill();
  }
  wait_dma_and_barrier<(NS - 2) * N_DMA>();   // slice 0 has landed
#pragma unroll
  for (int u = 0; u < NB; ++u) {
    fa[0][u] = frag_a(0, u);
    fb[0][u] = frag_b(0, u);
  }

  for (int kt = 0; kt < nk; kt += NS) {
    static_for<NS>([&](auto r_c) {
      constexpr int r = decltype(r_c)::value, cur = r & 1, nxt = cur ^ 1;
      constexpr int st_next = (r + 1) % NS, st_fill = (r + NS - 1) % NS;
      const int t = kt + r;
      // slice t+1 has landed (only the copies of slice t+2 may still be in flight); every wave
      // has finished reading slices <= t from LDS
      wait_dma_and_barrier<N_DMA>();
      static_for<16>([&](auto g_c) {
        constexpr int g = decltype(g_c)::value;
        // four matrix instructions: block row g/2, block columns 4*(g%2) .. +3
        // (block columns run forwards in even block rows and backwards in odd ones, so that
        // exactly one operand changes from one instruction to the next)
        static_for<4>([&](auto q_c) {
          constexpr int ib = g / 2, j0 = 4 * (g % 2) + decltype(q_c)::value, jb = (ib & 1) ? NB - 1 - j0 : j0;
          mfma16_at<4 * (NB * ib + jb), F16>(fb[cur][jb], fa[cur][ib]);
        });
        __builtin_amdgcn_sched_barrier(0);
        // one fragment of the next slice
        if constexpr (g < NB) fa[nxt][g] = frag_a(st_next, g);
        else fb[nxt][g - NB] = frag_b(st_next, g - NB);
        // and after every second group one DMA instruction of slice t+3
        if constexpr (g % 2 == 1) dma(t + NS - 1, st_fill, g / 2);
        __builtin_amdgcn_sched_barrier(0);
      });
      advance_fill();
    });
  }
  // no DMA may still be writing LDS when the staging starts; the matrix pipeline must have
  // drained before the accumulators are read (the compiler does not know they were written)
  asm volatile("s_waitcnt vmcnt(0)\n\ts_nop 15\n\ts_nop 15\n\ts_nop 15" ::: "memory");

  auto write_pass = [&](auto pass_c, auto rp_c, float* stg) {
    constexpr int pass = decltype(pass_c)::value, BI = decltype(rp_c)::value / 16;   // block rows per pass
    static_for<BI * NB>([&](auto b_c) {
      constexpr int ii = decltype(b_c)::value / NB, jb = decltype(b_c)::value % NB;
      constexpr int R = 4 * (NB * (pass * BI + ii) + jb);
      f32x4 v;
      v[0] = agpr_read<R>();
      v[1] = agpr_read<R + 1>();
      v[2] = agpr_read<R + 2>();
      v[3] = agpr_read<R + 3>();
      *reinterpret_cast<f32x4*>(stg + stage_slot<WN>(ii * 16 + (lane & 15), jb * 4 + (lane >> 4))) = v;
    });
  };
  gemm_epilogue<BM, BN, EPI, NW, NS * STAGE, F16>(write_pass, a, lds, m0, n0, wm, wn, wave, lane);
}

template <int EPI, bool B_IMG, bool KM = false, bool F16 = false, bool BKM = false>
hipError_t launch_mi16(const MfmaArgs& a, hipStream_t st) {
  const int tiles = ((a.M + 255) / 256) * ((a.N + 255) / 256);
  hipLaunchKernelGGL((gemm_mi16_kernel<EPI, B_IMG, KM, F16, BKM>), dim3(tiles), dim3(256), 0, st, a);
  return hipGetLastError();
}

template <int BM, int BN, int BK, int NS, bool AK, bool BKM, int EPI, bool B_IMG = false, int NW = 4>
hipError_t launch(const MfmaArgs& a, hipStream_t st) {
  const int tiles = ((a.M + BM - 1) / BM) * ((a.N + BN - 1) / BN);
  hipLaunchKernelGGL((gemm_mfma_kernel<BM, BN, BK, NS, AK, BKM, EPI, B_IMG, NW>), dim3(tiles), dim3(64 * NW), 0,
                     st, a);
  return hipGetLastError();
}

// Tile choice: 256x256 (slices of 32, four LDS stages: three slices in flight) from 100 tiles
// up, else 128x128 (slices of 64, two stages, two workgroups per CU) to recover occupancy on
// small problems.  Measured on whole stages: at 144-192 tiles (M = 2048 or 4096 tokens against
// N = 4608 ... 5120) the large tile is 10-25 % faster per product although it leaves a third of
// the CUs idle; at 64 tiles it is 30 % slower.
#ifndef GPTS_BIG_TILE_MIN
#define GPTS_BIG_TILE_MIN 100
#endif
bool use_big_tiles(int M, int N) { return (long)((M + 255) / 256) * ((N + 255) / 256) >= GPTS_BIG_TILE_MIN; }

template <bool AK, bool BKM, int EPI> hipError_t pick_tile(const MfmaArgs& a, hipStream_t st) {
  if (use_big_tiles(a.M, a.N)) {
    // both operands K-contiguous (forward on raw weights) or both K-major (wgrad): the
    // 16x16x32 kernel
    if constexpr (AK == BKM) {
      if (a.K % 128 == 0) return launch_mi16<EPI, false, AK>(a, st);
    }
    // data gradient on the raw weight (A K-contiguous, B K-major): the mixed form of the same kernel
    if constexpr (!AK && BKM) {
      if (a.K % 128 == 0) return launch_mi16<EPI, false, false, false, true>(a, st);
    }
    // otherwise the 32x32x16 kernel (a K-contiguous A takes its five-stage ring with paired fetches)
    return launch<256, 256, 32, AK ? 4 : GPTS_KC_STAGES, AK, BKM, EPI, false, GPTS_BIG_WAVES>(a, st);
  }
  return launch<128, 128, 64, 2, AK, BKM, EPI>(a, st);
}

// ---- operand images -----------------------------------------------------------------
// image[tile][slice][slot] with slot = row*4 + physical chunk, holding logical chunk
// (physical ^ swizzle(row)) of row tile*256+row, k = slice*32 + chunk*8 .. +7, where
// element (n, k) of the operand is src[n*sn + k*sk].  Rows past N are zero.  One
// workgroup per (slice, tile): the 32 x 256 source patch goes through LDS so that both
// the reads (along whichever index is contiguous in src) and the writes are coalesced.
// TO_F16: the image holds the values converted to fp16 (exact for magnitudes in
// [2^-14, 65504]; smaller ones become fp16 subnormals, absolute error <= 2^-25; larger ones
// saturate), for products whose other operand is an fp16 activation.
template <bool TO_F16>
__global__ __launch_bounds__(256) void prepare_image_kernel(const bf16* __restrict__ src, bf16* __restrict__ img,
                                                            int N, int K, size_t sn, size_t sk) {
  __shared__ bf16 patch[256][32 + 2];   // [row n][k], padded
  const int kt = blockIdx.x, tn = blockIdx.y, nk = K / 32;
  const int n0 = tn * 256, k0 = kt * 32;
  if (sk == 1) {           // rows contiguous along k: thread loads 8 k of one row, 4 times
    for (int i = threadIdx.x; i < 256 * 4; i += 256) {
      const int r = i >> 2, c = i & 3;
      bf16x8 v;
      if (n0 + r < N) v = *reinterpret_cast<const bf16x8*>(src + (size_t)(n0 + r) * sn + k0 + c * 8);
      else for (int e = 0; e < 8; ++e) v[e] = (bf16)0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) patch[r][c * 8 + e] = v[e];
    }
  } else {                 // contiguous along n (sn == 1): thread loads 8 n of one k-row
    for (int i = threadIdx.x; i < 32 * 32; i += 256) {
      const int k = i >> 5, c = i & 31;
      bf16x8 v;
      if (n0 + c * 8 < N) v = *reinterpret_cast<const bf16x8*>(src + (size_t)(k0 + k) * sk + n0 + c * 8);
      else for (int e = 0; e < 8; ++e) v[e] = (bf16)0.f;
#pragma unroll
      for (int e = 0; e < 8; ++e) patch[c * 8 + e][k] = v[e];
    }
  }
  __syncthreads();
  bf16* out = img + ((size_t)tn * nk + kt) * (256 * 32);
  for (int slot = threadIdx.x; slot < 256 * 4; slot += 256) {
    const int r = slot >> 2, c = (slot & 3) ^ swz_kc<4>(r);
    if constexpr (TO_F16) {
      f16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = sat_f16((float)patch[r][c * 8 + e]);
      *reinterpret_cast<f16x8*>(out + (size_t)slot * 8) = v;
    } else {
      bf16x8 v;
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = patch[r][c * 8 + e];
      *reinterpret_cast<bf16x8*>(out + (size_t)slot * 8) = v;
    }
  }
}

}  // namespace

bool gemm_mfma_supported(int form, int M, int N, int K) {
  (void)form;
  return M >= 64 && N >= 64 && K >= 64 && M % 8 == 0 && N % 8 == 0 && K % 64 == 0 &&
         (size_t)M * K < (1ull << 31) && (size_t)N * K < (1ull << 31);
}

// A weight-gradient product whose contraction is split over several buffers runs as one launch
// of the 16x16x32 K-major kernel: the shape must be one that kernel takes (K here is the
// length of one segment).
bool gemm_wgrad_segments_supported(int form, int M, int N, int K) {
  return form == 2 && gemm_mfma_supported(form, M, N, K) && use_big_tiles(M, N) && K % 128 == 0;
}

int gemm_mfma_colsum_rows(int M, int N) {
  const int bm = use_big_tiles(M, N) ? 256 : 128;
  return 2 * ((M + bm - 1) / bm);
}

size_t gemm_image_elems(int N, int K) { return (size_t)((N + 255) / 256) * 256 * K; }

hipError_t gemm_prepare_image(const void* src, void* img, int N, int K, bool transposed, hipStream_t st,
                              bool to_f16) {
  // operand element (n, k) = src[n*K + k] (src is [N,K]) or src[k*N + n] (src is [K,N])
  dim3 g(K / 32, (N + 255) / 256);
  const size_t sn = transposed ? (size_t)1 : (size_t)K, sk = transposed ? (size_t)N : (size_t)1;
  if (to_f16)
    hipLaunchKernelGGL(prepare_image_kernel<true>, g, dim3(256), 0, st, (const bf16*)src, (bf16*)img, N, K, sn, sk);
  else
    hipLaunchKernelGGL(prepare_image_kernel<false>, g, dim3(256), 0, st, (const bf16*)src, (bf16*)img, N, K, sn, sk);
  return hipGetLastError();
}

bool gemm_fwd_f16_supported(int M, int N, int K) {
  return M >= 1 && N >= 8 && N % 8 == 0 && K >= 128 && K % 128 == 0 && (size_t)M * K < (1ull << 31) &&
         (size_t)((N + 255) / 256) * 256 * K < (1ull << 31);
}

hipError_t gemm_fwd_f16(int M, int N, int K, const void* A, const void* b_image, void* C,
                        const GemmEpilogue& ep, hipStream_t st) {
  if (!gemm_fwd_f16_supported(M, N, K) || !b_image) return hipErrorInvalidValue;
  MfmaArgs a;
  a.A = (const bf16*)A; a.B = (const bf16*)b_image; a.C = C;
  a.M = M; a.N = N; a.K = K;
  a.bias = (const bf16*)ep.bias; a.residual = ep.residual;
  a.gelu_out = (bf16*)ep.gelu_out; a.dgelu_u = nullptr; a.colsum = nullptr;
  if (ep.gelu_out)
    return ep.gelu_kind == 0 ? launch_mi16<EPI_GELU_TANH, true, false, true>(a, st)
                             : launch_mi16<EPI_GELU_ERF, true, false, true>(a, st);
  if (ep.residual) {
    if (!ep.residual_f32) return hipErrorInvalidValue;
    return ep.out_f32 ? launch_mi16<EPI_BIAS_RES32_OUT32, true, false, true>(a, st)
                      : launch_mi16<EPI_BIAS_RES32_OUT16, true, false, true>(a, st);
  }
  return launch_mi16<EPI_BIAS, true, false, true>(a, st);
}

hipError_t gemm_mfma(int form, int M, int N, int K, const void* A, const void* B, void* C,
                     const GemmEpilogue& ep, hipStream_t st) {
  MfmaArgs a;
  a.A = (const bf16*)A; a.B = (const bf16*)B; a.C = C;
  a.M = M; a.N = N; a.K = K;
  a.bias = (const bf16*)ep.bias; a.residual = ep.residual;
  a.gelu_out = (bf16*)ep.gelu_out; a.dgelu_u = (const bf16*)ep.dgelu_u;
  a.colsum = ep.dgelu_u ? ep.colsum_partial : nullptr;
  if (ep.k_segments > 1) {
    if (!gemm_wgrad_segments_supported(form, M, N, K)) return hipErrorInvalidValue;
    a.k_segments = ep.k_segments;
    a.seg_stride_a = ep.seg_stride_a;
    a.seg_stride_b = ep.seg_stride_b;
    return launch_mi16<EPI_ACCUM, false, true>(a, st);
  }
  if (ep.b_image && form != 2 && use_big_tiles(M, N)) {
    // B comes as the image of its [N rows, K] K-contiguous view: forward and dgrad are
    // then the same product with different epilogues.
    a.B = (const bf16*)ep.b_image;
    const bool mi16 = K % 128 == 0;
#define GPTS_IMG(EPI) (mi16 ? launch_mi16<EPI, true>(a, st) : launch<256, 256, 32, 4, false, false, EPI, true, GPTS_BIG_WAVES>(a, st))
    if (form == 0) {
      if (ep.gelu_out) return ep.gelu_kind == 0 ? GPTS_IMG(EPI_GELU_TANH) : GPTS_IMG(EPI_GELU_ERF);
      if (ep.residual && ep.residual_f32) return ep.out_f32 ? GPTS_IMG(EPI_BIAS_RES32_OUT32) : GPTS_IMG(EPI_BIAS_RES32_OUT16);
      return ep.residual ? GPTS_IMG(EPI_BIAS_RES) : GPTS_IMG(EPI_BIAS);
    }
    if (ep.dgelu_u) return ep.gelu_kind == 0 ? GPTS_IMG(EPI_DGELU_TANH) : GPTS_IMG(EPI_DGELU_ERF);
    return GPTS_IMG(EPI_PLAIN);
#undef GPTS_IMG
  }
  if (form == 0) {
    if (ep.gelu_out)
      return ep.gelu_kind == 0 ? pick_tile<false, false, EPI_GELU_TANH>(a, st)
                               : pick_tile<false, false, EPI_GELU_ERF>(a, st);
    if (ep.residual && ep.residual_f32)
      return ep.out_f32 ? pick_tile<false, false, EPI_BIAS_RES32_OUT32>(a, st)
                        : pick_tile<false, false, EPI_BIAS_RES32_OUT16>(a, st);
    return ep.residual ? pick_tile<false, false, EPI_BIAS_RES>(a, st) : pick_tile<false, false, EPI_BIAS>(a, st);
  }
  if (form == 1) {
    if (ep.dgelu_u)
      return ep.gelu_kind == 0 ? pick_tile<false, true, EPI_DGELU_TANH>(a, st)
                               : pick_tile<false, true, EPI_DGELU_ERF>(a, st);
    return pick_tile<false, true, EPI_PLAIN>(a, st);
  }
  return pick_tile<true, true, EPI_ACCUM>(a, st);
}

}  // namespace gpts
