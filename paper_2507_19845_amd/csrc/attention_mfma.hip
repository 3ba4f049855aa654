// Causal softmax attention on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// Forward, per (batch, head): a workgroup owns 128 query rows (4 waves x 32) and
// walks the key/value rows in tiles of 64 up to the diagonal with an online
// softmax.  Both products are computed TRANSPOSED so that no value ever has to
// move between lanes:
//   S^T[key][query] = K Q^T      A-operand = K fragment (ds_read_b128 from the
//                                K tile), B-operand = Q fragment (registers)
//   O^T[d][query]   = V^T P^T    A-operand = V^T fragment, B-operand = P^T, which
//                                is exactly the S^T accumulator of the same lane,
//                                rounded to bf16.
// A lane therefore owns one query column throughout: its running max, running
// sum and the rescaling of O are per-lane scalars; only the max needs one
// exchange with the lane that holds the other half of the keys (lane ^ 32).
//
// Every product that contracts over the sequence index (O^T = V^T P^T, and in the
// backward pass dV^T = dO^T P, dK^T = Q^T dS, dQ^T = K^T dS^T) needs its A operand
// with the sequence index running fastest.  The transposing LDS read delivers that from
// a row-major tile, but at well under half the bandwidth of a plain 16-byte read, and
// these kernels are bound by LDS bandwidth.  So a small kernel first writes a
// "transposed image" of each such matrix (attn_timage_kernel): per (batch, head) and
// 64-row tile, the tile as [D][64] with
//   * the 64 sequence positions permuted inside each group of 16 into the order in which
//     an MFMA accumulator hands out its rows (8t + 4*half + j  ->  8*half + 4t + j), so
//     that the 8 values a lane needs are one 16-byte chunk, and
//   * the 16-byte chunks of a row XOR-swizzled with the row for conflict-free reads,
// stored contiguously, so that a tile arrives in LDS by a flat DMA copy.
// K, V, Q and dO tiles in their natural [row][D] form go global -> LDS by DMA as well,
// double buffered.
#include "kernels.hpp"

namespace gpts {
namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));

// Wave priority inside the kernels: raised around a run of matrix instructions, so that of the
// two waves sharing a SIMD the one feeding the matrix pipe issues first and the other's softmax
// arithmetic fills the gaps (measured: forward +1.7 %, backward +1 %).
#define GPTS_PRIO(p) __builtin_amdgcn_s_setprio(p)

constexpr int BQ = 128;   // queries per workgroup of the forward kernel
constexpr int BKV = 64;   // rows per streamed tile
constexpr int BW = 256;   // rows owned by a workgroup of the backward kernels (8 waves x 32)

__device__ __forceinline__ int swz16(int row) { return (row & 7) ^ ((row >> 3) & 1); }

// Eight accumulator values rounded to 16 bits as the next product's operand.  All operand
// registers are typed bf16x8; with F16 they hold fp16 bits (forward activations kept in fp16).
template <bool F16 = false> __device__ __forceinline__ bf16x8 pack8(const f32x16& v, int base) {
  if constexpr (F16) {
    f16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (f16)v[base + e];
    return __builtin_bit_cast(bf16x8, r);
  } else {
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (bf16)v[base + e];
    return r;
  }
}
// acc += A (32 x 16) * B (16 x 32); F16: the operand registers hold fp16 values
template <bool F16 = false>
__device__ __forceinline__ f32x16 mma32(const bf16x8& a, const bf16x8& b, const f32x16& acc) {
  if constexpr (F16)
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), acc, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
}

// Marks a register value as used.  The tiles travel by DMA instructions the compiler
// does not track, while ordinary global loads it does track are waited for with
// "s_waitcnt vmcnt(n)" in front of their first use.  If that first use sits inside the
// tile loop, the wait stays there in every iteration and -- the counter being shared --
// also drains the next tile's DMA, which removes the double buffering.  Using the loaded
// registers once before the loop moves the wait in front of the loop.
__device__ __forceinline__ void settle(const bf16x8& v) {
  asm volatile("" ::"v"(__builtin_bit_cast(i32x4, v)));
}
__device__ __forceinline__ void settle(float v) { asm volatile("" ::"v"(v)); }

__device__ __forceinline__ uint32_t lds_addr(const void* p) {
  return (uint32_t)(size_t)(__attribute__((address_space(3))) const char*)p;
}

// One DMA instruction: lane i copies 16 bytes from src + off_i to LDS dst + 16*i.
// Inline assembly on purpose (see settle()): the kernels wait for these copies
// explicitly (s_waitcnt vmcnt(0)) before the barrier that publishes a tile.
__device__ __forceinline__ void dma16(const void* src, uint32_t off, uint32_t dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(dst), "v"(off), "s"(src) : "memory");
}
// 64 floats global -> LDS by one DMA instruction of one wave (lane i: src[idx_i] -> dst[i])
__device__ __forceinline__ void dma_floats(const float* __restrict__ src, int idx, float* dst) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_addr(dst)), "v"((uint32_t)idx * 4u), "s"(src) : "memory");
}

// A [64][D] bf16 tile in LDS: row r, 16-byte chunk c stored at
// r*(2D) + ((c ^ swz(r)) << 4), swz(r) = swz16(r) cut to the chunks a row has (the XOR only
// touches the low 3 bits of c; a row of head dimension 32 has 4 chunks, so 2 bits there).
// 64 rows starting at global row `row0` (clamped to < S) are copied by the NW waves
// of the workgroup; each DMA instruction moves 1 KiB (a tile of fewer instructions than waves
// is copied by the first waves only).
template <int D, int NW>
__device__ __forceinline__ void dma_tile(const bf16* __restrict__ src, size_t ld, int row0, int S,
                                         char* tile, int wave, int lane) {
  constexpr int ROWB = D * 2;              // bytes per row
  constexpr int CPR = ROWB / 16;           // chunks per row
  constexpr int NT = BKV * ROWB / 1024;        // instructions per tile
  constexpr int NI = NT >= NW ? NT / NW : 1;   // instructions per (issuing) wave
  static_assert(NT >= 1 && (NT >= NW ? NT % NW == 0 : true), "tile / wave count mismatch");
  if (NT < NW && wave >= NT) return;
  const uint32_t lds_tile = lds_addr(tile);
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int slot = (wave * NI + i) * 64 + lane;
    const int r = slot / CPR, pc = slot % CPR;
    const int c = pc ^ (swz16(r) & (CPR - 1));
    int gr = row0 + r;
    gr = gr < S ? gr : S - 1;
    dma16(src, (uint32_t)(((size_t)gr * ld + c * 8) * 2), lds_tile + (wave * NI + i) * 1024);
  }
}
// A transposed-image tile (D*128 contiguous bytes) global -> LDS, flat.
template <int D, int NW>
__device__ __forceinline__ void dma_image(const bf16* __restrict__ tile_src, char* tile, int wave, int lane) {
  constexpr int NT = D * 128 / 1024;
  constexpr int NI = NT >= NW ? NT / NW : 1;
  static_assert(NT >= 1 && (NT >= NW ? NT % NW == 0 : true), "tile / wave count mismatch");
  if (NT < NW && wave >= NT) return;
  const uint32_t lds_tile = lds_addr(tile);
#pragma unroll
  for (int i = 0; i < NI; ++i)
    dma16(tile_src, (uint32_t)(((wave * NI + i) * 64 + lane) * 16), lds_tile + (wave * NI + i) * 1024);
}

// ---- transposed images ----------------------------------------------------------------
struct TImageArgs {
  const bf16* src[3];  // element (b, s, head n, d) at src + (b*S + s)*ld + n*D + d
  size_t ld[3];
  bf16* dst[3];        // image: [b][n][tile][D][64]
  int n_src;
};
// chunk c (8 positions) of a transposed row holds the sequence positions
//   16*(c>>1) + 8*(p>>2) + 4*(c&1) + (p&3),  p = 0..7
// and is stored at chunk position c ^ ((d>>1)&7) of row d.  Rows past S are zero.
template <int D>
__global__ __launch_bounds__(256) void attn_timage_kernel(const TImageArgs args, int S, int a) {
  constexpr int PITCH = D + 2;  // bf16 elements; odd number of 32-bit words per row
  __shared__ __attribute__((aligned(16))) bf16 stage[BKV * PITCH];
  const int t = blockIdx.x, n = blockIdx.y;
  const int b = blockIdx.z / args.n_src, w = blockIdx.z % args.n_src;
  const bf16* src = args.src[w] + (size_t)b * S * args.ld[w] + (size_t)n * D;
  constexpr int TPR = D / 8, RPP = 256 / TPR;  // threads per row, rows per pass
#pragma unroll
  for (int p = 0; p < BKV / RPP; ++p) {
    const int r = p * RPP + threadIdx.x / TPR, cc = threadIdx.x % TPR;
    const int s = t * BKV + r;
    bf16x8 v;
    if (s < S) {
      v = *reinterpret_cast<const bf16x8*>(src + (size_t)s * args.ld[w] + cc * 8);
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[e] = (bf16)0.f;
    }
    uint32_t* dstw = reinterpret_cast<uint32_t*>(stage + r * PITCH + cc * 8);
    const i32x4 vi = __builtin_bit_cast(i32x4, v);
#pragma unroll
    for (int e = 0; e < 4; ++e) dstw[e] = (uint32_t)vi[e];
  }
  __syncthreads();
  const int ntile = (S + BKV - 1) / BKV;
  bf16* out = args.dst[w] + (((size_t)b * a + n) * ntile + t) * (size_t)(D * BKV);
#pragma unroll
  for (int it = 0; it < D * 8 / 256; ++it) {
    const int slot = it * 256 + threadIdx.x;
    const int d = slot >> 3, cpos = slot & 7;
    const int c = cpos ^ ((d >> 1) & 7);
    bf16x8 v;
#pragma unroll
    for (int p = 0; p < 8; ++p) {
      const int s = 16 * (c >> 1) + 8 * (p >> 2) + 4 * (c & 1) + (p & 3);
      v[p] = stage[s * PITCH + d];
    }
    *reinterpret_cast<bf16x8*>(out + (size_t)slot * 8) = v;
  }
}

// Image fragment (A operand, 32 rows d x 16 sequence positions): the lane's byte offset
// inside an image tile for d-block 0 and 16-group 0; d-block db adds db*4096, 16-group g
// XORs g<<5 (the chunk index is 2g + half, swizzled with (d>>1)&7 -- and (32*db)>>1 is a
// multiple of 8).
__device__ __forceinline__ int image_frag_off(int ql, int h) { return ql * 128 + ((h ^ ((ql >> 1) & 7)) << 4); }
// Natural-tile fragment (A operand, 32 rows x 16 d): byte offset for row block 0 and
// k-step 0; row block rb adds rb*32*ROWB, k-step kk XORs kk<<5.
template <int D> __device__ __forceinline__ int natural_frag_off(int ql, int h) {
  return ql * (D * 2) + ((h ^ (swz16(ql) & (D / 8 - 1))) << 4);
}
__device__ __forceinline__ bf16x8 lds_frag(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

// ---- forward -----------------------------------------------------------------------------
// grid (heads, batch, query tiles): the heaviest query tiles of all heads start first.
// F16: qkv, the V image, the probabilities and out are fp16 (same layouts, f16 instructions).
template <int D, bool F16 = false>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv,
                                                               const bf16* __restrict__ vt_img,
                                                               bf16* __restrict__ out,
                                                               float* __restrict__ lse, int S, int a) {
  constexpr int KSTEPS = D / 16;   // MFMA k-steps over the head dimension
  constexpr int DB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;
  constexpr int TILE = BKV * ROWB;  // bytes of one K tile or one V^T image tile
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];  // [stage][K | V^T image]

  const int lane = threadIdx.x & 63;
  const int lane_id = lane;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = gridDim.z - 1 - blockIdx.z;
  const int n = blockIdx.x, b = blockIdx.y;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const int ntile = (S + BKV - 1) / BKV;
  const bf16* vimg = vt_img + ((size_t)b * a + n) * ntile * (size_t)(D * BKV);
  const int q0 = qt * BQ;
  const int ql = lane & 31, h = lane >> 5;
  const int qrow = q0 + wave * 32 + ql;          // this lane's query
  const int qclamp = qrow < S ? qrow : S - 1;
  const int qmax_wave = min(q0 + wave * 32 + 31, S - 1);

  // Q fragments (B operand: column = query, 8 consecutive d per lane and k-step)
  bf16x8 qf[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk)
    qf[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)qclamp * ld + kk * 16 + h * 8);
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) settle(qf[kk]);

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = 1.4426950408889634f / sqrtf((float)D);  // log2(e)/sqrt(D)

  const int koff = natural_frag_off<D>(ql, h);
  const int voff = image_frag_off(ql, h);

  const int last_key = min(q0 + BQ, S);               // keys [0, last_key) are needed
  const int nkv = (last_key + BKV - 1) / BKV;
  dma_tile<D, 4>(base + P, ld, 0, S, lds, wave, lane);
  dma_image<D, 4>(vimg, lds + TILE, wave, lane);

  for (int kt = 0; kt < nkv; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int k0 = kt * BKV;
    const char* tK = lds + (kt & 1) * 2 * TILE;
    const char* tV = tK + TILE;
    if (kt + 1 < nkv) {
      char* nK = lds + ((kt + 1) & 1) * 2 * TILE;
      dma_tile<D, 4>(base + P, ld, k0 + BKV, S, nK, wave, lane);
      dma_image<D, 4>(vimg + (size_t)(kt + 1) * (D * BKV), nK + TILE, wave, lane);
    }
    if (k0 > qmax_wave) continue;  // every key of this tile is masked for this wave

    // ---- S^T = K Q^T for the two 32-key blocks -------------------------------------
    f32x16 sacc[2];
    GPTS_PRIO(1);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const bf16x8 kf = lds_frag(tK + kb * 32 * ROWB + (koff ^ (kk << 5)));
        sacc[kb] = mma32<F16>(kf, qf[kk], sacc[kb]);
      }
    }
    GPTS_PRIO(0);
    // ---- causal mask (only tiles that reach past the first query of the wave) --------
    if (k0 + BKV - 1 > q0 + wave * 32) {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int key = k0 + kb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
          if (key > qrow) sacc[kb][e] = -INFINITY;
        }
    }
    // ---- online softmax ------------------------------------------------------------------
    float mx = sacc[0][0];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[kb][e]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float mc = m_new * c;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -mc));
        sacc[kb][e] = p;
        psum += p;
      }
    // the running maximum rarely moves after the first tiles: skip the rescaling of the
    // output accumulators when no lane of the wave needs it
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
      const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
      l_run *= alpha;
#pragma unroll
      for (int i = 0; i < DB; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
      m_run = m_new;
    }
    l_run += psum;
    // ---- O^T += V^T P^T ------------------------------------------------------------------------
    GPTS_PRIO(1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {           // 16 keys per step
      const bf16x8 pf = pack8<F16>(sacc[ks >> 1], (ks & 1) * 8);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const bf16x8 vf = lds_frag(tV + db * 4096 + (voff ^ (ks << 5)));
        oacc[db] = mma32<F16>(vf, pf, oacc[db]);
      }
    }
    GPTS_PRIO(0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // ---- finish: combine the two key halves' sums, normalise, store ------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qrow < S) {
    const float inv = 1.f / l_tot;
    bf16* orow = out + ((size_t)b * S + qrow) * P + (size_t)n * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        if constexpr (F16) {
          f16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = sat_f16(oacc[db][g * 4 + e] * inv);
          *reinterpret_cast<f16x4*>(orow + db * 32 + g * 8 + h * 4) = o;
        } else {
          bf16x4 o;
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = (bf16)(oacc[db][g * 4 + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + db * 32 + g * 8 + h * 4) = o;
        }
      }
    if (h == 0) lse[((size_t)b * a + n) * S + qrow] = (m_run * c + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
  }
}


// delta[b,n,i] = sum_d dO[b,i,n*D+d] * O[b,i,n*D+d]; one 16-lane group per (row, head).
// O16: out holds fp16 values.
template <int D, bool O16 = false>
__global__ __launch_bounds__(256) void attn_delta_kernel(const bf16* __restrict__ out,
                                                         const bf16* __restrict__ dout,
                                                         float* __restrict__ delta, int S, int a,
                                                         int total) {
  constexpr int PER = D / 16;  // elements per lane
  const int gid = (blockIdx.x * 256 + threadIdx.x) >> 4, sub = threadIdx.x & 15;
  float acc = 0.f;
  if (gid < total) {
    const int n = gid % a;
    const size_t row = gid / a;  // b*S + i
    const size_t off = row * (size_t)a * D + (size_t)n * D + sub * PER;
    if constexpr (PER >= 4) {
#pragma unroll
      for (int e = 0; e < PER; e += 4) {
        const bf16x4 o = *reinterpret_cast<const bf16x4*>(out + off + e);
        const bf16x4 g = *reinterpret_cast<const bf16x4*>(dout + off + e);
#pragma unroll
        for (int k = 0; k < 4; ++k)
          acc = fmaf(O16 ? (float)__builtin_bit_cast(f16x4, o)[k] : (float)o[k], (float)g[k], acc);
      }
    } else {   // head dimension 32: two elements per lane
      typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
      typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
      const bf16x2 o = *reinterpret_cast<const bf16x2*>(out + off);
      const bf16x2 g = *reinterpret_cast<const bf16x2*>(dout + off);
#pragma unroll
      for (int k = 0; k < 2; ++k)
        acc = fmaf(O16 ? (float)__builtin_bit_cast(f16x2, o)[k] : (float)o[k], (float)g[k], acc);
    }
  }
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (gid < total && sub == 0) {
    const int n = gid % a;
    const size_t row = gid / a;
    const size_t b = row / S, i = row % S;
    delta[(b * a + n) * S + i] = acc;
  }
}

// Backward, key side.  A workgroup owns 256 keys (8 waves x 32) and streams the
// query rows at and after them in tiles of 64: the Q and dO tiles in natural form, their
// transposed images, lse and delta, all by DMA.  Per wave and 32-query block:
//   S[q][k]  = Q K^T       (A = Q fragment from LDS, B = K fragment in registers)
//   dP[q][k] = dO V^T      (A = dO fragment from LDS, B = V fragment in registers)
//   P = exp(S/sqrt(D) - lse_q),  dS = P (dP - delta_q)
//   dV^T[d][k] += dO^T P   (A = fragment of the dO image, B = P from the accumulator)
//   dK^T[d][k] += Q^T dS   (A = fragment of the Q image,  B = dS)
// so a lane owns one key column and nothing moves between lanes.
// grid (heads, batch, key blocks): the key blocks with the most queries start first.
// F16S: the logits are recomputed from fp16 copies of Q and K (qk16, laid out like qkv) with
// the f16 instruction -- the operands the forward pass formed them from; everything else
// (V, the images, dO) is bf16.  Without F16S qk16 == qkv.
template <int D, bool F16S = false>
__global__ __launch_bounds__(512) void attn_bwd_dkv_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ qk16, const bf16* __restrict__ dout, const bf16* __restrict__ qt_img,
    const bf16* __restrict__ dot_img, const float* __restrict__ lse, const float* __restrict__ delta,
    bf16* __restrict__ dqkv, int S, int a) {
  constexpr int KSTEPS = D / 16, DB = D / 32, ROWB = D * 2, TILE = BKV * ROWB;
  __shared__ __attribute__((aligned(1024))) char lds[8 * TILE];  // [stage][Q | dO | Q image | dO image]
  __shared__ __attribute__((aligned(256))) float stat[2][2][BKV];  // [stage][lse | delta][row]

  const int lane = threadIdx.x & 63;
  const int lane_id = lane;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = blockIdx.x, b = blockIdx.y;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const bf16* base16 = qk16 + (size_t)b * S * ld + (size_t)n * D;
  const bf16* dobase = dout + (size_t)b * S * P + (size_t)n * D;
  const int ntile = (S + BKV - 1) / BKV;
  const size_t img_off = ((size_t)b * a + n) * ntile * (size_t)(D * BKV);
  const bf16* qimg = qt_img + img_off;
  const bf16* doimg = dot_img + img_off;
  const float* lse_h = lse + ((size_t)b * a + n) * S;
  const float* delta_h = delta + ((size_t)b * a + n) * S;
  const int k0 = blockIdx.z * BW;
  const int kw0 = k0 + wave * 32;
  const int ql = lane & 31, h = lane >> 5;
  const int key = kw0 + ql;
  const int kclamp = key < S ? key : S - 1;
  const float rsd = 1.f / sqrtf((float)D);

  bf16x8 kfr[KSTEPS], vfr[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    kfr[kk] = *reinterpret_cast<const bf16x8*>(base16 + (size_t)kclamp * ld + P + kk * 16 + h * 8);
    vfr[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)kclamp * ld + 2 * P + kk * 16 + h * 8);
  }
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    settle(kfr[kk]);
    settle(vfr[kk]);
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[i][e] = dv[i][e] = 0.f;

  const int aoff = natural_frag_off<D>(ql, h);
  const int ioff = image_frag_off(ql, h);

  // The query tiles are walked from the LAST one down to the key block's own diagonal: every
  // key block of a head then starts at the same tile and they move in step, so the tiles one
  // workgroup streams are the ones its neighbours (same head, same XCD) are streaming at that
  // moment and come out of the L2 instead of HBM.  (Walking upwards from the diagonal, each
  // block is 256 rows ahead of the next one and the window does not fit the cache.)
  const int qt0 = k0 / BKV;
  auto fetch = [&](int qt, int stage) {
    // the lane index is made opaque here so that the per-lane DMA offsets are recomputed
    // (a dozen integer operations per tile) instead of being kept in registers across the
    // loop, where there are none to spare
    int lane = lane_id;
    asm volatile("" : "+v"(lane));
    char* t = lds + stage * 4 * TILE;
    dma_tile<D, 8>(base16, ld, qt * BKV, S, t, wave, lane);
    dma_tile<D, 8>(dobase, (size_t)P, qt * BKV, S, t + TILE, wave, lane);
    dma_image<D, 8>(qimg + (size_t)qt * (D * BKV), t + 2 * TILE, wave, lane);
    dma_image<D, 8>(doimg + (size_t)qt * (D * BKV), t + 3 * TILE, wave, lane);
    const int qi = qt * BKV + lane;
    const int qc = qi < S ? qi : S - 1;
    if (wave == 0) dma_floats(lse_h, qc, stat[stage][0]);
    if (wave == 1) dma_floats(delta_h, qc, stat[stage][1]);
  };
  fetch(ntile - 1, 0);

  for (int qt = ntile - 1; qt >= qt0; --qt) {
    const int stage = (ntile - 1 - qt) & 1;
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const char* tQ = lds + stage * 4 * TILE;
    const char* tO = tQ + TILE;
    const char* tQT = tQ + 2 * TILE;
    const char* tOT = tQ + 3 * TILE;
    if (qt > qt0) fetch(qt - 1, stage ^ 1);
#pragma unroll 1
    for (int qb = 0; qb < 2; ++qb) {
      const int qmin = qt * BKV + qb * 32;
      if (qmin + 31 < kw0 || qmin >= S) continue;  // block fully masked for this wave
      // S, then P = exp(S/sqrt(D) - lse) rounded to bf16 right away (the fp32 block dies
      // here: registers are the scarce resource of this kernel), then dP and
      // dS = P (dP - delta) with the rounded P -- the one that also enters dV.
      const char* aQ = tQ + qb * 32 * ROWB;
      const char* aO = tO + qb * 32 * ROWB;
      const float* Ls = &stat[stage][0][qb * 32 + h * 4];
      const float* Ds = &stat[stage][1][qb * 32 + h * 4];
      const bool masked = (qmin < kw0 + 31) || (qmin + 31 >= S);  // diagonal or ragged block
      bf16x8 pf[2], dsf[2];
      {
        f32x16 sacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
        GPTS_PRIO(1);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
          sacc = mma32<F16S>(lds_frag(aQ + (aoff ^ (kk << 5))), kfr[kk], sacc);
        GPTS_PRIO(0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 L = *reinterpret_cast<const f32x4*>(Ls + g * 8);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            sacc[g * 4 + e] = __builtin_amdgcn_exp2f(fmaf(sacc[g * 4 + e], rsd, -L[e]) * 1.4426950408889634f);
        }
        if (masked) {
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int query = qmin + (e >> 2) * 8 + h * 4 + (e & 3);
            if (key > query || query >= S) sacc[e] = 0.f;
          }
        }
        pf[0] = pack8(sacc, 0);
        pf[1] = pack8(sacc, 8);
      }
      {
        f32x16 dpacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) dpacc[e] = 0.f;
        GPTS_PRIO(1);
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk)
          dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(aO + (aoff ^ (kk << 5))), vfr[kk], dpacc, 0, 0, 0);
        GPTS_PRIO(0);
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const f32x4 Dl = *reinterpret_cast<const f32x4*>(Ds + g * 8);
#pragma unroll
          for (int e = 0; e < 4; ++e)
            dpacc[g * 4 + e] = (float)pf[g >> 1][(g & 1) * 4 + e] * (dpacc[g * 4 + e] - Dl[e]);
        }
        dsf[0] = pack8(dpacc, 0);
        dsf[1] = pack8(dpacc, 8);
      }
      GPTS_PRIO(1);
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {   // 16 queries per step
        const int off = ioff ^ ((qb * 2 + ks) << 5);
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(tOT + db * 4096 + off), pf[ks], dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(tQT + db * 4096 + off), dsf[ks], dk[db], 0, 0, 0);
        }
      }
      GPTS_PRIO(0);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  if (key < S) {
    const float scale = 1.f / sqrtf((float)D);
    bf16* drow = dqkv + ((size_t)b * S + key) * ld + (size_t)n * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 ok, ov;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          ok[e] = (bf16)(dk[db][g * 4 + e] * scale);
          ov[e] = (bf16)dv[db][g * 4 + e];
        }
        *reinterpret_cast<bf16x4*>(drow + P + db * 32 + g * 8 + h * 4) = ok;
        *reinterpret_cast<bf16x4*>(drow + 2 * P + db * 32 + g * 8 + h * 4) = ov;
      }
  }
}

// Backward, query side.  A workgroup owns 256 queries (8 waves x 32) and walks the key
// tiles of 64 up to the diagonal, everything transposed:
//   S^T = K Q^T,  dP^T = V dO^T  (A = K / V fragments from LDS, B = Q / dO in registers)
//   dS^T = P^T (dP^T - delta_q),  dQ^T[d][q] += K^T dS^T (A = fragment of the K image).
// grid (heads, batch, query blocks), heaviest first.
template <int D, bool F16S = false>
__global__ __launch_bounds__(512) void attn_bwd_dq_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ qk16, const bf16* __restrict__ dout, const bf16* __restrict__ kt_img,
    const float* __restrict__ lse, const float* __restrict__ delta, bf16* __restrict__ dqkv, int S, int a) {
  constexpr int KSTEPS = D / 16, DB = D / 32, ROWB = D * 2, TILE = BKV * ROWB;
  __shared__ __attribute__((aligned(1024))) char lds[6 * TILE];  // [stage][K | V | K image]

  const int lane = threadIdx.x & 63;
  const int lane_id = lane;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = gridDim.z - 1 - blockIdx.z;
  const int n = blockIdx.x, b = blockIdx.y;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const bf16* base16 = qk16 + (size_t)b * S * ld + (size_t)n * D;
  const int ntile = (S + BKV - 1) / BKV;
  const bf16* kimg = kt_img + ((size_t)b * a + n) * ntile * (size_t)(D * BKV);
  const int q0 = qt * BW;
  const int ql = lane & 31, h = lane >> 5;
  const int qrow = q0 + wave * 32 + ql;
  const int qclamp = qrow < S ? qrow : S - 1;
  const int qmax_wave = min(q0 + wave * 32 + 31, S - 1);
  const float c = 1.4426950408889634f / sqrtf((float)D);

  bf16x8 qf[KSTEPS], dof[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    qf[kk] = *reinterpret_cast<const bf16x8*>(base16 + (size_t)qclamp * ld + kk * 16 + h * 8);
    dof[kk] = *reinterpret_cast<const bf16x8*>(dout + ((size_t)b * S + qclamp) * P + (size_t)n * D + kk * 16 + h * 8);
  }
  const float L2 = lse[((size_t)b * a + n) * S + qclamp] * 1.4426950408889634f;
  const float Dl = delta[((size_t)b * a + n) * S + qclamp];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    settle(qf[kk]);
    settle(dof[kk]);
  }
  settle(L2);
  settle(Dl);
  f32x16 dq[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;

  const int koff = natural_frag_off<D>(ql, h);
  const int ioff = image_frag_off(ql, h);

  const int last_key = min(q0 + BW, S);
  const int nkv = (last_key + BKV - 1) / BKV;
  auto fetch = [&](int kt, int stage) {
    int lane = lane_id;  // opaque: recompute the DMA offsets per tile rather than keep them
    asm volatile("" : "+v"(lane));
    char* t = lds + stage * 3 * TILE;
    dma_tile<D, 8>(base16 + P, ld, kt * BKV, S, t, wave, lane);
    dma_tile<D, 8>(base + 2 * P, ld, kt * BKV, S, t + TILE, wave, lane);
    dma_image<D, 8>(kimg + (size_t)kt * (D * BKV), t + 2 * TILE, wave, lane);
  };
  fetch(0, 0);

  for (int kt = 0; kt < nkv; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int k0 = kt * BKV;
    const char* tK = lds + (kt & 1) * 3 * TILE;
    const char* tV = tK + TILE;
    const char* tKT = tK + 2 * TILE;
    if (kt + 1 < nkv) fetch(kt + 1, (kt + 1) & 1);
    if (k0 > qmax_wave) continue;
    f32x16 sacc[2], dpacc[2];
    GPTS_PRIO(1);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = dpacc[kb][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int off = kb * 32 * ROWB + (koff ^ (kk << 5));
        sacc[kb] = mma32<F16S>(lds_frag(tK + off), qf[kk], sacc[kb]);
        dpacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(tV + off), dof[kk], dpacc[kb], 0, 0, 0);
      }
    }
    GPTS_PRIO(0);
    if (k0 + BKV - 1 > q0 + wave * 32) {  // tile reaches past the first query of the wave: mask
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -L2));
          const int key = k0 + kb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
          if (key > qrow) p = 0.f;
          dpacc[kb][e] = p * (dpacc[kb][e] - Dl);
        }
    } else {
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -L2));
          dpacc[kb][e] = p * (dpacc[kb][e] - Dl);
        }
    }
    GPTS_PRIO(1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 dsf = pack8(dpacc[ks >> 1], (ks & 1) * 8);
#pragma unroll
      for (int db = 0; db < DB; ++db)
        dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lds_frag(tKT + db * 4096 + (ioff ^ (ks << 5))), dsf, dq[db], 0, 0, 0);
    }
    GPTS_PRIO(0);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  if (qrow < S) {
    const float scale = 1.f / sqrtf((float)D);
    bf16* drow = dqkv + ((size_t)b * S + qrow) * ld + (size_t)n * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)(dq[db][g * 4 + e] * scale);
        *reinterpret_cast<bf16x4*>(drow + db * 32 + g * 8 + h * 4) = o;
      }
  }
}

size_t image_bytes(int B, int S, int a, int d) {
  return (size_t)B * a * ((S + BKV - 1) / BKV) * (size_t)(d * BKV) * 2;
}
size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

template <int D>
void launch_timage(const TImageArgs& t, int B, int S, int a, hipStream_t st) {
  dim3 g((S + BKV - 1) / BKV, a, B * t.n_src);
  hipLaunchKernelGGL(attn_timage_kernel<D>, g, dim3(256), 0, st, t, S, a);
}

}  // namespace

// The kernels address a tile row with a 32-bit byte offset from the (batch, head) base and
// count (batch, row, head) triples in an int.
bool attention_mfma_supported(int B, int S, int a, int d) {
  return (d == 32 || d == 64 || d == 128) && B >= 1 && S >= 1 && a >= 1 && (size_t)S * 3 * a * d < (1ull << 31) &&
         (size_t)B * S * a < (1ull << 27);
}

size_t attention_mfma_scratch_bytes(int B, int S, int a, int d, int phase) {
  const size_t img = align256(image_bytes(B, S, a, d));
  if (phase == 0) return img;                                     // V image
  return align256((size_t)B * a * S * sizeof(float)) + 3 * img;   // delta, Q / K / dO images
}

hipError_t attention_fwd_mfma(int B, int S, int a, int d, const void* qkv, void* out, float* lse,
                              void* scratch, hipStream_t st, bool f16) {
  if (!attention_mfma_supported(B, S, a, d)) return hipErrorInvalidValue;
  const int P = a * d;
  const bf16* q = (const bf16*)qkv;
  bf16* vimg = (bf16*)scratch;
  TImageArgs t{};
  t.n_src = 1;
  t.src[0] = q + 2 * P;
  t.ld[0] = 3 * (size_t)P;
  t.dst[0] = vimg;
  dim3 g(a, B, (S + BQ - 1) / BQ), blk(256);
  // the image kernel only moves 16-bit values, so it serves fp16 as it serves bf16
  if (d == 128) {
    launch_timage<128>(t, B, S, a, st);
    if (f16) hipLaunchKernelGGL((attn_fwd_mfma_kernel<128, true>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
    else hipLaunchKernelGGL((attn_fwd_mfma_kernel<128, false>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
  } else if (d == 64) {
    launch_timage<64>(t, B, S, a, st);
    if (f16) hipLaunchKernelGGL((attn_fwd_mfma_kernel<64, true>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
    else hipLaunchKernelGGL((attn_fwd_mfma_kernel<64, false>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
  } else {
    launch_timage<32>(t, B, S, a, st);
    if (f16) hipLaunchKernelGGL((attn_fwd_mfma_kernel<32, true>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
    else hipLaunchKernelGGL((attn_fwd_mfma_kernel<32, false>), g, blk, 0, st, q, vimg, (bf16*)out, lse, S, a);
  }
  return hipGetLastError();
}

template <int D, bool F16>
static void launch_bwd(dim3 gd, dim3 gw, const TImageArgs& t, int B, int S, int a, int total, const bf16* q,
                const bf16* q16, const bf16* o, const bf16* g, bf16* qimg, bf16* kimg, bf16* doimg,
                const float* lse, float* delta, bf16* dq, hipStream_t st) {
  hipLaunchKernelGGL((attn_delta_kernel<D, F16>), gd, dim3(256), 0, st, o, g, delta, S, a, total);
  launch_timage<D>(t, B, S, a, st);
  hipLaunchKernelGGL((attn_bwd_dkv_mfma_kernel<D, F16>), gw, dim3(512), 0, st, q, q16, g, qimg, doimg, lse, delta, dq, S, a);
  hipLaunchKernelGGL((attn_bwd_dq_mfma_kernel<D, F16>), gw, dim3(512), 0, st, q, q16, g, kimg, lse, delta, dq, S, a);
}

hipError_t attention_bwd_mfma(int B, int S, int a, int d, const void* qkv, const void* out,
                              const float* lse, const void* dout, void* dqkv, void* scratch,
                              hipStream_t st, const void* qkv_f16) {
  if (!attention_mfma_supported(B, S, a, d)) return hipErrorInvalidValue;
  const int total = B * S * a, P = a * d;
  const size_t img = align256(image_bytes(B, S, a, d));
  char* sc = static_cast<char*>(scratch);
  float* delta = reinterpret_cast<float*>(sc);
  bf16* qimg = reinterpret_cast<bf16*>(sc + align256((size_t)total * sizeof(float)));
  bf16* kimg = reinterpret_cast<bf16*>(reinterpret_cast<char*>(qimg) + img);
  bf16* doimg = reinterpret_cast<bf16*>(reinterpret_cast<char*>(kimg) + img);
  const bf16* q = (const bf16*)qkv;
  const bf16* o = (const bf16*)out;
  const bf16* g = (const bf16*)dout;
  bf16* dq = (bf16*)dqkv;
  TImageArgs t{};
  t.n_src = 3;
  t.src[0] = q;         t.ld[0] = 3 * (size_t)P; t.dst[0] = qimg;
  t.src[1] = q + P;     t.ld[1] = 3 * (size_t)P; t.dst[1] = kimg;
  t.src[2] = g;         t.ld[2] = (size_t)P;     t.dst[2] = doimg;
  dim3 gd((unsigned)(((size_t)total * 16 + 255) / 256)), gw(a, B, (S + BW - 1) / BW);
  const bf16* q16 = (const bf16*)qkv_f16;
  if (d == 128) {
    if (q16) launch_bwd<128, true>(gd, gw, t, B, S, a, total, q, q16, o, g, qimg, kimg, doimg, lse, delta, dq, st);
    else launch_bwd<128, false>(gd, gw, t, B, S, a, total, q, q, o, g, qimg, kimg, doimg, lse, delta, dq, st);
  } else if (d == 64) {
    if (q16) launch_bwd<64, true>(gd, gw, t, B, S, a, total, q, q16, o, g, qimg, kimg, doimg, lse, delta, dq, st);
    else launch_bwd<64, false>(gd, gw, t, B, S, a, total, q, q, o, g, qimg, kimg, doimg, lse, delta, dq, st);
  } else {
    if (q16) launch_bwd<32, true>(gd, gw, t, B, S, a, total, q, q16, o, g, qimg, kimg, doimg, lse, delta, dq, st);
    else launch_bwd<32, false>(gd, gw, t, B, S, a, total, q, q, o, g, qimg, kimg, doimg, lse, delta, dq, st);
  }
  return hipGetLastError();
}

}  // namespace gpts
