// Causal softmax attention on the gfx950 matrix cores (bf16 in, fp32 accumulate).
//
// Forward, per (batch, head): a workgroup owns 128 query rows (4 waves x 32) and
// walks the key/value rows in tiles of 64 up to the diagonal with an online
// softmax.  Both products are computed TRANSPOSED so that no value ever has to
// move between lanes:
//   S^T[key][query] = K Q^T      A-operand = K fragment (ds_read_b128 from the
//                                K tile), B-operand = Q fragment (registers)
//   O^T[d][query]   = V^T P^T    A-operand = V^T fragment (transposing LDS read
//                                of the V tile as it sits in memory),
//                                B-operand = P^T, which is exactly the S^T
//                                accumulator of the same lane, rounded to bf16.
// A lane therefore owns one query column throughout: its running max, running
// sum and the rescaling of O are per-lane scalars; only the max needs one
// exchange with the lane that holds the other half of the keys (lane ^ 32).
// The order of keys inside the P^T fragment is the order the accumulator
// provides (8t + 4*half + j); V is read with the same order.
// K and V tiles go global -> LDS with the DMA path, double buffered.
#include "kernels.hpp"

namespace gpts {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(1))) const void* glb_ptr;

constexpr int BQ = 128;   // queries per workgroup
constexpr int BKV = 64;   // keys per tile

__device__ __forceinline__ int swz16(int row) { return (row & 7) ^ ((row >> 3) & 1); }

__device__ __forceinline__ bf16x8 tr_frag(const char* p0, const char* p1) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p0);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)p1);
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

__device__ __forceinline__ bf16x8 pack8(const f32x16& v, int base) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16)v[base + e];
  return r;
}

// A [rows][D] bf16 tile in LDS: row r, 16-byte chunk c stored at
// r*(2D) + ((c ^ swz16(r)) << 4) (the XOR only touches the low 3 bits of c).
// `rows` rows starting at global row `row0` (clamped to < S) are copied by the
// whole workgroup; each DMA instruction moves 1 KiB.
template <int D>
__device__ __forceinline__ void dma_tile(const bf16* __restrict__ src, size_t ld, int row0, int S,
                                         char* tile, int wave, int lane) {
  constexpr int ROWB = D * 2;              // bytes per row
  constexpr int CPR = ROWB / 16;           // chunks per row
  constexpr int NI = BKV * ROWB / 1024 / 4;  // instructions per wave
  const uint32_t lds_tile = (uint32_t)(size_t)(__attribute__((address_space(3))) char*)tile;
#pragma unroll
  for (int i = 0; i < NI; ++i) {
    const int slot = (wave * NI + i) * 64 + lane;
    const int r = slot / CPR, pc = slot % CPR;
    const int c = pc ^ swz16(r);
    int gr = row0 + r;
    gr = gr < S ? gr : S - 1;
    // Inline assembly on purpose: the compiler does not track these copies, so it does
    // not drain them in front of every transposing LDS read; the kernels wait for them
    // explicitly (s_waitcnt vmcnt(0)) before the barrier that publishes a tile.
    const uint32_t off = (uint32_t)(((size_t)gr * ld + c * 8) * 2);
    const uint32_t dst = lds_tile + (wave * NI + i) * 1024;
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 ::"s"(dst), "v"(off), "s"(src)
                 : "memory");
  }
}

template <int D>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma_kernel(const bf16* __restrict__ qkv,
                                                               bf16* __restrict__ out,
                                                               float* __restrict__ lse, int S, int a) {
  constexpr int KSTEPS = D / 16;   // MFMA k-steps over the head dimension
  constexpr int DB = D / 32;       // 32-row blocks of O^T
  constexpr int ROWB = D * 2;
  constexpr int TILE = BKV * ROWB;  // bytes of one K or V tile
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];  // [stage][K|V]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = gridDim.x - 1 - blockIdx.x;  // heaviest query tiles first
  const int n = blockIdx.y, b = blockIdx.z;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
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

  f32x16 oacc[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) oacc[i][e] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;
  const float c = 1.4426950408889634f / sqrtf((float)D);  // log2(e)/sqrt(D)

  // LDS read offsets.  K fragment (row = key): lane reads chunk 2*kk+h of row kb*32+ql.
  const int krow_off = ql * ROWB;
  const int ksw = swz16(ql);
  // V^T fragment via transposing reads: 16-lane group g = lane>>4: d-half mh = g&1,
  // key group kg = g>>1 (= h); inside the group lane i: key j = i>>2, d-quad q4 = i&3.
  // The lane supplies the address of 4 consecutive d of key row j: byte offset inside
  // the row = db*64 + mh*32 + q4*8, i.e. chunk db*4 + mh*2 + (q4>>1), byte (q4&1)*8.
  const int vi = lane & 15, vmh = (lane >> 4) & 1, vj = vi >> 2, vq4 = vi & 3;
  const int vch = vmh * 2 + (vq4 >> 1), vlow = (vq4 & 1) * 8;
  int vrow[2], vsw[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int k = 8 * t + 4 * h + vj;  // key inside a 16-key step
    vrow[t] = k * ROWB;
    vsw[t] = swz16(k);
  }

  const int last_key = min(q0 + BQ, S);               // keys [0, last_key) are needed
  const int nkv = (last_key + BKV - 1) / BKV;
  dma_tile<D>(base + P, ld, 0, S, lds, wave, lane);
  dma_tile<D>(base + 2 * P, ld, 0, S, lds + TILE, wave, lane);

  for (int kt = 0; kt < nkv; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int k0 = kt * BKV;
    const char* tK = lds + (kt & 1) * 2 * TILE;
    const char* tV = tK + TILE;
    if (kt + 1 < nkv) {
      char* nK = lds + ((kt + 1) & 1) * 2 * TILE;
      dma_tile<D>(base + P, ld, k0 + BKV, S, nK, wave, lane);
      dma_tile<D>(base + 2 * P, ld, k0 + BKV, S, nK + TILE, wave, lane);
    }
    if (k0 > qmax_wave) continue;  // every key of this tile is masked for this wave

    // ---- S^T = K Q^T for the two 32-key blocks -------------------------------------
    f32x16 sacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int chunk = (2 * kk + h) ^ ksw;   // swizzle touches the low 3 bits only
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(tK + kb * 32 * ROWB + krow_off + (chunk << 4));
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb], 0, 0, 0);
      }
    }
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
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * c);
    const float mc = m_new * c;
    m_run = m_new;
    float psum = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -mc));
        sacc[kb][e] = p;
        psum += p;
      }
    l_run = l_run * alpha + psum;
#pragma unroll
    for (int i = 0; i < DB; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) oacc[i][e] *= alpha;
    // ---- O^T += V^T P^T ------------------------------------------------------------------------
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {           // 16 keys per step
      const bf16x8 pf = pack8(sacc[ks >> 1], (ks & 1) * 8);
      const char* vb = tV + ks * 16 * ROWB + vlow;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int ch = db * 4 + vch;           // logical 16-byte chunk of this lane's 4 d values
        const bf16x8 vf = tr_frag(vb + vrow[0] + ((ch ^ vsw[0]) << 4), vb + vrow[1] + ((ch ^ vsw[1]) << 4));
        oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, oacc[db], 0, 0, 0);
      }
    }
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
        bf16x4 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) o[e] = (bf16)(oacc[db][g * 4 + e] * inv);
        *reinterpret_cast<bf16x4*>(orow + db * 32 + g * 8 + h * 4) = o;
      }
    if (h == 0) lse[((size_t)b * a + n) * S + qrow] = (m_run * c + __builtin_amdgcn_logf(l_tot)) * 0.6931471805599453f;
  }
}


// delta[b,n,i] = sum_d dO[b,i,n*D+d] * O[b,i,n*D+d]; one 16-lane group per (row, head).
template <int D>
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
#pragma unroll
    for (int e = 0; e < PER; e += 4) {
      const bf16x4 o = *reinterpret_cast<const bf16x4*>(out + off + e);
      const bf16x4 g = *reinterpret_cast<const bf16x4*>(dout + off + e);
#pragma unroll
      for (int k = 0; k < 4; ++k) acc = fmaf((float)o[k], (float)g[k], acc);
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

// Backward, key side.  A workgroup owns 128 keys (4 waves x 32) and streams the
// query rows at and after them in tiles of 64 (Q and dO tiles by DMA, lse and
// delta through LDS).  Per wave and 32-query block:
//   S[q][k]  = Q K^T       (A = Q fragment from LDS, B = K fragment in registers)
//   dP[q][k] = dO V^T      (A = dO fragment from LDS, B = V fragment in registers)
//   P = exp(S/sqrt(D) - lse_q),  dS = P (dP - delta_q)
//   dV^T[d][k] += dO^T P   (A = transposing read of the dO tile, B = P from the accumulator)
//   dK^T[d][k] += Q^T dS   (A = transposing read of the Q tile,  B = dS)
// so a lane owns one key column and nothing moves between lanes.
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int S, int a) {
  constexpr int KSTEPS = D / 16, DB = D / 32, ROWB = D * 2, TILE = BKV * ROWB;
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];  // [stage][Q|dO]
  __shared__ __attribute__((aligned(16))) float stat[2][2][BKV];  // [stage][lse*log2e | delta][row]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int n = blockIdx.y, b = blockIdx.z;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const bf16* dobase = dout + (size_t)b * S * P + (size_t)n * D;
  const float* lse_h = lse + ((size_t)b * a + n) * S;
  const float* delta_h = delta + ((size_t)b * a + n) * S;
  const int k0 = blockIdx.x * 128;
  const int kw0 = k0 + wave * 32;
  const int ql = lane & 31, h = lane >> 5;
  const int key = kw0 + ql;
  const int kclamp = key < S ? key : S - 1;
  const float c = 1.4426950408889634f / sqrtf((float)D);

  bf16x8 kfr[KSTEPS], vfr[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    kfr[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)kclamp * ld + P + kk * 16 + h * 8);
    vfr[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)kclamp * ld + 2 * P + kk * 16 + h * 8);
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dk[i][e] = dv[i][e] = 0.f;

  const int arow_off = ql * ROWB, asw = swz16(ql);
  const int vi = lane & 15, vmh = (lane >> 4) & 1, vj = vi >> 2, vq4 = vi & 3;
  const int vch = vmh * 2 + (vq4 >> 1), vlow = (vq4 & 1) * 8;
  int trow[2], tsw[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int k = 8 * t + 4 * h + vj;
    trow[t] = k * ROWB;
    tsw[t] = swz16(k);
  }

  const int nq = (S + BKV - 1) / BKV;
  const int qt0 = k0 / BKV;
  auto stage_stats = [&](int qt, int stage) {
    if (threadIdx.x < BKV) {
      const int qi = qt * BKV + threadIdx.x;
      const int qc = qi < S ? qi : S - 1;
      stat[stage][0][threadIdx.x] = lse_h[qc] * 1.4426950408889634f;
      stat[stage][1][threadIdx.x] = delta_h[qc];
    }
  };
  dma_tile<D>(base, ld, qt0 * BKV, S, lds, wave, lane);
  dma_tile<D>(dobase, (size_t)P, qt0 * BKV, S, lds + TILE, wave, lane);
  stage_stats(qt0, 0);

  for (int qt = qt0; qt < nq; ++qt) {
    const int stage = (qt - qt0) & 1;
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const char* tQ = lds + stage * 2 * TILE;
    const char* tO = tQ + TILE;
    if (qt + 1 < nq) {
      char* nQ = lds + (stage ^ 1) * 2 * TILE;
      dma_tile<D>(base, ld, (qt + 1) * BKV, S, nQ, wave, lane);
      dma_tile<D>(dobase, (size_t)P, (qt + 1) * BKV, S, nQ + TILE, wave, lane);
      stage_stats(qt + 1, stage ^ 1);
    }
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      const int qmin = qt * BKV + qb * 32;
      if (qmin + 31 < kw0 || qmin >= S) continue;  // block fully masked for this wave
      f32x16 sacc, dpacc;
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[e] = dpacc[e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int off = qb * 32 * ROWB + arow_off + ((((2 * kk + h) ^ asw)) << 4);
        const bf16x8 qa = *reinterpret_cast<const bf16x8*>(tQ + off);
        const bf16x8 da = *reinterpret_cast<const bf16x8*>(tO + off);
        sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qa, kfr[kk], sacc, 0, 0, 0);
        dpacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(da, vfr[kk], dpacc, 0, 0, 0);
      }
      const bool need_mask = (qmin < kw0 + 31) || (qmin + 31 >= S);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int r = qb * 32 + g * 8 + h * 4;
        const f32x4 L = *reinterpret_cast<const f32x4*>(&stat[stage][0][r]);
        const f32x4 Dl = *reinterpret_cast<const f32x4*>(&stat[stage][1][r]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float p = __builtin_amdgcn_exp2f(fmaf(sacc[g * 4 + e], c, -L[e]));
          if (need_mask) {
            const int query = qt * BKV + r + e;
            if (key > query || query >= S) p = 0.f;
          }
          sacc[g * 4 + e] = p;
          dpacc[g * 4 + e] = p * (dpacc[g * 4 + e] - Dl[e]);
        }
      }
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {   // 16 queries per step
        const bf16x8 pf = pack8(sacc, ks * 8);
        const bf16x8 dsf = pack8(dpacc, ks * 8);
        const int rb = (qb * 32 + ks * 16) * ROWB + vlow;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
          const int ch = db * 4 + vch;
          const int o0 = rb + trow[0] + ((ch ^ tsw[0]) << 4), o1 = rb + trow[1] + ((ch ^ tsw[1]) << 4);
          const bf16x8 dot = tr_frag(tO + o0, tO + o1);
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dot, pf, dv[db], 0, 0, 0);
          const bf16x8 qT = tr_frag(tQ + o0, tQ + o1);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qT, dsf, dk[db], 0, 0, 0);
        }
      }
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

// Backward, query side.  Same walk as the forward pass (128 queries per workgroup,
// key tiles of 64 up to the diagonal), everything transposed:
//   S^T = K Q^T,  dP^T = V dO^T  (A = K / V fragments from LDS, B = Q / dO in registers)
//   dS^T = P^T (dP^T - delta_q),  dQ^T[d][q] += K^T dS^T (A = transposing read of the K tile).
template <int D>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_mfma_kernel(
    const bf16* __restrict__ qkv, const bf16* __restrict__ dout, const float* __restrict__ lse,
    const float* __restrict__ delta, bf16* __restrict__ dqkv, int S, int a) {
  constexpr int KSTEPS = D / 16, DB = D / 32, ROWB = D * 2, TILE = BKV * ROWB;
  __shared__ __attribute__((aligned(1024))) char lds[4 * TILE];  // [stage][K|V]

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qt = gridDim.x - 1 - blockIdx.x;
  const int n = blockIdx.y, b = blockIdx.z;
  const int P = a * D;
  const size_t ld = 3 * (size_t)P;
  const bf16* base = qkv + (size_t)b * S * ld + (size_t)n * D;
  const int q0 = qt * BQ;
  const int ql = lane & 31, h = lane >> 5;
  const int qrow = q0 + wave * 32 + ql;
  const int qclamp = qrow < S ? qrow : S - 1;
  const int qmax_wave = min(q0 + wave * 32 + 31, S - 1);
  const float c = 1.4426950408889634f / sqrtf((float)D);

  bf16x8 qf[KSTEPS], dof[KSTEPS];
#pragma unroll
  for (int kk = 0; kk < KSTEPS; ++kk) {
    qf[kk] = *reinterpret_cast<const bf16x8*>(base + (size_t)qclamp * ld + kk * 16 + h * 8);
    dof[kk] = *reinterpret_cast<const bf16x8*>(dout + ((size_t)b * S + qclamp) * P + (size_t)n * D + kk * 16 + h * 8);
  }
  const float L2 = lse[((size_t)b * a + n) * S + qclamp] * 1.4426950408889634f;
  const float Dl = delta[((size_t)b * a + n) * S + qclamp];
  f32x16 dq[DB];
#pragma unroll
  for (int i = 0; i < DB; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) dq[i][e] = 0.f;

  const int krow_off = ql * ROWB, ksw = swz16(ql);
  const int vi = lane & 15, vmh = (lane >> 4) & 1, vj = vi >> 2, vq4 = vi & 3;
  const int vch = vmh * 2 + (vq4 >> 1), vlow = (vq4 & 1) * 8;
  int trow[2], tsw[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const int k = 8 * t + 4 * h + vj;
    trow[t] = k * ROWB;
    tsw[t] = swz16(k);
  }

  const int last_key = min(q0 + BQ, S);
  const int nkv = (last_key + BKV - 1) / BKV;
  dma_tile<D>(base + P, ld, 0, S, lds, wave, lane);
  dma_tile<D>(base + 2 * P, ld, 0, S, lds + TILE, wave, lane);

  for (int kt = 0; kt < nkv; ++kt) {
    asm volatile("s_waitcnt vmcnt(0)\n\ts_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    const int k0 = kt * BKV;
    const char* tK = lds + (kt & 1) * 2 * TILE;
    const char* tV = tK + TILE;
    if (kt + 1 < nkv) {
      char* nK = lds + ((kt + 1) & 1) * 2 * TILE;
      dma_tile<D>(base + P, ld, k0 + BKV, S, nK, wave, lane);
      dma_tile<D>(base + 2 * P, ld, k0 + BKV, S, nK + TILE, wave, lane);
    }
    if (k0 > qmax_wave) continue;
    f32x16 sacc[2], dpacc[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int e = 0; e < 16; ++e) sacc[kb][e] = dpacc[kb][e] = 0.f;
#pragma unroll
      for (int kk = 0; kk < KSTEPS; ++kk) {
        const int off = kb * 32 * ROWB + krow_off + (((2 * kk + h) ^ ksw) << 4);
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(tK + off);
        const bf16x8 vf = *reinterpret_cast<const bf16x8*>(tV + off);
        sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[kk], sacc[kb], 0, 0, 0);
        dpacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[kk], dpacc[kb], 0, 0, 0);
      }
    }
    const bool need_mask = k0 + BKV - 1 > q0 + wave * 32;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        float p = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], c, -L2));
        if (need_mask) {
          const int key = k0 + kb * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
          if (key > qrow) p = 0.f;
        }
        dpacc[kb][e] = p * (dpacc[kb][e] - Dl);
      }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8 dsf = pack8(dpacc[ks >> 1], (ks & 1) * 8);
      const char* kb_ = tK + ks * 16 * ROWB + vlow;
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        const int ch = db * 4 + vch;
        const bf16x8 kT = tr_frag(kb_ + trow[0] + ((ch ^ tsw[0]) << 4), kb_ + trow[1] + ((ch ^ tsw[1]) << 4));
        dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kT, dsf, dq[db], 0, 0, 0);
      }
    }
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

}  // namespace

hipError_t attention_fwd_mfma(int B, int S, int a, int d, const void* qkv, void* out, float* lse,
                              hipStream_t st) {
  dim3 g((S + BQ - 1) / BQ, a, B), blk(256);
  if (d == 128)
    hipLaunchKernelGGL(attn_fwd_mfma_kernel<128>, g, blk, 0, st, (const bf16*)qkv, (bf16*)out, lse, S, a);
  else if (d == 64)
    hipLaunchKernelGGL(attn_fwd_mfma_kernel<64>, g, blk, 0, st, (const bf16*)qkv, (bf16*)out, lse, S, a);
  else
    return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace gpts

namespace gpts {

hipError_t attention_bwd_mfma(int B, int S, int a, int d, const void* qkv, const void* out,
                              const float* lse, const void* dout, void* dqkv, float* delta,
                              hipStream_t st) {
  const int total = B * S * a;
  dim3 gd((total * 16 + 255) / 256), gq((S + BQ - 1) / BQ, a, B), gk((S + 127) / 128, a, B), blk(256);
  const bf16* q = (const bf16*)qkv;
  const bf16* o = (const bf16*)out;
  const bf16* g = (const bf16*)dout;
  bf16* dq = (bf16*)dqkv;
  if (d == 128) {
    hipLaunchKernelGGL(attn_delta_kernel<128>, gd, blk, 0, st, o, g, delta, S, a, total);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel<128>, gk, blk, 0, st, q, g, lse, delta, dq, S, a);
    hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel<128>, gq, blk, 0, st, q, g, lse, delta, dq, S, a);
  } else if (d == 64) {
    hipLaunchKernelGGL(attn_delta_kernel<64>, gd, blk, 0, st, o, g, delta, S, a, total);
    hipLaunchKernelGGL(attn_bwd_dkv_mfma_kernel<64>, gk, blk, 0, st, q, g, lse, delta, dq, S, a);
    hipLaunchKernelGGL(attn_bwd_dq_mfma_kernel<64>, gq, blk, 0, st, q, g, lse, delta, dq, S, a);
  } else {
    return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace gpts
