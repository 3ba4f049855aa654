// C-ABI of libgptstage and the stage orchestrator: buffer layouts, argument
// validation and the per-layer launch sequence of the forward and backward
// phases.  All arithmetic lives in the kernels; this file only sequences them.
#include "../../include/gpt_stage.h"

#include <string.h>

#include <new>

#include "kernels.hpp"

using namespace gpts;

namespace {

// text and status of the calling thread's last failed call
thread_local char g_err[256] = "";
thread_local int g_err_code = GPTS_OK;

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline size_t esize(const gpt_stage_cfg& c) { return c.dtype == GPTS_BF16 ? 2 : 4; }
// The residual stream (x of every layer and x1) is carried in fp32 inside the stage,
// also for bf16 stages: rounding it to bf16 after every layer perturbs the attention
// logits of the following layers enough to cost several percent on their gradients
// when the logits are large.  Everything that branches off it is still bf16.
constexpr size_t kResBytes = 4;

struct Dims {
  int L, H, a, d, P, F, S, B, T;
  explicit Dims(const gpt_stage_cfg& c)
      : L(c.n_layers), H(c.hidden), a(c.n_heads), d(c.head_dim), P(c.n_heads * c.head_dim),
        F(c.ffn), S(c.seq), B(c.batch), T(c.batch * c.seq) {}
};

size_t tensor_elems(const Dims& D, int id) {
  switch (id) {
    case GPTS_LN1_G: case GPTS_LN1_B: case GPTS_LN2_G: case GPTS_LN2_B:
    case GPTS_B_O: case GPTS_B_FC2: return D.H;
    case GPTS_W_QKV: return (size_t)3 * D.P * D.H;
    case GPTS_B_QKV: return (size_t)3 * D.P;
    case GPTS_W_O: return (size_t)D.H * D.P;
    case GPTS_W_FC1: return (size_t)D.F * D.H;
    case GPTS_B_FC1: return D.F;
    case GPTS_W_FC2: return (size_t)D.H * D.F;
  }
  return 0;
}

size_t layer_elems(const Dims& D) {
  size_t n = 0;
  for (int i = 0; i < GPTS_N_TENSORS; ++i) n += tensor_elems(D, i);
  return n;
}

size_t tensor_off(const Dims& D, int layer, int id) {
  size_t o = (size_t)layer * layer_elems(D);
  for (int i = 0; i < id; ++i) o += tensor_elems(D, i);
  return o;
}

// ---- activation stash of one micro-batch: per layer, in this order ----------
//   X [T,H]f32  mean1,rstd1 [T]f32  A [T,H]  QKV [T,3P]  C [T,P]  LSE [B,a,S]f32
//   X1 [T,H]f32 mean2,rstd2 [T]f32  A2 [T,H] U [T,F]  G [T,F]
// every region 256-byte aligned.
constexpr size_t kAbsent = ~(size_t)0;
struct StashLayer {
  size_t X, stat1, A, QKV, C, LSE, X1, stat2, A2, U, G, end;   // kAbsent: not stashed
};
// layer_block(): every tensor one layer's backward reads, in the order above.  It is what a
// layer of the stash holds -- except with recompute == 2, where the stash keeps only X per layer
// (stash_layer()) and the block is a workspace buffer the backward phase refills, layer by
// layer, by running the layer's forward again.
StashLayer layer_block(const gpt_stage_cfg& c) {
  Dims D(c);
  const size_t e = esize(c);
  StashLayer s;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  // with the light recomputation, and always when the forward activations are fp16 (the backward
  // phase needs bf16 copies and rebuilds them), A, A2 and G are not kept; with fwd_fp16 the
  // kept QKV, C and U hold fp16 values (same size)
  const bool full = c.recompute != 1 && c.fwd_fp16 == 0;
  s.X = take((size_t)D.T * D.H * kResBytes);
  s.stat1 = take((size_t)2 * D.T * 4);
  s.A = full ? take((size_t)D.T * D.H * e) : kAbsent;
  s.QKV = take((size_t)D.T * 3 * D.P * e);
  s.C = take((size_t)D.T * D.P * e);
  s.LSE = take((size_t)D.B * D.a * D.S * 4);
  s.X1 = take((size_t)D.T * D.H * kResBytes);
  s.stat2 = take((size_t)2 * D.T * 4);
  s.A2 = full ? take((size_t)D.T * D.H * e) : kAbsent;
  s.U = take((size_t)D.T * D.F * e);
  s.G = full ? take((size_t)D.T * D.F * e) : kAbsent;
  s.end = o;
  return s;
}
StashLayer stash_layer(const gpt_stage_cfg& c) {
  if (c.recompute != 2) return layer_block(c);
  Dims D(c);
  StashLayer s;
  s.X = 0;
  s.stat1 = s.A = s.QKV = s.C = s.LSE = s.X1 = s.stat2 = s.A2 = s.U = s.G = kAbsent;
  s.end = align_up((size_t)D.T * D.H * kResBytes, 256);
  return s;
}

// ---- workspace ---------------------------------------------------------------------
// [forward region | backward region]: a forward and a backward call on different streams
// may share one workspace, their regions are disjoint.  The forward region is the
// attention kernels' scratch; offsets in BwdWs are relative to the whole workspace.
size_t attention_scratch_bytes(int dtype, int B, int S, int a, int d, int phase);
struct FwdWs {
  size_t attn, A, G, blk, end;   // A (shared by both LayerNorm outputs) and G only where they are
                                 // not kept; blk: the layer block with recompute == 2
};
FwdWs fwd_ws(const gpt_stage_cfg& c) {
  Dims D(c);
  const size_t e = esize(c);
  FwdWs w;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  w.attn = take(attention_scratch_bytes(c.dtype, D.B, D.S, D.a, D.d, 0));
  const bool transient = c.recompute == 1 || c.fwd_fp16;
  w.A = transient ? take((size_t)D.T * D.H * e) : kAbsent;
  w.G = transient ? take((size_t)D.T * D.F * e) : kAbsent;
  w.blk = c.recompute == 2 ? take(layer_block(c).end) : kAbsent;
  w.end = o;
  return w;
}
size_t fwd_ws_bytes(const gpt_stage_cfg& c) { return fwd_ws(c).end; }
struct BwdWs {
  size_t dU, dA, dX1, dC, dQKV, attn, ping, pong, ln_part, cs_part, rA, rG, rstat, end;
  size_t bQKV, bC, bU;   // fwd_fp16: bf16 copies of the fp16 QKV, C and U of the stash
  size_t fwd2;           // recompute == 2: a forward workspace of the backward phase's own
};
BwdWs bwd_ws(const gpt_stage_cfg& c) {
  Dims D(c);
  const size_t e = esize(c);
  BwdWs w;
  size_t o = fwd_ws_bytes(c);
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  w.dU = take((size_t)D.T * D.F * e);
  w.dA = take((size_t)D.T * D.H * e);
  w.dX1 = take((size_t)D.T * D.H * e);
  w.dC = take((size_t)D.T * D.P * e);
  w.dQKV = take((size_t)D.T * 3 * D.P * e);
  w.attn = take(attention_scratch_bytes(c.dtype, D.B, D.S, D.a, D.d, 1));
  w.ping = take((size_t)D.T * D.H * e);
  w.pong = take((size_t)D.T * D.H * e);
  w.ln_part = take(ln_bwd_scratch_bytes(D.T, D.H));
  int maxn = D.H;
  if (3 * D.P > maxn) maxn = 3 * D.P;
  if (D.F > maxn) maxn = D.F;
  w.cs_part = take(colsum_scratch_bytes(D.T, maxn));
  // recomputed LayerNorm output (one buffer, used for A2 and then A), GeLU output, statistics
  const bool rebuild = c.recompute == 1 || c.fwd_fp16;
  w.rA = rebuild ? take((size_t)D.T * D.H * e) : kAbsent;
  w.rG = rebuild ? take((size_t)D.T * D.F * e) : kAbsent;
  w.rstat = rebuild ? take((size_t)2 * D.T * 4) : kAbsent;
  w.bQKV = c.fwd_fp16 ? take((size_t)D.T * 3 * D.P * e) : kAbsent;
  w.bC = c.fwd_fp16 ? take((size_t)D.T * D.P * e) : kAbsent;
  w.bU = c.fwd_fp16 ? take((size_t)D.T * D.F * e) : kAbsent;
  w.fwd2 = c.recompute == 2 ? take(fwd_ws_bytes(c)) : kAbsent;
  w.end = o;
  return w;
}

// ---- gradient stash of one micro-batch (backward split into a data and a weight phase):
// per layer the output gradients of its four linears, the operands the weight-gradient
// products need besides the activation stash:  dY [T,H]  dU [T,F]  dX1 [T,H]  dQKV [T,3P]
struct GradStashLayer {
  size_t dY, dU, dX1, dQKV, end;
};
GradStashLayer grad_stash_layer(const gpt_stage_cfg& c) {
  Dims D(c);
  const size_t e = esize(c);
  GradStashLayer s;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
  s.dY = take((size_t)D.T * D.H * e);
  s.dU = take((size_t)D.T * D.F * e);
  s.dX1 = take((size_t)D.T * D.H * e);
  s.dQKV = take((size_t)D.T * 3 * D.P * e);
  s.end = o;
  return s;
}

// ---- prepared weights: per layer and linear (qkv, out-proj, fc1, fc2) the forward image of
// the weight ([out rows, in]).  The data gradients read the raw weight: its K-major form goes
// through the same 16x16x32 kernel at the speed an image gave, so none is built for them.
struct LinDims { int out, in, wid; };
inline void linears(const Dims& D, LinDims (&L)[4]) {
  L[0] = {3 * D.P, D.H, GPTS_W_QKV};
  L[1] = {D.H, D.P, GPTS_W_O};
  L[2] = {D.F, D.H, GPTS_W_FC1};
  L[3] = {D.H, D.F, GPTS_W_FC2};
}
// element offset of the image of (layer, linear); total when layer == L
size_t prepared_off(const Dims& D, int layer, int lin) {
  LinDims L[4];
  linears(D, L);
  size_t per_layer = 0, off = 0;
  for (int i = 0; i < 4; ++i) {
    const size_t f = gemm_image_elems(L[i].out, L[i].in);
    if (i < lin) off += f;
    per_layer += f;
  }
  return (size_t)layer * per_layer + (layer == D.L ? 0 : off);
}

int fail(int code, const char* msg) {
  strncpy(g_err, msg, sizeof(g_err) - 1);
  g_err[sizeof(g_err) - 1] = 0;
  g_err_code = code;
  return code;
}
int hip_fail(hipError_t e, const char* where) {
  snprintf(g_err, sizeof(g_err), "%s: %s", where, hipGetErrorString(e));
  g_err_code = GPTS_EHIP;
  return GPTS_EHIP;
}
bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

#define GPTS_TRY(expr, where)                          \
  do {                                                 \
    hipError_t e__ = (expr);                           \
    if (e__ != hipSuccess) return hip_fail(e__, where); \
  } while (0)

// ---- operator tracer -------------------------------------------------------------
// A start and an end hipEvent are recorded on the stream around every operator of a
// traced call; elapsed times are read back later, off the critical path
// (the event-pair scheme of the paper's section 3.2, MegaScan data collection).
struct TraceRec {
  hipEvent_t e0, e1;
  int op, sub, layer, phase;
  double flops, bytes;
};
struct Tracer {
  int capacity = 0, n = 0, dropped = 0;
  TraceRec* recs = nullptr;
};
struct TraceScope {
  Tracer* t;
  hipStream_t st;
  int idx = -1;
  TraceScope(Tracer* t_, hipStream_t st_, int op, int sub, int layer, int phase, double flops, double bytes)
      : t(t_), st(st_) {
    if (!t) return;
    if (t->n >= t->capacity) { ++t->dropped; return; }
    idx = t->n++;
    TraceRec& r = t->recs[idx];
    r.op = op; r.sub = sub; r.layer = layer; r.phase = phase; r.flops = flops; r.bytes = bytes;
    (void)hipEventRecord(r.e0, st);
  }
  ~TraceScope() {
    if (idx >= 0) (void)hipEventRecord(t->recs[idx].e1, st);
  }
};
#define GPTS_OP(op, sub, phase, fl, by, expr, where)                 \
  do {                                                               \
    TraceScope ts__(tr, st, (op), (sub), l, (phase), (fl), (by));    \
    GPTS_TRY(expr, where);                                           \
  } while (0)

// One matrix product of the stage: MFMA path for bf16 shapes it covers, the
// plain FMA path otherwise (always for fp32).
hipError_t gemm(int dtype, int form, int M, int N, int K, const void* A, const void* B, void* C,
                const GemmEpilogue& ep, hipStream_t st) {
  if (dtype == GPTS_BF16 && gemm_mfma_supported(form, M, N, K))
    return gemm_mfma(form, M, N, K, A, B, C, ep, st);
  return gemm_simple(dtype, form, M, N, K, A, B, C, ep, st);
}

// Attention: MFMA kernels for bf16 (head_dim 32, 64, 128), the plain FMA kernels for fp32.
// scratch: attention_scratch_bytes(.., phase) bytes of device memory.
bool attention_uses_mfma(int dtype, int B, int S, int a, int d) {
  return dtype == GPTS_BF16 && attention_mfma_supported(B, S, a, d);
}
size_t attention_scratch_bytes(int dtype, int B, int S, int a, int d, int phase) {
  if (attention_uses_mfma(dtype, B, S, a, d)) return attention_mfma_scratch_bytes(B, S, a, d, phase);
  return phase == 0 ? 0 : align_up((size_t)B * a * S * sizeof(float), 256);  // delta
}
// f16 / qkv_f16: the fp16 forward-activation variants (matrix-core path only)
hipError_t attention_fwd(int dtype, int B, int S, int a, int d, const void* qkv, void* out,
                         float* lse, void* scratch, hipStream_t st, bool f16 = false) {
  if (attention_uses_mfma(dtype, B, S, a, d)) return attention_fwd_mfma(B, S, a, d, qkv, out, lse, scratch, st, f16);
  if (f16) return hipErrorInvalidValue;
  return attention_fwd_simple(dtype, B, S, a, d, qkv, out, lse, st);
}
hipError_t attention_bwd(int dtype, int B, int S, int a, int d, const void* qkv, const void* out,
                         const float* lse, const void* dout, void* dqkv, void* scratch,
                         hipStream_t st, const void* qkv_f16 = nullptr) {
  if (attention_uses_mfma(dtype, B, S, a, d))
    return attention_bwd_mfma(B, S, a, d, qkv, out, lse, dout, dqkv, scratch, st, qkv_f16);
  if (qkv_f16) return hipErrorInvalidValue;
  return attention_bwd_simple(dtype, B, S, a, d, qkv, out, lse, dout, dqkv, static_cast<float*>(scratch), st);
}

int check_call(const gpt_stage_params* p) {
  if (!p) return fail(GPTS_EINVAL, "params is NULL");
  int rc = gpt_stage_validate(&p->cfg);
  if (rc != GPTS_OK) return rc;
  if (!p->weights || misaligned(p->weights)) return fail(GPTS_EINVAL, "weights NULL or not 16-byte aligned");
  if (p->workspace && misaligned(p->workspace)) return fail(GPTS_EINVAL, "workspace not 16-byte aligned");
  if (p->prepared && misaligned(p->prepared)) return fail(GPTS_EINVAL, "prepared not 16-byte aligned");
  return GPTS_OK;
}
int need_prepared(const gpt_stage_params* p) {
  if (p->cfg.fwd_fp16 && !p->prepared)
    return fail(GPTS_EINVAL, "cfg.fwd_fp16 needs prepared weights (gpt_stage_prepare with the same cfg)");
  return GPTS_OK;
}

// Forward of layer l.  X: the layer's input (residual stream); blk: the layer block that
// receives every tensor the backward phase reads (layer_block() layout; its X slot is not
// written here); Yout: the layer's output, or nullptr to stop after the GeLU (the re-run of a
// layer inside the backward phase needs nothing beyond it); fwk: a forward workspace (fwd_ws
// layout).  phase: what the tracer records (0 forward phase, 1 backward phase).
int fwd_layer(const gpt_stage_params* p, int l, const void* X, char* blk, void* Yout, bool y_f32,
              char* fwk, hipStream_t st, int phase) {
  Tracer* tr = static_cast<Tracer*>(p->trace);
  const gpt_stage_cfg& c = p->cfg;
  const Dims D(c);
  const size_t e = esize(c);
  const int dt = c.dtype;
  const StashLayer sl = layer_block(c);
  const FwdWs fw = fwd_ws(c);
  const char* W = static_cast<const char*>(p->weights);
  auto w = [&](int l_, int id) { return (const void*)(W + tensor_off(D, l_, id) * e); };
  // algorithmic work of one operator, for the tracer: flops of an M x N x K product and
  // the bytes it must move (operands once, result once)
  auto gf = [](double M, double N, double K) { return 2.0 * M * N * K; };
  auto gb = [&](double M, double N, double K, double out_bytes) { return (M * K + N * K) * e + M * N * out_bytes; };
  const double TH = (double)D.T * D.H, attn_fl = 4.0 * D.B * D.a * D.d * ((double)D.S * (D.S + 1) / 2.0);
  const bool bf = dt == GPTS_BF16;
  const bf16* prep = bf ? static_cast<const bf16*>(p->prepared) : nullptr;
  auto img = [&](int l_, int lin) -> const void* {
    return prep ? (const void*)(prep + prepared_off(D, l_, lin)) : nullptr;
  };
  const int top = phase == 0 ? GPTS_TR_LN_FWD : GPTS_TR_RECOMPUTE;   // a re-run counts as recomputation
  const int top_gemm = phase == 0 ? GPTS_TR_GEMM_FWD : GPTS_TR_RECOMPUTE;
  const int top_attn = phase == 0 ? GPTS_TR_ATTN_FWD : GPTS_TR_RECOMPUTE;
  char* s = blk;
  float* stat1 = reinterpret_cast<float*>(s + sl.stat1);
  float* stat2 = reinterpret_cast<float*>(s + sl.stat2);
  // with the light recomputation (and with fp16 forward activations) the LayerNorm and GeLU
  // outputs only live in the workspace
  const bool transient = c.recompute == 1 || c.fwd_fp16;
  const bool h16 = c.fwd_fp16 != 0;   // A, QKV, C, A2, U, G hold fp16 values
  void* A = transient ? fwk + fw.A : s + sl.A;
  void* A2 = transient ? fwk + fw.A : s + sl.A2;
  void* G = transient ? fwk + fw.G : s + sl.G;
  // one forward product: fp16 operands through the weight's fp16 image, or the bf16 paths
  auto fwd_gemm = [&](int N, int K, const void* Ain, int wid, void* Cout, const GemmEpilogue& ep_) {
    return h16 ? gemm_fwd_f16(D.T, N, K, Ain, ep_.b_image, Cout, ep_, st) : gemm(dt, 0, D.T, N, K, Ain, w(l, wid), Cout, ep_, st);
  };
  GPTS_OP(top, 0, phase, 0.0, TH * (kResBytes + e), ln_fwd(dt, bf, D.T, D.H, c.ln_eps, X, w(l, GPTS_LN1_G), w(l, GPTS_LN1_B), A, stat1,
                  stat1 + D.T, st, h16), "ln1 fwd");
  GemmEpilogue ep;
  ep.bias = w(l, GPTS_B_QKV);
  ep.b_image = img(l, 0);
  GPTS_OP(top_gemm, 0, phase, gf(D.T, 3 * D.P, D.H), gb(D.T, 3 * D.P, D.H, e), fwd_gemm(3 * D.P, D.H, A, GPTS_W_QKV, s + sl.QKV, ep), "qkv gemm");
  GPTS_OP(top_attn, 0, phase, attn_fl, (double)D.T * 4 * D.P * e, attention_fwd(dt, D.B, D.S, D.a, D.d, s + sl.QKV, s + sl.C,
                                reinterpret_cast<float*>(s + sl.LSE), fwk + fw.attn, st, h16), "attention fwd");
  ep = GemmEpilogue();
  ep.bias = w(l, GPTS_B_O);
  ep.residual = X;
  ep.residual_f32 = ep.out_f32 = bf;
  ep.b_image = img(l, 1);
  GPTS_OP(top_gemm, 1, phase, gf(D.T, D.H, D.P), gb(D.T, D.H, D.P, 2 * kResBytes), fwd_gemm(D.H, D.P, s + sl.C, GPTS_W_O, s + sl.X1, ep), "out-proj gemm");
  GPTS_OP(top, 1, phase, 0.0, TH * (kResBytes + e), ln_fwd(dt, bf, D.T, D.H, c.ln_eps, s + sl.X1, w(l, GPTS_LN2_G), w(l, GPTS_LN2_B), A2,
                  stat2, stat2 + D.T, st, h16), "ln2 fwd");
  ep = GemmEpilogue();
  ep.bias = w(l, GPTS_B_FC1);
  ep.gelu_out = G;
  ep.gelu_kind = c.gelu;
  ep.b_image = img(l, 2);
  GPTS_OP(top_gemm, 2, phase, gf(D.T, D.F, D.H), gb(D.T, D.F, D.H, 2 * e), fwd_gemm(D.F, D.H, A2, GPTS_W_FC1, s + sl.U, ep), "fc1 gemm");
  if (!Yout) return GPTS_OK;
  ep = GemmEpilogue();
  ep.bias = w(l, GPTS_B_FC2);
  ep.residual = s + sl.X1;
  ep.residual_f32 = bf;
  ep.out_f32 = bf && y_f32;   // the stage output y is bf16, the stream between layers fp32
  ep.b_image = img(l, 3);
  GPTS_OP(top_gemm, 3, phase, gf(D.T, D.H, D.F), gb(D.T, D.H, D.F, 2 * kResBytes), fwd_gemm(D.H, D.F, G, GPTS_W_FC2, Yout, ep), "fc2 gemm");
  return GPTS_OK;
}

int run_fwd(const gpt_stage_params* p, const void* x, void* act_stash, void* y, hipStream_t st) {
  int rc = check_call(p);
  if (rc != GPTS_OK) return rc;
  if ((rc = need_prepared(p)) != GPTS_OK) return rc;
  if (!x || !act_stash || !y || misaligned(x) || misaligned(act_stash) || misaligned(y))
    return fail(GPTS_EINVAL, "x / act_stash / y NULL or not 16-byte aligned");
  if (x == y) return fail(GPTS_EINVAL, "y must not alias x");
  if (!p->workspace && fwd_ws_bytes(p->cfg) > 0) return fail(GPTS_EINVAL, "forward needs a workspace");
  const gpt_stage_cfg& c = p->cfg;
  const Dims D(c);
  const size_t e = esize(c);
  const StashLayer sl = stash_layer(c);
  char* stash = static_cast<char*>(act_stash);
  // layer 0 keeps its own (fp32) copy of x so the backward phase never needs the caller's buffer
  if (c.dtype == GPTS_BF16)
    GPTS_TRY(widen_to_f32(x, reinterpret_cast<float*>(stash + sl.X), (size_t)D.T * D.H, st), "widen x");
  else
    GPTS_TRY(hipMemcpyAsync(stash + sl.X, x, (size_t)D.T * D.H * e, hipMemcpyDeviceToDevice, st), "copy x");
  const FwdWs fw = fwd_ws(c);
  char* fwk = static_cast<char*>(p->workspace);
  for (int l = 0; l < D.L; ++l) {
    char* s = stash + (size_t)l * sl.end;
    // with recompute == 2 only X stays in the stash; the rest of the block is transient
    char* blk = c.recompute == 2 ? fwk + fw.blk : s;
    const bool last = l == D.L - 1;
    void* Yout = last ? y : (void*)(s + sl.end + sl.X);
    rc = fwd_layer(p, l, s + sl.X, blk, Yout, !last, fwk, st, 0);
    if (rc != GPTS_OK) return rc;
  }
  return GPTS_OK;
}

// grad_stash != nullptr: data phase only -- the four weight-gradient products of every layer
// (and the rebuilding of their activation operands) are left out and the output gradients
// they need are written into grad_stash instead of the workspace.
int run_bwd(const gpt_stage_params* p, const void* act_stash, const void* dy, void* dx,
            void* dparams, hipStream_t st, void* grad_stash = nullptr) {
  int rc = check_call(p);
  if (rc != GPTS_OK) return rc;
  if ((rc = need_prepared(p)) != GPTS_OK) return rc;
  Tracer* tr = static_cast<Tracer*>(p->trace);
  if (!act_stash || !dy || !dx || !dparams || misaligned(act_stash) || misaligned(dy) ||
      misaligned(dx) || misaligned(dparams))
    return fail(GPTS_EINVAL, "act_stash / dy / dx / dparams NULL or not 16-byte aligned");
  if (!p->workspace) return fail(GPTS_EINVAL, "backward needs a workspace");
  const gpt_stage_cfg& c = p->cfg;
  const Dims D(c);
  const size_t e = esize(c);
  const int dt = c.dtype;
  const StashLayer xsl = stash_layer(c);   // what the stash holds per layer
  const StashLayer sl = layer_block(c);    // the block the backward of a layer reads
  const bool rerun = c.recompute == 2;     // the block is rebuilt by running the layer's forward again
  if (rerun && grad_stash)
    return fail(GPTS_EINVAL, "bwd_data_only: recompute == 2 keeps no activations for a later weight phase");
  const BwdWs ws = bwd_ws(c);
  const char* W = static_cast<const char*>(p->weights);
  const char* stash = static_cast<const char*>(act_stash);
  char* wk = static_cast<char*>(p->workspace);
  float* dP = static_cast<float*>(dparams);
  auto w = [&](int l, int id) { return (const void*)(W + tensor_off(D, l, id) * e); };
  auto g = [&](int l, int id) { return dP + tensor_off(D, l, id); };
  float* ln_part = reinterpret_cast<float*>(wk + ws.ln_part);
  float* cs_part = reinterpret_cast<float*>(wk + ws.cs_part);
  void* dU = wk + ws.dU;
  void* dA = wk + ws.dA;
  void* dX1 = wk + ws.dX1;
  void* dC = wk + ws.dC;
  void* dQKV = wk + ws.dQKV;
  void* attn_scratch = wk + ws.attn;
  const bool data_only = grad_stash != nullptr;
  if (data_only && misaligned(grad_stash)) return fail(GPTS_EINVAL, "grad_stash not 16-byte aligned");
  const GradStashLayer gl = grad_stash_layer(c);
  char* gs = static_cast<char*>(grad_stash);

  // algorithmic work of one operator, for the tracer: flops of an M x N x K product and
  // the bytes it must move (operands once, result once)
  auto gf = [](double M, double N, double K) { return 2.0 * M * N * K; };
  auto gb = [&](double M, double N, double K, double out_bytes) { return (M * K + N * K) * e + M * N * out_bytes; };
  const double TH = (double)D.T * D.H, attn_fl = 4.0 * D.B * D.a * D.d * ((double)D.S * (D.S + 1) / 2.0);
  const void* dY = dy;
  if (data_only) {
    // the top layer's output gradient is the caller's buffer: keep a copy for the weight phase
    void* top = gs + (size_t)(D.L - 1) * gl.end + gl.dY;
    GPTS_TRY(hipMemcpyAsync(top, dy, (size_t)D.T * D.H * e, hipMemcpyDeviceToDevice, st), "copy dy");
    dY = top;
  }
  for (int l = D.L - 1; l >= 0; --l) {
    const char* xs = stash + (size_t)l * xsl.end + xsl.X;    // the layer's input X
    const char* s = stash + (size_t)l * xsl.end;
    if (rerun) {
      // keep-only-X recomputation: run the layer's forward again, up to the GeLU, into the
      // workspace block (same kernels on the same inputs as in the forward phase: same bits)
      char* fwk2 = wk + ws.fwd2;
      char* blk = fwk2 + fwd_ws(c).blk;
      int rc2 = fwd_layer(p, l, xs, blk, nullptr, false, fwk2, st, 1);
      if (rc2 != GPTS_OK) return rc2;
      s = blk;
    }
    const float* stat1 = reinterpret_cast<const float*>(s + sl.stat1);
    const float* stat2 = reinterpret_cast<const float*>(s + sl.stat2);
    void* dXout = (l == 0) ? dx : (void*)(wk + (((D.L - 1 - l) & 1) ? ws.pong : ws.ping));
    if (data_only) {
      char* g0 = gs + (size_t)l * gl.end;
      dU = g0 + gl.dU;
      dX1 = g0 + gl.dX1;
      dQKV = g0 + gl.dQKV;
      if (l > 0) dXout = gs + (size_t)(l - 1) * gl.end + gl.dY;   // the layer below reads it as its dY
    }
    GemmEpilogue none;
    GemmEpilogue d_fc1, d_o, d_qkv;   // plain dgrads (on the raw weights)
    // y = x1 + g W2^T + b2 ;  g = gelu(u)
    const bool h16 = c.fwd_fp16 != 0;            // QKV, C, U of the stash hold fp16 values
    const bool rebuild = c.recompute == 1 || h16;     // A, A2, G are rebuilt here (as bf16)
    const void* U = s + sl.U;
    if (h16) {
      // gradients need bf16's range, so every backward product is bf16: it reads bf16 copies of
      // the fp16 forward activations (only the attention logits are recomputed from the fp16
      // Q and K, the operands the forward pass formed them from)
      GPTS_OP(GPTS_TR_CONVERT, 2, 1, 0.0, (double)D.T * D.F * 2 * e, f16_to_bf16(s + sl.U, wk + ws.bU, (size_t)D.T * D.F, st), "u to bf16");
      U = wk + ws.bU;
    }
    GemmEpilogue ep;
    ep.dgelu_u = U;
    ep.gelu_kind = c.gelu;
    // the matrix-core product also leaves the column sums of dU (the fc1 bias gradient) as
    // per-tile-row partials, when it runs and they fit the column-sum scratch
    const int cs_rows = (dt == GPTS_BF16 && gemm_mfma_supported(1, D.T, D.F, D.H)) ? gemm_mfma_colsum_rows(D.T, D.F) : 0;
    const bool fused_b1 = cs_rows > 0 && cs_rows <= colsum_splits(D.T);
    if (fused_b1) ep.colsum_partial = cs_part;
    GPTS_OP(GPTS_TR_GEMM_DGRAD, 3, 1, gf(D.T, D.F, D.H), gb(D.T, D.F, D.H, 2 * e), gemm(dt, 1, D.T, D.F, D.H, dY, w(l, GPTS_W_FC2), dU, ep, st), "fc2 dgrad");
    if (fused_b1)
      GPTS_OP(GPTS_TR_BIAS_GRAD, 2, 1, 0.0, (double)cs_rows * D.F * 4, reduce_colsum_partials(cs_part, cs_rows, D.F, g(l, GPTS_B_FC1), st), "fc1 bias grad (partials from the fc2 dgrad epilogue)");
    const void* G = s + sl.G;
    if (rebuild && !data_only) {
      GPTS_OP(GPTS_TR_RECOMPUTE, 2, 1, 0.0, (double)D.T * D.F * 2 * e, gelu_fwd(dt, c.gelu, s + sl.U, wk + ws.rG, (size_t)D.T * D.F, st, h16), "gelu recompute");
      G = wk + ws.rG;
    }
    if (!data_only)
      GPTS_OP(GPTS_TR_GEMM_WGRAD, 3, 1, gf(D.H, D.F, D.T), gb(D.H, D.F, D.T, 8), gemm(dt, 2, D.H, D.F, D.T, dY, G, g(l, GPTS_W_FC2), none, st), "fc2 wgrad");
    // the bias gradient of fc2 is the column sum of the layer's incoming gradient: below the
    // top layer the LayerNorm backward that produced that gradient has summed it already
    if (l == c.n_layers - 1)
      GPTS_OP(GPTS_TR_BIAS_GRAD, 3, 1, 0.0, TH * e, colsum(dt, D.T, D.H, dY, g(l, GPTS_B_FC2), cs_part, st), "fc2 bias grad");
    // u = a2 W1^T + b1
    GPTS_OP(GPTS_TR_GEMM_DGRAD, 2, 1, gf(D.T, D.H, D.F), gb(D.T, D.H, D.F, e), gemm(dt, 1, D.T, D.H, D.F, dU, w(l, GPTS_W_FC1), dA, d_fc1, st), "fc1 dgrad");
    const void* A2 = s + sl.A2;
    if (rebuild && !data_only) {
      float* rs = reinterpret_cast<float*>(wk + ws.rstat);
      GPTS_OP(GPTS_TR_RECOMPUTE, 1, 1, 0.0, TH * (kResBytes + e), ln_fwd(dt, dt == GPTS_BF16, D.T, D.H, c.ln_eps, s + sl.X1, w(l, GPTS_LN2_G), w(l, GPTS_LN2_B),
                      wk + ws.rA, rs, rs + D.T, st), "ln2 recompute");
      A2 = wk + ws.rA;
    }
    if (!data_only)
      GPTS_OP(GPTS_TR_GEMM_WGRAD, 2, 1, gf(D.F, D.H, D.T), gb(D.F, D.H, D.T, 8), gemm(dt, 2, D.F, D.H, D.T, dU, A2, g(l, GPTS_W_FC1), none, st), "fc1 wgrad");
    if (!fused_b1)
      GPTS_OP(GPTS_TR_BIAS_GRAD, 2, 1, 0.0, (double)D.T * D.F * e, colsum(dt, D.T, D.F, dU, g(l, GPTS_B_FC1), cs_part, st), "fc1 bias grad");
    // a2 = LN2(x1), x1 also feeds the residual
    GPTS_OP(GPTS_TR_LN_BWD, 1, 1, 0.0, TH * (3 * e + kResBytes), ln_bwd(dt, dt == GPTS_BF16, D.T, D.H, dA, s + sl.X1, stat2, stat2 + D.T, w(l, GPTS_LN2_G), dY, dX1,
                    g(l, GPTS_LN2_G), g(l, GPTS_LN2_B), g(l, GPTS_B_O), ln_part, st), "ln2 bwd (+ out-proj bias grad)");
    // x1 = x + c Wo^T + bo
    GPTS_OP(GPTS_TR_GEMM_DGRAD, 1, 1, gf(D.T, D.P, D.H), gb(D.T, D.P, D.H, e), gemm(dt, 1, D.T, D.P, D.H, dX1, w(l, GPTS_W_O), dC, d_o, st), "out-proj dgrad");
    const void* Cb = s + sl.C;
    const void* QKVb = s + sl.QKV;
    if (h16) {
      if (!data_only)
        GPTS_OP(GPTS_TR_CONVERT, 1, 1, 0.0, (double)D.T * D.P * 2 * e, f16_to_bf16(s + sl.C, wk + ws.bC, (size_t)D.T * D.P, st), "c to bf16");
      GPTS_OP(GPTS_TR_CONVERT, 0, 1, 0.0, (double)D.T * 3 * D.P * 2 * e, f16_to_bf16(s + sl.QKV, wk + ws.bQKV, (size_t)D.T * 3 * D.P, st), "qkv to bf16");
      Cb = wk + ws.bC;
      QKVb = wk + ws.bQKV;
    }
    if (!data_only)
      GPTS_OP(GPTS_TR_GEMM_WGRAD, 1, 1, gf(D.H, D.P, D.T), gb(D.H, D.P, D.T, 8), gemm(dt, 2, D.H, D.P, D.T, dX1, Cb, g(l, GPTS_W_O), none, st), "out-proj wgrad");
    // c = attention(qkv)
    GPTS_OP(GPTS_TR_ATTN_BWD, 0, 1, 2.0 * attn_fl, (double)D.T * 9 * D.P * e, attention_bwd(dt, D.B, D.S, D.a, D.d, QKVb, s + sl.C,
                                  reinterpret_cast<const float*>(s + sl.LSE), dC, dQKV, attn_scratch, st, h16 ? s + sl.QKV : nullptr),
             "attention bwd");
    // qkv = a Wqkv^T + bqkv
    GPTS_OP(GPTS_TR_GEMM_DGRAD, 0, 1, gf(D.T, D.H, 3 * D.P), gb(D.T, D.H, 3 * D.P, e), gemm(dt, 1, D.T, D.H, 3 * D.P, dQKV, w(l, GPTS_W_QKV), dA, d_qkv, st), "qkv dgrad");
    const void* A = s + sl.A;
    if (rebuild && !data_only) {
      float* rs = reinterpret_cast<float*>(wk + ws.rstat);
      GPTS_OP(GPTS_TR_RECOMPUTE, 0, 1, 0.0, TH * (kResBytes + e), ln_fwd(dt, dt == GPTS_BF16, D.T, D.H, c.ln_eps, xs, w(l, GPTS_LN1_G), w(l, GPTS_LN1_B),
                      wk + ws.rA, rs, rs + D.T, st), "ln1 recompute");
      A = wk + ws.rA;
    }
    if (!data_only)
      GPTS_OP(GPTS_TR_GEMM_WGRAD, 0, 1, gf(3 * D.P, D.H, D.T), gb(3 * D.P, D.H, D.T, 8), gemm(dt, 2, 3 * D.P, D.H, D.T, dQKV, A, g(l, GPTS_W_QKV), none, st), "qkv wgrad");
    GPTS_OP(GPTS_TR_BIAS_GRAD, 0, 1, 0.0, (double)D.T * 3 * D.P * e, colsum(dt, D.T, 3 * D.P, dQKV, g(l, GPTS_B_QKV), cs_part, st), "qkv bias grad");
    // a = LN1(x), x also feeds the residual
    GPTS_OP(GPTS_TR_LN_BWD, 0, 1, 0.0, TH * (3 * e + kResBytes), ln_bwd(dt, dt == GPTS_BF16, D.T, D.H, dA, xs, stat1, stat1 + D.T, w(l, GPTS_LN1_G), dX1, dXout,
                    g(l, GPTS_LN1_G), g(l, GPTS_LN1_B), l > 0 ? g(l - 1, GPTS_B_FC2) : nullptr, ln_part, st),
            "ln1 bwd (+ fc2 bias grad of the layer below)");
    dY = dXout;
  }
  return GPTS_OK;
}

// Weight phase: dW += sum over the n micro-batches of (output gradient)^T (input activation),
// for the four linears of every layer.  When the stash holds the input activations as bf16
// (full stash), the buffers are equally spaced and the shape suits the segmented kernel, one
// launch per linear contracts over all micro-batches' tokens (one read-modify-write of dW);
// otherwise one accumulating product per micro-batch, with the activations rebuilt first where
// the stash does not hold them (recompute, fwd_fp16).
int run_wgrad_flush(const gpt_stage_params* p, int n, const void* const* act_stashes,
                    const void* const* grad_stashes, void* dparams, hipStream_t st) {
  int rc = check_call(p);
  if (rc != GPTS_OK) return rc;
  if (n < 1 || !act_stashes || !grad_stashes || !dparams || misaligned(dparams))
    return fail(GPTS_EINVAL, "wgrad_flush: n < 1, NULL array or dparams NULL / misaligned");
  for (int m = 0; m < n; ++m)
    if (!act_stashes[m] || !grad_stashes[m] || misaligned(act_stashes[m]) || misaligned(grad_stashes[m]))
      return fail(GPTS_EINVAL, "wgrad_flush: a stash pointer is NULL or not 16-byte aligned");
  if (!p->workspace) return fail(GPTS_EINVAL, "wgrad_flush needs the backward workspace");
  Tracer* tr = static_cast<Tracer*>(p->trace);
  const gpt_stage_cfg& c = p->cfg;
  const Dims D(c);
  const size_t e = esize(c);
  const int dt = c.dtype;
  const StashLayer sl = stash_layer(c);
  const GradStashLayer gl = grad_stash_layer(c);
  const BwdWs ws = bwd_ws(c);
  const char* W = static_cast<const char*>(p->weights);
  char* wk = static_cast<char*>(p->workspace);
  float* dP = static_cast<float*>(dparams);
  auto w = [&](int l, int id) { return (const void*)(W + tensor_off(D, l, id) * e); };
  auto g = [&](int l, int id) { return dP + tensor_off(D, l, id); };
  auto gf = [](double M, double N, double K) { return 2.0 * M * N * K; };
  auto gb = [&](double M, double N, double K, double out_bytes) { return (M * K + N * K) * e + M * N * out_bytes; };
  if (c.recompute == 2) return fail(GPTS_EINVAL, "wgrad_flush: recompute == 2 keeps no activations for a weight phase");
  const bool h16 = c.fwd_fp16 != 0, rebuild = c.recompute == 1 || h16;
  // equal spacing of the micro-batches' buffers (byte strides; 0 when n == 1)
  auto stride_of = [&](const void* const* ptrs, ptrdiff_t* out) {
    *out = 0;
    if (n == 1) return true;
    const ptrdiff_t d0 = static_cast<const char*>(ptrs[1]) - static_cast<const char*>(ptrs[0]);
    if (d0 <= 0 || d0 % (ptrdiff_t)e) return false;
    for (int m = 2; m < n; ++m)
      if (static_cast<const char*>(ptrs[m]) - static_cast<const char*>(ptrs[m - 1]) != d0) return false;
    *out = d0;
    return true;
  };
  ptrdiff_t act_stride = 0, grad_stride = 0;
  const bool spaced = dt == GPTS_BF16 && !rebuild && stride_of(act_stashes, &act_stride) && stride_of(grad_stashes, &grad_stride);
  struct Lin { int sub, M, N, wid; size_t dout, in; };   // dW[M,N] += dOut[T,M]^T In[T,N]
  const Lin lins[4] = {{3, D.H, D.F, GPTS_W_FC2, gl.dY, sl.G}, {2, D.F, D.H, GPTS_W_FC1, gl.dU, sl.A2},
                       {1, D.H, D.P, GPTS_W_O, gl.dX1, sl.C}, {0, 3 * D.P, D.H, GPTS_W_QKV, gl.dQKV, sl.A}};
  for (int l = D.L - 1; l >= 0; --l) {
    for (const Lin& L : lins) {
      auto dout_of = [&](int m) { return static_cast<const char*>(grad_stashes[m]) + (size_t)l * gl.end + L.dout; };
      if (spaced && (n == 1 || gemm_wgrad_segments_supported(2, L.M, L.N, D.T))) {
        GemmEpilogue ep;
        ep.k_segments = n;
        ep.seg_stride_a = (size_t)grad_stride / e;
        ep.seg_stride_b = (size_t)act_stride / e;
        const void* in0 = static_cast<const char*>(act_stashes[0]) + (size_t)l * sl.end + L.in;
        GPTS_OP(GPTS_TR_GEMM_WGRAD, L.sub, 1, gf(L.M, L.N, (double)D.T * n), gb(L.M, L.N, (double)D.T * n, 8),
                gemm(dt, 2, L.M, L.N, D.T, dout_of(0), in0, g(l, L.wid), ep, st), "wgrad over all micro-batches");
        continue;
      }
      for (int m = 0; m < n; ++m) {
        const char* s = static_cast<const char*>(act_stashes[m]) + (size_t)l * sl.end;
        const void* in = rebuild ? nullptr : (const void*)(s + L.in);
        if (rebuild) {
          float* rs = reinterpret_cast<float*>(wk + ws.rstat);
          if (L.sub == 3) {
            GPTS_OP(GPTS_TR_RECOMPUTE, 2, 1, 0.0, (double)D.T * D.F * 2 * e, gelu_fwd(dt, c.gelu, s + sl.U, wk + ws.rG, (size_t)D.T * D.F, st, h16), "gelu recompute");
            in = wk + ws.rG;
          } else if (L.sub == 1) {
            in = s + sl.C;
            if (h16) {
              GPTS_OP(GPTS_TR_CONVERT, 1, 1, 0.0, (double)D.T * D.P * 2 * e, f16_to_bf16(s + sl.C, wk + ws.bC, (size_t)D.T * D.P, st), "c to bf16");
              in = wk + ws.bC;
            }
          } else {
            const bool second = L.sub == 2;
            GPTS_OP(GPTS_TR_RECOMPUTE, second ? 1 : 0, 1, 0.0, (double)D.T * D.H * (kResBytes + e),
                    ln_fwd(dt, dt == GPTS_BF16, D.T, D.H, c.ln_eps, s + (second ? sl.X1 : sl.X), w(l, second ? GPTS_LN2_G : GPTS_LN1_G),
                           w(l, second ? GPTS_LN2_B : GPTS_LN1_B), wk + ws.rA, rs, rs + D.T, st), "layernorm recompute");
            in = wk + ws.rA;
          }
        }
        GemmEpilogue none;
        GPTS_OP(GPTS_TR_GEMM_WGRAD, L.sub, 1, gf(L.M, L.N, D.T), gb(L.M, L.N, D.T, 8),
                gemm(dt, 2, L.M, L.N, D.T, dout_of(m), in, g(l, L.wid), none, st), "wgrad of one micro-batch");
      }
    }
  }
  return GPTS_OK;
}

}  // namespace

namespace gpts {
int set_error(int code, const char* msg) { return fail(code, msg); }
}  // namespace gpts

extern "C" {

int gpt_stage_validate(const gpt_stage_cfg* c) {
  if (!c) return fail(GPTS_EINVAL, "cfg is NULL");
  if (c->dtype != GPTS_FP32 && c->dtype != GPTS_BF16) return fail(GPTS_EINVAL, "dtype must be GPTS_FP32 or GPTS_BF16");
  if (c->gelu != GPTS_GELU_TANH && c->gelu != GPTS_GELU_ERF) return fail(GPTS_EINVAL, "gelu must be GPTS_GELU_TANH or GPTS_GELU_ERF");
  if (!(c->ln_eps >= 0.f)) return fail(GPTS_EINVAL, "ln_eps must be >= 0");
  if (c->recompute < 0 || c->recompute > 2) return fail(GPTS_EINVAL, "recompute must be 0, 1 or 2");
  if (c->fwd_fp16 != 0 && c->fwd_fp16 != 1) return fail(GPTS_EINVAL, "fwd_fp16 must be 0 or 1");
  if (c->fwd_fp16 && c->dtype != GPTS_BF16) return fail(GPTS_EINVAL, "fwd_fp16 applies to bf16 stages only");
  if (c->n_layers < 1 || c->batch < 1 || c->seq < 1 || c->n_heads < 1 || c->hidden < 1 || c->ffn < 1)
    return fail(GPTS_ESHAPE, "n_layers, batch, seq, n_heads, hidden, ffn must be >= 1");
  if (c->head_dim != 32 && c->head_dim != 64 && c->head_dim != 128)
    return fail(GPTS_ESHAPE, "head_dim must be 32, 64 or 128");
  const long long P = (long long)c->n_heads * c->head_dim, T = (long long)c->batch * c->seq;
  if (c->hidden % 8 || c->ffn % 8) return fail(GPTS_ESHAPE, "hidden and ffn must be multiples of 8");
  if (c->hidden > 16384) return fail(GPTS_ESHAPE, "hidden must be <= 16384");
  if (T > (1 << 24) || P > (1 << 20) || c->ffn > (1 << 20)) return fail(GPTS_ESHAPE, "tokens, attention width or ffn too large");
  if (c->dtype == GPTS_BF16 && (T % 64 || c->hidden % 64 || P % 64 || c->ffn % 64))
    return fail(GPTS_ESHAPE, "bf16 stages need tokens, hidden, attention width and ffn to be multiples of 64");
  if (c->fwd_fp16) {
    const int Pi = (int)P, Ti = (int)T;
    if (c->hidden % 128 || P % 128 || c->ffn % 128)
      return fail(GPTS_ESHAPE, "fwd_fp16 needs hidden, attention width and ffn to be multiples of 128");
    if (!attention_mfma_supported(c->batch, c->seq, c->n_heads, c->head_dim))
      return fail(GPTS_ESHAPE, "fwd_fp16 needs seq*3*width < 2^31 (32-bit offsets of the attention kernels)");
    if (!gemm_fwd_f16_supported(Ti, 3 * Pi, c->hidden) || !gemm_fwd_f16_supported(Ti, c->hidden, Pi) ||
        !gemm_fwd_f16_supported(Ti, c->ffn, c->hidden) || !gemm_fwd_f16_supported(Ti, c->hidden, c->ffn))
      return fail(GPTS_ESHAPE, "fwd_fp16: a forward product exceeds the 32-bit operand offsets of the kernels");
  }
  return GPTS_OK;
}

size_t gpt_stage_param_count(const gpt_stage_cfg* c) {
  if (gpt_stage_validate(c) != GPTS_OK) return 0;
  Dims D(*c);
  return layer_elems(D) * D.L;
}
size_t gpt_stage_param_bytes(const gpt_stage_cfg* c) { return gpt_stage_param_count(c) * (c ? esize(*c) : 0); }
size_t gpt_stage_grad_bytes(const gpt_stage_cfg* c) { return gpt_stage_param_count(c) * sizeof(float); }
size_t gpt_stage_stash_bytes(const gpt_stage_cfg* c) {
  if (gpt_stage_validate(c) != GPTS_OK) return 0;
  return stash_layer(*c).end * c->n_layers;
}
size_t gpt_stage_workspace_bytes(const gpt_stage_cfg* c, int phase) {
  if (gpt_stage_validate(c) != GPTS_OK) return 0;
  return phase == 0 ? fwd_ws_bytes(*c) : bwd_ws(*c).end;
}
int gpt_stage_param_offset(const gpt_stage_cfg* c, int layer, int tensor_id, size_t* elem_off, size_t* n_elem) {
  int rc = gpt_stage_validate(c);
  if (rc != GPTS_OK) return rc;
  if (layer < 0 || layer >= c->n_layers || tensor_id < 0 || tensor_id >= GPTS_N_TENSORS || !elem_off || !n_elem)
    return fail(GPTS_EINVAL, "layer / tensor_id out of range or NULL output pointer");
  Dims D(*c);
  *elem_off = tensor_off(D, layer, tensor_id);
  *n_elem = tensor_elems(D, tensor_id);
  return GPTS_OK;
}
double gpt_stage_model_flops(const gpt_stage_cfg* c, int causal_aware) {
  if (gpt_stage_validate(c) != GPTS_OK) return 0.0;
  Dims D(*c);
  const double lin = 2.0 * D.T * (4.0 * D.P * D.H + 2.0 * (double)D.H * D.F);
  const double pairs = causal_aware ? (double)D.S * (D.S + 1) / 2.0 : (double)D.S * D.S;
  const double att = 4.0 * D.B * D.a * D.d * pairs;
  return 3.0 * D.L * (lin + att);
}
const char* gpt_stage_strerror(int code) {
  // the detailed text of the thread's last failure when `code` is the status that failure
  // returned, else the generic meaning of `code`
  if (code != GPTS_OK && code == g_err_code && g_err[0]) return g_err;
  switch (code) {
    case GPTS_OK: return "ok";
    case GPTS_EINVAL: return "invalid argument (null or misaligned pointer, bad enum value)";
    case GPTS_ESHAPE: return "shape outside what the kernels support";
    case GPTS_EHIP: return "a HIP call failed";
    case GPTS_ENOMEM: return "a caller-provided pool or array is too small";
  }
  return "unknown status";
}

size_t gpt_stage_prepared_bytes(const gpt_stage_cfg* c) {
  if (gpt_stage_validate(c) != GPTS_OK || c->dtype != GPTS_BF16) return 0;
  Dims D(*c);
  return prepared_off(D, D.L, 0) * 2;
}
int gpt_stage_prepare(const gpt_stage_params* p, void* prepared, void* stream) {
  int rc = check_call(p);
  if (rc != GPTS_OK) return rc;
  if (p->cfg.dtype != GPTS_BF16) return fail(GPTS_EINVAL, "prepare: only bf16 stages have prepared weights");
  if (!prepared || misaligned(prepared)) return fail(GPTS_EINVAL, "prepare: prepared NULL or not 16-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const Dims D(p->cfg);
  LinDims L[4];
  linears(D, L);
  const bf16* W = static_cast<const bf16*>(p->weights);
  bf16* out = static_cast<bf16*>(prepared);
  for (int l = 0; l < D.L; ++l)
    for (int i = 0; i < 4; ++i) {
      const bf16* w = W + tensor_off(D, l, L[i].wid);
      GPTS_TRY(gemm_prepare_image(w, out + prepared_off(D, l, i), L[i].out, L[i].in, false, st, p->cfg.fwd_fp16 != 0), "prepare fwd image");
    }
  return GPTS_OK;
}

int gpt_stage_fwd(const gpt_stage_params* p, const void* x, void* act_stash, void* y, void* stream) {
  return run_fwd(p, x, act_stash, y, static_cast<hipStream_t>(stream));
}
int gpt_stage_bwd(const gpt_stage_params* p, const void* act_stash, const void* dy, void* dx,
                  void* dparams, void* stream) {
  return run_bwd(p, act_stash, dy, dx, dparams, static_cast<hipStream_t>(stream));
}
int gpt_stage_fwd_only(const gpt_stage_params* p, const void* x, void* act_stash, void* y,
                       void* stream, void* done_event) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = run_fwd(p, x, act_stash, y, st);
  if (rc != GPTS_OK) return rc;
  if (done_event) GPTS_TRY(hipEventRecord(static_cast<hipEvent_t>(done_event), st), "record done_event");
  return GPTS_OK;
}
int gpt_stage_bwd_only(const gpt_stage_params* p, const void* act_stash, const void* dy, void* dx,
                       void* dparams, void* stream, void* wait_event) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = check_call(p);  // validate before touching the stream
  if (rc != GPTS_OK) return rc;
  if (wait_event) GPTS_TRY(hipStreamWaitEvent(st, static_cast<hipEvent_t>(wait_event), 0), "wait on wait_event");
  return run_bwd(p, act_stash, dy, dx, dparams, st);
}
size_t gpt_stage_grad_stash_bytes(const gpt_stage_cfg* c) {
  if (gpt_stage_validate(c) != GPTS_OK) return 0;
  return grad_stash_layer(*c).end * c->n_layers;
}
int gpt_stage_bwd_data_only(const gpt_stage_params* p, const void* act_stash, const void* dy, void* dx,
                            void* dparams, void* grad_stash, void* stream, void* wait_event) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = check_call(p);  // validate before touching the stream
  if (rc != GPTS_OK) return rc;
  if (!grad_stash) return fail(GPTS_EINVAL, "bwd_data_only: grad_stash is NULL");
  if (wait_event) GPTS_TRY(hipStreamWaitEvent(st, static_cast<hipEvent_t>(wait_event), 0), "wait on wait_event");
  return run_bwd(p, act_stash, dy, dx, dparams, st, grad_stash);
}
int gpt_stage_wgrad_flush(const gpt_stage_params* p, int n_microbatches, const void* const* act_stashes,
                          const void* const* grad_stashes, void* dparams, void* stream) {
  return run_wgrad_flush(p, n_microbatches, act_stashes, grad_stashes, dparams, static_cast<hipStream_t>(stream));
}
int gpt_stage_fwd_bwd(const gpt_stage_params* p, const void* x, const void* dy, void* act_stash,
                      void* y, void* dx, void* dparams, void* stream) {
  hipStream_t st = static_cast<hipStream_t>(stream);
  int rc = run_fwd(p, x, act_stash, y, st);
  if (rc != GPTS_OK) return rc;
  return run_bwd(p, act_stash, dy, dx, dparams, st);
}

// ---- operator tracer ----------------------------------------------------------------
int gpt_stage_trace_create(int capacity, void** trace) {
  if (capacity < 1 || !trace) return fail(GPTS_EINVAL, "trace_create: capacity must be >= 1 and trace non-NULL");
  Tracer* t = new (std::nothrow) Tracer;
  if (!t) return fail(GPTS_EINVAL, "trace_create: out of host memory");
  t->recs = new (std::nothrow) TraceRec[capacity];
  if (!t->recs) { delete t; return fail(GPTS_EINVAL, "trace_create: out of host memory"); }
  for (int i = 0; i < capacity; ++i) {
    if (hipEventCreate(&t->recs[i].e0) != hipSuccess || hipEventCreate(&t->recs[i].e1) != hipSuccess) {
      t->capacity = i;  // events created so far are released by destroy
      gpt_stage_trace_destroy(t);
      return fail(GPTS_EHIP, "trace_create: hipEventCreate failed");
    }
    t->capacity = i + 1;
  }
  *trace = t;
  return GPTS_OK;
}
int gpt_stage_trace_destroy(void* trace) {
  Tracer* t = static_cast<Tracer*>(trace);
  if (!t) return GPTS_OK;
  for (int i = 0; i < t->capacity; ++i) {
    (void)hipEventDestroy(t->recs[i].e0);
    (void)hipEventDestroy(t->recs[i].e1);
  }
  delete[] t->recs;
  delete t;
  return GPTS_OK;
}
int gpt_stage_trace_reset(void* trace) {
  Tracer* t = static_cast<Tracer*>(trace);
  if (!t) return fail(GPTS_EINVAL, "trace_reset: trace is NULL");
  t->n = 0;
  t->dropped = 0;
  return GPTS_OK;
}
int gpt_stage_trace_collect(void* trace, gpt_stage_trace_rec* out, int max_records, int* n_records,
                            int* n_dropped) {
  Tracer* t = static_cast<Tracer*>(trace);
  if (!t || !n_records || (max_records > 0 && !out)) return fail(GPTS_EINVAL, "trace_collect: bad argument");
  const int n = t->n < max_records ? t->n : max_records;
  for (int i = 0; i < n; ++i) {
    const TraceRec& r = t->recs[i];
    GPTS_TRY(hipEventSynchronize(r.e1), "trace_collect: event synchronize");
    float ms = 0.f, ts = 0.f;
    GPTS_TRY(hipEventElapsedTime(&ms, r.e0, r.e1), "trace_collect: elapsed");
    GPTS_TRY(hipEventElapsedTime(&ts, t->recs[0].e0, r.e0), "trace_collect: elapsed");
    out[i].op = r.op; out[i].sub = r.sub; out[i].layer = r.layer; out[i].phase = r.phase;
    out[i].start_ms = ts; out[i].dur_ms = ms; out[i].flops = r.flops; out[i].bytes = r.bytes;
  }
  *n_records = n;
  if (n_dropped) *n_dropped = t->dropped + (t->n - n);
  return GPTS_OK;
}
const char* gpt_stage_trace_op_name(int op) {
  switch (op) {
    case GPTS_TR_LN_FWD: return "layernorm_fwd";
    case GPTS_TR_GEMM_FWD: return "gemm_fwd";
    case GPTS_TR_ATTN_FWD: return "attention_fwd";
    case GPTS_TR_GEMM_DGRAD: return "gemm_dgrad";
    case GPTS_TR_GEMM_WGRAD: return "gemm_wgrad";
    case GPTS_TR_BIAS_GRAD: return "bias_grad";
    case GPTS_TR_LN_BWD: return "layernorm_bwd";
    case GPTS_TR_ATTN_BWD: return "attention_bwd";
    case GPTS_TR_RECOMPUTE: return "recompute";
    case GPTS_TR_CONVERT: return "convert";
  }
  return "unknown";
}

// ---- single operations ------------------------------------------------------------
static int op_dtype_ok(int dtype) { return dtype == GPTS_FP32 || dtype == GPTS_BF16; }

int gpt_stage_op_layernorm_fwd(int dtype, int x_f32, int T, int H, float eps, const void* x, const void* gamma,
                               const void* beta, void* out, float* mean, float* rstd, void* stream) {
  if (!op_dtype_ok(dtype) || !x || !gamma || !beta || !out || !mean || !rstd) return fail(GPTS_EINVAL, "layernorm_fwd: bad argument");
  if (T < 1 || H < 8 || H % 8 || H > 16384) return fail(GPTS_ESHAPE, "layernorm_fwd: H must be a multiple of 8, <= 16384");
  GPTS_TRY(ln_fwd(dtype, x_f32 != 0, T, H, eps, x, gamma, beta, out, mean, rstd, static_cast<hipStream_t>(stream)), "layernorm_fwd");
  return GPTS_OK;
}
size_t gpt_stage_op_layernorm_bwd_scratch_bytes(int T, int H) { return ln_bwd_scratch_bytes(T, H); }
int gpt_stage_op_layernorm_bwd(int dtype, int x_f32, int T, int H, const void* dout, const void* x,
                               const float* mean, const float* rstd, const void* gamma,
                               const void* dres, void* dx, float* dgamma, float* dbeta,
                               float* dxsum, float* partial, void* stream) {
  if (!op_dtype_ok(dtype) || !dout || !x || !mean || !rstd || !gamma || !dx || !dgamma || !dbeta || !partial)
    return fail(GPTS_EINVAL, "layernorm_bwd: bad argument");
  if (T < 1 || H < 8 || H % 8 || H > 16384) return fail(GPTS_ESHAPE, "layernorm_bwd: H must be a multiple of 8, <= 16384");
  GPTS_TRY(ln_bwd(dtype, x_f32 != 0, T, H, dout, x, mean, rstd, gamma, dres, dx, dgamma, dbeta, dxsum, partial,
                  static_cast<hipStream_t>(stream)), "layernorm_bwd");
  return GPTS_OK;
}
int gpt_stage_op_gemm(int dtype, int form, int M, int N, int K, const void* A, const void* B, void* C,
                      const void* bias, const void* residual, void* C2, const void* dgelu_u,
                      int gelu_kind, int f32_flags, void* stream) {
  if (!op_dtype_ok(dtype) || form < 0 || form > 2 || !A || !B || !C) return fail(GPTS_EINVAL, "gemm: bad argument");
  if (M < 1 || N < 1 || K < 1) return fail(GPTS_ESHAPE, "gemm: M, N, K must be >= 1");
  if (form == 2 && (bias || residual || C2 || dgelu_u)) return fail(GPTS_EINVAL, "gemm: the wgrad form takes no epilogue");
  if (form == 1 && C2) return fail(GPTS_EINVAL, "gemm: gelu output only with form 0");
  if (form == 0 && dgelu_u) return fail(GPTS_EINVAL, "gemm: dgelu only with form 1");
  if (f32_flags && (form != 0 || !residual || C2 || (f32_flags & 2 && !(f32_flags & 1)) || f32_flags > 3))
    return fail(GPTS_EINVAL, "gemm: fp32 residual/output only for form 0 with a residual and no gelu output");
  GemmEpilogue ep;
  ep.bias = bias; ep.residual = residual; ep.gelu_out = C2; ep.dgelu_u = dgelu_u; ep.gelu_kind = gelu_kind;
  ep.residual_f32 = dtype == GPTS_BF16 && (f32_flags & 1); ep.out_f32 = dtype == GPTS_BF16 && (f32_flags & 2);
  GPTS_TRY(gemm(dtype, form, M, N, K, A, B, C, ep, static_cast<hipStream_t>(stream)), "gemm");
  return GPTS_OK;
}
size_t gpt_stage_op_colsum_scratch_bytes(int M, int N) { return colsum_scratch_bytes(M, N); }
int gpt_stage_op_colsum(int dtype, int M, int N, const void* A, float* out, float* partial, void* stream) {
  if (!op_dtype_ok(dtype) || !A || !out || !partial) return fail(GPTS_EINVAL, "colsum: bad argument");
  if (M < 1 || N < 8 || N % 8) return fail(GPTS_ESHAPE, "colsum: N must be a multiple of 8");
  GPTS_TRY(colsum(dtype, M, N, A, out, partial, static_cast<hipStream_t>(stream)), "colsum");
  return GPTS_OK;
}
size_t gpt_stage_op_attention_scratch_bytes(int dtype, int B, int S, int n_heads, int head_dim, int phase) {
  if (!op_dtype_ok(dtype) || B < 1 || S < 1 || n_heads < 1 || (head_dim != 32 && head_dim != 64 && head_dim != 128) ||
      (phase != 0 && phase != 1))
    return 0;
  return attention_scratch_bytes(dtype, B, S, n_heads, head_dim, phase);
}
int gpt_stage_op_attention_fwd(int dtype, int B, int S, int n_heads, int head_dim, const void* qkv,
                               void* out, float* lse, void* scratch, void* stream) {
  if (!op_dtype_ok(dtype) || !qkv || !out || !lse) return fail(GPTS_EINVAL, "attention_fwd: bad argument");
  if (B < 1 || S < 1 || n_heads < 1 || (head_dim != 32 && head_dim != 64 && head_dim != 128))
    return fail(GPTS_ESHAPE, "attention_fwd: head_dim must be 32, 64 or 128");
  if (!scratch && attention_scratch_bytes(dtype, B, S, n_heads, head_dim, 0) > 0)
    return fail(GPTS_EINVAL, "attention_fwd: scratch is NULL");
  GPTS_TRY(attention_fwd(dtype, B, S, n_heads, head_dim, qkv, out, lse, scratch, static_cast<hipStream_t>(stream)), "attention_fwd");
  return GPTS_OK;
}
int gpt_stage_op_attention_bwd(int dtype, int B, int S, int n_heads, int head_dim, const void* qkv,
                               const void* out, const float* lse, const void* dout, void* dqkv,
                               void* scratch, void* stream) {
  if (!op_dtype_ok(dtype) || !qkv || !out || !lse || !dout || !dqkv || !scratch) return fail(GPTS_EINVAL, "attention_bwd: bad argument");
  if (B < 1 || S < 1 || n_heads < 1 || (head_dim != 32 && head_dim != 64 && head_dim != 128))
    return fail(GPTS_ESHAPE, "attention_bwd: head_dim must be 32, 64 or 128");
  GPTS_TRY(attention_bwd(dtype, B, S, n_heads, head_dim, qkv, out, lse, dout, dqkv, scratch,
                                static_cast<hipStream_t>(stream)), "attention_bwd");
  return GPTS_OK;
}

}  // extern "C"
