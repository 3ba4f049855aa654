/*
 * gpt_stage.h -- C ABI of libgptstage: forward and backward pass of one GPT
 * pipeline stage (L pre-LayerNorm decoder layers) on one MI355X (gfx950).
 *
 * What the calls compute.  The paper's schedulers treat a pipeline stage as two
 * separable phases: a "forward phase" and a "backward phase (gradient
 * computation)" (MegaFBD, section 4.1), and one unit of work is "one model
 * chunk applied to one micro-batch" (MegaDPP, section 5.2, parallel scheduler).
 * The layer mathematics is that of the GPT/Megatron-LM decoder layer the paper
 * builds on (section 2.2-2.3).  Per layer, for x in R^{T x H}, T = batch*seq:
 *     a   = LayerNorm(x; ln1_g, ln1_b)
 *     qkv = a W_qkv^T + b_qkv          (columns: [Q heads | K heads | V heads])
 *     c   = causal softmax attention per head, scale 1/sqrt(head_dim)
 *     x1  = x + c W_o^T + b_o
 *     a2  = LayerNorm(x1; ln2_g, ln2_b)
 *     u   = a2 W_fc1^T + b_fc1 ;  g = gelu(u)
 *     y   = x1 + g W_fc2^T + b_fc2
 * The backward phase returns dx = d<y,dy>/dx and ADDS d<y,dy>/dparam to the
 * caller's gradient buffer (accumulation over micro-batches, as the
 * breadth-first traversal of section 5.2 needs).
 *
 * General rules (all entry points)
 *  - Every pointer named "device" is GPU memory owned by the caller; the library
 *    allocates no device memory and frees nothing.  Its only state is the calling
 *    thread's last error text, the host objects the caller creates (tracers,
 *    coordinators) and the fixed scratch array of gpt_stage_op_colsum_noalloc.
 *  - Every call only enqueues kernels on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream) and returns; it never synchronises
 *    (exceptions, documented where they are declared: gpt_stage_trace_collect and
 *    gpt_dpp_run_ready block the calling host thread).
 *  - Device pointers must be 16-byte aligned.
 *  - Return value: GPTS_OK (0) or a negative gpts_status; nothing is launched
 *    when validation fails.  No exceptions cross this boundary.
 *  - Results are run-to-run bitwise deterministic (no floating-point atomics).
 *  - bf16 stages: x, y, dy, dx, weights and every tensor that branches off the
 *    residual stream are bf16 with fp32 accumulation; LayerNorm statistics, softmax,
 *    parameter gradients and the residual stream between layers are fp32.
 */
#ifndef GPT_STAGE_H_
#define GPT_STAGE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GPTS_OK = 0,
  GPTS_EINVAL = -1, /* null or misaligned pointer, bad enum value            */
  GPTS_ESHAPE = -2, /* shape outside what the kernels support (see validate) */
  GPTS_EHIP = -3,   /* a HIP launch failed; text via gpt_stage_strerror      */
  GPTS_ENOMEM = -4  /* a caller-provided pool or array is too small           */
} gpts_status;

enum { GPTS_FP32 = 0, GPTS_BF16 = 1 };     /* cfg.dtype */
enum { GPTS_GELU_TANH = 0, GPTS_GELU_ERF = 1 }; /* cfg.gelu  */

/* Per-layer tensor ids, in the order they sit in the flat parameter buffer and
 * in the flat fp32 gradient buffer.  Weights are row-major [out, in].
 * W_QKV rows [0,P) are Q, [P,2P) K, [2P,3P) V, P = n_heads*head_dim; head n owns
 * rows n*head_dim .. (n+1)*head_dim-1 of each block. */
enum {
  GPTS_LN1_G = 0, GPTS_LN1_B, GPTS_W_QKV, GPTS_B_QKV, GPTS_W_O, GPTS_B_O,
  GPTS_LN2_G, GPTS_LN2_B, GPTS_W_FC1, GPTS_B_FC1, GPTS_W_FC2, GPTS_B_FC2,
  GPTS_N_TENSORS
};

typedef struct {
  int32_t n_layers;  /* L >= 1                                               */
  int32_t hidden;    /* H                                                    */
  int32_t n_heads;   /* a : heads held by this GPU (P = a*head_dim may != H) */
  int32_t head_dim;  /* d in {32, 64, 128}                                   */
  int32_t ffn;       /* F                                                    */
  int32_t seq;       /* S                                                    */
  int32_t batch;     /* B : micro-batch size; tokens T = B*S                 */
  int32_t dtype;     /* GPTS_FP32: every tensor fp32.  GPTS_BF16: activations,
                        weights, x, y, dy, dx bf16; statistics, accumulators
                        and parameter gradients fp32.                        */
  int32_t gelu;      /* GPTS_GELU_TANH or GPTS_GELU_ERF                      */
  float   ln_eps;    /* LayerNorm epsilon (inside the square root)           */
  int32_t recompute; /* Activation recomputation (sections 4.1, 5.2: the backward phase
                        "involves ... activation recomputation"; the traversal choice is tied
                        to activation memory).  Identical results at every level.
                        0: the stash holds every tensor the backward phase reads.
                        1: the two LayerNorm outputs and the GeLU output are not stashed; the
                           backward phase rebuilds them from the stashed x, x1 and u.  One third
                           less stash, about 2 % more time per step.
                        2: the stash keeps only each layer's input x; the backward phase runs
                           the layer's forward again (up to the GeLU) into its workspace before
                           the layer's backward.  One ninth of the stash at hidden = width,
                           ffn = 4 hidden; one more forward minus the last product per layer.
                           The split backward (bwd_data_only / wgrad_flush) is not available
                           at this level: it would need the activations a second time.     */
  int32_t fwd_fp16;  /* bf16 stages only.  0: forward activations are bf16.  1: the forward
                        phase keeps the activations that branch off the residual stream
                        (both LayerNorm outputs, qkv, the attention probabilities and
                        output, u, g) in fp16 -- 11 significand bits instead of 8 at the
                        same size -- and runs its products on the matrix cores' f16
                        instructions against fp16 images of the weights, still with fp32
                        accumulation; x, y, weights, gradients and every backward product
                        stay bf16 (gradients need bf16's range), the backward phase reading
                        bf16 copies of the stashed fp16 tensors and rebuilding the
                        LayerNorm and GeLU outputs as with `recompute`.  For stages whose
                        attention logits are large enough that bf16 rounding of the forward
                        activations, amplified by the softmax, shows in the gradients.
                        Needs p->prepared (built by gpt_stage_prepare() with the SAME cfg: the
                        forward images then hold fp16) and hidden, attention width and ffn
                        multiples of 128.  Forward activations are bounded
                        by LayerNorm and the softmax; values beyond fp16's range saturate. */
} gpt_stage_cfg;

typedef struct {
  gpt_stage_cfg cfg;
  const void* weights;   /* device; gpt_stage_param_bytes(); layout from
                            gpt_stage_param_offset(); read-only              */
  void*       workspace; /* device scratch of gpt_stage_workspace_bytes();
                            contents undefined between calls; two calls that
                            may overlap in time must not share it            */
  const void* prepared;  /* NULL, or device buffer filled by gpt_stage_prepare() for the
                            CURRENT contents of `weights` and THIS cfg (bf16 stages): the weight
                            matrices re-laid-out as tiled images the forward matrix products
                            copy with fully contiguous transfers (fp16 images with
                            cfg.fwd_fp16).  Same results bit for bit, faster forward
                            products.  Must be rebuilt whenever the weights change.        */
  void*       trace;     /* NULL, or a tracer from gpt_stage_trace_create(): every
                            operator of the call is then bracketed by a pair of
                            hipEvents on the stream (see "operator tracer")    */
} gpt_stage_params;

/* ---- host-side queries (no GPU needed) ---------------------------------- */

/* GPTS_OK if the kernels support cfg: L,B,S >= 1; head_dim in {32,64,128};
 * H, P, F multiples of 8; H <= 16384; dtype/gelu valid.  bf16 additionally
 * needs T = B*S, H, P, F multiples of 64 (MFMA tile granularity); fwd_fp16 see cfg. */
int gpt_stage_validate(const gpt_stage_cfg* cfg);

size_t gpt_stage_param_count(const gpt_stage_cfg* cfg);  /* elements, all layers */
size_t gpt_stage_param_bytes(const gpt_stage_cfg* cfg);  /* weights buffer (cfg.dtype elements) */
size_t gpt_stage_grad_bytes(const gpt_stage_cfg* cfg);   /* dparams buffer (fp32 elements, same order) */
size_t gpt_stage_stash_bytes(const gpt_stage_cfg* cfg);  /* ONE micro-batch's activation stash */
size_t gpt_stage_workspace_bytes(const gpt_stage_cfg* cfg, int phase); /* 0 = forward, 1 = backward */

/* Element offset and element count of tensor `tensor_id` of `layer` inside the
 * parameter buffer (identical for the gradient buffer).  Offsets are multiples
 * of 8 elements. */
int gpt_stage_param_offset(const gpt_stage_cfg* cfg, int layer, int tensor_id,
                           size_t* elem_off, size_t* n_elem);

/* Model FLOPs of one forward+backward of one micro-batch: 3 x forward, forward =
 * 2*T*(3PH + PH + 2HF) for the four linears + attention 4*B*a*d*S*(S+1)/2
 * (causal_aware != 0) or 4*B*a*d*S*S (dense convention).  Recomputation is
 * never counted. */
double gpt_stage_model_flops(const gpt_stage_cfg* cfg, int causal_aware);

/* Text for a status: the detailed message of the calling thread's last failed call when
 * `code` is the status that call returned, otherwise the generic meaning of `code`
 * ("unknown status" for values that are not a gpts_status).  The pointer stays valid until
 * the thread's next failing call. */
const char* gpt_stage_strerror(int code);

/* Prepared weights (optional, bf16 stages; required with cfg.fwd_fp16).  gpt_stage_prepare()
 * enqueues kernels that read p->weights and write `prepared` (device,
 * gpt_stage_prepared_bytes(): about the weight bytes -- one image per weight matrix, for the
 * forward products; the data gradients read the raw weights at the same speed).  Rebuilding
 * costs a read and a write of the weights, and pays once a few micro-batches share the images:
 * call it once per weight update (e.g. once per optimizer step), then pass the buffer as
 * p->prepared.  p->prepared is ignored here. */
size_t gpt_stage_prepared_bytes(const gpt_stage_cfg* cfg);   /* 0 for fp32 stages */
int gpt_stage_prepare(const gpt_stage_params* p, void* prepared, void* stream);

/* ---- the stage calls ----------------------------------------------------- */

/* Forward phase (section 4.1 "forward phase"; section 5.2 one task).
 *   x         device, [B,S,H] cfg.dtype, read-only, must not alias y
 *   act_stash device, gpt_stage_stash_bytes(); written; opaque; one per
 *             in-flight micro-batch; stays valid until its backward has run
 *   y         device, [B,S,H] cfg.dtype, written
 * Needs p->workspace of workspace_bytes(cfg, 0) (may be NULL when that is 0); it uses
 * the first workspace_bytes(cfg, 0) bytes.  Concurrent forward calls must not share
 * a workspace. */
int gpt_stage_fwd(const gpt_stage_params* p, const void* x, void* act_stash,
                  void* y, void* stream);

/* Backward phase (section 4.1 "gradient computation").
 *   act_stash device, as written by the forward of the same micro-batch; not modified
 *   dy        device, [B,S,H] cfg.dtype, read-only
 *   dx        device, [B,S,H] cfg.dtype, written; may alias dy
 *   dparams   device, fp32, gpt_stage_grad_bytes(); ACCUMULATED into (+=): the
 *             caller zeroes it before the first micro-batch
 * Needs p->workspace of workspace_bytes(cfg, 1), which includes workspace_bytes(cfg, 0)
 * at its start: the backward phase only touches the bytes after those, so ONE forward and
 * ONE backward call may run concurrently (different streams) on the same workspace.
 * Concurrent backward calls must not share dparams or workspace. */
int gpt_stage_bwd(const gpt_stage_params* p, const void* act_stash, const void* dy,
                  void* dx, void* dparams, void* stream);

/* Decoupled entry points (MegaFBD section 4.1 "instance-level decoupled
 * scheduling": the two phases run as separate instances and meet only at the
 * stash).  Same mathematics as the two calls above plus event plumbing so a
 * forward stream and a backward stream never need a host synchronisation:
 *   done_event  hipEvent_t or NULL; recorded on `stream` after the last kernel
 *   wait_event  hipEvent_t or NULL; `stream` waits on it before the first kernel */
int gpt_stage_fwd_only(const gpt_stage_params* p, const void* x, void* act_stash,
                       void* y, void* stream, void* done_event);
int gpt_stage_bwd_only(const gpt_stage_params* p, const void* act_stash, const void* dy,
                       void* dx, void* dparams, void* stream, void* wait_event);

/* Backward phase split into a data phase and a weight phase (section 5.2: with a breadth-first
 * traversal a chunk's weight gradients are only needed once ALL its micro-batches have been
 * through it, which is when its gradient exchange starts).
 *
 * gpt_stage_bwd_data_only: gpt_stage_bwd_only without the weight-gradient products.  Writes dx,
 * adds the bias and LayerNorm parameter gradients to dparams (exactly as gpt_stage_bwd does),
 * and leaves in grad_stash (device, gpt_stage_grad_stash_bytes(), one per in-flight
 * micro-batch, written, opaque) the output gradients of every linear layer.  The activation
 * stash must stay alive until the weight phase has run.
 *
 * gpt_stage_wgrad_flush: the weight phase for n micro-batches at once: for every linear layer
 * dW += sum_m (output gradient of micro-batch m)^T (its input activation), added to dparams.
 * act_stashes / grad_stashes are HOST arrays of n device pointers.  When the n buffers of each
 * kind are equally spaced in memory (e.g. slices of one allocation), the stash holds the
 * activations (no recompute, no fwd_fp16) and the shape suits the 256x256 tiles, each linear
 * is ONE product contracting over all micro-batches' tokens: the fp32 gradient matrix is read
 * and written once instead of n times.  Otherwise it is one accumulating product per
 * micro-batch, as in gpt_stage_bwd.  Same mathematics either way; the fp32 summation order
 * over tokens differs from n separate calls of gpt_stage_bwd.  Needs p->workspace of
 * workspace_bytes(cfg, 1).  Deterministic. */
size_t gpt_stage_grad_stash_bytes(const gpt_stage_cfg* cfg);
int gpt_stage_bwd_data_only(const gpt_stage_params* p, const void* act_stash, const void* dy,
                            void* dx, void* dparams, void* grad_stash, void* stream,
                            void* wait_event);
int gpt_stage_wgrad_flush(const gpt_stage_params* p, int n_microbatches,
                          const void* const* act_stashes, const void* const* grad_stashes,
                          void* dparams, void* stream);

/* Coupled convenience: forward then backward of one micro-batch on one stream.
 * p->workspace must hold max(workspace_bytes(cfg,0), workspace_bytes(cfg,1)). */
int gpt_stage_fwd_bwd(const gpt_stage_params* p, const void* x, const void* dy,
                      void* act_stash, void* y, void* dx, void* dparams, void* stream);

/* ---- operator tracer -------------------------------------------------------
 * The paper's tracer (section 3.2, MegaScan data collection) records a start and an
 * end event on the stream around each operator and reads the elapsed time later, off
 * the critical path, together with the operator's arguments.  Same scheme here with
 * hipEvents: a traced call only records events; gpt_stage_trace_collect() waits for
 * them and returns one record per operator.  A tracer is a host object owning
 * 2*capacity events; it is not thread-safe and must not be shared by calls that
 * run concurrently on the host.  Records beyond capacity are dropped and counted. */
enum {
  GPTS_TR_LN_FWD = 0, GPTS_TR_GEMM_FWD, GPTS_TR_ATTN_FWD, GPTS_TR_GEMM_DGRAD, GPTS_TR_GEMM_WGRAD,
  GPTS_TR_BIAS_GRAD, GPTS_TR_LN_BWD, GPTS_TR_ATTN_BWD, GPTS_TR_RECOMPUTE, GPTS_TR_CONVERT, GPTS_TR_N_OPS
};
typedef struct {
  int32_t op;       /* GPTS_TR_*                                                     */
  int32_t sub;      /* which linear: 0 qkv, 1 out-proj, 2 fc1, 3 fc2; LayerNorm 0/1   */
  int32_t layer;
  int32_t phase;    /* 0 forward, 1 backward                                         */
  float   start_ms; /* start, relative to the first record of the tracer             */
  float   dur_ms;   /* end - start                                                   */
  double  flops;    /* algorithmic flops of the operator (0 for memory-bound ones)   */
  double  bytes;    /* algorithmic HBM bytes: operands read once, results written once */
} gpt_stage_trace_rec;
int gpt_stage_trace_create(int capacity, void** trace);
int gpt_stage_trace_destroy(void* trace);
int gpt_stage_trace_reset(void* trace);   /* forget all records, keep the events */
/* Waits for the recorded events (host-blocking) and copies up to max_records records in
 * launch order; *n_dropped (may be NULL) = records lost to capacity or to max_records. */
int gpt_stage_trace_collect(void* trace, gpt_stage_trace_rec* out, int max_records,
                            int* n_records, int* n_dropped);
const char* gpt_stage_trace_op_name(int op);

/* ---- single operations (the kernels the stage is built from) -------------
 * Exposed so each kernel can be checked and timed on its own.  `dtype` is
 * GPTS_FP32 or GPTS_BF16 as in cfg; all pointers device. */

/* out[t,:] = (x[t,:]-mu_t) * rstd_t * gamma + beta ; mean/rstd fp32 [T] written.
 * x_f32 != 0: x is fp32 although dtype is bf16 (inside a bf16 stage the residual
 * stream -- the tensor LayerNorm reads -- is carried in fp32; everything else is bf16). */
int gpt_stage_op_layernorm_fwd(int dtype, int x_f32, int T, int H, float eps, const void* x,
                               const void* gamma, const void* beta, void* out,
                               float* mean, float* rstd, void* stream);

/* dx = dres + LN-backward(dout) ; dgamma += sum_t dout*xhat ; dbeta += sum_t dout.
 * dres may be NULL (treated as 0).  dxsum may be NULL; otherwise fp32 [H] and
 * dxsum += sum_t dx[t,:] (dx as stored in `dtype`): dx is the gradient of the output of
 * the linear layer that feeds the residual stream, so this is that layer's bias gradient,
 * obtained without another pass over dx.  partial: fp32 scratch of
 * gpt_stage_op_layernorm_bwd_scratch_bytes(T,H). */
size_t gpt_stage_op_layernorm_bwd_scratch_bytes(int T, int H);
int gpt_stage_op_layernorm_bwd(int dtype, int x_f32, int T, int H, const void* dout, const void* x,
                               const float* mean, const float* rstd, const void* gamma,
                               const void* dres, void* dx, float* dgamma, float* dbeta,
                               float* dxsum, float* partial, void* stream);

/* Matrix products of the three forms the stage uses; fp32 accumulation.
 *   form 0 (NT, forward):  C[M,N]  = A[M,K] B[N,K]^T (+ bias[N]) (+ residual[M,N])
 *                          gelu != 0: also writes C2 = gelu(C) (C keeps the pre-activation)
 *   form 1 (NN, dgrad):    C[M,N]  = A[M,K] B[K,N] ; dgelu_u != NULL: C *= gelu'(dgelu_u[M,N])
 *   form 2 (TN, wgrad):    Cf[M,N] += A[K,M]^T B[K,N]   (Cf fp32, accumulated into)
 * A, B, C, C2, residual, dgelu_u are `dtype`; bias is `dtype`; gelu_kind as cfg.gelu.
 * f32_flags (bf16, form 0 with a residual only): bit 0 = residual is fp32, bit 1 = C is
 * written as fp32 (needs bit 0): the epilogues that extend the fp32 residual stream. */
int gpt_stage_op_gemm(int dtype, int form, int M, int N, int K, const void* A, const void* B,
                      void* C, const void* bias, const void* residual, void* C2,
                      const void* dgelu_u, int gelu_kind, int f32_flags, void* stream);

/* colsum[n] += sum_m A[m,n]   (bias gradients); A `dtype`, colsum fp32;
 * partial: fp32 scratch of gpt_stage_op_colsum_scratch_bytes(M,N). */
size_t gpt_stage_op_colsum_scratch_bytes(int M, int N);
int gpt_stage_op_colsum(int dtype, int M, int N, const void* A, float* colsum,
                        float* partial, void* stream);

/* The same column sums for callers that cannot allocate device memory or pass a scratch
 * buffer: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The partial sums go to a fixed 4 MiB array the library holds on each GPU it runs on (until
 * the process ends); the call allocates and frees nothing.  Same kernels, same summation
 * order, same bits as gpt_stage_op_colsum.  N <= 16384, otherwise GPTS_ESHAPE and nothing is
 * launched.  All calls on one GPU share that array: calls that may overlap in time (different
 * streams) race on it and must be serialised by the caller.  The array is addressed on the
 * device that is current when the call is made, which must be the device of `stream`. */
int gpt_stage_op_colsum_noalloc(int dtype, int M, int N, const void* A, float* colsum,
                                void* stream);

/* Causal attention.  qkv [B,S,3P] ([Q|K|V], P = n_heads*head_dim); out [B,S,P];
 * lse fp32 [B,n_heads,S] = log sum_j exp(s_ij) of each causal row.
 * scratch: device memory of gpt_stage_op_attention_scratch_bytes(.., phase) bytes,
 * 256-byte aligned, phase 0 for the forward and 1 for the backward call (may be NULL
 * where that size is 0); contents are not kept between calls.  The size query returns
 * 0 for arguments the calls would reject. */
size_t gpt_stage_op_attention_scratch_bytes(int dtype, int B, int S, int n_heads, int head_dim,
                                            int phase);
int gpt_stage_op_attention_fwd(int dtype, int B, int S, int n_heads, int head_dim,
                               const void* qkv, void* out, float* lse, void* scratch,
                               void* stream);
/* dqkv [B,S,3P] written. */
int gpt_stage_op_attention_bwd(int dtype, int B, int S, int n_heads, int head_dim,
                               const void* qkv, const void* out, const float* lse,
                               const void* dout, void* dqkv, void* scratch, void* stream);

/* ---- traversal of the (micro-batch, model chunk) task matrix ---------------------------
 * Section 5.2 (MegaDPP, "parallel scheduler"): the compute tasks of one iteration form a
 * matrix indexed by (model chunk, micro-batch) and a schedule is a traversal order of it.
 * Here the chunks are stages that sit on one GPU one after the other (chunk j+1 consumes the
 * output of chunk j); every forward task F(i,j) = micro-batch i on chunk j has a backward
 * task B(i,j).  Dependencies: F(i,j) after F(i,j-1); B(i,j) after F(i,j) and B(i,j+1).
 *   GPT_DPP_DFC  depth first: the same micro-batch through all chunks, forward then
 *                backward, before the next micro-batch (earliest backward, smallest stash)
 *   GPT_DPP_BFC  breadth first: all micro-batches on the same chunk before the next chunk;
 *                a chunk's gradients are complete as early as possible, the stash is largest
 *   GPT_DPP_BFC_BEST_EFFORT  breadth first over windows of W consecutive micro-batches, W the
 *                largest number whose stash fits: W = clamp(max_live_stash / n_chunks, 1, M)
 *                (section 5.2: breadth first "as long as it does not cause" out-of-memory)
 * A window of W micro-batches runs F(i,0) for its i, then F(i,1), ..., then B(i,C-1) for its
 * i, ..., B(i,0); DFC is W = 1, BFC is W = M.  Inside a chunk micro-batches always run in
 * ascending order, so gradient accumulation order -- and every result bit -- is the same for
 * all three policies. */
enum { GPT_DPP_DFC = 0, GPT_DPP_BFC = 1, GPT_DPP_BFC_BEST_EFFORT = 2 };
enum { GPT_DPP_FWD = 0, GPT_DPP_BWD = 1 };
typedef struct {
  int32_t phase;      /* GPT_DPP_FWD or GPT_DPP_BWD */
  int32_t microbatch; /* i */
  int32_t chunk;      /* j */
} gpt_dpp_task;

/* Host only.  Writes the 2*n_chunks*n_microbatches tasks in execution order into tasks
 * (capacity entries; GPTS_ENOMEM if too few).  max_live_stash: for BEST_EFFORT the number of
 * (micro-batch, chunk) activation stashes that may be alive at once (ignored otherwise; values
 * below n_chunks still schedule one micro-batch at a time).  peak_live_stash (may be NULL)
 * receives the largest number of stashes alive at once under the order written.
 * Returns the number of tasks, or a negative gpts_status. */
int gpt_dpp_plan(int policy, int n_chunks, int n_microbatches, int max_live_stash,
                 gpt_dpp_task* tasks, int capacity, int* peak_live_stash);

typedef struct {
  int32_t n_chunks, n_microbatches, policy;
  int32_t max_live_stash;         /* BEST_EFFORT: stashes that may be alive at once; <= 0: as many
                                     as stash_pool holds (the memory at hand decides)          */
  const gpt_stage_params* chunks; /* host array [n_chunks]; all chunks share batch, seq,
                                     hidden and dtype; workspaces may be shared (one stream) */
  const void* const* x;           /* host array [M] of device pointers: inputs of chunk 0   */
  const void* const* dy;          /* [M]: gradients w.r.t. the last chunk's outputs         */
  void* const* y;                 /* [M]: outputs of the last chunk, written                */
  void* const* dx;                /* [M]: gradients w.r.t. x, written                       */
  void* const* dparams;           /* [n_chunks]: fp32 gradient buffer of each chunk (+=)    */
  void* stash_pool;               /* device; slots of gpt_dpp_stash_slot_bytes() each       */
  size_t stash_pool_bytes;
  void* act_pool;                 /* device; chunk-boundary activations and gradients,
                                     slots of gpt_dpp_act_slot_bytes() each                 */
  size_t act_pool_bytes;
  void* const* grad_ready;        /* NULL, or [n_chunks] hipEvent_t: event j is recorded when
                                     the last backward task of chunk j (and, with grad_pool,
                                     its last weight phase) has been enqueued              */
  void* grad_pool;                /* NULL: every backward task is a whole gpt_stage_bwd_only.
                                     Otherwise (gpt_dpp_run only) device memory for W slots of
                                     gpt_dpp_grad_slot_bytes(), W the window of the policy:
                                     backward tasks run the data phase only and, as soon as a
                                     chunk has seen the backward tasks of all micro-batches of
                                     a window, ONE weight phase (gpt_stage_wgrad_flush) adds
                                     the chunk's weight gradients over those micro-batches --
                                     what breadth first buys on top of the early gradient
                                     exchange: the wider the window, the fewer passes over the
                                     fp32 gradient matrices.  The stash pool must then hold
                                     n_chunks * W slots (handed out in a fixed, equally spaced
                                     pattern, which the one-launch weight phase needs); a
                                     stash is released after its chunk's weight phase.      */
  size_t grad_pool_bytes;
} gpt_dpp_job;

typedef struct {
  int32_t n_tasks;
  int32_t peak_live_stash;   /* stashes alive at once                  */
  int32_t peak_live_act;     /* boundary buffers alive at once         */
  size_t  stash_slot_bytes;
  size_t  act_slot_bytes;
} gpt_dpp_report;

size_t gpt_dpp_stash_slot_bytes(const gpt_stage_params* chunks, int n_chunks); /* 0 on bad input */
size_t gpt_dpp_grad_slot_bytes(const gpt_stage_params* chunks, int n_chunks);  /* 0 on bad input */
size_t gpt_dpp_act_slot_bytes(const gpt_stage_cfg* cfg);                        /* 0 on bad input */

/* The best-effort allowance from the memory that is free right now on the current device
 * (section 5.2: breadth first "as long as it does not cause" out-of-memory): how many
 * (micro-batch, chunk) activation stashes can be alive at once if the stash pool takes what
 * hipMemGetInfo reports free, minus reserve_bytes (whatever else the caller still has to
 * allocate) and minus the boundary-buffer pool.  Rounded down to whole windows (a multiple of
 * n_chunks), at most n_chunks*n_microbatches, 0 if not even one micro-batch fits.  Writes the
 * pool sizes to allocate for it (either pointer may be NULL).  Returns the allowance or a
 * negative gpts_status.  Allocates nothing. */
int gpt_dpp_allowance_from_free_memory(const gpt_stage_params* chunks, int n_chunks,
                                       int n_microbatches, size_t reserve_bytes,
                                       size_t* stash_pool_bytes, size_t* act_pool_bytes);

/* Enqueues every task of the job on `stream` in the order gpt_dpp_plan gives, through the
 * decoupled entry points; stash slots and boundary buffers are taken from the two pools and
 * returned as soon as their consumer has been enqueued (one stream: in-order execution makes
 * that safe).  GPTS_ENOMEM if a pool is too small for the policy -- nothing has been enqueued
 * then.  report may be NULL.  Asynchronous like every other call. */
int gpt_dpp_run(const gpt_dpp_job* job, void* stream, gpt_dpp_report* report);

/* ---- communication coordinator, simulated on the host ------------------------------------
 * Section 4.2 (MegaFBD, "communication coordinator"): training threads (virtual ranks) of one
 * GPU share a control thread; a collective starts only after every rank of its group has
 * posted the same request.  Per control thread a table holds one bit vector per communication
 * group, one bit per virtual rank (flattened to one array).  Steps: registration (a rank sets
 * its bit in the vector of the group it wants to communicate in), alignment (bitwise-OR
 * all-reduce of the tables), readiness check (vector == the group's expected mask), ordered
 * execution (ready groups in ascending group order; their vectors are cleared).
 * Everything here runs on the host and moves no data: it models the protocol only.
 *   group g has members group_members[group_start[g] .. group_start[g+1]-1]
 *   control_of_rank[r] = control thread (GPU) that virtual rank r lives on */
int gpt_fbd_coord_create(int n_ranks, int n_groups, const int32_t* group_start,
                         const int32_t* group_members, int n_control,
                         const int32_t* control_of_rank, void** coord);
int gpt_fbd_coord_destroy(void* coord);
/* bits: n_ranks + 1 chars; bits[r] = '1' if rank r is in the group (rank 0 leftmost, as in the
 * paper's example: eight threads, group {0,1,2,3} -> "11110000") */
int gpt_fbd_coord_expected(void* coord, int group, char* bits);
int gpt_fbd_coord_register(void* coord, int rank, int group);            /* step 1 */
int gpt_fbd_coord_align(void* coord);                                    /* step 2 */
/* step 3, as seen by one control thread: ready groups in ascending order; returns the count */
int gpt_fbd_coord_ready(void* coord, int control, int32_t* groups, int capacity);
/* step 4: all control threads run the ready collectives in ascending group order (the tables
 * must be aligned); their vectors are cleared; returns the count, groups[] the order */
int gpt_fbd_coord_execute(void* coord, int32_t* groups, int capacity);
/* Runs whole rank programs: rank r performs collectives in groups prog[prog_start[r] ..
 * prog_start[r+1]-1], in that order, posting the next request only when the previous
 * collective is done.  verify = 1: the coordinator protocol above, in rounds (every idle rank
 * registers, align, execute).  verify = 0: no verification -- a control thread starts the
 * oldest request it holds and is busy until that collective completes (the situation the
 * section describes as deadlock-prone).  log receives the executed groups in order;
 * *deadlocked = 1 when requests remain and nothing can proceed. */
int gpt_fbd_coord_simulate(void* coord, const int32_t* prog_start, const int32_t* prog, int verify,
                           int32_t* log, int log_capacity, int32_t* n_executed,
                           int32_t* deadlocked);

/* ---- run-time scheduling of the task matrix: the ready set ----------------------------------
 * Section 5.2: with asynchronous transfers "a compute thread can always pick the highest-priority
 * ready input for execution", and the scheduler is to be "resource-aware".  A task is READY when
 * the tasks it depends on have been issued and its external input has arrived: x of micro-batch i
 * for F(i,0), dy of micro-batch i for B(i,C-1).  Its priority is its position in the static plan
 * of the policy (gpt_dpp_plan), so with every input present from the start the order IS that
 * plan.  Two rules keep results and memory those of the plan: backward tasks of one chunk go in
 * ascending micro-batch order (the order the chunk's gradients accumulate in, hence every result
 * bit), and a micro-batch is only started while the free stash slots, after setting aside what
 * the micro-batches in flight still need, cover all its chunks -- twice that when it would start
 * ahead of a lower-numbered one, which must still be able to pass through (a started
 * micro-batch can always finish; the width follows the memory at hand).
 *
 * gpt_dpp_simulate_ready (host only, discrete time, one task per step): x_at[i] / dy_at[i] = the
 * step from which the input / output gradient of micro-batch i is present (NULL: all from step 0).
 * dynamic = 0: the static plan, idling whenever its next task's input is missing; dynamic = 1:
 * the first ready task of the plan.  order receives the tasks in order of issue; *n_steps the
 * steps used, *idle_steps those without a task (either may be NULL).  Returns the number of
 * tasks or a negative gpts_status.
 *
 * gpt_dpp_run_ready: the same scheduler driving the GPU.  x_ready[i] / dy_ready[i] are hipEvent_t
 * (NULL array or NULL entry: present from the start) that whoever delivers the data records on
 * its own stream; they are polled with hipEventQuery.  Tasks are issued on `stream` as in
 * gpt_dpp_run.  Unlike every other call this one BLOCKS the calling host thread until all tasks
 * have been issued, waiting (yielding) while nothing is ready, and gives up with GPTS_EHIP after
 * timeout_seconds without progress -- tasks issued until then have been enqueued.  The stash
 * pool needs at least one slot per chunk, the boundary pool min(micro-batches, stash slots) + 1
 * buffers.  order_out (may be NULL) receives the order of issue. */
int gpt_dpp_simulate_ready(int policy, int n_chunks, int n_microbatches, int max_live_stash,
                           const int32_t* x_at, const int32_t* dy_at, int dynamic,
                           gpt_dpp_task* order, int capacity, int32_t* n_steps, int32_t* idle_steps);
int gpt_dpp_run_ready(const gpt_dpp_job* job, const void* const* x_ready, const void* const* dy_ready,
                      double timeout_seconds, void* stream, gpt_dpp_task* order_out, int capacity,
                      gpt_dpp_report* report);

#ifdef __cplusplus
}
#endif
#endif /* GPT_STAGE_H_ */
