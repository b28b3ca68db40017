/*
 * tbp.h - C ABI of the two-stage-backpropagation (2BP) stage library for AMD MI355X (gfx950).
 *
 * One object, a "stage", is one pipeline stage of a LLaMa-like decoder stack (RMSNorm, rotary
 * embedding, causal attention, SwiGLU MLP, no linear bias: the paper's Transformer-7b, Section 3.2).
 * Its backward pass is split as the paper's Section 3.1 defines:
 *   backward-p1  gradient w.r.t. the output of the preceding layer (input gradients), per micro-batch;
 *   backward-p2  gradient w.r.t. the layer parameters, deferred, computed later from what p1 left behind.
 *
 * General rules for every entry point
 *   - Plain C.  No exceptions cross the boundary.  Every function returns a tbp_status; on failure
 *     tbp_last_error() gives a human-readable reason (thread-local, valid until the next call).
 *   - "device" pointers are HIP device addresses valid on the current device; "host" pointers are
 *     ordinary process memory.  The library never allocates or frees device memory: weights,
 *     gradients, the stash arena, inputs, outputs and the stream all belong to the caller and must
 *     outlive the calls (and, for the arena / weights / gradients, the stage) that use them.
 *   - All device work is enqueued on the hipStream_t passed as `void* stream` (NULL = the null
 *     stream) and the call returns without synchronising.  Device-side failures detectable at
 *     launch time are reported as TBP_EDEVICE.
 *   - What a call enqueues is kernels and device-to-device copies only (no allocation, no memset, no
 *     synchronisation, no host callback), and nothing on the device depends on an earlier call except
 *     through the buffers themselves: the calls can be recorded into a HIP graph with stream capture
 *     and replayed.  A stage's per-micro-batch state advances when a call is recorded, not when the
 *     graph runs, so record sequences that a replay may repeat as they are (a whole step returns every
 *     micro-batch to EMPTY).
 *   - Argument errors are detected on the host before anything is launched (TBP_EINVAL /
 *     TBP_ESTATE / TBP_ENOMEM): such a call launches nothing and changes no state.  A launch that HIP
 *     refuses in the middle of a call (TBP_EDEVICE) is different: the kernels enqueued before it still
 *     run, the micro-batch's state does not advance, and what the call was writing (its stash rows,
 *     workspace, outputs) is undefined; reset the stage (tbp_stage_reset) or repeat the call.
 *   - Streams.  A stage has ONE workspace (temporaries of a call, the rotation table, scratch of split
 *     products) and recycles activation slots and stash rows on the host when a call is enqueued.  Forward
 *     and backward-p1 calls of a stage must therefore be ordered with respect to each other on the device
 *     (same stream, or events), and so must any two calls that touch the same micro-batch index or
 *     activation slot.  backward-p2 shares no workspace with them: a p2 call may run on another stream concurrently
 *     with forward / p1 calls of OTHER micro-batches, provided it is ordered after the p1 calls of its own
 *     set and before any forward that reuses those micro-batch indices; two p2 calls must not overlap each other.
 *   - Layouts: activations and gradients are token-major, row-major [tokens, width] with
 *     tokens = micro_batch * seq and sequence b in rows b*seq .. (b+1)*seq-1.  Weights are
 *     row-major [in, out] so that Y = X W, dX = dY W^T, dW = X^T dY.  q/k/v projections are one
 *     fused matrix [d_model, 3*d_model] (column blocks q, k, v); gate/up are fused [d_model, 2*d_ffn]
 *     (column blocks gate, up).  Head h owns columns h*head_dim .. (h+1)*head_dim-1.
 *   - Storage type: TBP_BF16 (bfloat16 storage, fp32 accumulation, MFMA matrix cores) or TBP_F32
 *     (fp32 everywhere).  Parameter gradients are always fp32.
 *   - Size limits (TBP_EINVAL otherwise): bf16 needs d_model, d_ffn, head_dim and seq to be multiples
 *     of 8; d_model <= 8192 (bf16) or 4096 (f32); seq <= 4096; head_dim even.
 */
#ifndef TBP_H
#define TBP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tbp_stage tbp_stage; /* opaque; host-side bookkeeping only */

typedef enum {
  TBP_OK = 0,
  TBP_EINVAL = 1,  /* bad argument (null pointer, size outside the limits, bad micro-batch set) */
  TBP_ESTATE = 2,  /* call order violates the per-micro-batch state machine */
  TBP_ENOMEM = 3,  /* arena too small, or no free activation slot */
  TBP_EDEVICE = 4  /* HIP reported an error at launch */
} tbp_status;

typedef enum { TBP_F32 = 0, TBP_BF16 = 1 } tbp_dtype;

/* How backward-p2 walks a set of micro-batches (Section 3.2, Figure 2; Section 4.4, Table 3):
 *   LOOP     one weight-gradient product per micro-batch, accumulated in fp32;
 *   KCONCAT  the micro-batches are treated as one batch concatenated over the batch dimension,
 *            i.e. one product whose contraction length is n_mbs * tokens.  The stash keeps each
 *            tensor's micro-batches in consecutive rows of one slab, so no copy is made; the set
 *            must therefore be ascending consecutive indices (TBP_EINVAL otherwise). */
typedef enum { TBP_P2_LOOP = 0, TBP_P2_KCONCAT = 1 } tbp_p2_mode;

/* Attention is a functional operation: no backward-p2, everything it keeps is released in backward-p1 (Section 4.2).
 *   MATERIALISED  scores -> softmax -> P v as separate products; the probabilities P [batch, heads, seq, seq] are
 *                 stashed from forward to p1 (any dtype, any head_dim);
 *   FUSED         one forward kernel and one backward kernel that never write scores or probabilities: only the
 *                 row log-sum-exp [batch, heads, seq] is stashed and p1 rebuilds the probabilities from it
 *                 (bf16 storage, head_dim 64 or 128; TBP_EINVAL otherwise);
 *   FUSED_RECOMPUTE  FUSED, with a backward whose dq comes from a second pass over the keys that rebuilds the scores
 *                 and dP instead of from a product with dS^T written out by the first pass: three more products
 *                 per tile, no dS^T workspace (batch * heads * seq^2 storage-type elements less per stage), the same
 *                 speed within 1 % at the benchmark shapes; same availability rule as FUSED;
 *   AUTO          FUSED where it is available, MATERIALISED elsewhere. */
typedef enum { TBP_ATTN_AUTO = 0, TBP_ATTN_MATERIALISED = 1, TBP_ATTN_FUSED = 2, TBP_ATTN_FUSED_RECOMPUTE = 3 } tbp_attention;

/* Where the gradient of an RMSNorm gain, dg = sum over tokens of dy * x * rsqrt(mean(x^2) + eps), is computed.  A gain
 * is a parameter, so by Section 3.1 its gradient is backward-p2 work; the two settings give the same result:
 *   PARTIALS  p1, which has x and dy in registers anyway, leaves the gain gradient of each norm and micro-batch in the
 *             stash as at most 256 fp32 partial rows [d_model] (one per workgroup of its row kernel) and p2 adds up
 *             the partial rows of its set (no activation is kept for the norms past p1);
 *   LITERAL   p1 computes nothing for the gains; each norm's input x and output derivative dy are stashed until p2
 *             like a linear layer's operands (4 more [tokens, d_model] tensors per layer and micro-batch, 2 for an
 *             MLP-only layer) and p2 computes dg from them, over the concatenated rows for KCONCAT. */
typedef enum { TBP_GAIN_PARTIALS = 0, TBP_GAIN_LITERAL = 1 } tbp_gain_grad;

typedef struct {
  int32_t n_layers;
  int32_t d_model;
  int32_t n_heads;          /* 0 => MLP-only blocks: x + Wd(silu(g)*u), [g,u] = RMSNorm(x) Wgu */
  int32_t head_dim;         /* n_heads * head_dim must equal d_model when n_heads > 0 */
  int32_t d_ffn;
  int32_t seq;
  int32_t micro_batch;      /* sequences per micro-batch */
  int32_t max_microbatches; /* micro-batch indices are 0 .. max_microbatches-1 (rows of every slab) */
  int32_t act_slots;        /* micro-batches that may be between forward and p1 at once;
                               0 => max_microbatches.  Sizes the forward->p1 part of the stash. */
  int32_t causal;           /* 1: query i attends to keys j <= i */
  int32_t dtype;            /* tbp_dtype */
  float rms_eps;            /* added to the mean square inside the square root */
  float rope_base;
  int32_t attention;        /* tbp_attention: how the attention of each layer is computed and what it stashes */
  int32_t gain_grad;        /* tbp_gain_grad: which phase computes the RMSNorm gain gradients */
} tbp_config;

/* Per-layer arrays (host arrays of length n_layers holding DEVICE pointers).  The w_* / g* arrays hold
 * tensors of the storage type; the d* arrays hold fp32 gradients of the same shapes.
 * For MLP-only stages the attention entries (w_qkv, w_o, g1 and their gradients) may be NULL. */
typedef struct {
  const void* const* w_qkv; /* [d_model, 3 d_model] */
  const void* const* w_o;   /* [d_model, d_model]   */
  const void* const* g1;    /* [d_model] gain of the pre-attention RMSNorm */
  const void* const* w_gu;  /* [d_model, 2 d_ffn]   */
  const void* const* w_d;   /* [d_ffn, d_model]     */
  const void* const* g2;    /* [d_model] gain of the pre-MLP RMSNorm */
  float* const* dw_qkv;
  float* const* dw_o;
  float* const* dg1;
  float* const* dw_gu;
  float* const* dw_d;
  float* const* dg2;
} tbp_params;

/* Bytes held by the stash (Section 4.2: linear layers keep their input activation and output
 * derivative until p2; functional operations release their activations in p1). */
typedef struct {
  size_t w_stash_bytes;    /* slabs that live until p2: linear-layer inputs and output derivatives */
  size_t a_stash_bytes;    /* slots that live from forward to p1 only */
  size_t workspace_bytes;  /* per-call scratch (never live between calls) */
  size_t arena_bytes;      /* total the caller must provide (sum of the above plus alignment) */
} tbp_stash_sizes;

typedef struct {
  size_t w_live_bytes;     /* bytes of p2 operands currently held */
  size_t a_live_bytes;     /* bytes of forward->p1 activations currently held */
  size_t high_water_bytes; /* maximum of w_live + a_live since creation or the last reset */
} tbp_stash_stats;

/* Size query.  Host pointers.  No device access. */
tbp_status tbp_stash_query(const tbp_config* cfg, tbp_stash_sizes* out);

/* Create a stage over a caller-provided device arena of at least arena_bytes (256-byte aligned).
 * The pointer arrays inside `params` are copied; the tensors they point to are not. */
tbp_status tbp_stage_create(const tbp_config* cfg, const tbp_params* params, void* arena_device,
                            size_t arena_bytes, tbp_stage** out);
void tbp_stage_destroy(tbp_stage* st);

/* Forward of micro-batch mb (state EMPTY -> FWD): x_in [tokens, d_model] -> x_out, both device, storage
 * type.  Fills the stash.  Needs a free activation slot (TBP_ENOMEM otherwise). */
tbp_status tbp_stage_forward(tbp_stage* st, int mb, const void* x_in, void* x_out, void* stream);

/* backward-p1 of micro-batch mb (state FWD -> P1_DONE), Section 3.1: dy = gradient w.r.t. the stage
 * output, dx = gradient w.r.t. the stage input, device, storage type.  Leaves every linear layer's
 * output derivative (and the per-micro-batch RMSNorm gain partials) in the stash and releases the
 * micro-batch's activation slot. */
tbp_status tbp_stage_backward_p1(tbp_stage* st, int mb, const void* dy, void* dx, void* stream);

/* backward-p2 of a set of micro-batches, all in state P1_DONE (-> EMPTY), Sections 3.1 and 3.2:
 * parameter gradients from the stash.  `mbs` is a host array.  accumulate != 0: gradients += result;
 * accumulate == 0: gradients = result (for LOOP the first micro-batch of the set overwrites).
 * Calling p1(mb) then p2({mb}, LOOP) reproduces unsplit backpropagation. */
tbp_status tbp_stage_backward_p2(tbp_stage* st, const int* mbs, int n_mbs, int p2_mode, int accumulate,
                                 void* stream);

tbp_status tbp_stage_stash_stats(const tbp_stage* st, tbp_stash_stats* out);
/* All micro-batches back to EMPTY, all slots free, high-water mark cleared.  Gradients untouched. */
tbp_status tbp_stage_reset(tbp_stage* st);

/* ---- single operations (the kernels the stage is made of), exposed for parity tests and roofline
 * measurement.  All pointers device unless noted; dtype is a tbp_dtype; leading dimensions in elements. */

/* C[M,N] (= or +=) alpha * op(A) op(B) (+ R).  layout: 0 = NN (A [M,K], B [K,N]), 1 = NT (A [M,K],
 * B [N,K]: dX = dY W^T, Section 3.1), 2 = TN (A [K,M], B [K,N]: dW = X^T dY, Section 3.1).
 * out_f32 != 0: C is fp32 (and may accumulate); else C has the storage type and R (optional,
 * same shape and leading dimension as C) is added before rounding.
 * bf16 storage: A, B, C and R must be 16-byte aligned; the contiguous extent of A and of B, N, lda, ldb and
 * ldc must be multiples of 8 (every lane moves 16 bytes) and lda, ldb below 2^22 elements; TBP_EINVAL otherwise.
 * fp32 storage has no such rule.
 * K == 0 writes zeros (or leaves an accumulated C alone); M == 0 or N == 0 does nothing. */
tbp_status tbp_gemm(int dtype, int layout, int M, int N, int K, float alpha, const void* A, int lda,
                    const void* B, int ldb, void* C, int ldc, int out_f32, int accumulate, const void* R,
                    void* stream);
/* The same product with scratch memory.  A bf16 NN or NT product with a storage-type output of fewer than 192 tiles of
 * 256 x 256 cannot fill the chip with one workgroup per tile; given `workspace` (device, 256-byte aligned, at least
 * tbp_gemm_workspace_bytes(...) bytes) the contraction is split over several workgroups per tile whose fp32 partial
 * sums meet in the workspace and are added in a fixed order (the result does not depend on timing).
 * tbp_gemm_workspace_bytes returns 0 for a product that would not be split; workspace may then be NULL.  The call
 * clears the part of the workspace it relies on; calls that share a workspace must not overlap.  The stage gives its
 * forward and backward-p1 linear products such a workspace out of its arena (Section 3.1: dX = dY W^T). */
size_t tbp_gemm_workspace_bytes(int dtype, int layout, int M, int N, int K, int out_f32);
tbp_status tbp_gemm_ws(int dtype, int layout, int M, int N, int K, float alpha, const void* A, int lda,
                       const void* B, int ldb, void* C, int ldc, int out_f32, int accumulate, const void* R,
                       void* workspace, size_t workspace_bytes, void* stream);
tbp_status tbp_rmsnorm_fwd(int dtype, int rows, int d, float eps, const void* x, const void* g, void* y,
                           void* stream);
/* RMSNorm backward, split as Section 3.1 splits every parametrised module.  The backward-p1 half,
 * tbp_rmsnorm_p1_partials: dx = resid + dL/dx (resid may be NULL), and the gain gradient dg = sum over rows of
 * dy * x * rsqrt(mean(x^2) + eps) is left as tbp_rmsnorm_partial_rows(dtype, rows, d) partial rows (at most 256; a
 * function of the three arguments only) in partials_out [partial rows][d] fp32, each the sum over a fixed subset of the
 * rows.  The backward-p2 half, tbp_gain_partials_sum: dg_out [d] fp32 (= or +=) the sum of the first n_rows rows of
 * partials [n_rows][d] (partial rows of several micro-batches stored one after the other are summed in one call).
 * This is how the stage computes the gain gradients with TBP_GAIN_PARTIALS.  rows == 0 writes nothing. */
int tbp_rmsnorm_partial_rows(int dtype, int rows, int d);
tbp_status tbp_rmsnorm_p1_partials(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                                   const void* resid, void* dx, float* partials_out, void* stream);
tbp_status tbp_gain_partials_sum(const float* partials, int n_rows, int d, int accumulate, float* dg_out, void* stream);
/* Both halves in one call: dx as above and dg_out [d] fp32 = the gain gradient (overwritten).
 * scratch: device, >= tbp_rmsnorm_p1_scratch_bytes(d) (receives the partial rows). */
tbp_status tbp_rmsnorm_p1(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                          const void* resid, void* dx, float* dg_out, void* scratch, void* stream);
size_t tbp_rmsnorm_p1_scratch_bytes(int d);
/* tbp_rmsnorm_p1 for callers that cannot allocate device memory or carry a workspace (code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments minus `scratch`, same kernels, same results
 * bit for bit.  The row-block partials of the gain gradient live in an 8 MiB array inside the library's code object
 * (256 rows of at most 8192 fp32 columns), resident on every GPU the library is used on until the process ends; its
 * device address is looked up on the first call on each device (make that first call outside a stream capture).
 * The call allocates and frees nothing.  d above the limit of the storage type (8192 bf16, 4096 f32) is TBP_EINVAL.
 * Nothing in the array needs clearing between calls, but every call on a GPU uses that GPU's one array: calls that may
 * overlap on one GPU (different streams, or threads) race on it and must be ordered by the caller. */
tbp_status tbp_rmsnorm_p1_static(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                                 const void* resid, void* dx, float* dg_out, void* stream);
/* The gain gradient alone, as a backward-p2 operation (Section 3.1): dg_out [d] fp32 (= or +=) sum over rows of
 * dy * x * rsqrt(mean(x^2) + eps).  dy, x [rows, d] device, storage type; scratch as for tbp_rmsnorm_p1. */
tbp_status tbp_rmsnorm_gain_p2(int dtype, int rows, int d, float eps, const void* dy, const void* x, int accumulate,
                               float* dg_out, void* scratch, void* stream);
/* gu [rows, 2f] (gate | up) -> m [rows, f];  p1: dm [rows, f], gu -> dgu [rows, 2f]. */
tbp_status tbp_swiglu_fwd(int dtype, int rows, int f, const void* gu, void* m, void* stream);
tbp_status tbp_swiglu_p1(int dtype, int rows, int f, const void* dm, const void* gu, void* dgu, void* stream);
/* Rotary embedding in place on n_heads heads starting at column 0 of x [rows, ld]; position = row % seq.
 * inverse != 0 rotates by the negated angle (backward-p1).  table: device scratch of
 * tbp_rope_table_bytes(seq, head_dim), filled by tbp_rope_table. */
size_t tbp_rope_table_bytes(int seq, int head_dim);
tbp_status tbp_rope_table(int seq, int head_dim, float base, void* table, void* stream);
tbp_status tbp_rope(int dtype, int rows, int seq, int n_heads, int head_dim, int ld, const void* table,
                    int inverse, void* x, void* stream);
/* Row softmax of n_mat matrices [seq, seq]: scores fp32 -> P (storage type).  causal: columns j > i get
 * probability 0.  p1: dS = P * (dP - rowsum(dP * P)), written over dP. */
tbp_status tbp_softmax_fwd(int dtype, int n_mat, int seq, int causal, const float* scores, void* P, void* stream);
tbp_status tbp_softmax_p1(int dtype, int n_mat, int seq, int causal, const void* P, void* dP_dS, void* stream);

/* Fused scaled-dot-product attention per (sequence, head) (an operation with no backward-p2 and a significant
 * backward-p1, Section 4.1), bf16 storage, head_dim 64 or 128.  qkv: device [batch*seq, ld_qkv], column blocks
 * q | k | v of n_heads*head_dim each (q and k already rotated); out: device [batch*seq, ld_out], heads concatenated;
 * lse: device [batch, n_heads, seq] fp32 = log2 of the row's sum of exp2(score * log2(e) / sqrt(head_dim)), all that
 * backward-p1 needs to rebuild the probabilities.  causal != 0: query i sees keys j <= i.  Pointers 16-byte aligned,
 * leading dimensions multiples of 8, seq * ld_qkv * 2 below 2^32 (one sequence's rows span less than 4 GiB).  Neither
 * scores nor probabilities are written to memory. */
tbp_status tbp_attention_fwd(int dtype, int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv,
                             int ld_qkv, void* out, int ld_out, float* lse, void* stream);

/* Backward-p1 of the fused attention: dq, dk, dv (not yet rotated back) into the q | k | v column blocks of dqkv
 * [batch*seq, ld_dqkv], from qkv, the forward's out and lse, and d_out = derivative of out (out and d_out dense:
 * ld_out == n_heads*head_dim).  The probabilities are rebuilt from lse; dS = P * (dP - rowsum(d_out * out)).
 * scratch: device, 256-byte aligned, >= tbp_attention_p1_scratch_bytes(batch, n_heads, seq) (row sums and dS^T).
 * tbp_attention_p1_recompute is the same operation with dq from a recompute pass (see TBP_ATTN_FUSED_RECOMPUTE): its
 * scratch holds the row sums only, tbp_attention_p1_recompute_scratch_bytes(batch, n_heads, seq) bytes. */
size_t tbp_attention_p1_scratch_bytes(int batch, int n_heads, int seq);
size_t tbp_attention_p1_recompute_scratch_bytes(int batch, int n_heads, int seq);
tbp_status tbp_attention_p1_recompute(int dtype, int batch, int n_heads, int seq, int head_dim, int causal,
                                      const void* qkv, int ld_qkv, const void* out, const void* d_out, int ld_out,
                                      const float* lse, void* dqkv, int ld_dqkv, void* scratch, void* stream);
tbp_status tbp_attention_p1(int dtype, int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv,
                            int ld_qkv, const void* out, const void* d_out, int ld_out, const float* lse, void* dqkv,
                            int ld_dqkv, void* scratch, void* stream);

/* Measurement aid (no paper passage: it prices the hardware, not the method): a register-resident loop of
 * 32x32x16 bf16 MFMAs, blocks x 4 wavefronts x iters x 16 instructions = blocks*iters*2^21 FLOP, touching no memory
 * inside the loop.  What it sustains is the practical ceiling of the matrix pipes under the chip's power management,
 * which depends on the operand values (all-zero operands run about 1.4 times as fast as N(0,1) operands): seed it
 * with data like the workload's.
 * seed: device, 4096 bf16 values (any finite data); sink: device, blocks*256 floats (written once). */
tbp_status tbp_mfma_ceiling(int blocks, int iters, const void* seed, float* sink, void* stream);

const char* tbp_last_error(void);
/* Library version string (static storage). */
const char* tbp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* TBP_H */
