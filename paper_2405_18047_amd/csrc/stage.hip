// Host side of the C ABI: configuration checks, the stash allocator, the per-micro-batch state machine
// and the kernel sequence of forward / backward-p1 / backward-p2 for a LLaMa-like decoder stage.
#include "../../include/tbp.h"
#include "kernels.h"

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

namespace {

thread_local char g_err[512] = "";

tbp_status fail(tbp_status code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

#define TBP_HIP(expr)                                                                        \
  do {                                                                                       \
    hipError_t e__ = (expr);                                                                 \
    if (e__ != hipSuccess) return fail(TBP_EDEVICE, "%s: %s", #expr, hipGetErrorString(e__)); \
  } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- stash layout ------------------------------------------------------------------------------------
// Tensors that backward-p2 consumes ("W" class: inputs and output derivatives of the linear layers) live in
// slabs [max_microbatches * tokens, width]; micro-batch j owns rows j*tokens .. (j+1)*tokens-1, so any run of
// consecutive micro-batches is already the batch-concatenated operand of one weight-gradient product.
// Tensors needed only from forward to backward-p1 ("A" class) live in per-slot buffers handed out by a small
// free list; a slot is taken at forward and returned at the end of backward-p1.
// W_N1X .. W_N2DY exist only with the literal gain-gradient p2: the inputs of the two RMSNorms and the derivatives of
// their outputs, kept until p2 like a linear layer's operands.
enum WTensor { W_H1, W_A, W_H2, W_M, W_N1X, W_N2X, W_DQKV, W_DX1, W_DGU, W_DX2, W_N1DY, W_N2DY, W_COUNT };
enum ATensor { A_X0, A_QKV, A_P, A_LSE, A_X1, A_GU, A_COUNT };

struct Dims {
  int L, d, H, dh, f, S, B, T, Mmax, slots, dtype, causal;
  size_t e;       // bytes per stored element
  bool attn;
  bool fused;     // attention without stored probabilities (row log-sum-exp only)
  bool dq_recompute;   // fused attention backward without a dS^T buffer: dq by a recompute pass
  bool literal;   // RMSNorm gain gradients computed in p2 from stashed (x, dy) instead of p1's per-micro-batch partials
  float eps, base;
};

size_t w_width(const Dims& c, int t) {
  switch (t) {
    case W_H1: case W_A: case W_DX1: return c.attn ? c.d : 0;
    case W_DQKV: return c.attn ? 3 * (size_t)c.d : 0;
    case W_H2: case W_DX2: return c.d;
    case W_M: return c.f;
    case W_DGU: return 2 * (size_t)c.f;
    case W_N1X: case W_N1DY: return (c.literal && c.attn) ? c.d : 0;
    case W_N2X: case W_N2DY: return c.literal ? c.d : 0;
  }
  return 0;
}
bool w_from_forward(int t) { return t == W_H1 || t == W_A || t == W_H2 || t == W_M || t == W_N1X || t == W_N2X; }

size_t a_bytes(const Dims& c, int t) {      // bytes per slot
  switch (t) {
    case A_X0: return (c.attn && !c.literal) ? (size_t)c.T * c.d * c.e : 0;     // (literal gain p2: lives in the W class)
    case A_QKV: return c.attn ? (size_t)c.T * 3 * c.d * c.e : 0;
    case A_P: return (c.attn && !c.fused) ? (size_t)c.B * c.H * c.S * c.S * c.e : 0;
    case A_LSE: return (c.attn && c.fused) ? (size_t)c.B * c.H * c.S * sizeof(float) : 0;
    case A_X1: return c.literal ? 0 : (size_t)c.T * c.d * c.e;
    case A_GU: return (size_t)c.T * 2 * c.f * c.e;
  }
  return 0;
}

struct Layout {
  size_t w_off[W_COUNT];        // per layer: offset of each slab inside the layer's W block
  size_t w_layer_bytes;
  size_t a_off[A_COUNT];        // per (layer, slot)
  size_t a_slot_bytes;          // one slot of one layer
  size_t gain_part_off;         // fp32 [L][2][Mmax][gain_rows][d]: per micro-batch, the partial rows of a norm's gain gradient (W class)
  size_t gain_part_bytes;
  int gain_rows;                // partial rows that backward-p1 of one micro-batch leaves per norm
  size_t w_total, a_base, a_total, ws_base, ws_total, arena;
  // workspace pieces
  size_t ws_t_f, ws_t_d0, ws_t_d1, ws_scores, ws_norm_partials_p2, ws_rope, ws_delta, ws_split;
  size_t ws_split_bytes;        // scratch of the products that split their contraction (0: none does)
  // accounting units
  size_t w_fwd_bytes_per_mb, w_p1_bytes_per_mb, a_bytes_per_mb;
};

Layout plan(const Dims& c) {
  Layout y{};
  size_t off = 0;
  for (int t = 0; t < W_COUNT; t++) {
    y.w_off[t] = off;
    off += align_up((size_t)c.Mmax * c.T * w_width(c, t) * c.e, 256);
  }
  y.w_layer_bytes = off;
  y.gain_part_off = y.w_layer_bytes * c.L;
  y.gain_rows = c.literal ? 0 : tbp::rmsnorm_partial_rows(c.dtype, c.T, c.d);
  y.gain_part_bytes = align_up((size_t)c.L * 2 * c.Mmax * y.gain_rows * c.d * sizeof(float), 256);
  y.w_total = y.gain_part_off + y.gain_part_bytes;
  off = 0;
  for (int t = 0; t < A_COUNT; t++) {
    y.a_off[t] = off;
    off += align_up(a_bytes(c, t), 256);
  }
  y.a_slot_bytes = off;
  y.a_base = y.w_total;
  y.a_total = y.a_slot_bytes * c.slots * c.L;
  y.ws_base = y.a_base + y.a_total;
  off = 0;
  y.ws_t_f = off; off += align_up((size_t)c.T * c.f * c.e, 256);
  y.ws_t_d0 = off; off += align_up((size_t)c.T * c.d * c.e, 256);
  y.ws_t_d1 = off; off += align_up((size_t)c.T * c.d * c.e, 256);
  // fp32 scores, then dS (materialised attention) or dS^T in the storage type (fused)
  y.ws_scores = off; off += (!c.attn || c.dq_recompute) ? 0 : align_up(c.fused ? (size_t)c.B * c.H * tbp::attn_ds_elems(c.S) * c.e
                                                           : (size_t)c.B * c.H * c.S * c.S * sizeof(float), 256);
  y.ws_norm_partials_p2 = off; off += c.literal ? align_up((size_t)tbp::kNormPartialBlocks * c.d * sizeof(float), 256) : 0;
  y.ws_rope = off; off += c.attn ? align_up((size_t)c.S * (c.dh / 2) * sizeof(float2), 256) : 0;
  y.ws_delta = off; off += c.attn ? align_up((size_t)c.T * c.H * sizeof(float), 256) : 0;
  {  // the forward and backward-p1 products of a layer, [T, out] = [T, in] x W: the largest scratch any of them wants
    const int outs[4] = {3 * c.d, c.d, 2 * c.f, c.d}, ins[4] = {c.d, c.d, c.d, c.f};
    size_t need = 0;
    for (int i = 0; i < 4; i++) {
      if (!c.attn && i < 2) continue;
      need = std::max(need, tbp::gemm_split_plan(c.dtype, tbp::NN, c.T, outs[i], ins[i], 0, 1).bytes);
      need = std::max(need, tbp::gemm_split_plan(c.dtype, tbp::NT, c.T, ins[i], outs[i], 0, 1).bytes);
    }
    y.ws_split_bytes = need;
    y.ws_split = off; off += align_up(need, 256);
  }
  y.ws_total = off;
  y.arena = y.ws_base + y.ws_total;
  size_t fw = 0, p1 = 0;
  for (int t = 0; t < W_COUNT; t++) {
    const size_t b = (size_t)c.T * w_width(c, t) * c.e;
    if (w_from_forward(t)) fw += b; else p1 += b;
  }
  y.w_fwd_bytes_per_mb = fw * c.L;
  y.w_p1_bytes_per_mb = (p1 + (c.attn ? 2 : 1) * (size_t)y.gain_rows * c.d * sizeof(float)) * c.L;
  size_t a = 0;
  for (int t = 0; t < A_COUNT; t++) a += a_bytes(c, t);
  y.a_bytes_per_mb = a * c.L;
  return y;
}

tbp_status check_config(const tbp_config* cfg, Dims* out) {
  if (!cfg) return fail(TBP_EINVAL, "config is null");
  Dims c{};
  c.L = cfg->n_layers; c.d = cfg->d_model; c.H = cfg->n_heads; c.dh = cfg->head_dim; c.f = cfg->d_ffn;
  c.S = cfg->seq; c.B = cfg->micro_batch; c.Mmax = cfg->max_microbatches; c.dtype = cfg->dtype;
  c.causal = cfg->causal ? 1 : 0; c.eps = cfg->rms_eps; c.base = cfg->rope_base;
  c.slots = cfg->act_slots > 0 ? cfg->act_slots : cfg->max_microbatches;
  c.attn = c.H > 0;
  if (c.dtype != TBP_F32 && c.dtype != TBP_BF16) return fail(TBP_EINVAL, "dtype must be TBP_F32 or TBP_BF16");
  c.e = c.dtype == TBP_BF16 ? 2 : 4;
  const int q = c.dtype == TBP_BF16 ? 8 : 4;     // elements per 16-byte vector
  if (c.L < 1 || c.d < 1 || c.f < 1 || c.S < 1 || c.B < 1 || c.Mmax < 1)
    return fail(TBP_EINVAL, "n_layers, d_model, d_ffn, seq, micro_batch, max_microbatches must be >= 1");
  if (c.H < 0 || cfg->act_slots < 0 || c.slots > c.Mmax)
    return fail(TBP_EINVAL, "n_heads >= 0 and 0 <= act_slots <= max_microbatches required");
  if (c.d % q || c.f % q) return fail(TBP_EINVAL, "d_model and d_ffn must be multiples of %d for this dtype", q);
  if (c.d > tbp::max_d_model(c.dtype)) return fail(TBP_EINVAL, "d_model %d above the limit %d", c.d, tbp::max_d_model(c.dtype));
  if (c.attn) {
    if ((long)c.H * c.dh != c.d) return fail(TBP_EINVAL, "n_heads * head_dim must equal d_model");
    if (c.dh % (2 * q)) return fail(TBP_EINVAL, "head_dim must be a multiple of %d for this dtype", 2 * q);
    if (c.S % q) return fail(TBP_EINVAL, "seq must be a multiple of %d for this dtype", q);
    if (c.S > tbp::kMaxSeq) return fail(TBP_EINVAL, "seq %d above the limit %d", c.S, tbp::kMaxSeq);
    if (!(c.base > 0.f)) return fail(TBP_EINVAL, "rope_base must be positive");
  }
  if (cfg->attention < TBP_ATTN_AUTO || cfg->attention > TBP_ATTN_FUSED_RECOMPUTE) return fail(TBP_EINVAL, "attention must be a tbp_attention value");
  {
    const bool can_fuse = c.attn && c.dtype == TBP_BF16 && (c.dh == 64 || c.dh == 128);
    if ((cfg->attention == TBP_ATTN_FUSED || cfg->attention == TBP_ATTN_FUSED_RECOMPUTE) && c.attn && !can_fuse)
      return fail(TBP_EINVAL, "fused attention needs bf16 storage and head_dim 64 or 128");
    c.fused = can_fuse && cfg->attention != TBP_ATTN_MATERIALISED;
    c.dq_recompute = c.fused && cfg->attention == TBP_ATTN_FUSED_RECOMPUTE;
  }
  if (cfg->gain_grad != TBP_GAIN_PARTIALS && cfg->gain_grad != TBP_GAIN_LITERAL) return fail(TBP_EINVAL, "gain_grad must be a tbp_gain_grad value");
  c.literal = cfg->gain_grad == TBP_GAIN_LITERAL;
  if (!(c.eps >= 0.f)) return fail(TBP_EINVAL, "rms_eps must be >= 0");
  if ((long)c.S * c.B > (1L << 24)) return fail(TBP_EINVAL, "tokens per micro-batch above 2^24");
  c.T = c.S * c.B;
  *out = c;
  return TBP_OK;
}

enum MbState { MB_EMPTY = 0, MB_FWD = 1, MB_P1 = 2 };

}  // namespace

struct tbp_stage {
  Dims c;
  Layout y;
  unsigned char* arena;
  std::vector<const void*> w_qkv, w_o, g1, w_gu, w_d, g2;
  std::vector<float*> dw_qkv, dw_o, dg1, dw_gu, dw_d, dg2;
  std::vector<int> state;       // per micro-batch
  std::vector<int> slot_of;     // per micro-batch, -1 if none
  std::vector<int> free_slots;
  std::vector<tbp::GroupedProduct> grouped;      // loop-mode p2: the products of one micro-batch (capacity fixed at creation)
  size_t w_live, a_live, high;

  void* wslab(int layer, int t, int mb) const {
    return arena + layer * y.w_layer_bytes + y.w_off[t] + (size_t)mb * c.T * w_width(c, t) * c.e;
  }
  void* aslot(int layer, int t, int slot) const {
    return arena + y.a_base + ((size_t)layer * c.slots + slot) * y.a_slot_bytes + y.a_off[t];
  }
  float* gain_part(int layer, int which, int mb) const {      // [gain_rows][d] of micro-batch mb; consecutive micro-batches are consecutive rows
    return reinterpret_cast<float*>(arena + y.gain_part_off) + (((size_t)layer * 2 + which) * c.Mmax + mb) * y.gain_rows * c.d;
  }
  void* ws(size_t off) const { return arena + y.ws_base + off; }
  // inputs of the two RMSNorms of a layer: forward->p1 slot, or a slab kept until p2 (literal gain gradient)
  void* x0_of(int layer, int mb, int slot) const { return c.literal ? wslab(layer, W_N1X, mb) : aslot(layer, A_X0, slot); }
  void* x1_of(int layer, int mb, int slot) const { return c.literal ? wslab(layer, W_N2X, mb) : aslot(layer, A_X1, slot); }
  void bump() { if (w_live + a_live > high) high = w_live + a_live; }
};

namespace {

using tbp::GemmArgs;
using tbp::gemm_args;

// One attention product per (sequence, head): z = b * H + h.
GemmArgs head_gemm(const Dims& c, int layout, int M, int N, int K) {
  GemmArgs g{};
  g.layout = layout; g.M = M; g.N = N; g.K = K; g.alpha = 1.f;
  g.batch = c.B * c.H; g.batch_inner = c.H;
  return g;
}

// A linear-layer product of the forward or backward-p1 pass: handed the stage's scratch when its output is small
// enough for the contraction to be split over several workgroups per tile.
hipError_t linear_gemm(tbp_stage* st, GemmArgs g, hipStream_t s) {
  const Dims& c = st->c;
  if (st->y.ws_split_bytes) {
    const tbp::SplitPlan plan = tbp::gemm_split_plan(c.dtype, g.layout, g.M, g.N, g.K, g.out_f32, g.batch);
    if (plan.split > 1 && plan.bytes <= st->y.ws_split_bytes) {
      g.ws = st->ws(st->y.ws_split);
      g.ws_bytes = st->y.ws_split_bytes;
      // The arrival counters are cleared before every such product (one small launch) rather than once: a flag kept on
      // the host would be wrong for a caller who records the first call into a graph and replays it later.
      g.ws_counters_zero = 0;
    }
  }
  return tbp::gemm(c.dtype, g, s);
}

tbp_status run_forward(tbp_stage* st, int mb, int slot, const void* x_in, void* x_out, hipStream_t s) {
  const Dims& c = st->c;
  const int dt = c.dtype, T = c.T, d = c.d, f = c.f;
  const size_t act_bytes = (size_t)T * d * c.e;
  // The rotation table is rebuilt by every forward call (a few microseconds) instead of once behind a host-side flag:
  // the flag would be wrong for a caller who records the first call into a graph and replays it later, and for one who
  // moves to another stream without synchronising.  (Every build writes the same values, so a backward-p1 call that
  // reads the table on another stream meanwhile reads them either way.)
  if (c.attn) TBP_HIP(tbp::rope_table(c.S, c.dh, c.base, (float2*)st->ws(st->y.ws_rope), s));
  const void* x_cur = x_in;
  for (int l = 0; l < c.L; l++) {
    void* x1 = st->x1_of(l, mb, slot);
    if (c.attn) {
      void* x0 = st->x0_of(l, mb, slot);
      // the layer input is kept for the RMSNorm backward; for layer 0 it is copied from the caller
      if (l == 0) TBP_HIP(hipMemcpyAsync(x0, x_in, act_bytes, hipMemcpyDeviceToDevice, s));
      (void)x_cur;
      void* h1 = st->wslab(l, W_H1, mb);
      void* qkv = st->aslot(l, A_QKV, slot);
      void* P = st->aslot(l, A_P, slot);
      void* a = st->wslab(l, W_A, mb);
      TBP_HIP(tbp::rmsnorm_fwd(dt, T, d, c.eps, x0, st->g1[l], h1, s));
      TBP_HIP(linear_gemm(st, gemm_args(tbp::NN, T, 3 * d, d, h1, d, st->w_qkv[l], 3 * d, qkv, 3 * d), s));
      TBP_HIP(tbp::rope(dt, T, c.S, 2 * c.H, c.dh, 3 * d, (const float2*)st->ws(st->y.ws_rope), 0, qkv, s));
      if (c.fused) {
        TBP_HIP(tbp::attention_fwd(c.B, c.H, c.S, c.dh, c.causal, qkv, 3 * d, a, d, (float*)st->aslot(l, A_LSE, slot), s));
      } else {
        float* scores = (float*)st->ws(st->y.ws_scores);
        {  // scores = q k^T / sqrt(dh), fp32
          GemmArgs g = head_gemm(c, tbp::NT, c.S, c.S, c.dh);
          g.alpha = 1.f / sqrtf((float)c.dh);
          g.A = qkv; g.lda = 3 * d; g.sAo = (long)c.S * 3 * d; g.sAi = c.dh;
          g.B = (const char*)qkv + (size_t)d * c.e; g.ldb = 3 * d; g.sBo = g.sAo; g.sBi = c.dh;
          g.C = scores; g.ldc = c.S; g.sCo = (long)c.H * c.S * c.S; g.sCi = (long)c.S * c.S;
          g.out_f32 = 1; g.causal = c.causal ? tbp::CAUSAL_SKIP_UPPER : tbp::CAUSAL_NONE;
          TBP_HIP(tbp::gemm(dt, g, s));
        }
        TBP_HIP(tbp::softmax_fwd(dt, (long)c.B * c.H * c.S, c.S, c.causal, scores, P, s));
        {  // a = P v
          GemmArgs g = head_gemm(c, tbp::NN, c.S, c.dh, c.S);
          g.A = P; g.lda = c.S; g.sAo = (long)c.H * c.S * c.S; g.sAi = (long)c.S * c.S;
          g.B = (const char*)qkv + (size_t)2 * d * c.e; g.ldb = 3 * d; g.sBo = (long)c.S * 3 * d; g.sBi = c.dh;
          g.C = a; g.ldc = d; g.sCo = (long)c.S * d; g.sCi = c.dh;
          g.causal = c.causal ? tbp::CAUSAL_K_END : tbp::CAUSAL_NONE;
          TBP_HIP(tbp::gemm(dt, g, s));
        }
      }
      {  // x1 = x0 + a Wo
        GemmArgs g = gemm_args(tbp::NN, T, d, d, a, d, st->w_o[l], d, x1, d);
        g.R = x0;
        TBP_HIP(linear_gemm(st, g, s));
      }
    } else if (l == 0) {
      TBP_HIP(hipMemcpyAsync(x1, x_in, act_bytes, hipMemcpyDeviceToDevice, s));
    }
    void* h2 = st->wslab(l, W_H2, mb);
    void* gu = st->aslot(l, A_GU, slot);
    void* m = st->wslab(l, W_M, mb);
    TBP_HIP(tbp::rmsnorm_fwd(dt, T, d, c.eps, x1, st->g2[l], h2, s));
    TBP_HIP(linear_gemm(st, gemm_args(tbp::NN, T, 2 * f, d, h2, d, st->w_gu[l], 2 * f, gu, 2 * f), s));
    TBP_HIP(tbp::swiglu_fwd(dt, T, f, gu, m, s));
    {  // x2 = x1 + m Wd, written where the next layer (or the caller) wants its input
      void* dst = (l + 1 < c.L) ? (c.attn ? st->x0_of(l + 1, mb, slot) : st->x1_of(l + 1, mb, slot)) : x_out;
      GemmArgs g = gemm_args(tbp::NN, T, d, f, m, f, st->w_d[l], d, dst, d);
      g.R = x1;
      TBP_HIP(linear_gemm(st, g, s));
    }
  }
  return TBP_OK;
}

tbp_status run_p1(tbp_stage* st, int mb, int slot, const void* dy, void* dx, hipStream_t s) {
  const Dims& c = st->c;
  const int dt = c.dtype, T = c.T, d = c.d, f = c.f;
  const size_t act_bytes = (size_t)T * d * c.e;
  // the stage's upstream gradient is the output derivative of the last layer's down projection: keep it
  TBP_HIP(hipMemcpyAsync(st->wslab(c.L - 1, W_DX2, mb), dy, act_bytes, hipMemcpyDeviceToDevice, s));
  for (int l = c.L - 1; l >= 0; l--) {
    void* dx2 = st->wslab(l, W_DX2, mb);
    void* dm = st->ws(st->y.ws_t_f);
    void* dgu = st->wslab(l, W_DGU, mb);
    // derivative of a norm's output: a temporary, or (literal gain gradient) a slab that p2 reads
    void* dh = c.literal ? st->wslab(l, W_N2DY, mb) : st->ws(st->y.ws_t_d0);
    void* gu = st->aslot(l, A_GU, slot);
    void* x1 = st->x1_of(l, mb, slot);
    // where this layer's input gradient goes: previous layer's dx2 slab, or the caller
    void* dx_out = (l > 0) ? st->wslab(l - 1, W_DX2, mb) : dx;
    // dm = dx2 Wd^T
    TBP_HIP(linear_gemm(st, gemm_args(tbp::NT, T, f, d, dx2, d, st->w_d[l], d, dm, f), s));
    TBP_HIP(tbp::swiglu_p1(dt, T, f, dm, gu, dgu, s));
    // dh2 = [dg, du] Wgu^T
    TBP_HIP(linear_gemm(st, gemm_args(tbp::NT, T, d, 2 * f, dgu, 2 * f, st->w_gu[l], 2 * f, dh, d), s));
    void* dx1 = c.attn ? st->wslab(l, W_DX1, mb) : dx_out;
    // (the partial rows of the gain gradient stay in the stash as they leave the row kernel: backward-p2 adds them up)
    TBP_HIP(tbp::rmsnorm_p1_rows(dt, T, d, c.eps, dh, x1, st->g2[l], dx2, dx1,
                                 c.literal ? nullptr : st->gain_part(l, 1, mb), s));
    if (!c.attn) continue;
    void* da = st->ws(st->y.ws_t_d1);
    void* qkv = st->aslot(l, A_QKV, slot);
    void* P = st->aslot(l, A_P, slot);
    void* x0 = st->x0_of(l, mb, slot);
    void* dqkv = st->wslab(l, W_DQKV, mb);
    void* dP = st->ws(st->y.ws_scores);       // dS, storage type, reuses the score workspace
    const float scale = 1.f / sqrtf((float)c.dh);
    const long hs = (long)c.S * c.S, bs = (long)c.H * hs, tok3 = (long)c.S * 3 * d;
    // da = dx1 Wo^T
    TBP_HIP(linear_gemm(st, gemm_args(tbp::NT, T, d, d, dx1, d, st->w_o[l], d, da, d), s));
    if (c.fused) {
      // probabilities rebuilt from the stashed row log-sum-exp; dq, dk, dv straight into the dqkv slab
      TBP_HIP(tbp::attention_p1(c.B, c.H, c.S, c.dh, c.causal, qkv, 3 * d, st->wslab(l, W_A, mb), da, d,
                                (const float*)st->aslot(l, A_LSE, slot), dqkv, 3 * d, (float*)st->ws(st->y.ws_delta),
                                c.dq_recompute ? nullptr : dP, s));
    } else {
      // rowsum(dP * P) per (token, head) = rowsum(da * a): no S x S tensor needed for it
      float* delta = (float*)st->ws(st->y.ws_delta);
      TBP_HIP(tbp::head_rowdot(dt, T, c.H, c.dh, da, st->wslab(l, W_A, mb), delta, s));
      {  // dS = P * (da v^T - delta): the softmax backward is the epilogue of the dP product (dP is never stored)
        GemmArgs g = head_gemm(c, tbp::NT, c.S, c.S, c.dh);
        g.A = da; g.lda = d; g.sAo = (long)c.S * d; g.sAi = c.dh;
        g.B = (const char*)qkv + (size_t)2 * d * c.e; g.ldb = 3 * d; g.sBo = tok3; g.sBi = c.dh;
        g.C = dP; g.ldc = c.S; g.sCo = bs; g.sCi = hs;
        g.R = P;
        g.delta = delta; g.ldd = c.H; g.sDo = (long)c.S * c.H; g.sDi = 1; g.delta_causal = c.causal;
        g.causal = c.causal ? tbp::CAUSAL_SKIP_UPPER : tbp::CAUSAL_NONE;
        TBP_HIP(tbp::gemm(dt, g, s));
      }
      {  // dv = P^T da
        GemmArgs g = head_gemm(c, tbp::TN, c.S, c.dh, c.S);
        g.A = P; g.lda = c.S; g.sAo = bs; g.sAi = hs;
        g.B = da; g.ldb = d; g.sBo = (long)c.S * d; g.sBi = c.dh;
        g.C = (char*)dqkv + (size_t)2 * d * c.e; g.ldc = 3 * d; g.sCo = tok3; g.sCi = c.dh;
        g.causal = c.causal ? tbp::CAUSAL_K_BEGIN : tbp::CAUSAL_NONE;
        TBP_HIP(tbp::gemm(dt, g, s));
      }
      {  // dq = dS k / sqrt(dh)
        GemmArgs g = head_gemm(c, tbp::NN, c.S, c.dh, c.S);
        g.alpha = scale;
        g.A = dP; g.lda = c.S; g.sAo = bs; g.sAi = hs;
        g.B = (const char*)qkv + (size_t)d * c.e; g.ldb = 3 * d; g.sBo = tok3; g.sBi = c.dh;
        g.C = dqkv; g.ldc = 3 * d; g.sCo = tok3; g.sCi = c.dh;
        g.causal = c.causal ? tbp::CAUSAL_K_END : tbp::CAUSAL_NONE;
        TBP_HIP(tbp::gemm(dt, g, s));
      }
      {  // dk = dS^T q / sqrt(dh)
        GemmArgs g = head_gemm(c, tbp::TN, c.S, c.dh, c.S);
        g.alpha = scale;
        g.A = dP; g.lda = c.S; g.sAo = bs; g.sAi = hs;
        g.B = qkv; g.ldb = 3 * d; g.sBo = tok3; g.sBi = c.dh;
        g.C = (char*)dqkv + (size_t)d * c.e; g.ldc = 3 * d; g.sCo = tok3; g.sCi = c.dh;
        g.causal = c.causal ? tbp::CAUSAL_K_BEGIN : tbp::CAUSAL_NONE;
        TBP_HIP(tbp::gemm(dt, g, s));
      }
    }
    TBP_HIP(tbp::rope(dt, T, c.S, 2 * c.H, c.dh, 3 * d, (const float2*)st->ws(st->y.ws_rope), 1, dqkv, s));
    // dh1 = [dq, dk, dv] Wqkv^T
    void* dh1 = c.literal ? st->wslab(l, W_N1DY, mb) : dh;
    TBP_HIP(linear_gemm(st, gemm_args(tbp::NT, T, d, 3 * d, dqkv, 3 * d, st->w_qkv[l], 3 * d, dh1, d), s));
    TBP_HIP(tbp::rmsnorm_p1_rows(dt, T, d, c.eps, dh1, x0, st->g1[l], dx1, dx_out,
                                 c.literal ? nullptr : st->gain_part(l, 0, mb), s));
  }
  return TBP_OK;
}

// dW (=, +=) X^T dY over rows [row0, row0 + K) of the two slabs.  rests != nullptr: the part of the output that does
// not make whole rounds of large tiles is not launched but appended to *rests, for one grouped launch at the end.
tbp_status p2_product(tbp_stage* st, int layer, int xt, int dyt, int mb0, int K, float* dW, int accumulate,
                      hipStream_t s, std::vector<tbp::GroupedProduct>* rests = nullptr) {
  const Dims& c = st->c;
  const int M = (int)w_width(c, xt), N = (int)w_width(c, dyt);
  GemmArgs g = gemm_args(tbp::TN, M, N, K, st->wslab(layer, xt, mb0), M, st->wslab(layer, dyt, mb0), N, dW, N);
  g.out_f32 = 1;
  g.accumulate = accumulate;
  tbp::GroupedProduct rest{};
  if (rests) g.defer_rest = &rest;
  TBP_HIP(tbp::gemm(c.dtype, g, s));
  if (rests && rest.M > 0) rests->push_back(rest);        // (capacity reserved at creation: no allocation here)
  return TBP_OK;
}

tbp_status run_p2(tbp_stage* st, const int* mbs, int n, int mode, int accumulate, hipStream_t s) {
  const Dims& c = st->c;
  struct Prod { int x, dy; float* const* dw; bool attn_only; };
  auto prods_of = [&](Prod (&out)[4]) {
    const Prod all[4] = {{W_H1, W_DQKV, st->dw_qkv.data(), true}, {W_A, W_DX1, st->dw_o.data(), true},
                         {W_H2, W_DGU, st->dw_gu.data(), false}, {W_M, W_DX2, st->dw_d.data(), false}};
    for (int i = 0; i < 4; i++) out[i] = all[i];
  };
  Prod prods[4];
  prods_of(prods);
  if (c.dtype == TBP_BF16 && mode == TBP_P2_LOOP) {
    // bf16, one micro-batch per product: all weight-gradient products of the stage for that micro-batch go into one
    // grouped launch, each launch accumulating on the previous one.  (The K-concatenated products are long enough
    // that one launch per weight, which starts its tiles in step, is the faster arrangement.)
    std::vector<tbp::GroupedProduct>& table = st->grouped;     // (no host allocation here: the capacity is reserved)
    for (int i = 0; i < n; i++) {
      table.clear();
      const int mb0 = mbs[i];
      const int K = c.T;
      for (int l = 0; l < c.L; l++)
        for (const Prod& p : prods) {
          if (p.attn_only && !c.attn) continue;
          tbp::GroupedProduct g{};
          g.M = (int)w_width(c, p.x); g.N = (int)w_width(c, p.dy); g.K = K;
          g.A = st->wslab(l, p.x, mb0); g.lda = g.M;
          g.B = st->wslab(l, p.dy, mb0); g.ldb = g.N;
          g.C = p.dw[l]; g.ldc = g.N;
          g.accumulate = (accumulate || i > 0) ? 1 : 0;
          table.push_back(g);
        }
      TBP_HIP(tbp::gemm_tn_grouped(table.data(), (int)table.size(), s));
    }
  } else {
    // K-concatenated bf16 products: one launch per weight for the whole rounds of large tiles (tiles that start in step
    // share operand panels through the L2), and the remainders of all the stage's products together in one grouped
    // launch at the end, where they fill rounds with each other instead of each running a last, mostly empty round
    std::vector<tbp::GroupedProduct>* rests = (mode == TBP_P2_KCONCAT && c.dtype == TBP_BF16) ? &st->grouped : nullptr;
    if (rests) rests->clear();
    for (int l = 0; l < c.L; l++)
      for (const Prod& p : prods) {
        if (p.attn_only && !c.attn) continue;
        if (mode == TBP_P2_KCONCAT) {
          tbp_status r = p2_product(st, l, p.x, p.dy, mbs[0], n * c.T, p.dw[l], accumulate, s, rests);
          if (r != TBP_OK) return r;
        } else {
          for (int i = 0; i < n; i++) {
            tbp_status r = p2_product(st, l, p.x, p.dy, mbs[i], c.T, p.dw[l], (accumulate || i > 0) ? 1 : 0, s);
            if (r != TBP_OK) return r;
          }
        }
      }
    if (rests && !rests->empty()) TBP_HIP(tbp::gemm_tn_grouped(rests->data(), (int)rests->size(), s));
  }
  if (c.literal) {
    // gain gradients from the stashed norm inputs and output derivatives (Section 3.1 treats a norm's gain like any
    // other parameter: its gradient belongs to backward-p2); rows of consecutive micro-batches are one operand
    float* part = (float*)st->ws(st->y.ws_norm_partials_p2);
    const int runs = mode == TBP_P2_KCONCAT ? 1 : n;
    const int rows = mode == TBP_P2_KCONCAT ? n * c.T : c.T;
    for (int l = 0; l < c.L; l++)
      for (int i = 0; i < runs; i++) {
        const int acc = (accumulate || i > 0) ? 1 : 0;
        if (c.attn)
          TBP_HIP(tbp::rmsnorm_gain_p2(c.dtype, rows, c.d, c.eps, st->wslab(l, W_N1DY, mbs[i]), st->wslab(l, W_N1X, mbs[i]),
                                       acc, st->dg1[l], part, s));
        TBP_HIP(tbp::rmsnorm_gain_p2(c.dtype, rows, c.d, c.eps, st->wslab(l, W_N2DY, mbs[i]), st->wslab(l, W_N2X, mbs[i]),
                                     acc, st->dg2[l], part, s));
      }
    return TBP_OK;
  }
  // gain gradients: the partial rows that backward-p1 left, added up run by run of consecutive micro-batches (whose
  // partial rows are consecutive in the stash; a K-concatenated set is one run)
  for (int l = 0; l < c.L; l++)
    for (int i = 0; i < n;) {
      int j = i + 1;
      while (j < n && mbs[j] == mbs[j - 1] + 1) j++;
      const int acc = (accumulate || i > 0) ? 1 : 0, nrows = (j - i) * st->y.gain_rows;
      if (c.attn) TBP_HIP(tbp::gain_partials_sum(st->gain_part(l, 0, mbs[i]), nrows, c.d, acc, st->dg1[l], s));
      TBP_HIP(tbp::gain_partials_sum(st->gain_part(l, 1, mbs[i]), nrows, c.d, acc, st->dg2[l], s));
      i = j;
    }
  return TBP_OK;
}

bool copy_ptrs(std::vector<const void*>& dst, const void* const* src, int n) {
  if (!src) return false;
  dst.assign(src, src + n);
  for (const void* p : dst) if (!p) return false;
  return true;
}
bool copy_ptrs(std::vector<float*>& dst, float* const* src, int n) {
  if (!src) return false;
  dst.assign(src, src + n);
  for (float* p : dst) if (!p) return false;
  return true;
}

}  // namespace

extern "C" {

const char* tbp_last_error(void) { return g_err; }
const char* tbp_version(void) { return "tbp 0.1 (gfx950)"; }

tbp_status tbp_stash_query(const tbp_config* cfg, tbp_stash_sizes* out) {
  Dims c;
  tbp_status r = check_config(cfg, &c);
  if (r != TBP_OK) return r;
  if (!out) return fail(TBP_EINVAL, "out is null");
  const Layout y = plan(c);
  out->w_stash_bytes = y.w_total;
  out->a_stash_bytes = y.a_total;
  out->workspace_bytes = y.ws_total;
  out->arena_bytes = y.arena;
  return TBP_OK;
}

tbp_status tbp_stage_create(const tbp_config* cfg, const tbp_params* params, void* arena, size_t arena_bytes,
                            tbp_stage** out) {
  Dims c;
  tbp_status r = check_config(cfg, &c);
  if (r != TBP_OK) return r;
  if (!params || !arena || !out) return fail(TBP_EINVAL, "params, arena and out must be non-null");
  if (reinterpret_cast<uintptr_t>(arena) % 256) return fail(TBP_EINVAL, "arena must be 256-byte aligned");
  const Layout y = plan(c);
  if (arena_bytes < y.arena)
    return fail(TBP_ENOMEM, "arena of %zu bytes is smaller than the %zu bytes this configuration needs", arena_bytes, y.arena);
  tbp_stage* st = new (std::nothrow) tbp_stage();
  if (!st) return fail(TBP_ENOMEM, "host allocation failed");
  st->c = c; st->y = y; st->arena = static_cast<unsigned char*>(arena);
  bool ok = false;
  try {                                        // (no exception may leave through the C boundary)
    ok = copy_ptrs(st->w_gu, params->w_gu, c.L) && copy_ptrs(st->w_d, params->w_d, c.L) &&
         copy_ptrs(st->g2, params->g2, c.L) && copy_ptrs(st->dw_gu, params->dw_gu, c.L) &&
         copy_ptrs(st->dw_d, params->dw_d, c.L) && copy_ptrs(st->dg2, params->dg2, c.L);
    if (ok && c.attn)
      ok = copy_ptrs(st->w_qkv, params->w_qkv, c.L) && copy_ptrs(st->w_o, params->w_o, c.L) &&
           copy_ptrs(st->g1, params->g1, c.L) && copy_ptrs(st->dw_qkv, params->dw_qkv, c.L) &&
           copy_ptrs(st->dw_o, params->dw_o, c.L) && copy_ptrs(st->dg1, params->dg1, c.L);
    st->state.assign(c.Mmax, MB_EMPTY);
    st->slot_of.assign(c.Mmax, -1);
    st->free_slots.reserve(c.slots);
    for (int i = c.slots - 1; i >= 0; i--) st->free_slots.push_back(i);
    st->grouped.reserve((size_t)4 * c.L);
  } catch (...) {
    delete st;
    return fail(TBP_ENOMEM, "host allocation failed");
  }
  if (!ok) {
    delete st;
    return fail(TBP_EINVAL, "a parameter or gradient pointer (array or entry) is null");
  }
  st->w_live = st->a_live = st->high = 0;
  *out = st;
  return TBP_OK;
}

void tbp_stage_destroy(tbp_stage* st) { delete st; }

tbp_status tbp_stage_forward(tbp_stage* st, int mb, const void* x_in, void* x_out, void* stream) {
  if (!st || !x_in || !x_out) return fail(TBP_EINVAL, "stage, x_in and x_out must be non-null");
  if (mb < 0 || mb >= st->c.Mmax) return fail(TBP_EINVAL, "micro-batch %d outside 0..%d", mb, st->c.Mmax - 1);
  if (st->state[mb] != MB_EMPTY) return fail(TBP_ESTATE, "forward(%d): micro-batch is not EMPTY", mb);
  if (st->free_slots.empty()) return fail(TBP_ENOMEM, "forward(%d): all %d activation slots are in use", mb, st->c.slots);
  const int slot = st->free_slots.back();
  tbp_status r = run_forward(st, mb, slot, x_in, x_out, static_cast<hipStream_t>(stream));
  if (r != TBP_OK) return r;
  st->free_slots.pop_back();
  st->slot_of[mb] = slot;
  st->state[mb] = MB_FWD;
  st->w_live += st->y.w_fwd_bytes_per_mb;
  st->a_live += st->y.a_bytes_per_mb;
  st->bump();
  return TBP_OK;
}

tbp_status tbp_stage_backward_p1(tbp_stage* st, int mb, const void* dy, void* dx, void* stream) {
  if (!st || !dy || !dx) return fail(TBP_EINVAL, "stage, dy and dx must be non-null");
  if (mb < 0 || mb >= st->c.Mmax) return fail(TBP_EINVAL, "micro-batch %d outside 0..%d", mb, st->c.Mmax - 1);
  if (st->state[mb] != MB_FWD) return fail(TBP_ESTATE, "backward_p1(%d): forward has not run (or p1 already has)", mb);
  tbp_status r = run_p1(st, mb, st->slot_of[mb], dy, dx, static_cast<hipStream_t>(stream));
  if (r != TBP_OK) return r;
  st->w_live += st->y.w_p1_bytes_per_mb;
  st->bump();                        // the derivatives exist before the activations are dropped
  st->a_live -= st->y.a_bytes_per_mb;
  st->free_slots.push_back(st->slot_of[mb]);
  st->slot_of[mb] = -1;
  st->state[mb] = MB_P1;
  return TBP_OK;
}

tbp_status tbp_stage_backward_p2(tbp_stage* st, const int* mbs, int n_mbs, int p2_mode, int accumulate, void* stream) {
  if (!st || !mbs) return fail(TBP_EINVAL, "stage and mbs must be non-null");
  if (n_mbs < 1 || n_mbs > st->c.Mmax) return fail(TBP_EINVAL, "n_mbs %d outside 1..%d", n_mbs, st->c.Mmax);
  if (p2_mode != TBP_P2_LOOP && p2_mode != TBP_P2_KCONCAT) return fail(TBP_EINVAL, "unknown p2 mode %d", p2_mode);
  for (int i = 0; i < n_mbs; i++) {          // argument errors first, for the whole set
    const int mb = mbs[i];
    if (mb < 0 || mb >= st->c.Mmax) return fail(TBP_EINVAL, "micro-batch %d outside 0..%d", mb, st->c.Mmax - 1);
    for (int j = 0; j < i; j++)
      if (mbs[j] == mb) return fail(TBP_EINVAL, "micro-batch %d listed twice", mb);
    if (p2_mode == TBP_P2_KCONCAT && i > 0 && mb != mbs[i - 1] + 1)
      return fail(TBP_EINVAL, "KCONCAT needs ascending consecutive micro-batches (got %d after %d)", mb, mbs[i - 1]);
  }
  for (int i = 0; i < n_mbs; i++)            // then the state of every member: the set is taken whole or not at all
    if (st->state[mbs[i]] != MB_P1)
      return fail(TBP_ESTATE, "backward_p2: micro-batch %d has not finished backward_p1", mbs[i]);
  tbp_status r = run_p2(st, mbs, n_mbs, p2_mode, accumulate, static_cast<hipStream_t>(stream));
  if (r != TBP_OK) return r;
  for (int i = 0; i < n_mbs; i++) {
    st->state[mbs[i]] = MB_EMPTY;
    st->w_live -= st->y.w_fwd_bytes_per_mb + st->y.w_p1_bytes_per_mb;
  }
  return TBP_OK;
}

tbp_status tbp_stage_stash_stats(const tbp_stage* st, tbp_stash_stats* out) {
  if (!st || !out) return fail(TBP_EINVAL, "stage and out must be non-null");
  out->w_live_bytes = st->w_live;
  out->a_live_bytes = st->a_live;
  out->high_water_bytes = st->high;
  return TBP_OK;
}

tbp_status tbp_stage_reset(tbp_stage* st) {
  if (!st) return fail(TBP_EINVAL, "stage is null");
  st->state.assign(st->c.Mmax, MB_EMPTY);
  st->slot_of.assign(st->c.Mmax, -1);
  st->free_slots.clear();
  for (int i = st->c.slots - 1; i >= 0; i--) st->free_slots.push_back(i);
  st->w_live = st->a_live = st->high = 0;
  return TBP_OK;
}

// ---- single operations -------------------------------------------------------------------------------
static int vecq(int dtype) { return dtype == TBP_BF16 ? 8 : 4; }
static tbp_status check_dtype(int dtype) {
  return (dtype == TBP_F32 || dtype == TBP_BF16) ? TBP_OK : fail(TBP_EINVAL, "dtype must be TBP_F32 or TBP_BF16");
}

size_t tbp_gemm_workspace_bytes(int dtype, int layout, int M, int N, int K, int out_f32) {
  if (M <= 0 || N <= 0 || K <= 0 || layout < 0 || layout > 2) return 0;
  return tbp::gemm_split_plan(dtype, layout, M, N, K, out_f32, 1).bytes;
}

tbp_status tbp_gemm(int dtype, int layout, int M, int N, int K, float alpha, const void* A, int lda, const void* B,
                    int ldb, void* C, int ldc, int out_f32, int accumulate, const void* R, void* stream) {
  return tbp_gemm_ws(dtype, layout, M, N, K, alpha, A, lda, B, ldb, C, ldc, out_f32, accumulate, R, nullptr, 0, stream);
}

tbp_status tbp_gemm_ws(int dtype, int layout, int M, int N, int K, float alpha, const void* A, int lda, const void* B,
                       int ldb, void* C, int ldc, int out_f32, int accumulate, const void* R, void* workspace,
                       size_t workspace_bytes, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (layout < 0 || layout > 2) return fail(TBP_EINVAL, "layout must be 0 (NN), 1 (NT) or 2 (TN)");
  if (M < 0 || N < 0 || K < 0) return fail(TBP_EINVAL, "negative size");
  if (M == 0 || N == 0) return TBP_OK;
  if (!C || (K > 0 && (!A || !B))) return fail(TBP_EINVAL, "A, B, C must be non-null");
  const int a_cols = layout == tbp::TN ? M : K, b_cols = layout == tbp::NT ? K : N;
  if (lda < a_cols || ldb < b_cols || ldc < N) return fail(TBP_EINVAL, "leading dimension smaller than the row length");
  if (dtype == TBP_BF16) {
    if (a_cols % 8 || b_cols % 8 || lda % 8 || ldb % 8)
      return fail(TBP_EINVAL, "bf16 operands need contiguous extents and leading dimensions that are multiples of 8");
    if ((uintptr_t)A % 16 || (uintptr_t)B % 16 || (uintptr_t)C % 16 || (R && (uintptr_t)R % 16))
      return fail(TBP_EINVAL, "bf16-path operands, output and residual must be 16-byte aligned");
    if (N % 8 || ldc % 8) return fail(TBP_EINVAL, "bf16 path needs N and ldc to be multiples of 8");
    // (a tile's 256 rows are addressed through a 31-bit buffer range)
    if (lda >= (1 << 22) || ldb >= (1 << 22)) return fail(TBP_EINVAL, "bf16 path needs leading dimensions below 2^22 elements");
  }
  if (dtype == TBP_F32) out_f32 = 1;
  if (accumulate && !out_f32) return fail(TBP_EINVAL, "accumulate needs an fp32 output");
  if (R && out_f32 && dtype == TBP_BF16) return fail(TBP_EINVAL, "residual is only added to storage-type outputs");
  tbp::GemmArgs g = gemm_args(layout, M, N, K, A, lda, B, ldb, C, ldc);
  g.alpha = alpha; g.out_f32 = out_f32; g.accumulate = accumulate; g.R = R;
  if (workspace) {
    if ((uintptr_t)workspace % 256) return fail(TBP_EINVAL, "workspace must be 256-byte aligned");
    g.ws = workspace; g.ws_bytes = workspace_bytes; g.ws_counters_zero = 0;     // a caller's buffer: cleared here
  }
  TBP_HIP(tbp::gemm(dtype, g, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_attention_fwd(int dtype, int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv,
                             int ld_qkv, void* out, int ld_out, float* lse, void* stream) {
  if (dtype != TBP_BF16) return fail(TBP_EINVAL, "fused attention is built for bf16 storage only");
  if (head_dim != 64 && head_dim != 128) return fail(TBP_EINVAL, "fused attention needs head_dim 64 or 128");
  if (batch < 0 || n_heads < 0 || seq < 0) return fail(TBP_EINVAL, "negative size");
  if (batch == 0 || n_heads == 0 || seq == 0) return TBP_OK;
  if (!qkv || !out || !lse) return fail(TBP_EINVAL, "qkv, out and lse must be non-null");
  if (ld_qkv < 3 * n_heads * head_dim || ld_out < n_heads * head_dim || ld_qkv % 8 || ld_out % 8)
    return fail(TBP_EINVAL, "leading dimensions must cover the head columns and be multiples of 8");
  if ((uintptr_t)qkv % 16 || (uintptr_t)out % 16) return fail(TBP_EINVAL, "qkv and out must be 16-byte aligned");
  // (the kernels address one sequence's rows through a 32-bit buffer range)
  if ((long)seq * ld_qkv * 2 >= (1L << 32)) return fail(TBP_EINVAL, "seq * ld_qkv too large: a sequence's rows must span less than 4 GiB");
  if (seq % 8) return fail(TBP_EINVAL, "seq must be a multiple of 8");
  if (seq > tbp::kMaxSeq) return fail(TBP_EINVAL, "seq %d above the limit %d", seq, tbp::kMaxSeq);
  TBP_HIP(tbp::attention_fwd(batch, n_heads, seq, head_dim, causal ? 1 : 0, qkv, ld_qkv, out, ld_out, lse,
                             static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

size_t tbp_attention_p1_scratch_bytes(int batch, int n_heads, int seq) {
  if (batch <= 0 || n_heads <= 0 || seq <= 0) return 0;
  return align_up((size_t)batch * seq * n_heads * sizeof(float), 256) + (size_t)batch * n_heads * tbp::attn_ds_elems(seq) * 2;
}

static tbp_status attention_p1_checked(int dtype, int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv,
                                       int ld_qkv, const void* out, const void* d_out, int ld_out, const float* lse, void* dqkv,
                                       int ld_dqkv, void* scratch, int recompute, void* stream) {
  if (dtype != TBP_BF16) return fail(TBP_EINVAL, "fused attention is built for bf16 storage only");
  if (head_dim != 64 && head_dim != 128) return fail(TBP_EINVAL, "fused attention needs head_dim 64 or 128");
  if (batch < 0 || n_heads < 0 || seq < 0) return fail(TBP_EINVAL, "negative size");
  if (batch == 0 || n_heads == 0 || seq == 0) return TBP_OK;
  if (!qkv || !out || !d_out || !lse || !dqkv || !scratch) return fail(TBP_EINVAL, "null pointer");
  const int d = n_heads * head_dim;
  if (ld_qkv < 3 * d || ld_dqkv < 3 * d || ld_qkv % 8 || ld_dqkv % 8) return fail(TBP_EINVAL, "leading dimensions must cover 3*n_heads*head_dim and be multiples of 8");
  if (ld_out != d) return fail(TBP_EINVAL, "out and d_out must be dense [batch*seq, n_heads*head_dim]");
  if ((long)seq * ld_qkv * 2 >= (1L << 32) || (long)seq * ld_dqkv * 2 >= (1L << 32))
    return fail(TBP_EINVAL, "seq * leading dimension too large: a sequence's rows must span less than 4 GiB");
  if (seq % 8) return fail(TBP_EINVAL, "seq must be a multiple of 8");
  if (seq > tbp::kMaxSeq) return fail(TBP_EINVAL, "seq %d above the limit %d", seq, tbp::kMaxSeq);
  if ((uintptr_t)qkv % 16 || (uintptr_t)out % 16 || (uintptr_t)d_out % 16 || (uintptr_t)dqkv % 16 || (uintptr_t)scratch % 256)
    return fail(TBP_EINVAL, "tensors must be 16-byte aligned, scratch 256-byte aligned");
  float* delta = static_cast<float*>(scratch);
  void* ds_t = recompute ? nullptr : static_cast<char*>(scratch) + align_up((size_t)batch * seq * n_heads * sizeof(float), 256);
  TBP_HIP(tbp::attention_p1(batch, n_heads, seq, head_dim, causal ? 1 : 0, qkv, ld_qkv, out, d_out, ld_out, lse, dqkv,
                            ld_dqkv, delta, ds_t, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_attention_p1(int dtype, int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv,
                            int ld_qkv, const void* out, const void* d_out, int ld_out, const float* lse, void* dqkv,
                            int ld_dqkv, void* scratch, void* stream) {
  return attention_p1_checked(dtype, batch, n_heads, seq, head_dim, causal, qkv, ld_qkv, out, d_out, ld_out, lse, dqkv,
                              ld_dqkv, scratch, 0, stream);
}

size_t tbp_attention_p1_recompute_scratch_bytes(int batch, int n_heads, int seq) {
  if (batch <= 0 || n_heads <= 0 || seq <= 0) return 0;
  return align_up((size_t)batch * seq * n_heads * sizeof(float), 256);
}

tbp_status tbp_attention_p1_recompute(int dtype, int batch, int n_heads, int seq, int head_dim, int causal,
                                      const void* qkv, int ld_qkv, const void* out, const void* d_out, int ld_out,
                                      const float* lse, void* dqkv, int ld_dqkv, void* scratch, void* stream) {
  return attention_p1_checked(dtype, batch, n_heads, seq, head_dim, causal, qkv, ld_qkv, out, d_out, ld_out, lse, dqkv,
                              ld_dqkv, scratch, 1, stream);
}

tbp_status tbp_mfma_ceiling(int blocks, int iters, const void* seed, float* sink, void* stream) {
  if (blocks < 1 || blocks > 65536 || iters < 0 || !seed || !sink) return fail(TBP_EINVAL, "bad mfma ceiling arguments");
  TBP_HIP(tbp::mfma_ceiling(blocks, iters, seed, sink, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_rmsnorm_fwd(int dtype, int rows, int d, float eps, const void* x, const void* g, void* y, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || d < 1 || d % vecq(dtype) || d > tbp::max_d_model(dtype)) return fail(TBP_EINVAL, "bad rows / d");
  if (rows == 0) return TBP_OK;
  if (!x || !g || !y) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::rmsnorm_fwd(dtype, rows, d, eps, x, g, y, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

size_t tbp_rmsnorm_p1_scratch_bytes(int d) { return d > 0 ? (size_t)tbp::kNormPartialBlocks * d * sizeof(float) : 0; }

int tbp_rmsnorm_partial_rows(int dtype, int rows, int d) {
  if ((dtype != TBP_F32 && dtype != TBP_BF16) || d < 1 || d > tbp::max_d_model(dtype)) return 0;
  return tbp::rmsnorm_partial_rows(dtype, rows, d);
}

tbp_status tbp_rmsnorm_p1_partials(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                                   const void* resid, void* dx, float* partials_out, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || d < 1 || d % vecq(dtype) || d > tbp::max_d_model(dtype)) return fail(TBP_EINVAL, "bad rows / d");
  if (rows == 0) return TBP_OK;
  if (!g || !partials_out || !dy || !x || !dx) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::rmsnorm_p1_rows(dtype, rows, d, eps, dy, x, g, resid, dx, partials_out, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_gain_partials_sum(const float* partials, int n_rows, int d, int accumulate, float* dg_out, void* stream) {
  if (n_rows < 0 || d < 1) return fail(TBP_EINVAL, "bad n_rows / d");
  if (!dg_out || (n_rows > 0 && !partials)) return fail(TBP_EINVAL, "null pointer");
  if (n_rows == 0 && accumulate) return TBP_OK;
  TBP_HIP(tbp::gain_partials_sum(partials, n_rows, d, accumulate ? 1 : 0, dg_out, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_rmsnorm_p1(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                          const void* resid, void* dx, float* dg_out, void* scratch, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || d < 1 || d % vecq(dtype) || d > tbp::max_d_model(dtype)) return fail(TBP_EINVAL, "bad rows / d");
  if (!g || !dg_out || !scratch || (rows > 0 && (!dy || !x || !dx))) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::rmsnorm_p1(dtype, rows, d, eps, dy, x, g, resid, dx, dg_out, (float*)scratch, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

// ---- the entry point that allocates nothing ---------------------------------------------------------------------
// Scratch of tbp_rmsnorm_p1_static: the row-block partials of the gain gradient, kNormPartialBlocks rows of up to
// max_d_model(bf16) fp32 columns (8 MiB), resident on every GPU the library runs on until the process ends.  In host
// code the array's name is only a stand-in for the symbol: its device address is asked for once per device
// (hipGetSymbolAddress with that device current) and kept in g_static_scratch[device]; only that pointer is ever
// handed to a kernel.
constexpr size_t kStaticScratchFloats = (size_t)tbp::kNormPartialBlocks * 8192;
static __device__ __align__(256) float scratch[kStaticScratchFloats];
constexpr int kMaxDevices = 64;
static std::atomic<float*> g_static_scratch[kMaxDevices];

static tbp_status static_scratch(float** out) {
  int dev = -1;
  TBP_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(TBP_EDEVICE, "device index %d outside 0..%d", dev, kMaxDevices - 1);
  float* p = g_static_scratch[dev].load(std::memory_order_acquire);
  if (!p) {           // first call on this device (two threads racing here both obtain the same address)
    void* sym = nullptr;
    TBP_HIP(hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)));
    if (!sym) return fail(TBP_EDEVICE, "hipGetSymbolAddress returned a null address for the static scratch");
    p = static_cast<float*>(sym);
    g_static_scratch[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return TBP_OK;
}

tbp_status tbp_rmsnorm_p1_static(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                                 const void* resid, void* dx, float* dg_out, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || d < 1 || d % vecq(dtype)) return fail(TBP_EINVAL, "bad rows / d");
  if (d > tbp::max_d_model(dtype) || (size_t)tbp::kNormPartialBlocks * d > kStaticScratchFloats)
    return fail(TBP_EINVAL, "d = %d is above the %d columns (%s) the static scratch of %zu bytes is built for", d,
                tbp::max_d_model(dtype), dtype == TBP_BF16 ? "bf16" : "f32", kStaticScratchFloats * sizeof(float));
  if (!g || !dg_out || (rows > 0 && (!dy || !x || !dx))) return fail(TBP_EINVAL, "null pointer");
  float* part = nullptr;
  const tbp_status r = static_scratch(&part);
  if (r != TBP_OK) return r;
  // nothing in the scratch has to start at zero: the row kernel writes every partial row that the column sum then reads
  TBP_HIP(tbp::rmsnorm_p1(dtype, rows, d, eps, dy, x, g, resid, dx, dg_out, part, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_rmsnorm_gain_p2(int dtype, int rows, int d, float eps, const void* dy, const void* x, int accumulate,
                               float* dg_out, void* scratch, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || d < 1 || d % vecq(dtype) || d > tbp::max_d_model(dtype)) return fail(TBP_EINVAL, "bad rows / d");
  if (!dg_out || !scratch || (rows > 0 && (!dy || !x))) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::rmsnorm_gain_p2(dtype, rows, d, eps, dy, x, accumulate ? 1 : 0, dg_out, (float*)scratch,
                               static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_swiglu_fwd(int dtype, int rows, int f, const void* gu, void* m, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || f < 1 || f % vecq(dtype)) return fail(TBP_EINVAL, "bad rows / f");
  if (rows == 0) return TBP_OK;
  if (!gu || !m) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::swiglu_fwd(dtype, rows, f, gu, m, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_swiglu_p1(int dtype, int rows, int f, const void* dm, const void* gu, void* dgu, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (rows < 0 || f < 1 || f % vecq(dtype)) return fail(TBP_EINVAL, "bad rows / f");
  if (rows == 0) return TBP_OK;
  if (!dm || !gu || !dgu) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::swiglu_p1(dtype, rows, f, dm, gu, dgu, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

size_t tbp_rope_table_bytes(int seq, int head_dim) {
  return (seq > 0 && head_dim > 1) ? (size_t)seq * (head_dim / 2) * sizeof(float2) : 0;
}

tbp_status tbp_rope_table(int seq, int head_dim, float base, void* table, void* stream) {
  if (seq < 1 || head_dim < 2 || head_dim % 2 || !(base > 0.f) || !table) return fail(TBP_EINVAL, "bad rope table arguments");
  TBP_HIP(tbp::rope_table(seq, head_dim, base, (float2*)table, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_rope(int dtype, int rows, int seq, int n_heads, int head_dim, int ld, const void* table, int inverse,
                    void* x, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  const int q = vecq(dtype);
  if (rows < 0 || seq < 1 || n_heads < 0 || head_dim < 2 || head_dim % (2 * q) || ld < n_heads * head_dim || ld % q)
    return fail(TBP_EINVAL, "bad rope arguments");
  if (rows == 0 || n_heads == 0) return TBP_OK;
  if (!table || !x) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::rope(dtype, rows, seq, n_heads, head_dim, ld, (const float2*)table, inverse, x, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_softmax_fwd(int dtype, int n_mat, int seq, int causal, const float* scores, void* P, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (n_mat < 0 || seq < 1 || seq % vecq(dtype) || seq % 4 || seq > tbp::kMaxSeq) return fail(TBP_EINVAL, "bad n_mat / seq");
  if (n_mat == 0) return TBP_OK;
  if (!scores || !P) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::softmax_fwd(dtype, (long)n_mat * seq, seq, causal, scores, P, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

tbp_status tbp_softmax_p1(int dtype, int n_mat, int seq, int causal, const void* P, void* dP_dS, void* stream) {
  if (check_dtype(dtype) != TBP_OK) return TBP_EINVAL;
  if (n_mat < 0 || seq < 1 || seq % vecq(dtype) || seq > tbp::kMaxSeq) return fail(TBP_EINVAL, "bad n_mat / seq");
  if (n_mat == 0) return TBP_OK;
  if (!P || !dP_dS) return fail(TBP_EINVAL, "null pointer");
  TBP_HIP(tbp::softmax_p1(dtype, (long)n_mat * seq, seq, causal, P, dP_dS, static_cast<hipStream_t>(stream)));
  return TBP_OK;
}

}  // extern "C"
