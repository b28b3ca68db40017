// Internal launch interface between the stage executor and the gfx950 kernels.
// Nothing here is part of the public C ABI (see include/tbp.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tbp {

enum Layout { NN = 0, NT = 1, TN = 2 };

// How a product that involves the causal probability matrix restricts its work.  Rows of the
// probability (and score-gradient) matrices are zero-filled from the diagonal to the next multiple
// of kCausalPad columns, which is what lets whole K-tiles be skipped safely.
enum Causal {
  CAUSAL_NONE = 0,
  CAUSAL_SKIP_UPPER = 1,  // output [S,S] tiles strictly above the diagonal are not computed (q k^T, do v^T)
  CAUSAL_K_END = 2,       // A = P or dS [S,S]: contraction stops at the end of the row tile (P v, dS k)
  CAUSAL_K_BEGIN = 3      // A = P^T or dS^T:   contraction starts at the row tile's first index (P^T do, dS^T q)
};
constexpr int kCausalPad = 256;

struct GroupedProduct;
struct GemmArgs {
  int layout;            // Layout
  int M, N, K;
  float alpha;
  const void* A; long lda;
  const void* B; long ldb;
  void* C; long ldc;
  const void* R;         // optional residual added before rounding (storage-type output only), same ld as C
  int out_f32;           // C is fp32
  int accumulate;        // C += (fp32 output only)
  int batch;             // grid z; z -> (zo = z / batch_inner, zi = z % batch_inner)
  int batch_inner;
  long sAo, sAi, sBo, sBi, sCo, sCi;   // element strides of the outer / inner batch index
  int causal;            // Causal
  // Softmax backward fused into the epilogue of dP = do v^T (per-head batched product with a storage-type output):
  // when delta is set, R points at the probabilities P (same layout as C) and the kernel stores
  // dS = P * (alpha * acc - delta[row]) for columns <= row and exact zeros above the diagonal (causal) instead of dP.
  // delta[(zo * sDo + zi * sDi) + row * ldd] = rowsum(dP * P) = sum over the head's columns of do * o.
  const float* delta; long ldd, sDo, sDi;
  int delta_causal;
  // Optional scratch for products whose output has too few large tiles to fill the chip (see gemm_split_plan):
  // device memory of at least gemm_split_plan(...).bytes bytes, 256-byte aligned.  Its first kSplitCounterBytes hold
  // per-tile arrival counters that must be zero when a product starts and are zero again when it ends;
  // ws_counters_zero = 0 makes gemm() clear them first (a small fill launch).
  void* ws; size_t ws_bytes;
  int ws_counters_zero;
  // TN layout, storage-type operands only: A is stored in panels of kPanel output rows, element (k, m) at
  // A[(m / kPanel) * a_panel + k * lda + m % kPanel] with lda == kPanel, so that the K x kPanel slab an output tile
  // contracts over is one contiguous stream.  0: plain [K, lda] matrix.  Such a product runs on kPanel-wide tiles.
  long a_panel;
  // Weight-gradient products (TN layout, bf16 storage, fp32 C, alpha = 1) whose tiles do not fill whole rounds of the
  // 256 compute units: when set, gemm() launches only the part of the output that makes whole rounds of large tiles
  // and describes the remainder in *defer_rest (M = 0 there: nothing was held back) instead of launching it on
  // smaller tiles.  The caller collects the remainders of several products and runs them as one gemm_tn_grouped
  // launch, in which they fill rounds together.
  GroupedProduct* defer_rest;
};
constexpr int kPanel = 128;
// elements of one (sequence, head) entry of the fused attention's dS^T scratch, stored in such panels
constexpr size_t attn_ds_elems(int seq) { return (size_t)((seq + kPanel - 1) / kPanel) * seq * kPanel; }

// Split of the contraction over several workgroups per output tile.  An output with fewer than 192 tiles of
// 256 x 256 leaves compute units idle (or falls back to small tiles that move twice the operand bytes per FLOP);
// with `split` workgroups per tile, each summing a slice of the contraction into fp32 partials in the scratch buffer,
// the chip is full again.  The workgroup that arrives last at a tile adds the partials up in slice order (so the result
// does not depend on arrival order), and runs the ordinary epilogue.  split == 1: not worth it / not applicable.
struct SplitPlan { int split; size_t bytes; };
constexpr size_t kSplitCounterBytes = 1024;
SplitPlan gemm_split_plan(int dtype, int layout, int M, int N, int K, int out_f32, int batch);

inline GemmArgs gemm_args(int layout, int M, int N, int K, const void* A, long lda, const void* B, long ldb,
                          void* C, long ldc) {
  GemmArgs g{};
  g.layout = layout; g.M = M; g.N = N; g.K = K; g.alpha = 1.f;
  g.A = A; g.lda = lda; g.B = B; g.ldb = ldb; g.C = C; g.ldc = ldc;
  g.batch = 1; g.batch_inner = 1;
  return g;
}

// dtype: 0 = fp32 storage, 1 = bf16 storage (matches tbp_dtype).
hipError_t gemm(int dtype, const GemmArgs& g, hipStream_t s);

// Several bf16 weight-gradient products C (=, +=) A^T B (TN layout, fp32 C, alpha = 1) run as ONE launch.
// Same operand rules as the bf16 TN product of gemm(): 16-byte aligned pointers, extents and leading dimensions
// multiples of 8.
struct GroupedProduct {
  const void* A; const void* B; float* C;     // A [K, M] (lda), B [K, N] (ldb), C [M, N] (ldc)
  int M, N, K;
  int lda, ldb, ldc;
  int accumulate;
};
constexpr int kMaxGrouped = 40;               // products per launch (the table travels as a kernel argument)
struct GroupedTable {
  int n;
  int first_block[kMaxGrouped];
  GroupedProduct prod[kMaxGrouped];
};
hipError_t gemm_tn_grouped(const GroupedProduct* prods, int n, hipStream_t s);

hipError_t rmsnorm_fwd(int dtype, int rows, int d, float eps, const void* x, const void* g, void* y, hipStream_t s);
constexpr int kNormPartialBlocks = 256;     // at most this many row-block partials of the gain gradient per call
// RMSNorm backward-p1.  The gain gradient dg = sum over rows of dy * x * r leaves the row kernel as
// rmsnorm_partial_rows(dtype, rows, d) <= kNormPartialBlocks partial rows [d] fp32 (one per workgroup, each a sum over
// that workgroup's rows in a fixed order); gain_partials_sum adds partial rows up.
int rmsnorm_partial_rows(int dtype, int rows, int d);
// dx = resid + dL/dx; partials (may be null: nothing is computed for the gain) receives the partial rows.
hipError_t rmsnorm_p1_rows(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                           const void* resid, void* dx, float* partials, hipStream_t s);
// out[d] (= or +=) sum of the first n_rows rows of partials [n_rows][d]  (n_rows == 0: zero, or out left alone)
hipError_t gain_partials_sum(const float* partials, int n_rows, int d, int accumulate, float* out, hipStream_t s);
// Both in one call: rows, then the sum into dg_out (dg_out == nullptr: nothing is computed for the gain).
hipError_t rmsnorm_p1(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                      const void* resid, void* dx, float* dg_out, float* partials, hipStream_t s);
hipError_t rmsnorm_gain_p2(int dtype, int rows, int d, float eps, const void* dy, const void* x, int accumulate,
                           float* dg_out, float* partials, hipStream_t s);
hipError_t swiglu_fwd(int dtype, int rows, int f, const void* gu, void* m, hipStream_t s);
hipError_t swiglu_p1(int dtype, int rows, int f, const void* dm, const void* gu, void* dgu, hipStream_t s);
hipError_t rope_table(int seq, int head_dim, float base, float2* table, hipStream_t s);
hipError_t rope(int dtype, int rows, int seq, int n_heads, int head_dim, long ld, const float2* table, int inverse,
                void* x, hipStream_t s);
hipError_t softmax_fwd(int dtype, long n_rows_total, int seq, int causal, const float* scores, void* P, hipStream_t s);
hipError_t softmax_p1(int dtype, long n_rows_total, int seq, int causal, const void* P, void* dP, hipStream_t s);
// delta[t * n_heads + h] = sum_c a[t, h*dh + c] * b[t, h*dh + c]   (fp32; a, b are [rows, n_heads*head_dim])
hipError_t head_rowdot(int dtype, int rows, int n_heads, int head_dim, const void* a, const void* b, float* delta,
                       hipStream_t s);
// Fused attention (bf16 storage only, head_dim 64 or 128).  qkv: [batch*seq, ld_qkv] with column blocks q | k | v of
// n_heads*head_dim each (q and k already rotated); out: [batch*seq, ld_out]; lse: [batch, n_heads, seq] fp32, the log2
// of each row's sum of exp2(score / sqrt(head_dim) * log2 e).
hipError_t attention_fwd(int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv, long ld_qkv,
                         void* out, long ld_out, float* lse, hipStream_t s);

// Backward-p1 of the same: dq, dk, dv into the column blocks of dqkv from qkv, the forward's output and lse and the
// output derivative d_out (dense rows: ld_out == n_heads*head_dim).  delta: scratch [batch*seq, n_heads] fp32;
// ds_t: scratch of batch * n_heads * attn_ds_elems(seq) storage-type elements (receives dS^T in panels of kPanel
// queries: per (sequence, head) [ceil(seq / kPanel)][seq keys][kPanel queries]; dq is then one batched product
// dS K), or nullptr: dq is computed by a second pass over the keys that rebuilds S and dP (no dS^T anywhere).
hipError_t attention_p1(int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv, long ld_qkv,
                        const void* out, const void* d_out, long ld_out, const float* lse, void* dqkv, long ld_dqkv,
                        float* delta, void* ds_t, hipStream_t s);

// Register-resident MFMA loop (measurement aid): blocks x 4 waves x iters x 16 MFMAs of 32x32x16.
// seed: 8 x 64 x 8 bf16 values; sink: blocks * 256 floats.
hipError_t mfma_ceiling(int blocks, int iters, const void* seed, float* sink, hipStream_t s);

// A kernel that wants more than 64 KiB of dynamic LDS must be told so once per DEVICE (the attribute belongs to the
// kernel's image on that device).  One instance per kernel instantiation; racing threads repeat a harmless call.
struct AttrOnce {
  static constexpr int kMaxDev = 64;
  bool done[kMaxDev] = {};
  hipError_t set(const void* kern, size_t smem) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < kMaxDev && done[dev]) return hipSuccess;
    e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess && dev >= 0 && dev < kMaxDev) done[dev] = true;
    return e;
  }
};

// Limits enforced by the host before any launch.
inline int max_d_model(int dtype) { return dtype == 1 ? 8192 : 4096; }
constexpr int kMaxSeq = 4096;

}  // namespace tbp
