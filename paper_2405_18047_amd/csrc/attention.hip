// Fused scaled-dot-product attention for gfx950 (bf16 storage, fp32 accumulation, head_dim 64 or 128): the forward
// keeps neither scores nor probabilities, only the log-sum-exp of every row; backward-p1 recomputes the
// probabilities from it.  Attention is one of the operations with no backward-p2 and a significant backward-p1
// (Section 4.1), so everything here is on the critical path of the pipeline.
//
// Orientation.  With the 32x32x16 MFMA an accumulator lane owns ONE column and 16 rows of a 32x32 tile.  The
// kernels arrange every product so that the softmax row statistics belong to the lane's column:
//   forward, dQ pass   S^T = K Q^T   (column = query): row max / row sum of a query are a reduction over the lane's own
//                      registers plus one exchange with lane ^ 32; the running rescale of the output is a per-lane
//                      scalar;
//   dK/dV pass         S   = Q K^T   (column = key), the statistics come from memory (one value per register row).
// In both cases the probabilities (and score gradients) leave the accumulators straight into the B operand of the next
// product: B lane (column c, half g) wants 8 contraction indices, and accumulator registers 8u .. 8u+7 of the
// lane are rows 16u + {0..3, 8..11} + 4g of its column, so k-step u of the next product simply DEFINES its
// contraction order to be that row order and the A operand is fetched in the same order (transpose reads of four
// consecutive rows at 16u + 4g and at 16u + 8 + 4g).  No shuffles, no LDS round trip for P.
#include "kernels.h"
#include "gfx950.h"

namespace tbp {

struct AttnParams {
  const bf16_t* qkv; long ld_qkv;      // [B*S, >= 3*H*DH]: q | k | v column blocks of H*DH each
  bf16_t* out; long ld_out;            // [B*S, >= H*DH]
  float* lse;                          // [B, H, S]: log2 of the row's sum of exp2(score * scale * log2 e)
  int B, H, S, causal;
  float scale_log2e;
};

// LDS image of `rows` x DH bf16, filled by asynchronous copies (a wave-wide copy writes 1 KiB = 4 or 8 rows).
// The 16-byte granule G of row r sits in slot G ^ swz(r).  swz is a bit permutation of the row index chosen so that
// both access patterns are free of bank conflicts: 16 consecutive rows at one granule (row fragments, ds_read_b128)
// and 4 consecutive rows x 2 adjacent granules (transpose fragments, ds_read_b64_tr_b16).
template <int DH>
struct HeadTile {
  static constexpr int RB = DH * 2, GPRW = DH / 8, RPC = 1024 / RB;
  static __device__ __forceinline__ int swz(int r) {
    if constexpr (DH == 128) return ((r & 3) << 1) | ((r >> 2) & 1) | (r & 8);
    else return (((r >> 1) & 1) << 1) | ((r >> 2) & 1) | (((r >> 3) & 1) << 2);
  }
  static __device__ __forceinline__ int at(int r, int G) { return r * RB + ((G ^ swz(r)) << 4); }
  // Copy plan of lane p of chunk c: tile row and byte offset inside the source row block.
  static __device__ __forceinline__ void plan(int c, int p, long ld, int& row, unsigned& goff) {
    row = RPC * c + p / GPRW;
    const int G = (p % GPRW) ^ swz(row);
    goff = (unsigned)((long)row * ld * 2 + G * 16);
  }
  // Per-lane byte offsets of the fragment reads, computed once per kernel (the swizzle makes them non-affine in the
  // k-step, so they are kept in registers; everything else - image, 32-row block, k-step pair - is an immediate).
  //   rows[s]: A-operand fragment of MFMA rows 0..31 of the image, contraction = columns 16 s .. 16 s + 15.
  //   cols[t][0/1]: A-operand fragment of the TRANSPOSED image: MFMA rows = columns 32 t .. 32 t + 31, contraction =
  //            image rows 16 u + {0..3} + 4 (lane / 32) (first read) and 16 u + 8 + {0..3} + 4 (lane / 32) (second):
  //            the accumulator row order, see the file header.  16 u rows further is an immediate too.
  struct Offsets { int rows[DH / 16]; int cols[DH / 32][2]; };
  static __device__ __forceinline__ Offsets offsets(int lane) {
    Offsets o;
#pragma unroll
    for (int s = 0; s < DH / 16; s++) o.rows[s] = at(lane & 31, 2 * s + (lane >> 5));
    const int i = lane & 15, q = (lane >> 4) & 1, g = lane >> 5;
    const int r = 4 * g + (i >> 2);
#pragma unroll
    for (int t = 0; t < DH / 32; t++) {
      const int G = 2 * (2 * t + q) + ((i & 3) >> 1);
      o.cols[t][0] = at(r, G) + 8 * (i & 1);
      o.cols[t][1] = at(r + 8, G) + 8 * (i & 1);
    }
    return o;
  }
  static __device__ __forceinline__ bf16x8 rows_frag(lds_u8* img, const Offsets& o, int r0, int s) {   // r0 % 16 == 0
    return *reinterpret_cast<LDS_AS const bf16x8*>(img + o.rows[s] + r0 * RB);
  }
  static __device__ __forceinline__ bf16x8 cols_frag(lds_u8* img, const Offsets& o, int r0, int u, int t) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(img + o.cols[t][0] + (r0 + 16 * u) * RB));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(img + o.cols[t][1] + (r0 + 16 * u) * RB));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

__device__ __forceinline__ float xor32(float v) { return __shfl_xor(v, 32, 64); }

__device__ __forceinline__ bf16x8 pack8(const f32x16& c, int u) {
  bf16x8 b;
#pragma unroll
  for (int t = 0; t < 8; t++) b[t] = (bf16_t)c[8 * u + t];
  return b;
}

// ------------------------------------------------------------------------------------------ forward
// One workgroup = 4 waves x 32 queries of one (sequence, head); keys and values stream through LDS in blocks of 64,
// double-buffered.  Per block and wave: S^T (64 keys x 32 queries), online softmax per lane, O^T += V^T P^T.
template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_kernel(AttnParams p) {
  using HT = HeadTile<DH>;
  constexpr int KS = DH / 16, DT = DH / 32, BKV = 64;
  constexpr int IMG = BKV * HT::RB, SLOT = 2 * IMG;
  constexpr int NCH = IMG / 1024 / 4;                 // copies per wave per operand per block

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  lds_u8* const lds = LDS_PTR(unsigned char, smem_raw);
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

  const int lane = threadIdx.x & 63, ql = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  // workgroup ids run over (head, sequence) fastest and query blocks slowest, longest (last) query blocks first: with
  // causal masking the work of a block grows with its index, and the blocks still to start near the end are short ones
  const int qb = (int)gridDim.y - 1 - (int)blockIdx.y;
  const int h = (int)blockIdx.x % p.H, b = (int)blockIdx.x / p.H;
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, query = qw0 + ql;
  const int d = p.H * DH;
  const long tok0 = (long)b * p.S;

  const typename HT::Offsets fo = HT::offsets(lane);
  // ---- the block's 128 query rows: copied (coalesced) into the second slot, which the loop fills only after its first
  // barrier; fetched per lane they would be 32-byte pieces of 32 rows per instruction
  {
    const u32x4 dq = make_desc(p.qkv + (tok0 + q0) * p.ld_qkv + h * DH, (uint32_t)((long)(p.S - q0) * p.ld_qkv * 2));
#pragma unroll
    for (int i = 0; i < 2 * NCH; i++) {
      int row; unsigned go;
      HT::plan(wave + 4 * i, lane, p.ld_qkv, row, go);
      dma16(lds0 + SLOT + (wave + 4 * i) * 1024, dq, q0 + row < p.S ? go : kOob);
    }
  }
  // ---- copy plan of this wave: chunks wave, wave + 4, ... of the K image and of the V image
  int c_row[NCH];
  unsigned c_off[NCH];
#pragma unroll
  for (int i = 0; i < NCH; i++) HT::plan(wave + 4 * i, lane, p.ld_qkv, c_row[i], c_off[i]);
  const int kv_end = p.causal ? (q0 + 128 < p.S ? q0 + 128 : p.S) : p.S;
  const int nblk = (kv_end + BKV - 1) / BKV;
  auto issue = [&](int j) {
    const int kv0 = j * BKV;
    const bf16_t* kb = p.qkv + (tok0 + kv0) * p.ld_qkv + d + h * DH;
    const uint32_t bytes = (uint32_t)((long)(p.S - kv0) * p.ld_qkv * 2);     // rows of this sequence only
    const u32x4 dk = make_desc(kb, bytes), dv = make_desc(kb + d, bytes);
    const uint32_t base = lds0 + (j & 1) * SLOT + wave * 1024;
#pragma unroll
    for (int i = 0; i < NCH; i++) {
      const unsigned off = (kv0 + c_row[i] < p.S) ? c_off[i] : kOob;
      dma16(base + i * 4096, dk, off);
      dma16(base + IMG + i * 4096, dv, off);
    }
  };

  f32x16 ot[DT];
#pragma unroll
  for (int t = 0; t < DT; t++)
#pragma unroll
    for (int e = 0; e < 16; e++) ot[t][e] = 0.f;
  float m = -INFINITY, l = 0.f;

  issue(0);
  wait_vmem<0>();
  __syncthreads();
  // ---- this lane's query row as B operand of S^T = K Q^T: 8 consecutive head-dim values per k-step
  bf16x8 qf[KS];
#pragma unroll
  for (int s = 0; s < KS; s++) qf[s] = HT::rows_frag(lds + SLOT, fo, 32 * wave, s);
  for (int j = 0; j < nblk; j++) {
    wait_vmem<0>();
    __syncthreads();                   // block j has landed; every wave is done with the other slot (and has its query row)
    if (j + 1 < nblk) issue(j + 1);
    const int kv0 = j * BKV;
    if (p.causal && kv0 > qw0 + 31) continue;          // every key of the block is after every query of this wave
    lds_u8* const kimg = lds + (j & 1) * SLOT;
    lds_u8* const vimg = kimg + IMG;
    // S^T for the two key tiles of the block as two interleaved accumulation chains (consecutive MFMAs are
    // independent), fragments fetched one k-step ahead
    f32x16 st[2];
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int e = 0; e < 16; e++) st[kt][e] = 0.f;
    {
      bf16x8 k0 = HT::rows_frag(kimg, fo, 0, 0), k1 = HT::rows_frag(kimg, fo, 32, 0);
#pragma unroll
      for (int s = 0; s < KS; s++) {
        bf16x8 n0 = k0, n1 = k1;
        if (s + 1 < KS) { n0 = HT::rows_frag(kimg, fo, 0, s + 1); n1 = HT::rows_frag(kimg, fo, 32, s + 1); }
        st[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0, qf[s], st[0], 0, 0, 0);
        st[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1, qf[s], st[1], 0, 0, 0);
        k0 = n0; k1 = n1;
      }
    }
    // keys beyond the query (causal) or beyond the sequence do not take part (blocks on the diagonal / at the end only)
    if ((p.causal && kv0 + BKV - 1 > qw0) || kv0 + BKV > p.S) {
      const int last = p.causal ? (query < p.S - 1 ? query : p.S - 1) : p.S - 1;      // last key this lane's query sees
      const int rel = last - kv0 - 4 * g;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int e = 0; e < 16; e++)
          st[kt][e] = (32 * kt + 8 * (e >> 2) + (e & 3) > rel) ? -INFINITY : st[kt][e];
    }
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int e = 0; e < 16; e++) mx = fmaxf(mx, st[kt][e]);
    mx = fmaxf(mx, xor32(mx)) * p.scale_log2e;          // scale > 0: the maximum commutes with it
    // The reference point m of the exponentials only has to stay within a safe distance of the running maximum, not
    // on it: o / l and lse = m + log2 l are the same for any m.  It is moved (and what is accumulated rescaled) only
    // when some query's maximum has risen by more than kSlack octaves above it; until then p <= 2^kSlack, far inside
    // the range of fp32 sums and of the storage type.  With the maximum itself as reference nearly every block moves
    // some lane's maximum and pays 16 * DT multiplications per lane; this way typically only the first block does.
    constexpr float kSlack = 8.f;
    const float mnew = fmaxf(m, mx);
    if (__any(mnew > m + kSlack)) {
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);    // first block: m = -inf, exp2(-inf) = 0
      l *= alpha;
#pragma unroll
      for (int t = 0; t < DT; t++)
#pragma unroll
        for (int e = 0; e < 16; e++) ot[t][e] *= alpha;
      m = mnew;
    }
    float rs = 0.f;
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int e = 0; e < 16; e++) {
        const float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(st[kt][e], p.scale_log2e, -m));
        st[kt][e] = pe;
        rs += pe;
      }
    l += rs + xor32(rs);
    // O^T += V^T P^T: 4 (kt, u) steps x DT independent accumulators, fragments one step ahead
    bf16x8 vf[DT];
#pragma unroll
    for (int t = 0; t < DT; t++) vf[t] = HT::cols_frag(vimg, fo, 0, 0, t);
#pragma unroll
    for (int ku = 0; ku < 4; ku++) {
      const bf16x8 pb = pack8(st[ku >> 1], ku & 1);
      bf16x8 nf[DT];
#pragma unroll
      for (int t = 0; t < DT; t++) nf[t] = ku < 3 ? HT::cols_frag(vimg, fo, 32 * ((ku + 1) >> 1), (ku + 1) & 1, t) : vf[t];
#pragma unroll
      for (int t = 0; t < DT; t++) ot[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t], pb, ot[t], 0, 0, 0);
#pragma unroll
      for (int t = 0; t < DT; t++) vf[t] = nf[t];
    }
  }

  // ---- o = O^T / l, transposed back on the way out.  A lane holds 4 consecutive head-dim values of its query per
  // register group (8 bytes, 32 rows per instruction if stored directly): each wave passes its 32 rows through LDS
  // (the ring is free after one more barrier; rows padded to DH * 2 + 16 bytes against bank conflicts) and writes them
  // whole, 16 bytes per lane.
  __syncthreads();
  constexpr int EROW = DH * 2 + 16;
  static_assert(128 * EROW <= 2 * SLOT, "the output tile must fit in the ring");
  lds_u8* const erow = lds + 32 * wave * EROW;
  {
    const float inv = 1.f / l;
#pragma unroll
    for (int t = 0; t < DT; t++)
#pragma unroll
      for (int e4 = 0; e4 < 4; e4++) {
        bf16x4 v;
#pragma unroll
        for (int r = 0; r < 4; r++) v[r] = (bf16_t)(ot[t][4 * e4 + r] * inv);
        *reinterpret_cast<LDS_AS bf16x4*>(erow + ql * EROW + (32 * t + 8 * e4 + 4 * g) * 2) = v;
      }
    if (g == 0 && query < p.S) p.lse[((long)b * p.H + h) * p.S + query] = m + __builtin_amdgcn_logf(l);
  }
  {  // (LDS operations of a wave execute in order: the reads below see this wave's own writes above)
    constexpr int LPR = DH / 8, RPI = 64 / LPR;
    const int rl = lane / LPR, piece = lane % LPR;
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPI) {
      const int qrow = qw0 + r0 + rl;
      if (qrow < p.S)
        *reinterpret_cast<u32x4*>(p.out + (tok0 + qrow) * p.ld_out + h * DH + 8 * piece) =
            *reinterpret_cast<const LDS_AS u32x4*>(erow + (r0 + rl) * EROW + 16 * piece);
    }
  }
}

// ------------------------------------------------------------------------------------------ backward-p1: dK, dV, dS^T
// One workgroup = 128 keys of one (sequence, head), 32 per wave pair; queries, their output derivatives and their row
// statistics stream through LDS in steps of 64 queries, three steps deep.  Per 32 queries and wave pair:
//   S = Q K^T and dP = dO V^T (column = key; K and V rows of the lane's key stay in registers as B operands),
//   P = exp2(S c - lse), dS = P (dP - delta), then dV^T += dO^T P and dK^T += Q^T dS with P and dS fed from the
//   accumulators (see the file header).  dS^T is also written out ([key][query], storage type): dQ = dS K is a
//   contraction over keys, which this kernel splits over workgroups, and is left to a batched product.
struct AttnBwdParams {
  const bf16_t* qkv; long ld_qkv;
  const bf16_t* dout; long ld_do;      // [B*S, >= H*DH] derivative of the attention output
  const float* lse;                    // [B, H, S] from the forward
  const float* delta;                  // [B*S, H]: rowsum(dout * out) per (token, head)
  bf16_t* dqkv; long ld_dqkv;          // dk and dv blocks are written (columns H*DH.. and 2*H*DH..)
  bf16_t* dst;                         // dS^T per (b, h) in panels of 128 queries: [ceil(S / 128)][S keys][128 queries]
  int B, H, S, causal;
  float scale, scale_log2e;
};

// The two kinds of work run on different waves.  A single wave issues in order: while it works through the ~200 vector
// instructions that turn S and dP into P and dS, the matrix pipe of its SIMD idles, and the other way round (a
// single-wave form of this kernel, software-pipelined three tiles deep, kept the matrix pipe 27 % busy and was 5 %
// slower).  A workgroup is 8 waves, two per SIMD, of which
//   waves 0..3 ("left")   compute S = Q K^T and dP = dO V^T for their 32 keys, then P and dS, write dS^T out and hand
//                         P and dS (already in B-operand form, 64 bytes per lane) over through LDS;
//   waves 4..7 ("right")  take P and dS of the previous tile from LDS and accumulate dV^T += dO^T P, dK^T += Q^T dS.
// The hardware interleaves the two instruction streams of a SIMD, so the vector work of one tile runs under the MFMAs
// of its neighbours.  One workgroup barrier per 32-query tile; the hand-over buffers and the query-step images are
// double / triple buffered so that neither side ever waits for the other beyond that barrier.  The right waves also
// issue all asynchronous copies (they have no other vector-memory operations, so their copy counter is exact).
template <int DH, bool WRITE_DST>
__global__ __launch_bounds__(512) void attn_bwd_kv_split_kernel(AttnBwdParams p) {
  using HT = HeadTile<DH>;
  constexpr int KS = DH / 16, DT = DH / 32, BQ = 64;
  constexpr int IMG = BQ * HT::RB, SLOT = 2 * IMG + 1024;     // Q image, dO image, 64 x (lse, delta); three slots
  constexpr int NCH = IMG / 1024 / 4;                         // copies per right wave and image
  constexpr int OPS = 2 * NCH + 1;                            // vector-memory operations of one issue(), per right wave
  constexpr int HAND = 4 * 4096;                              // one hand-over buffer: 4 wave pairs x 64 lanes x 64 bytes
  constexpr int HALF = 32 * HT::RB;                           // the second tile's rows inside an image

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  lds_u8* const lds = LDS_PTR(unsigned char, smem_raw);
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;
  lds_u8* const hand = lds + 3 * SLOT;

  const int tid = threadIdx.x, lane = tid & 63, kl = lane & 31, g = lane >> 5;
  const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int right = wave8 >> 2, wave = wave8 & 3;             // role, and which 32 keys of the block
  const int kb = blockIdx.y;
  const int h = (int)blockIdx.x % p.H, b = (int)blockIdx.x / p.H;
  const int kv0 = kb * 128, kw0 = kv0 + 32 * wave, key = kw0 + kl;
  const int d = p.H * DH;
  const long tok0 = (long)b * p.S;
  const long bh = (long)b * p.H + h;
  const typename HT::Offsets fo = HT::offsets(lane);
  const int step0 = p.causal ? kv0 / BQ : 0;                  // queries before the first key of the block see none of it
  const int nstep = (p.S + BQ - 1) / BQ;
  const int t0 = 2 * step0, nt = 2 * (nstep - step0);         // first tile, number of tiles
  typedef LDS_AS float lds_f32;
  lds_u8* const my_hand = hand + wave * 4096 + lane * 16;     // + buffer * HAND + 1024 * {p0, p1, s0, s1}
  constexpr int KVIMG = 128 * HT::RB;                         // image of the block's 128 K (then V) rows
  lds_u8* const kvimg = lds + 2 * SLOT;
  static_assert(2 * KVIMG <= SLOT + 2 * HAND, "K and V images must fit in the third slot plus the hand-over area");

  if (!right) {
    // ------------------------------------------------------------------ left: S, dP, P, dS, dS^T out
    bf16x8 kfb[KS], vfb[KS];
    const long ds_elems = (long)attn_ds_elems(p.S);
    const u32x4 rst = make_desc(p.dst + bh * ds_elems, (uint32_t)(ds_elems * 2));
    // The tiles of dS^T (32 keys x 32 queries each) leave through a per-wave LDS buffer that collects the two tiles of a
    // 64-query step (rows padded to 144 bytes against bank conflicts): a lane holds 4 consecutive queries of its key row
    // per register group, which stored directly is 8 bytes per lane and 32 rows per instruction; read back row-major
    // after the second tile it is 16 bytes per lane and 128 contiguous bytes (a whole cache line of the panel) per key row.
    constexpr int STG_ROW = 144;
    lds_u8* const stg = hand + 2 * HAND + wave * (32 * STG_ROW);
    lds_u8* const stg_wr = stg + kl * STG_ROW + 8 * g;          // + 64 (tile & 1) + 16 e4
    unsigned st_row[4];
#pragma unroll
    for (int r = 0; r < 4; r++) {
      const int row = (lane + 64 * r) >> 3;
      st_row[r] = kw0 + row < p.S ? (unsigned)(((kw0 + row) * kPanel + 8 * (lane & 7)) * 2) : kOob;
    }
    __syncthreads();                                          // steps step0, step0 + 1 and the K / V rows have landed
    // the lane's key row and value row as B operands (8 consecutive head-dim values per k-step), from the images the
    // right waves copied into the third slot and the hand-over area, which nothing else uses yet
#pragma unroll
    for (int s = 0; s < KS; s++) {
      kfb[s] = HT::rows_frag(kvimg, fo, 32 * wave, s);
      vfb[s] = HT::rows_frag(kvimg + KVIMG, fo, 32 * wave, s);
    }
    __syncthreads();                                          // every left wave has its rows: the area is free again
    for (int it = 0; it <= nt; it++) {
      if (it < nt) {
        const int tile = t0 + it, qt0 = tile * 32;
        lds_u8* const slot = lds + (((tile >> 1) - step0) % 3) * SLOT;
        lds_u8* const qimg = slot + (tile & 1) * HALF;
        lds_u8* const dimg = qimg + IMG;
        const lds_f32* const stat = reinterpret_cast<const lds_f32*>(slot + 2 * IMG) + 32 * (tile & 1);
        f32x16 sa, da;
#pragma unroll
        for (int e = 0; e < 16; e++) { sa[e] = 0.f; da[e] = 0.f; }
        constexpr int PF = KS < 4 ? KS : 4;
        bf16x8 fq[KS], fd[KS];
#pragma unroll
        for (int s = 0; s < PF; s++) { fq[s] = HT::rows_frag(qimg, fo, 0, s); fd[s] = HT::rows_frag(dimg, fo, 0, s); }
#pragma unroll
        for (int s = 0; s < KS; s++) {
          if (s + PF < KS) { fq[s + PF] = HT::rows_frag(qimg, fo, 0, s + PF); fd[s + PF] = HT::rows_frag(dimg, fo, 0, s + PF); }
          sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fq[s], kfb[s], sa, 0, 0, 0);
          da = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fd[s], vfb[s], da, 0, 0, 0);
        }
        // register e of the tile is query qt0 + 8 (e / 4) + 4 g + e % 4
        const int rel = p.causal ? key - qt0 - 4 * g : -1;
        float pv[16], sv[16];
#pragma unroll
        for (int e4 = 0; e4 < 4; e4++) {
          const f32x4 ls = *reinterpret_cast<const LDS_AS f32x4*>(stat + 8 * e4 + 4 * g);
          const f32x4 dl = *reinterpret_cast<const LDS_AS f32x4*>(stat + BQ + 8 * e4 + 4 * g);
#pragma unroll
          for (int q = 0; q < 4; q++) {
            const int e = 4 * e4 + q;
            float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(sa[e], p.scale_log2e, -ls[q]));
            pe = (8 * e4 + q < rel) ? 0.f : pe;
            pv[e] = pe;
            sv[e] = pe * (da[e] - dl[q]);
          }
        }
        bf16x8 kp[2], ks[2];
#pragma unroll
        for (int u = 0; u < 2; u++)
#pragma unroll
          for (int t = 0; t < 8; t++) { kp[u][t] = (bf16_t)pv[8 * u + t]; ks[u][t] = (bf16_t)sv[8 * u + t]; }
        lds_u8* const out = my_hand + (tile & 1) * HAND;
        *reinterpret_cast<LDS_AS bf16x8*>(out) = kp[0];
        *reinterpret_cast<LDS_AS bf16x8*>(out + 1024) = kp[1];
        *reinterpret_cast<LDS_AS bf16x8*>(out + 2048) = ks[0];
        *reinterpret_cast<LDS_AS bf16x8*>(out + 3072) = ks[1];
        // dS^T out: the two halves of each packed k-step are four consecutive queries of the lane's key row.  Nobody
        // reads it before the kernel ends, so the stores go out untracked: the barrier below must not wait for them
        // (tracked, their acknowledgements cost a quarter of the kernel's time).
        const u32x4 s0 = __builtin_bit_cast(u32x4, ks[0]), s1 = __builtin_bit_cast(u32x4, ks[1]);
        const u32x2 dsv[4] = {u32x2{s0[0], s0[1]}, u32x2{s0[2], s0[3]}, u32x2{s1[0], s1[1]}, u32x2{s1[2], s1[3]}};
        if constexpr (WRITE_DST) {
#pragma unroll
          for (int e4 = 0; e4 < 4; e4++) *reinterpret_cast<LDS_AS u32x2*>(stg_wr + 64 * (tile & 1) + 16 * e4) = dsv[e4];
        }
        // (LDS operations of a wave execute in order: the reads below see the writes above and those of the tile before)
        if (WRITE_DST && (tile & 1)) {
          const int qe = qt0 - 32;                              // first query of the step; the step lies inside one panel
          const long pan = ((long)(qe / kPanel) * p.S * kPanel + qe % kPanel) * 2;
#pragma unroll
          for (int r = 0; r < 4; r++) {
            const int idx = lane + 64 * r;
            const u32x4 v = *reinterpret_cast<const LDS_AS u32x4*>(stg + (idx >> 3) * STG_ROW + 16 * (idx & 7));
            store16_async(v, rst, qe + 8 * (lane & 7) < p.S ? st_row[r] : kOob, (uint32_t)__builtin_amdgcn_readfirstlane((int)pan));
          }
        }
      }
      __syncthreads();
    }
    __syncthreads();                                          // every right wave's copies have landed: the ring is free
    __syncthreads();                                          // the right waves have put dK and dV into LDS (below)
    return;
  }

  // -------------------------------------------------------------------- right: copies, dV^T, dK^T
  int c_row[NCH];
  unsigned cq_off[NCH], cd_off[NCH];
#pragma unroll
  for (int i = 0; i < NCH; i++) {
    HT::plan(wave + 4 * i, lane, p.ld_qkv, c_row[i], cq_off[i]);
    HT::plan(wave + 4 * i, lane, p.ld_do, c_row[i], cd_off[i]);
  }
  // Every call issues exactly OPS operations per wave (steps past the end write zeros into their slot and fetch
  // nothing), so a wait for "all but the last issue" is a fixed count.
  auto issue = [&](int i) {
    const int q0 = i * BQ;
    const bool live = i < nstep;
    const uint32_t slot = lds0 + ((i - step0) % 3) * SLOT;      // slots count from the block's first step
    const int qs = live ? q0 : 0;
    const u32x4 dq = make_desc(p.qkv + (tok0 + qs) * p.ld_qkv + h * DH, (uint32_t)((long)(p.S - qs) * p.ld_qkv * 2));
    const u32x4 dd = make_desc(p.dout + (tok0 + qs) * p.ld_do + h * DH, (uint32_t)((long)(p.S - qs) * p.ld_do * 2));
#pragma unroll
    for (int c = 0; c < NCH; c++) {
      const bool ok = live && q0 + c_row[c] < p.S;
      dma16(slot + wave * 1024 + c * 4096, dq, ok ? cq_off[c] : kOob);
      dma16(slot + IMG + wave * 1024 + c * 4096, dd, ok ? cd_off[c] : kOob);
    }
    // row statistics: wave 0 fetches lse[0..63], wave 1 delta[0..63]; waves 2 and 3 issue the same instruction out of
    // range (nothing moves) to keep the count uniform.  Their 256 bytes land behind the two statistics rows.
    const int q = q0 + lane;
    const u32x4 ds = (wave & 1) == 0 ? make_desc(p.lse + bh * p.S, (uint32_t)(p.S * 4))
                                     : make_desc(p.delta + tok0 * p.H + h, (uint32_t)(((long)(p.S - 1) * p.H + 1) * 4));
    const unsigned off = (live && wave < 2 && q < p.S) ? (unsigned)((wave & 1) == 0 ? q * 4 : (long)q * p.H * 4) : kOob;
    dma4(slot + 2 * IMG + wave * 256, ds, off);
  };
  // A right wave owns 32 head-dim columns (its index) of dV^T and dK^T for all four key blocks of the workgroup: it then
  // reads only its quarter of the Q and dO tiles as transposed fragments (the expensive reads) and all four left waves'
  // P and dS (cheap, lane-contiguous).  With head_dim 64 waves 2 and 3 have no columns and only copy.
  f32x16 dvt[4], dkt[4];
#pragma unroll
  for (int t = 0; t < 4; t++)
#pragma unroll
    for (int e = 0; e < 16; e++) { dvt[t][e] = 0.f; dkt[t][e] = 0.f; }
  const bool has_cols = wave < DT;
  int col0 = 0, col1 = 0;                                     // fragment offsets of this wave's column block
#pragma unroll
  for (int t = 0; t < DT; t++)
    if (t == wave) { col0 = fo.cols[t][0]; col1 = fo.cols[t][1]; }
  auto my_cols = [&](lds_u8* img, int u) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(img + col0 + 16 * u * HT::RB));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(img + col1 + 16 * u * HT::RB));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  };

  {  // the block's K and V rows, for the left waves (coalesced here; fetched per lane they are 32-byte pieces of 32 rows)
    const bf16_t* kb0 = p.qkv + (tok0 + kv0) * p.ld_qkv + d + h * DH;
    const uint32_t bytes = (uint32_t)((long)(p.S - kv0) * p.ld_qkv * 2);
    const u32x4 dk = make_desc(kb0, bytes), dv = make_desc(kb0 + d, bytes);
#pragma unroll
    for (int i = 0; i < 2 * NCH; i++) {
      int row; unsigned go;
      HT::plan(wave + 4 * i, lane, p.ld_qkv, row, go);
      const unsigned off = kv0 + row < p.S ? go : kOob;
      dma16(lds0 + 2 * SLOT + (wave + 4 * i) * 1024, dk, off);
      dma16(lds0 + 2 * SLOT + KVIMG + (wave + 4 * i) * 1024, dv, off);
    }
  }
  issue(step0);
  issue(step0 + 1);
  wait_vmem<0>();
  __syncthreads();
  __syncthreads();                                            // the left waves have read their K and V rows
  for (int it = 0; it <= nt; it++) {
    const int tp = t0 + it;                                   // the tile the left waves are on
    if (it > 0 && has_cols) {
      const int tile = tp - 1;
      lds_u8* const qimg = lds + (((tile >> 1) - step0) % 3) * SLOT + (tile & 1) * HALF;
      lds_u8* const dimg = qimg + IMG;
      // this wave's 32 head-dim columns of dO^T and Q^T (two k-steps of 16 queries), then every key block's P and dS
      bf16x8 fo_d[2], fo_q[2];
#pragma unroll
      for (int u = 0; u < 2; u++) { fo_d[u] = my_cols(dimg, u); fo_q[u] = my_cols(qimg, u); }
      const lds_u8* const in = hand + (tile & 1) * HAND + lane * 16;
#pragma unroll
      for (int kbk = 0; kbk < 4; kbk++) {
        bf16x8 kp[2], ks[2];
        kp[0] = *reinterpret_cast<const LDS_AS bf16x8*>(in + kbk * 4096);
        kp[1] = *reinterpret_cast<const LDS_AS bf16x8*>(in + kbk * 4096 + 1024);
        ks[0] = *reinterpret_cast<const LDS_AS bf16x8*>(in + kbk * 4096 + 2048);
        ks[1] = *reinterpret_cast<const LDS_AS bf16x8*>(in + kbk * 4096 + 3072);
#pragma unroll
        for (int u = 0; u < 2; u++) {
          dvt[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo_d[u], kp[u], dvt[kbk], 0, 0, 0);
          dkt[kbk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fo_q[u], ks[u], dkt[kbk], 0, 0, 0);
        }
      }
    }
    // step (tp + 1) / 2 + 1 is what the left waves start two barriers from now, when tp is odd: it was issued three
    // barriers ago and only the issue after it may still be in flight
    if (tp & 1) wait_vmem<OPS>();
    __syncthreads();
    // after this barrier nobody reads the step before tp / 2 any more (tp even): its slot takes step tp / 2 + 2
    if (!(tp & 1)) issue((tp >> 1) + 2);
  }
  wait_vmem<0>();                                             // (copies past the end: zeros, no traffic)
  __syncthreads();                                            // ... of every wave, before the ring is reused below

  // ---- dk = scale * dK^T transposed, dv = dV^T transposed.  A lane holds 4 consecutive head-dim values of one key per
  // register group; stored directly that is 8 bytes per lane scattered over 32 rows per instruction, and the 64 MB of
  // dK and dV of a launch then cost a tenth of the kernel's time.  The waves put their column blocks together in LDS
  // (the copy ring is free by now; rows padded to 272 bytes against bank conflicts) and each writes 32 whole key
  // rows, 16 bytes per lane, 256 contiguous bytes per row.
  constexpr int EROW = DH * 2 + 16;
  lds_u8* const edk = lds;
  lds_u8* const edv = lds + 128 * EROW;
  static_assert(2 * 128 * EROW <= 3 * SLOT, "dK and dV tiles must fit in the ring");
  if (has_cols) {
#pragma unroll
    for (int kbk = 0; kbk < 4; kbk++)
#pragma unroll
      for (int e4 = 0; e4 < 4; e4++) {
        bf16x4 vk, vv;
#pragma unroll
        for (int r = 0; r < 4; r++) { vk[r] = (bf16_t)(dkt[kbk][4 * e4 + r] * p.scale); vv[r] = (bf16_t)dvt[kbk][4 * e4 + r]; }
        const int off = (32 * kbk + kl) * EROW + (32 * wave + 8 * e4 + 4 * g) * 2;
        *reinterpret_cast<LDS_AS bf16x4*>(edk + off) = vk;
        *reinterpret_cast<LDS_AS bf16x4*>(edv + off) = vv;
      }
  }
  __syncthreads();
  {
    constexpr int LPR = DH / 8, RPI = 64 / LPR;               // lanes per row, rows per wave-wide store
    const int rl = lane / LPR, piece = lane % LPR;
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPI) {
      const int row = 32 * wave + r0 + rl;                    // this wave's 32 key rows
      const int krow = kv0 + row;
      if (krow < p.S) {
        bf16_t* const out = p.dqkv + (tok0 + krow) * p.ld_dqkv + d + h * DH + 8 * piece;
        *reinterpret_cast<u32x4*>(out) = *reinterpret_cast<const LDS_AS u32x4*>(edk + row * EROW + 16 * piece);
        *reinterpret_cast<u32x4*>(out + d) = *reinterpret_cast<const LDS_AS u32x4*>(edv + row * EROW + 16 * piece);
      }
    }
  }
}

// ------------------------------------------------------------------------------------------ backward-p1: dQ
// dQ = scale * dS K is a contraction over keys.  This pass is oriented like the forward (S^T = K Q^T: a lane owns one
// query, so lse and delta of the row are per-lane scalars): per block of 64 keys it recomputes S^T and dP^T = V dO^T,
// forms P^T = exp2(S^T c - lse) and dS^T = P^T (dP^T - delta) in the accumulators and feeds dS^T straight into
// dQ^T += K^T dS^T (the B-operand trick of the file header), accumulating dQ^T in registers over all key blocks.
// Three products per tile instead of one, but no dS^T is written to or read from memory, nothing is added
// atomically, and the result is bit-reproducible.  Workgroup = 4 waves x 32 queries, K and V blocks double-buffered
// through LDS exactly as in the forward.
struct AttnDqParams {
  const bf16_t* qkv; long ld_qkv;
  const bf16_t* dout; long ld_do;
  const float* lse;                    // [B, H, S]
  const float* delta;                  // [B*S, H]
  bf16_t* dqkv; long ld_dqkv;          // dq block is written (columns h * DH ..)
  int B, H, S, causal;
  float scale, scale_log2e;
};

template <int DH>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_bwd_dq_kernel(AttnDqParams p) {
  using HT = HeadTile<DH>;
  constexpr int KS = DH / 16, DT = DH / 32, BKV = 64;
  constexpr int IMG = BKV * HT::RB, SLOT = 2 * IMG;
  constexpr int NCH = IMG / 1024 / 4;

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  lds_u8* const lds = LDS_PTR(unsigned char, smem_raw);
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

  const int lane = threadIdx.x & 63, ql = lane & 31, g = lane >> 5;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qb = (int)gridDim.y - 1 - (int)blockIdx.y;             // longest (last) query blocks first
  const int h = (int)blockIdx.x % p.H, b = (int)blockIdx.x / p.H;
  const int q0 = qb * 128, qw0 = q0 + 32 * wave, query = qw0 + ql;
  const int d = p.H * DH;
  const long tok0 = (long)b * p.S;
  const long bh = (long)b * p.H + h;

  const typename HT::Offsets fo = HT::offsets(lane);
  // ---- the block's 128 query rows into the second slot and their output derivatives into the first (coalesced copies)
  {
    const u32x4 dq = make_desc(p.qkv + (tok0 + q0) * p.ld_qkv + h * DH, (uint32_t)((long)(p.S - q0) * p.ld_qkv * 2));
    const u32x4 dd = make_desc(p.dout + (tok0 + q0) * p.ld_do + h * DH, (uint32_t)((long)(p.S - q0) * p.ld_do * 2));
#pragma unroll
    for (int i = 0; i < 2 * NCH; i++) {
      int row; unsigned go, gd;
      HT::plan(wave + 4 * i, lane, p.ld_qkv, row, go);
      HT::plan(wave + 4 * i, lane, p.ld_do, row, gd);
      const bool ok = q0 + row < p.S;
      dma16(lds0 + SLOT + (wave + 4 * i) * 1024, dq, ok ? go : kOob);
      dma16(lds0 + (wave + 4 * i) * 1024, dd, ok ? gd : kOob);
    }
  }
  int c_row[NCH];
  unsigned c_off[NCH];
#pragma unroll
  for (int i = 0; i < NCH; i++) HT::plan(wave + 4 * i, lane, p.ld_qkv, c_row[i], c_off[i]);
  const int kv_end = p.causal ? (q0 + 128 < p.S ? q0 + 128 : p.S) : p.S;
  const int nblk = (kv_end + BKV - 1) / BKV;
  auto issue = [&](int j) {
    const int kv0 = j * BKV;
    const bf16_t* kb = p.qkv + (tok0 + kv0) * p.ld_qkv + d + h * DH;
    const uint32_t bytes = (uint32_t)((long)(p.S - kv0) * p.ld_qkv * 2);
    const u32x4 dk = make_desc(kb, bytes), dv = make_desc(kb + d, bytes);
    const uint32_t base = lds0 + (j & 1) * SLOT + wave * 1024;
#pragma unroll
    for (int i = 0; i < NCH; i++) {
      const unsigned off = (kv0 + c_row[i] < p.S) ? c_off[i] : kOob;
      dma16(base + i * 4096, dk, off);
      dma16(base + IMG + i * 4096, dv, off);
    }
  };
  // the row statistics of this lane's query
  const bool qlive = query < p.S;
  const float lse_q = qlive ? p.lse[bh * p.S + query] : 0.f;
  const float dl_q = qlive ? p.delta[(tok0 + query) * p.H + h] : 0.f;

  f32x16 dqt[DT];
#pragma unroll
  for (int t = 0; t < DT; t++)
#pragma unroll
    for (int e = 0; e < 16; e++) dqt[t][e] = 0.f;

  wait_vmem<0>();
  __syncthreads();
  bf16x8 qf[KS], dof[KS];            // this lane's query row and output-derivative row as B operands
#pragma unroll
  for (int s = 0; s < KS; s++) {
    qf[s] = HT::rows_frag(lds + SLOT, fo, 32 * wave, s);
    dof[s] = HT::rows_frag(lds, fo, 32 * wave, s);
  }
  __syncthreads();                   // every wave has its rows: both slots are free for the key blocks
  issue(0);
  for (int j = 0; j < nblk; j++) {
    wait_vmem<0>();
    __syncthreads();                 // block j has landed; every wave is done with the other slot
    if (j + 1 < nblk) issue(j + 1);
    const int kv0 = j * BKV;
    if (p.causal && kv0 > qw0 + 31) continue;
    lds_u8* const kimg = lds + (j & 1) * SLOT;
    lds_u8* const vimg = kimg + IMG;
    // keys beyond the query (causal) or beyond the sequence do not take part: their probability is zero
    const bool edge = (p.causal && kv0 + BKV - 1 > qw0) || kv0 + BKV > p.S;
    const int last = p.causal ? (query < p.S - 1 ? query : p.S - 1) : p.S - 1;
    const int rel = edge ? last - kv0 - 4 * g : 1 << 20;
    // one 32-key tile at a time (both tiles at once would need 64 more accumulator registers than a wave has):
    // S^T and dP^T as two interleaved accumulation chains, fragments one k-step ahead; then dS^T in place and
    // dQ^T += K^T dS^T over the tile's two k-steps on DT independent accumulators
#pragma unroll 1
    for (int kt = 0; kt < 2; kt++) {
      f32x16 st, dp;
#pragma unroll
      for (int e = 0; e < 16; e++) { st[e] = 0.f; dp[e] = 0.f; }
      bf16x8 kf = HT::rows_frag(kimg, fo, 32 * kt, 0), vf = HT::rows_frag(vimg, fo, 32 * kt, 0);
#pragma unroll
      for (int s = 0; s < KS; s++) {
        bf16x8 nk = kf, nv = vf;
        if (s + 1 < KS) { nk = HT::rows_frag(kimg, fo, 32 * kt, s + 1); nv = HT::rows_frag(vimg, fo, 32 * kt, s + 1); }
        st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], st, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, dof[s], dp, 0, 0, 0);
        kf = nk; vf = nv;
      }
      bf16x8 ktf[DT];
#pragma unroll
      for (int t = 0; t < DT; t++) ktf[t] = HT::cols_frag(kimg, fo, 32 * kt, 0, t);
#pragma unroll
      for (int e = 0; e < 16; e++) {
        float pe = __builtin_amdgcn_exp2f(__builtin_fmaf(st[e], p.scale_log2e, -lse_q));
        pe = (32 * kt + 8 * (e >> 2) + (e & 3) > rel) ? 0.f : pe;
        st[e] = pe * (dp[e] - dl_q);                         // dS^T
      }
#pragma unroll
      for (int u = 0; u < 2; u++) {
        const bf16x8 sb = pack8(st, u);
#pragma unroll
        for (int t = 0; t < DT; t++) {
          dqt[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktf[t], sb, dqt[t], 0, 0, 0);
          if (u == 0) ktf[t] = HT::cols_frag(kimg, fo, 32 * kt, 1, t);     // the second k-step's fragment, behind the MFMA that used the first
        }
      }
    }
  }

  // ---- dq = scale * dQ^T, transposed back through LDS and written as whole rows (as the forward writes its output)
  __syncthreads();
  constexpr int EROW = DH * 2 + 16;
  static_assert(128 * EROW <= 2 * SLOT, "the output tile must fit in the ring");
  lds_u8* const erow = lds + 32 * wave * EROW;
#pragma unroll
  for (int t = 0; t < DT; t++)
#pragma unroll
    for (int e4 = 0; e4 < 4; e4++) {
      bf16x4 v;
#pragma unroll
      for (int r = 0; r < 4; r++) v[r] = (bf16_t)(dqt[t][4 * e4 + r] * p.scale);
      *reinterpret_cast<LDS_AS bf16x4*>(erow + ql * EROW + (32 * t + 8 * e4 + 4 * g) * 2) = v;
    }
  {  // (LDS operations of a wave execute in order: the reads below see this wave's own writes above)
    constexpr int LPR = DH / 8, RPI = 64 / LPR;
    const int rl = lane / LPR, piece = lane % LPR;
#pragma unroll
    for (int r0 = 0; r0 < 32; r0 += RPI) {
      const int qrow = qw0 + r0 + rl;
      if (qrow < p.S)
        *reinterpret_cast<u32x4*>(p.dqkv + (tok0 + qrow) * p.ld_dqkv + h * DH + 8 * piece) =
            *reinterpret_cast<const LDS_AS u32x4*>(erow + (r0 + rl) * EROW + 16 * piece);
    }
  }
}

template <int DH>
static hipError_t launch_fwd(const AttnParams& p, hipStream_t s) {
  constexpr size_t smem = 2 * 2 * 64 * DH * 2;
  auto kern = attn_fwd_kernel<DH>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(p.H * p.B), (unsigned)((p.S + 127) / 128)), dim3(256), smem, s, p);
  return hipGetLastError();
}

hipError_t attention_fwd(int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv, long ld_qkv,
                         void* out, long ld_out, float* lse, hipStream_t s) {
  if (batch <= 0 || n_heads <= 0 || seq <= 0) return hipSuccess;
  AttnParams p{};
  p.qkv = (const bf16_t*)qkv; p.ld_qkv = ld_qkv; p.out = (bf16_t*)out; p.ld_out = ld_out; p.lse = lse;
  p.B = batch; p.H = n_heads; p.S = seq; p.causal = causal;
  p.scale_log2e = 1.4426950408889634f / sqrtf((float)head_dim);
  if (head_dim == 128) return launch_fwd<128>(p, s);
  if (head_dim == 64) return launch_fwd<64>(p, s);
  return hipErrorInvalidValue;
}

template <int DH>
static hipError_t launch_bwd_dq(const AttnDqParams& p, hipStream_t s) {
  constexpr size_t smem = 2 * 2 * 64 * DH * 2;
  auto kern = attn_bwd_dq_kernel<DH>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(p.H * p.B), (unsigned)((p.S + 127) / 128)), dim3(256), smem, s, p);
  return hipGetLastError();
}

template <int DH, bool WRITE_DST>
static hipError_t launch_bwd_kv_split(const AttnBwdParams& p, hipStream_t s) {
  constexpr size_t smem = 3 * (2 * 64 * DH * 2 + 1024) + 2 * 4 * 4096 + 4 * 32 * 144;     // three slots, two hand-over buffers, dS^T staging
  auto kern = attn_bwd_kv_split_kernel<DH, WRITE_DST>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)(p.H * p.B), (unsigned)((p.S + 127) / 128)), dim3(512), smem, s, p);
  return hipGetLastError();
}

hipError_t attention_p1(int batch, int n_heads, int seq, int head_dim, int causal, const void* qkv, long ld_qkv,
                        const void* out, const void* d_out, long ld_out, const float* lse, void* dqkv, long ld_dqkv,
                        float* delta, void* ds_t, hipStream_t s) {
  if (batch <= 0 || n_heads <= 0 || seq <= 0) return hipSuccess;
  if (ld_out != (long)n_heads * head_dim) return hipErrorInvalidValue;      // the row-dot kernel takes dense rows
  hipError_t e = head_rowdot(1, batch * seq, n_heads, head_dim, d_out, out, delta, s);
  if (e != hipSuccess) return e;
  AttnBwdParams p{};
  p.qkv = (const bf16_t*)qkv; p.ld_qkv = ld_qkv; p.dout = (const bf16_t*)d_out; p.ld_do = ld_out;
  p.lse = lse; p.delta = delta; p.dqkv = (bf16_t*)dqkv; p.ld_dqkv = ld_dqkv; p.dst = (bf16_t*)ds_t;
  p.B = batch; p.H = n_heads; p.S = seq; p.causal = causal;
  p.scale = 1.f / sqrtf((float)head_dim);
  p.scale_log2e = 1.4426950408889634f * p.scale;
  if (!ds_t) {
    // no dS^T buffer: dQ by the recompute pass
    if (head_dim == 128) e = launch_bwd_kv_split<128, false>(p, s);
    else if (head_dim == 64) e = launch_bwd_kv_split<64, false>(p, s);
    else return hipErrorInvalidValue;
    if (e != hipSuccess) return e;
    AttnDqParams q{};
    q.qkv = p.qkv; q.ld_qkv = ld_qkv; q.dout = p.dout; q.ld_do = ld_out; q.lse = lse; q.delta = delta;
    q.dqkv = p.dqkv; q.ld_dqkv = ld_dqkv; q.B = batch; q.H = n_heads; q.S = seq; q.causal = causal;
    q.scale = p.scale; q.scale_log2e = p.scale_log2e;
    return head_dim == 128 ? launch_bwd_dq<128>(q, s) : launch_bwd_dq<64>(q, s);
  }
  if (head_dim == 128) e = launch_bwd_kv_split<128, true>(p, s);
  else if (head_dim == 64) e = launch_bwd_kv_split<64, true>(p, s);
  else return hipErrorInvalidValue;
  if (e != hipSuccess) return e;
  // dq = scale * dS k = scale * (dS^T)^T k per (sequence, head): contraction over keys, causal: keys <= query
  const long d = (long)n_heads * head_dim;
  GemmArgs g = gemm_args(TN, seq, head_dim, seq, ds_t, kPanel, (const char*)qkv + d * 2, ld_qkv, dqkv, ld_dqkv);
  g.alpha = p.scale;
  g.a_panel = (long)seq * kPanel;
  g.batch = batch * n_heads; g.batch_inner = n_heads;
  g.sAi = (long)attn_ds_elems(seq); g.sAo = n_heads * g.sAi;
  g.sBo = (long)seq * ld_qkv; g.sBi = head_dim;
  g.sCo = (long)seq * ld_dqkv; g.sCi = head_dim;
  g.causal = causal ? CAUSAL_K_END : CAUSAL_NONE;
  return gemm(1, g, s);
}

}  // namespace tbp
