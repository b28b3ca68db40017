// GEMM kernels for gfx950 (MI355X).
//
// bf16 path: C = alpha * op(A) op(B) on the 32x32x16 bf16 MFMA instruction, fp32 accumulation.
//   One workgroup = 4 wavefronts (2 x 2), block tile BM x BN (256 x 256, 256 x 192 or 128 x 128, chosen per product by
//   how well the tiles fill the 256 compute units), contraction consumed in slices of 32 through a 4-slot LDS ring, or
//   in slices of 64 through two slots where the contraction index is contiguous in memory, filled by asynchronous
//   global -> LDS copies (no staging registers) that stay in flight while the previous slices are multiplied.
//   Outputs too small for any of that can split the contraction over several workgroups per tile (scratch memory).
//   An operand whose contraction index is contiguous in memory ("KC": A of NN/NT, B of NT) is kept in
//   LDS as [row][k] and read as 16-byte vectors; an operand whose contraction index is the slow,
//   strided one ("KS": A of TN, B of NN/TN, i.e. both operands of dW = X^T dY) is kept as [k][row]
//   exactly as it sits in memory and transposed on the way to the registers by the LDS
//   transpose-read instruction (ds_read_b64_tr_b16), so no operand is ever transposed in HBM.
//   Out-of-range lanes of a copy are redirected past the end of the buffer descriptor (they deliver zero),
//   which handles ragged M, N and K without branches.
// fp32 path: plain FMA tile kernel with generic strides (the fp32 configuration is tiny).
#include "kernels.h"
#include "gfx950.h"

namespace tbp {

struct GemmParams {
  const void* A; const void* B; void* C; const void* R;
  long lda, ldb, ldc;
  long sAo, sAi, sBo, sBi, sCo, sCi;
  int M, N, K;
  int batch_inner;
  int tiles_m, tiles_n;
  float alpha;
  int accumulate;
  int causal;
  // fp32 kernel only: element strides of A(m,k) and B(k,n)
  long sam, sak, sbk, sbn;
  // fused softmax backward (see GemmArgs)
  const float* delta; long ldd, sDo, sDi;
  int delta_causal;
  long a_panel;                 // see GemmArgs
  // contraction split over `split` workgroups per tile (see SplitPlan)
  int split;
  float* split_ws;
  unsigned* split_cnt;
};

constexpr int BK = 32;                     // contraction depth of one LDS slot
constexpr int STAGES = 4;                  // LDS ring: one slot being multiplied, three in flight


// Workgroup id -> (tile row, tile column).  Workgroups are handed to the 8 XCDs round-robin; the first
// step makes each XCD own a contiguous range of the tile sequence (so its private L2 sees neighbouring
// tiles), the second walks that sequence in groups of 8 tile rows so that concurrently running tiles
// share A and B panels.
__device__ __forceinline__ void tile_of_block(int pid, int tiles_m, int tiles_n, int& tm, int& tn) {
  const int nt = tiles_m * tiles_n;
  const int xcd = pid & 7, q = pid >> 3;
  const int per = nt >> 3, rem = nt & 7;
  int id = xcd * per + (xcd < rem ? xcd : rem) + q;
  const int GROUP = 8;
  const int width = GROUP * tiles_n;
  const int grp = id / width;
  const int first = grp * GROUP;
  const int gsz = (tiles_m - first) < GROUP ? (tiles_m - first) : GROUP;
  const int r = id - grp * width;
  tm = first + r % gsz;
  tn = r / gsz;
}

// LDS image of one operand tile (R rows/columns of the output x BK of the contraction), laid out so that
// (a) every 1 KiB piece is what one wave-wide 16-byte-per-lane copy writes (64 consecutive 16-byte granules),
// (b) the MFMA fragment reads are free of bank conflicts without padding:
//   KC (contraction index contiguous in memory): image [R][depth], 4 or 8 granules per row; granule g of row r sits
//       in slot g ^ ((r >> 2) & 3) (depth 32) or g ^ ((r >> 1) & 7) (depth 64): the 16 lanes served per clock (256
//       bytes) then touch 16 different 16-byte bank groups.  A fragment read is one ds_read_b128 per lane.
//   KS (contraction index strided in memory): image [BK][R] as in memory, R/8 granules per row; granule
//       pairs (32 bytes = 16 columns) are swizzled: pair q of row k sits in pair slot q ^ (k & 3).  A fragment
//       read is two ds_read_b64_tr_b16 (transpose reads), each covering 4 k x 16 columns per 16-lane group:
//       within a group lane j addresses row k + j/4, columns 4*(j%4)..+3 and receives 4 consecutive k of column j.
template <int R, bool KC, int KD = BK>
struct OperandTile {
  static constexpr int BYTES = R * KD * 2;
  static constexpr int CHUNKS = BYTES / 1024;       // wave-wide copies per tile
  static constexpr int PER_WAVE = CHUNKS / 4;
  static constexpr int GPR = R / 8;                 // granules per image row (KS)
  static constexpr int GR = KD / 8;                 // granules per image row (KC): 4 (64-byte rows) or 8 (128-byte rows)
  static constexpr int RPB = 16 / GR;               // KC rows per 256 bytes (one pass over all banks)
  static_assert(CHUNKS % 4 == 0, "tile must split evenly over 4 waves");
  static_assert(KD == 32 || KD == 64, "slot depth");

  // KC swizzle: granule g of row r sits in slot g ^ ((r / RPB) % GR), so 16 consecutive rows at one logical granule
  // cover the 16 bank groups once.
  static __device__ __forceinline__ int kc_swz(int row) { return (row / RPB) & (GR - 1); }

  // Global byte offset (relative to the tile origin) and contraction index covered by lane p of chunk c.
  static __device__ __forceinline__ void copy_plan(int c, int p, long ld, int origin, int extent, unsigned& goff,
                                                   int& kidx) {
    if constexpr (KC) {
      const int row = (64 / GR) * c + p / GR;
      const int g = (p % GR) ^ kc_swz(row);
      goff = (origin + row < extent) ? (unsigned)((long)row * ld * 2 + g * 16) : kOob;
      kidx = g * 8;
    } else {
      const int P = 64 * c + p;
      const int k = P / GPR, sl = P % GPR;
      const int g = ((((sl >> 1) ^ (k & 3)) << 1) | (sl & 1));
      goff = (origin + g * 8 < extent) ? (unsigned)((long)k * ld * 2 + g * 16) : kOob;
      kidx = k;
    }
  }
  // Per-lane byte offset inside the image of the fragment of MFMA tile 0 (rows/columns w0..w0+31), variant v:
  // KC: v = k-step (0 .. KD/16 - 1);  KS: v = parity of the MFMA tile index.
  static __device__ __forceinline__ int frag_base(int lane, int w0, int v) {
    if constexpr (KC) {
      const int row = w0 + (lane & 31);
      const int g = 2 * v + (lane >> 5);
      return row * (KD * 2) + ((g ^ kc_swz(row)) << 4);
    } else {
      const int k = 8 * (lane >> 5) + ((lane & 15) >> 2);
      const int q = w0 / 16 + ((lane >> 4) & 1) + 2 * v;
      return k * (R * 2) + ((q ^ (k & 3)) << 5) + 8 * (lane & 3);
    }
  }
  static constexpr int VARIANTS = KC ? KD / 16 : 2;
  static __device__ __forceinline__ constexpr int variant(int ks, int t) { return KC ? ks : (t & 1); }
  // Byte offset of (k-step ks, MFMA tile t) relative to frag_base(..., variant(ks, t)).
  static __device__ __forceinline__ constexpr int frag_step(int ks, int t) {
    return KC ? t * 32 * KD * 2 : ks * 16 * R * 2 + (t >> 1) * 128;
  }
};

template <int R, bool KC>
__device__ __forceinline__ bf16x8 read_frag(lds_u8* q) {
  if constexpr (KC) {
    return *reinterpret_cast<LDS_AS const bf16x8*>(q);
  } else {
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(q));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<LDS_AS s16x4*>(q + 4 * R * 2));
    s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
  }
}

// One output tile (tm_i, tn_i) of batch entry z of the product described by p.
// KD = contraction depth of one LDS slot: 32 with a ring of 4 slots, or 64 with 2 slots.  The deeper slot is for
// operands whose contraction index is contiguous in memory: their copies then fetch 128 contiguous bytes per tile
// row, a whole cache line, where the 32-deep slot fetches every line in two halves one iteration apart and doubles
// the number of requests to the L2.
template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD = BK, bool SPLIT = false, int RING = 0>
__device__ __forceinline__ void gemm_bf16_tile(const GemmParams& p, int tm_i, int tn_i, int z, int split_idx = 0,
                                               int tile_seq = 0) {
  // RING == 0: the default pipeline of the slot depth (32: ring of STAGES slots; 64: two slots); RING >= 3: the ring
  // pipeline with that many slots, for either depth
  constexpr bool RINGPIPE = KD == 32 || RING >= 3;
  constexpr int NS = RING >= 3 ? RING : (KD == 32 ? STAGES : 2);       // ring slots
  constexpr int KSTEPS = KD / 16;
  constexpr int WM = BM / 2, WN = BN / 2;       // per-wave tile
  constexpr int TM = WM / 32, TN = WN / 32;     // MFMA tiles per wave
  using TA = OperandTile<BM, AKC, KD>;
  using TB = OperandTile<BN, BKC, KD>;
  constexpr int STAGE_BYTES = TA::BYTES + TB::BYTES;
  constexpr int NA = TA::PER_WAVE, NB = TB::PER_WAVE;
  constexpr int L = NA + NB;                    // asynchronous copies per thread per slot

  extern __shared__ __attribute__((aligned(1024))) unsigned char smem_raw[];
  lds_u8* const lds = LDS_PTR(unsigned char, smem_raw);
  const uint32_t lds0 = (uint32_t)(uintptr_t)lds;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;

  const int m0 = tm_i * BM, n0 = tn_i * BN;

  int k_lo = 0, k_hi = p.K;
  if (p.causal == CAUSAL_SKIP_UPPER) {
    if (n0 > m0 + BM - 1) return;
  } else if (p.causal == CAUSAL_K_END) {
    k_hi = (m0 + BM < p.K) ? m0 + BM : p.K;
  } else if (p.causal == CAUSAL_K_BEGIN) {
    k_lo = m0;
  }
  if constexpr (SPLIT) {      // this workgroup's slice of the contraction, in whole slots (may be empty)
    const int per = ((p.K + KD - 1) / KD + p.split - 1) / p.split * KD;
    k_lo = split_idx * per < p.K ? split_idx * per : p.K;
    k_hi = k_lo + per < p.K ? k_lo + per : p.K;
  }
  const int nk = (k_hi - k_lo + KD - 1) / KD;

  const int zo = z / p.batch_inner, zi = z - zo * p.batch_inner;
  const bf16_t* A = reinterpret_cast<const bf16_t*>(p.A) + zo * p.sAo + zi * p.sAi;
  const bf16_t* B = reinterpret_cast<const bf16_t*>(p.B) + zo * p.sBo + zi * p.sBi;

  // ---- this wave's share of the global -> LDS copies of one slot: chunks wave, wave + 4, ...
  unsigned a_goff[NA], b_goff[NB];
  int a_kidx[NA], b_kidx[NB];
#pragma unroll
  for (int i = 0; i < NA; i++) TA::copy_plan(wave + 4 * i, lane, p.lda, m0, p.M, a_goff[i], a_kidx[i]);
#pragma unroll
  for (int i = 0; i < NB; i++) TB::copy_plan(wave + 4 * i, lane, p.ldb, n0, p.N, b_goff[i], b_kidx[i]);
  // tile origin at k = 0 (an operand stored in panels is only ever given to the kernel whose BM is the panel width)
  const bf16_t* Ablk = AKC ? A + (long)m0 * p.lda : (p.a_panel ? A + (long)tm_i * p.a_panel : A + m0);
  const bf16_t* Bblk = BKC ? B + (long)n0 * p.ldb : B + n0;
  const long a_kstep = AKC ? 1 : p.lda;                          // elements per unit of k
  const long b_kstep = BKC ? 1 : p.ldb;

  // Copies of the next K tile into the next ring slot.  One code path serves full tiles, the ragged last tile
  // and tiles past the end ( every lane is redirected out of range, zeros land in a slot nobody reads
  // again, no memory traffic), so the main loop needs no branch around it.
  struct CopyJob { u32x4 dA, dB; uint32_t sa, sb; int krem; };
  // Running state of the copy stream (all wave-uniform): next tile's operand addresses, ring slot and remaining k.
  uint64_t a_next = reinterpret_cast<uint64_t>(Ablk + (long)k_lo * a_kstep);
  uint64_t b_next = reinterpret_cast<uint64_t>(Bblk + (long)k_lo * b_kstep);
  const uint64_t a_adv = (uint64_t)(KD * a_kstep * 2), b_adv = (uint64_t)(KD * b_kstep * 2);
  int slot_next = 0, krem_next = k_hi - k_lo;
  auto next_job = [&]() {
    CopyJob j;
    j.dA = make_desc(reinterpret_cast<const void*>(a_next));
    j.dB = make_desc(reinterpret_cast<const void*>(b_next));
    j.sa = lds0 + slot_next * STAGE_BYTES + wave * 1024;
    j.sb = j.sa + TA::BYTES;
    j.krem = krem_next;
    a_next += a_adv; b_next += b_adv;
    slot_next = (slot_next + 1 == NS) ? 0 : slot_next + 1;
    krem_next -= KD;
    return j;
  };
  auto copy_one = [&](const CopyJob& j, int c) {     // c-th of this wave's L copies of the job
    if (c < NA) dma16(j.sa + c * 4096, j.dA, a_kidx[c] < j.krem ? a_goff[c] : kOob);
    else dma16(j.sb + (c - NA) * 4096, j.dB, b_kidx[c - NA] < j.krem ? b_goff[c - NA] : kOob);
  };

  int a_base[TA::VARIANTS], b_base[TB::VARIANTS];
#pragma unroll
  for (int v = 0; v < TA::VARIANTS; v++) a_base[v] = TA::frag_base(lane, wm * WM, v);
#pragma unroll
  for (int v = 0; v < TB::VARIANTS; v++) b_base[v] = TB::frag_base(lane, wn * WN, v) + TA::BYTES;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; i++)
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;

  // ---- main loop, software-pipelined over the two k-steps of a slot and scheduled by hand:
  //   while (tile t, k-step 0) is multiplied the fragments of (t, k-step 1) are fetched from LDS; then the wait
  //   for tile t+1 and the workgroup barrier; while (t, k-step 1) is multiplied the fragments of (t+1, k-step 0)
  //   are fetched and the asynchronous copies of tile t+STAGES-1 are started.  Reads and copies are spread
  //   between the MFMAs (an MFMA occupies the matrix pipe for 32 cycles, the other instructions issue in its
  //   shadow); sched_barrier pins that order.
  // Ring invariant: while tile t is multiplied, tiles t+1 .. t+STAGES-2 are landed or in flight; slot
  // (t-1) % STAGES is refilled only after a barrier that every wave passes after its last read of tile t-1.
  // The loop body has no data-dependent join around LDS reads (a join makes the compiler merge wait states and
  // stall MFMAs on reads they do not need): the last iteration also fetches "tile nk" fragments, stale but
  // in-bounds LDS contents that are never used.
  constexpr int MM = TM * TN, UNITS = TM + TN;
  // Fragment fetch order = order of first use by the MFMA sequence (i-major): a0, then every b, then a1, a2, ...;
  // one fetch per MFMA from the start of the region, so the fragments the NEXT region needs first have the whole
  // region to arrive and the last fetches still have MM - UNITS MFMAs of cover.  The copies fill the second half.
  // job != null: copies c0 .. c1-1 of the job are issued, spread over MFMAs m0 .. MM-1 of the region
  auto region = [&](const bf16x8* fa, const bf16x8* fb, bf16x8* na, bf16x8* nb, lds_u8* st, int nks, const CopyJob* job,
                    int c0 = 0, int c1 = -1, int m0 = -1) {
    if (c1 < 0) c1 = L;
    if (m0 < 0) m0 = MM >= 2 * L ? MM - L : 0;
#pragma unroll
    for (int m = 0; m < MM; m++) {
      const int i = m / TN, j = m % TN;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      constexpr int UPM = (UNITS + MM - 1) / MM;           // fetches per MFMA (1 for the tiles used here)
#pragma unroll
      for (int q = 0; q < UPM; q++) {
        const int u = m * UPM + q;                         // position in the fetch order
        if (u < UNITS) {
          if (u == 0) na[0] = read_frag<BM, AKC>(st + a_base[TA::variant(nks, 0)] + TA::frag_step(nks, 0));
          else if (u <= TN) nb[u - 1] = read_frag<BN, BKC>(st + b_base[TB::variant(nks, u - 1)] + TB::frag_step(nks, u - 1));
          else na[u - TN] = read_frag<BM, AKC>(st + a_base[TA::variant(nks, u - TN)] + TA::frag_step(nks, u - TN));
        }
      }
      if (job) {
        const int n = c1 - c0;
#pragma unroll
        for (int c = c0 + ((m - m0) * n) / (MM - m0); m >= m0 && c < c0 + ((m - m0 + 1) * n) / (MM - m0); c++) copy_one(*job, c);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  static_assert(BK == 32 && (!RINGPIPE || (NS - 2) * L < 64), "the wait counter has 6 bits");
  bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
  auto first_fragments = [&]() {
#pragma unroll
    for (int i = 0; i < TM; i++) fa0[i] = read_frag<BM, AKC>(lds + a_base[TA::variant(0, i)] + TA::frag_step(0, i));
#pragma unroll
    for (int j = 0; j < TN; j++) fb0[j] = read_frag<BN, BKC>(lds + b_base[TB::variant(0, j)] + TB::frag_step(0, j));
  };
  if constexpr (RINGPIPE) {
    // Ring of NS slots, KSTEPS k-steps per slot (an even number: the two fragment register sets alternate).  While
    // k-step ks - 1 of tile t is multiplied, the fragments of k-step ks are fetched; before the last k-step of a slot
    // (its fragments are in registers by then) come the wait for tile t + 1 and the workgroup barrier, and during that
    // last k-step the fragments of (t + 1, k-step 0) are fetched and the copies of tile t + NS - 1 are started.
    if (nk > 0) {
#pragma unroll
      for (int t = 0; t < NS - 1; t++) {
        const CopyJob j = next_job();
#pragma unroll
        for (int c = 0; c < L; c++) copy_one(j, c);
      }
      wait_vmem<(NS - 2) * L>();              // tile 0 has landed (this wave's share)
      __syncthreads();
      first_fragments();
      for (int t = 0; t < nk; t++) {
        lds_u8* const cur = lds + (t % NS) * STAGE_BYTES;
#pragma unroll
        for (int ks = 1; ks < KSTEPS; ks++) {
          if (ks & 1) region(fa0, fb0, fa1, fb1, cur, ks, nullptr);
          else region(fa1, fb1, fa0, fb0, cur, ks, nullptr);
        }
        wait_vmem<(NS - 3) * L>();            // tile t+1 has landed (this wave's share)
        __syncthreads();                      // everyone's share of t+1 landed; everyone is done with tile t-1
        const CopyJob j = next_job();         // tile t + NS - 1
        __builtin_amdgcn_sched_barrier(0);
        region(fa1, fb1, fa0, fb0, lds + ((t + 1) % NS) * STAGE_BYTES, 0, &j);
      }
      wait_vmem<0>();                         // drain the (empty) copies issued past the end
    }
  } else {
    // 64-deep slots, two of them: four k-steps per iteration.  The barrier sits before the last k-step: by then every
    // wave has fetched its last fragments of slot t (they are multiplied from registers in the last k-step), so the
    // barrier both publishes slot t+1 and frees slot t for tile t+2.
    // That refill is issued in two halves: one in the k-step after the barrier, one in the first k-step of the next
    // iteration (it still has three k-steps to land), so the texture path sees no burst of 16 copies per wave.
    // Invariant at the top of iteration t: tile t is landed or fully in flight, the first half of tile t+1 is in
    // flight and j is the job of tile t+1.
    if (nk > 0) {
      {
        const CopyJob j0 = next_job();
#pragma unroll
        for (int c = 0; c < L; c++) copy_one(j0, c);
      }
      CopyJob j = next_job();
#pragma unroll
      for (int c = 0; c < L / 2; c++) copy_one(j, c);
      wait_vmem<L / 2>();                     // tile 0 has landed (this wave's share)
      __syncthreads();
      first_fragments();
      for (int t = 0; t < nk; t++) {
        lds_u8* const cur = lds + (t & 1) * STAGE_BYTES;
        lds_u8* const nxt = lds + ((t + 1) & 1) * STAGE_BYTES;
        region(fa0, fb0, fa1, fb1, cur, 1, &j, L / 2, L, 0);
        region(fa1, fb1, fa0, fb0, cur, 2, nullptr);
        region(fa0, fb0, fa1, fb1, cur, 3, nullptr);
        wait_vmem<0>();                       // tile t+1 has landed (this wave's share)
        __syncthreads();
        j = next_job();                       // tile t + 2 into the slot of tile t
        __builtin_amdgcn_sched_barrier(0);
        region(fa1, fb1, fa0, fb0, nxt, 0, &j, 0, L / 2, 0);
      }
      wait_vmem<0>();
    }
  }

  // ---- epilogue.  Accumulator element e of a 32x32 tile sits at row 8*(e/4) + 4*(lane/32) + e%4, column lane%32:
  // a lane owns single elements of many rows.  Each wave therefore passes its tile through LDS one 32-row strip at
  // a time (the ring is free by now) and reads it back row-major, so that every lane stores 16 contiguous bytes
  // and a wave-wide store covers whole rows of the tile.
  if constexpr (SPLIT) {
    // Partial sums meet in memory: every workgroup of a tile leaves its accumulators there in register order (lane-
    // contiguous stores), takes a ticket, and the one that draws the last ticket adds all slices up in slice order,
    // clears the counter for the next product and goes on to the epilogue.  Nobody waits for anybody: a workgroup that
    // is not last is simply done.
    // The exchange does not depend on where the workgroups run.  The partial sums are written and read with
    // device-scope accesses (16-byte buffer stores / loads with the sc1 cache-policy bit: they go through to, and come
    // from, the level of the memory system that all XCDs share, whatever L2 the workgroup sits behind) and the ticket
    // is a device-scope atomic.
    // Order: every lane waits until its own stores have completed (vmcnt(0)), the workgroup barrier collects all
    // lanes, only then does lane 0 take the ticket; a workgroup that sees the last ticket therefore follows, in
    // time, the completion of every slice's stores, and its loads cannot be served from a stale cached copy.  No
    // cache-wide write-back or invalidate is involved (such a fence would flush the L2 under every other workgroup's
    // operand panels).  The launch map still puts the slices of a tile on one XCD, but only for speed.
    constexpr long TILE = (long)BM * BN;
    constexpr int kDeviceScope = 16;        // cache-policy bit "sc1" of the buffer instructions: device scope
    float* const mine = p.split_ws + ((long)tile_seq * p.split + split_idx) * TILE;
    {
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(mine, (uint32_t)(TILE * sizeof(float)));
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
          for (int e4 = 0; e4 < 4; e4++) {
            u32x4 v;
#pragma unroll
            for (int q = 0; q < 4; q++) v[q] = __float_as_uint(acc[i][j][4 * e4 + q]);
            __builtin_amdgcn_raw_buffer_store_b128(v, rs, ((((i * TN + j) * 4 + e4) * 256 + tid) << 4), 0, kDeviceScope);
          }
    }
    wait_vmem<0>();                         // this lane's partial sums have been written
    LDS_AS int* const last_arrival = reinterpret_cast<LDS_AS int*>(lds);     // (the ring is free once all waves are here)
    __syncthreads();
    if (tid == 0)
      *last_arrival = __hip_atomic_fetch_add(p.split_cnt + tile_seq, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                      (unsigned)(p.split - 1);
    __syncthreads();
    if (!*last_arrival) return;
#pragma unroll
    for (int i = 0; i < TM; i++)
#pragma unroll
      for (int j = 0; j < TN; j++)
#pragma unroll
        for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
    for (int sl = 0; sl < p.split; sl++) {
      const __amdgpu_buffer_rsrc_t rs = make_rsrc(p.split_ws + ((long)tile_seq * p.split + sl) * TILE, (uint32_t)(TILE * sizeof(float)));
#pragma unroll
      for (int i = 0; i < TM; i++)
#pragma unroll
        for (int j = 0; j < TN; j++)
#pragma unroll
          for (int e4 = 0; e4 < 4; e4++) {
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rs, ((((i * TN + j) * 4 + e4) * 256 + tid) << 4), 0, kDeviceScope);
#pragma unroll
            for (int q = 0; q < 4; q++) acc[i][j][4 * e4 + q] += __uint_as_float(v[q]);
          }
    }
    if (tid == 0) __hip_atomic_store(p.split_cnt + tile_seq, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
  __syncthreads();                          // every wave is done with the ring
  OutT* C = reinterpret_cast<OutT*>(p.C) + zo * p.sCo + zi * p.sCi;
  const bf16_t* R = reinterpret_cast<const bf16_t*>(p.R);
  if (R) R += zo * p.sCo + zi * p.sCi;
  constexpr int SW = WN + 4;                // strip row stride in floats
  typedef LDS_AS float lds_f32;
  lds_f32* const strip = reinterpret_cast<lds_f32*>(lds + wave * (32 * SW * 4));
  static_assert(4 * 32 * SW * 4 <= NS * STAGE_BYTES, "strips must fit in the ring");
  constexpr int V = sizeof(OutT) == 4 ? 4 : 8;          // elements per 16-byte store
  // A strip is 32 rows of LPR 16-byte vectors; vector q (row q / LPR) is stored by lane q % 64 in pass q / 64, so
  // a wave-wide store covers whole rows when LPR divides 64 and consecutive rows otherwise (WN = 96).
  constexpr int LPR = WN / V, NVEC = 32 * LPR;
  static_assert(NVEC % 64 == 0, "a strip must be a whole number of wave-wide stores");
#pragma unroll
  for (int i = 0; i < TM; i++) {
#pragma unroll
    for (int j = 0; j < TN; j++)
#pragma unroll
      for (int e = 0; e < 16; e++)
        strip[(8 * (e >> 2) + 4 * (lane >> 5) + (e & 3)) * SW + j * 32 + (lane & 31)] = p.alpha * acc[i][j][e];
    // what the strip needs from memory (old C for +=, residual or probabilities) is requested for the whole strip
    // first, so the stores below wait for one memory latency per strip instead of one per row group
    constexpr int NIT = NVEC / 64;                            // stores per strip, and per request batch:
    constexpr int GRP = NIT <= 8 ? NIT : (NIT % 8 == 0 ? 8 : (NIT % 6 == 0 ? 6 : (NIT % 5 == 0 ? 5 : 4)));
    static_assert(NIT % GRP == 0, "request batches must tile the strip");
    const bool need_pre = (sizeof(OutT) == 4) ? false : (R != nullptr);   // (fp32 += reads its old value in place)
    __builtin_amdgcn_sched_barrier(0);      // keep the next strip's requests from being hoisted over this one
#pragma unroll
    for (int g0 = 0; g0 < NIT; g0 += GRP) {
      u32x4 pre[GRP];
      float dl[GRP];
#pragma unroll
      for (int u = 0; u < GRP; u++) {
        const int q = (g0 + u) * 64 + lane;
        const int grow = m0 + wm * WM + i * 32 + q / LPR, gcol = n0 + wn * WN + (q % LPR) * V;
        if (need_pre && grow < p.M && gcol < p.N) {
          const long idx = (long)grow * p.ldc + gcol;
          pre[u] = *reinterpret_cast<const u32x4*>(R + idx);
          if (p.delta) dl[u] = p.delta[zo * p.sDo + zi * p.sDi + (long)grow * p.ldd];
        }
      }
#pragma unroll
      for (int u = 0; u < GRP; u++) {
        const int qv = (g0 + u) * 64 + lane;
        const int r = qv / LPR, sc = (qv % LPR) * V;
        const int grow = m0 + wm * WM + i * 32 + r, gcol = n0 + wn * WN + sc;
        if (grow < p.M && gcol < p.N) {     // N is a multiple of 8: a vector is inside or outside as a whole
          const long idx = (long)grow * p.ldc + gcol;
          float v[V];
#pragma unroll
          for (int q = 0; q < V; q += 4) {
            const f32x4 t4 = *reinterpret_cast<LDS_AS const f32x4*>(strip + r * SW + sc + q);
            v[q] = t4[0]; v[q + 1] = t4[1]; v[q + 2] = t4[2]; v[q + 3] = t4[3];
          }
          if constexpr (sizeof(OutT) == 4) {
            if (p.accumulate) {
              const f32x4 o = *reinterpret_cast<const f32x4*>(C + idx);
              v[0] += o[0]; v[1] += o[1]; v[2] += o[2]; v[3] += o[3];
            }
            f32x4 w4;
            w4[0] = v[0]; w4[1] = v[1]; w4[2] = v[2]; w4[3] = v[3];
            *reinterpret_cast<f32x4*>(C + idx) = w4;
          } else {
            if (p.delta) {                  // dS = P * (dP - delta[row]); zero above the diagonal
#pragma unroll
              for (int q = 0; q < 4; q++) {
                const float p0 = __uint_as_float(pre[u][q] << 16), p1 = __uint_as_float(pre[u][q] & 0xffff0000u);
                v[2 * q] = (!p.delta_causal || gcol + 2 * q <= grow) ? p0 * (v[2 * q] - dl[u]) : 0.f;
                v[2 * q + 1] = (!p.delta_causal || gcol + 2 * q + 1 <= grow) ? p1 * (v[2 * q + 1] - dl[u]) : 0.f;
              }
            } else if (R) {
#pragma unroll
              for (int q = 0; q < 4; q++) {
                v[2 * q] += __uint_as_float(pre[u][q] << 16);
                v[2 * q + 1] += __uint_as_float(pre[u][q] & 0xffff0000u);
              }
            }
            bf16x8 o;
#pragma unroll
            for (int q = 0; q < 8; q++) o[q] = (bf16_t)v[q];
            *reinterpret_cast<bf16x8*>(C + idx) = o;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
}

template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD, int RING = 0>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmParams p) {
  int tm_i, tn_i, z = (int)blockIdx.z;
  if (gridDim.z == 1) {
    tile_of_block(blockIdx.x, p.tiles_m, p.tiles_n, tm_i, tn_i);
  } else {
    // Batched (per-head) products.  The hardware hands consecutive workgroup ids (x fastest, then z) to the 8 XCDs in
    // turn, and each XCD has its own L2: with the plain id -> (tile, batch entry) map the tiles of one batch entry,
    // which share its operands, would be spread over all 8 XCDs and every L2 would fetch those operands again.  When
    // the batch count is a multiple of 8 the map is therefore regrouped so that an XCD walks whole batch entries; a
    // causal contraction that grows with the tile row starts with the longest tiles of each entry.
    const int nt = (int)gridDim.x;
    int id;
    if ((gridDim.z & 7) == 0) {
      const int lin = (int)blockIdx.x + nt * (int)blockIdx.z;
      const int xcd = lin & 7, j = lin >> 3;
      z = xcd + 8 * (j / nt);
      id = j % nt;
      if (p.causal == CAUSAL_K_END) id = nt - 1 - id;
    } else {
      // otherwise rotating the map by the batch index at least keeps one XCD from getting all the long tiles
      id = ((int)blockIdx.x + 3 * z) % nt;
    }
    if (p.causal == CAUSAL_SKIP_UPPER && p.tiles_m == p.tiles_n) {
      // only the lower-triangular tiles are launched: id = tm (tm + 1) / 2 + tn
      tm_i = (int)((__builtin_sqrtf(8.f * (float)id + 1.f) - 1.f) * 0.5f);
      while (tm_i * (tm_i + 1) / 2 > id) tm_i--;
      while ((tm_i + 1) * (tm_i + 2) / 2 <= id) tm_i++;
      tn_i = id - tm_i * (tm_i + 1) / 2;
    } else {
      tm_i = id % p.tiles_m;
      tn_i = id / p.tiles_m;
    }
  }
  gemm_bf16_tile<BM, BN, AKC, BKC, OutT, KD, false, RING>(p, tm_i, tn_i, z);
}

// Batched product with a causal contraction end (rows of tile i contract over (i + 1) * BM indices) and one tile column:
// a workgroup takes tile nt - 1 - i and then tile i, so every workgroup does the same amount of work, nt + 1 units,
// there are half as many of them (each pays its start-up once per two tiles' worth of streaming) and no compute unit
// is left with a long tile at the end.  Batch entries are regrouped by XCD as in gemm_bf16_kernel.
template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD>
__global__ __launch_bounds__(256) void gemm_bf16_causal_pair_kernel(GemmParams p) {
  const int np = (int)gridDim.x, nt = p.tiles_m;              // np = ceil(nt / 2) workgroups per batch entry
  int z = (int)blockIdx.z, id = (int)blockIdx.x;
  if ((gridDim.z & 7) == 0) {
    const int lin = (int)blockIdx.x + np * (int)blockIdx.z;
    const int xcd = lin & 7, j = lin >> 3;
    z = xcd + 8 * (j / np);
    id = j % np;
  }
  const int reps = (nt - 1 - id > id) ? 2 : 1;                // the middle tile of an odd count stands alone
  for (int r = 0; r < reps; r++) {
    gemm_bf16_tile<BM, BN, AKC, BKC, OutT, KD>(p, r == 0 ? nt - 1 - id : id, 0, z);
    __syncthreads();                          // every wave has read its strip back: the ring may be refilled
  }
}

// `split` workgroups per output tile, each over its slice of the contraction.  Workgroup ids that differ by 8 are made
// the slices of one tile: where the hardware hands consecutive ids to the 8 XCDs in turn, a tile's slices then run
// on one XCD and fetch the tile's operand panels through one L2 (a matter of speed only: the exchange of the partial
// sums is correct wherever the workgroups run).
template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD>
__global__ __launch_bounds__(256) void gemm_bf16_splitk_kernel(GemmParams p) {
  const int v = (int)blockIdx.x, xcd = v & 7, q = v >> 3;
  const int split_idx = q % p.split;
  const int tq = q / p.split;                 // which of this XCD's tiles
  const int nt = p.tiles_m * p.tiles_n;
  if (tq >= (nt >> 3) + (xcd < (nt & 7) ? 1 : 0)) return;
  // the same tile order as the unsplit kernel: an XCD owns a contiguous stretch of it, i.e. a compact patch of tiles
  int tm_i, tn_i;
  tile_of_block(tq * 8 + xcd, p.tiles_m, p.tiles_n, tm_i, tn_i);
  const int tile_seq = tn_i * p.tiles_m + tm_i;
  gemm_bf16_tile<BM, BN, AKC, BKC, OutT, KD, true>(p, tm_i, tn_i, 0, split_idx, tile_seq);
}

__global__ void fill_u32_kernel(unsigned* dst, int n, unsigned value) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = value;
}

// Several independent weight-gradient products (TN layout, fp32 output) in one launch: the tiles of all products form
// one sequence of workgroups, so the compute units that run out of tiles of one product start on the next one
// instead of idling until the slowest tile of a round has finished, and there is one launch instead of one per weight.
// Each product's first workgroup id is a multiple of 8, which keeps the id -> XCD correspondence that the tile map
// relies on; the surplus ids do nothing.
// This pays for short contractions (one micro-batch per product).  For long ones it loses: the 32 tiles an XCD runs at
// a time share operand panels through its L2 only while they walk the contraction in step, which they do when a
// launch starts them together and stop doing once tiles of different products and start times are mixed.
__global__ __launch_bounds__(256) void gemm_tn_grouped_kernel(GroupedTable g) {
  int lo = 0, hi = g.n - 1;                   // last product whose first workgroup id is <= blockIdx.x
  const int bid = (int)blockIdx.x;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (g.first_block[mid] <= bid) lo = mid; else hi = mid - 1;
  }
  const GroupedProduct& q = g.prod[lo];
  const int pid = bid - g.first_block[lo];
  const int tiles_m = (q.M + 255) / 256, tiles_n = (q.N + 255) / 256;
  if (pid >= tiles_m * tiles_n) return;
  GemmParams p{};
  p.A = q.A; p.B = q.B; p.C = q.C;
  p.lda = q.lda; p.ldb = q.ldb; p.ldc = q.ldc;
  p.M = q.M; p.N = q.N; p.K = q.K;
  p.batch_inner = 1; p.tiles_m = tiles_m; p.tiles_n = tiles_n;
  p.alpha = 1.f; p.accumulate = q.accumulate; p.causal = CAUSAL_NONE;
  int tm_i, tn_i;
  tile_of_block(pid, tiles_m, tiles_n, tm_i, tn_i);
  gemm_bf16_tile<256, 256, false, false, float>(p, tm_i, tn_i, 0);
}

// ------------------------------------------------------------------------------------------ ceiling
// Register-resident MFMA loop: 4 waves per compute unit, 16 independent 32x32x16 bf16 MFMAs per iteration on
// operands that never leave the registers.  It measures what the matrix pipes sustain under the chip's power
// management with no memory system involved: the practical ceiling the GEMM kernel is compared with.
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(int iters, const bf16_t* __restrict__ seed,
                                                           float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; i++) {
    a[i] = *reinterpret_cast<const bf16x8*>(seed + (size_t)(i * 64 + lane) * 8);
    b[i] = *reinterpret_cast<const bf16x8*>(seed + (size_t)((4 + i) * 64 + lane) * 8);
  }
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) acc[i][j][e] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
      for (int j = 0; j < 4; j++)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < 4; i++)
#pragma unroll
    for (int j = 0; j < 4; j++)
#pragma unroll
      for (int e = 0; e < 16; e++) t += acc[i][j][e];
  sink[(size_t)blockIdx.x * 256 + threadIdx.x] = t;
}

hipError_t mfma_ceiling(int blocks, int iters, const void* seed, float* sink, hipStream_t s) {
  hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(blocks), dim3(256), 0, s, iters, (const bf16_t*)seed, sink);
  return hipGetLastError();
}

// ------------------------------------------------------------------------------------------ fp32
// 64 x 64 x 16 tile, 256 threads, 4 x 4 outputs per thread; operands addressed through element strides so
// one kernel serves NN, NT and TN.
template <typename OutT>
__global__ __launch_bounds__(256) void gemm_f32_kernel(GemmParams p) {
  constexpr int TB = 64, TK = 16;
  __shared__ float As[TK][TB + 4];
  __shared__ float Bs[TK][TB + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int tm_i = blockIdx.x / p.tiles_n, tn_i = blockIdx.x - tm_i * p.tiles_n;
  const int m0 = tm_i * TB, n0 = tn_i * TB;
  int k_lo = 0, k_hi = p.K;
  if (p.causal == CAUSAL_SKIP_UPPER) {
    if (n0 > m0 + TB - 1) return;
  } else if (p.causal == CAUSAL_K_END) {
    k_hi = (m0 + TB < p.K) ? m0 + TB : p.K;
  } else if (p.causal == CAUSAL_K_BEGIN) {
    k_lo = m0;
  }
  const int z = blockIdx.z;
  const int zo = z / p.batch_inner, zi = z - zo * p.batch_inner;
  const float* A = reinterpret_cast<const float*>(p.A) + zo * p.sAo + zi * p.sAi;
  const float* B = reinterpret_cast<const float*>(p.B) + zo * p.sBo + zi * p.sBi;
  float acc[4][4] = {};
  for (int k0 = k_lo; k0 < k_hi; k0 += TK) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      const int e = tid + 256 * i;            // 1024 elements of each tile
      // A tile: consecutive threads along the contiguous direction of the layout
      int am, ak, bn, bk;
      if (p.sak == 1) { ak = e & 15; am = e >> 4; } else { am = e & 63; ak = e >> 6; }
      if (p.sbn == 1) { bn = e & 63; bk = e >> 6; } else { bk = e & 15; bn = e >> 4; }
      const bool aok = (m0 + am < p.M) && (k0 + ak < k_hi);
      const bool bok = (n0 + bn < p.N) && (k0 + bk < k_hi);
      As[ak][am] = aok ? A[(long)(m0 + am) * p.sam + (long)(k0 + ak) * p.sak] : 0.f;
      Bs[bk][bn] = bok ? B[(long)(k0 + bk) * p.sbk + (long)(n0 + bn) * p.sbn] : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < TK; k++) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; i++) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; j++) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  OutT* C = reinterpret_cast<OutT*>(p.C) + zo * p.sCo + zi * p.sCi;
  const float* R = reinterpret_cast<const float*>(p.R);
  if (R) R += zo * p.sCo + zi * p.sCi;
#pragma unroll
  for (int i = 0; i < 4; i++) {
    const int row = m0 + ty * 4 + i;
    if (row >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int col = n0 + tx * 4 + j;
      if (col >= p.N) continue;
      const long idx = (long)row * p.ldc + col;
      float v = p.alpha * acc[i][j];
      if (p.delta) {
        const float dl = p.delta[zo * p.sDo + zi * p.sDi + (long)row * p.ldd];
        v = (!p.delta_causal || col <= row) ? R[idx] * (v - dl) : 0.f;
      } else {
        if (p.accumulate) v += C[idx];
        if (R) v += R[idx];
      }
      C[idx] = v;
    }
  }
}

// ------------------------------------------------------------------------------------------ host
template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD, int RING = 0>
static hipError_t launch_bf16(const GemmParams& p0, int batch, hipStream_t s) {
  GemmParams p = p0;
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  constexpr size_t smem = (size_t)(RING >= 3 ? RING : (KD == 32 ? STAGES : 2)) * (BM + BN) * KD * sizeof(bf16_t);
  static_assert(smem <= 160 * 1024, "LDS budget of one gfx950 compute unit");
  auto kern = gemm_bf16_kernel<BM, BN, AKC, BKC, OutT, KD, RING>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  unsigned nt = (unsigned)(p.tiles_m * p.tiles_n);
  if (batch > 1 && p.causal == CAUSAL_SKIP_UPPER && p.tiles_m == p.tiles_n)
    nt = (unsigned)(p.tiles_m * (p.tiles_m + 1) / 2);       // lower-triangular tiles only
  dim3 grid(nt, 1, (unsigned)batch);
  hipLaunchKernelGGL(kern, grid, dim3(256), smem, s, p);
  return hipGetLastError();
}

template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD>
static hipError_t launch_bf16_causal_pair(const GemmParams& p0, int batch, hipStream_t s) {
  GemmParams p = p0;
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  if (p.tiles_n != 1 || p.causal != CAUSAL_K_END) return hipErrorInvalidValue;
  constexpr size_t smem = (size_t)(KD == 32 ? STAGES : 2) * (BM + BN) * KD * sizeof(bf16_t);
  auto kern = gemm_bf16_causal_pair_kernel<BM, BN, AKC, BKC, OutT, KD>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3((unsigned)((p.tiles_m + 1) / 2), 1, (unsigned)batch), dim3(256), smem, s, p);
  return hipGetLastError();
}

// Tiles 192 columns wide for the linear-layer products whose output fills the chip badly with 256 x 256 tiles (too
// few of them, or a last round that is mostly empty): e.g. [2048, 5120] is 160 large tiles (62 % of a round) but 216
// of the narrower ones (84 %).  Taken when the fraction of the rounds' capacity that is useful output, discounted
// 7 % for the narrower tile's lower operand reuse, beats what the other choice gives by 8 %; the small-tile kernel,
// which outputs of fewer than 192 large tiles otherwise use, counts as 0.60.
static bool narrow_tiles_pay(int M, int N, int K) {
  if (M < 256 || N < 192 || K <= 256) return false;
  const long tiles_m = (M + 255) / 256;
  const long t256 = tiles_m * ((N + 255) / 256), t192 = tiles_m * ((N + 191) / 192);
  const double area = (double)M * N;
  const double now = (N >= 256 && t256 >= 192) ? area / ((double)((t256 + 255) / 256) * 256 * 65536) : 0.60;
  const double narrow = 0.93 * area / ((double)((t192 + 255) / 256) * 256 * 49152);
  return t192 >= 192 && narrow > 1.08 * now;
}

// Cost model behind gemm_split_plan, fitted to measurements on this chip (microseconds): a round of large tiles costs
// 0.0245 per contraction index plus 12 of prologue and epilogue; the exchange of partial sums costs about 30 plus
// 0.67 per MiB of partials (they are written by every workgroup but read back by one workgroup per tile only); the
// small-tile kernel that such outputs otherwise use sustains about 800 TFLOP/s when it has a tile for every compute
// unit.  In practice only long contractions
// pay: e.g. [2048, 5120] x K = 27648 runs in 590 us split three ways against 810 us.
SplitPlan gemm_split_plan(int dtype, int layout, int M, int N, int K, int out_f32, int batch) {
  SplitPlan none{1, 0};
  if (dtype != 1 || out_f32 || batch != 1 || layout == TN || M < 256 || N < 256) return none;
  const long tiles = (long)((M + 255) / 256) * ((N + 255) / 256);
  if (tiles >= 192 || narrow_tiles_pay(M, N, K)) return none;
  const long small_tiles = (long)((M + 127) / 128) * ((N + 127) / 128);      // (fewer than 256 of them leave CUs idle)
  double best = 2.0 * M * N * (double)K / (800e6 * (small_tiles < 256 ? small_tiles / 256.0 : 1.0));
  int split = 1;
  for (int sp = 2; sp <= 8; sp++) {
    if (K / sp < 512) break;
    const long rounds = (tiles * sp + 255) / 256;
    const double t = rounds * (0.0245 * K / sp + 12.0) + 30.0 + 0.67 * (tiles * sp * 0.25);
    if (t < 0.9 * best) { best = t; split = sp; }
  }
  if (split == 1) return none;
  return SplitPlan{split, kSplitCounterBytes + (size_t)tiles * split * 256 * 256 * sizeof(float)};
}

template <int BM, int BN, bool AKC, bool BKC, typename OutT, int KD>
static hipError_t launch_bf16_split(const GemmParams& p0, int split, void* ws, int counters_zero, hipStream_t s) {
  GemmParams p = p0;
  p.tiles_m = (p.M + BM - 1) / BM;
  p.tiles_n = (p.N + BN - 1) / BN;
  p.split = split;
  p.split_cnt = static_cast<unsigned*>(ws);
  p.split_ws = reinterpret_cast<float*>(static_cast<char*>(ws) + kSplitCounterBytes);
  const int tiles = p.tiles_m * p.tiles_n;
  if ((size_t)tiles * sizeof(unsigned) > kSplitCounterBytes) return hipErrorInvalidValue;
  constexpr size_t smem = (size_t)(KD == 32 ? STAGES : 2) * (BM + BN) * KD * sizeof(bf16_t);
  auto kern = gemm_bf16_splitk_kernel<BM, BN, AKC, BKC, OutT, KD>;
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(kern), smem); e != hipSuccess) return e;
  if (!counters_zero) {
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(256), 0, s, p.split_cnt, (int)(kSplitCounterBytes / 4), 0u);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  const unsigned blocks = (unsigned)((tiles + 7) / 8 * 8 * split);
  hipLaunchKernelGGL(kern, dim3(blocks), dim3(256), smem, s, p);
  return hipGetLastError();
}

// Slot depth by layout and tile size: operands with a contiguous contraction index get the 64-deep slots on the
// large tiles (whole cache lines per tile row: up to 8 % faster); on the small tiles, which run two or three
// workgroups per compute unit and overlap that way, the 4-slot ring of 32-deep slots stays ahead.
#ifndef TBP_KC_DEPTH_SMALL
#define TBP_KC_DEPTH_SMALL 32
#endif
// The weight-gradient layout (both operands strided in the contraction index) on 64-deep slots, half the barriers
// and waits per unit of K: measured 0 to 4 % slower than the ring of four 32-deep slots.
#ifndef TBP_TN_DEPTH
#define TBP_TN_DEPTH 32
#endif
// The 256 x 192 tiles: two 64-deep slots (rings of four or five 32-deep slots measured 5 to 10 % slower: K-contiguous
// operands then arrive in half cache lines; a third 64-deep slot does not fit the LDS).
#ifndef TBP_NARROW_KD
#define TBP_NARROW_KD 64
#define TBP_NARROW_RING 0
#endif
#ifndef TBP_SMALL_DEEP_RING
#define TBP_SMALL_DEEP_RING 4
#endif
#ifndef TBP_SMALL_DEEP_KD
#define TBP_SMALL_DEEP_KD 64
#endif
// Small tiles with a deep ring: when the whole output is at most one small tile per compute unit (e.g. [1024, 4096]),
// no second workgroup shares the CU to cover the first one's waits, and a 32-deep slot of a 128 x 128 tile is
// multiplied in 256 clocks, so the three slots that a ring of four keeps in flight cover under 800 clocks of memory
// latency.  Such products get a ring of four 64-deep slots (128 KiB of LDS; one workgroup per CU anyway): three
// times 512 clocks of cover, and K-contiguous operands are fetched in whole 128-byte lines.  Measured on
// [1024, 4096] outputs: K = 12288 (NT) 126 -> 107 us, K = 22016 (NT) 237 -> 216 us, K = 11008 (NN) 104 -> 93 us;
// a ring of eight 32-deep slots gains 3 %, three 64-deep slots lose 5 %, five (all 160 KiB) lose too.
template <typename OutT>
static hipError_t dispatch_small_deep(int layout, const GemmParams& p, hipStream_t s) {
  switch (layout) {
    case NN: return launch_bf16<128, 128, true, false, OutT, TBP_SMALL_DEEP_KD, TBP_SMALL_DEEP_RING>(p, 1, s);
    case NT: return launch_bf16<128, 128, true, true, OutT, TBP_SMALL_DEEP_KD, TBP_SMALL_DEEP_RING>(p, 1, s);
    case TN: return launch_bf16<128, 128, false, false, OutT, 32, 8>(p, 1, s);
  }
  return hipErrorInvalidValue;
}

template <int BM, int BN, typename OutT>
static hipError_t dispatch_layout(int layout, const GemmParams& p, int batch, hipStream_t s) {
  constexpr int KD = BM >= 256 ? 64 : TBP_KC_DEPTH_SMALL;
  switch (layout) {
    case NN: return launch_bf16<BM, BN, true, false, OutT, KD>(p, batch, s);
    case NT: return launch_bf16<BM, BN, true, true, OutT, KD>(p, batch, s);
    case TN: return launch_bf16<BM, BN, false, false, OutT, (BM >= 256 ? TBP_TN_DEPTH : 32)>(p, batch, s);
  }
  return hipErrorInvalidValue;
}

hipError_t gemm_tn_grouped(const GroupedProduct* prods, int n, hipStream_t s) {
  constexpr size_t smem = (size_t)STAGES * (256 + 256) * BK * sizeof(bf16_t);
  static AttrOnce once;
  if (hipError_t e = once.set(reinterpret_cast<const void*>(gemm_tn_grouped_kernel), smem); e != hipSuccess) return e;
  for (int base = 0; base < n; base += kMaxGrouped) {
    GroupedTable g{};
    int blocks = 0;
    for (int i = base; i < n && g.n < kMaxGrouped; i++) {
      if (prods[i].M <= 0 || prods[i].N <= 0) continue;
      g.prod[g.n] = prods[i];
      g.first_block[g.n] = blocks;
      const int tiles = ((prods[i].M + 255) / 256) * ((prods[i].N + 255) / 256);
      blocks += (tiles + 7) & ~7;
      g.n++;
    }
    if (g.n == 0) continue;
    hipLaunchKernelGGL(gemm_tn_grouped_kernel, dim3((unsigned)blocks), dim3(256), smem, s, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t gemm(int dtype, const GemmArgs& g, hipStream_t s) {
  if (g.M <= 0 || g.N <= 0 || g.batch <= 0) return hipSuccess;     // empty product: nothing to write
  GemmParams p{};
  p.A = g.A; p.B = g.B; p.C = g.C; p.R = g.R;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc;
  p.sAo = g.sAo; p.sAi = g.sAi; p.sBo = g.sBo; p.sBi = g.sBi; p.sCo = g.sCo; p.sCi = g.sCi;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.batch_inner = g.batch_inner > 0 ? g.batch_inner : 1;
  p.alpha = g.alpha; p.accumulate = g.accumulate; p.causal = g.causal;
  p.delta = g.delta; p.ldd = g.ldd; p.sDo = g.sDo; p.sDi = g.sDi; p.delta_causal = g.delta_causal;
  if (dtype == 0) {
    if (g.a_panel) return hipErrorInvalidValue;
    switch (g.layout) {
      case NN: p.sam = g.lda; p.sak = 1; p.sbk = g.ldb; p.sbn = 1; break;
      case NT: p.sam = g.lda; p.sak = 1; p.sbk = 1; p.sbn = g.ldb; break;
      case TN: p.sam = 1; p.sak = g.lda; p.sbk = g.ldb; p.sbn = 1; break;
      default: return hipErrorInvalidValue;
    }
    p.tiles_m = (g.M + 63) / 64;
    p.tiles_n = (g.N + 63) / 64;
    dim3 grid((unsigned)(p.tiles_m * p.tiles_n), 1, (unsigned)g.batch);
    hipLaunchKernelGGL(gemm_f32_kernel<float>, grid, dim3(256), 0, s, p);   // fp32 storage: C is fp32 either way
    return hipGetLastError();
  }
  if (g.a_panel) {
    if (g.layout != TN || g.lda != kPanel || g.ws) return hipErrorInvalidValue;
    p.a_panel = g.a_panel;
    // (pairs only when they still give every compute unit its two workgroups)
    if (!g.out_f32 && g.causal == CAUSAL_K_END && g.N <= 128 && !g.delta &&
        (long)((g.M + kPanel - 1) / kPanel + 1) / 2 * g.batch >= 512)
      return launch_bf16_causal_pair<kPanel, 128, false, false, bf16_t, 32>(p, g.batch, s);
    return g.out_f32 ? launch_bf16<kPanel, 128, false, false, float, 32>(p, g.batch, s)
                     : launch_bf16<kPanel, 128, false, false, bf16_t, 32>(p, g.batch, s);
  }
  // bf16: large tiles when the output is big enough to fill 256 compute units with them
  const int tiles_m = (g.M + 255) / 256, tiles_n = (g.N + 255) / 256;
  const long tiles_big = (long)tiles_m * tiles_n * g.batch;
  // short contractions (the per-head q k^T and do v^T, K = head_dim) are all prologue and epilogue: small tiles let
  // two or three workgroups share a compute unit and overlap them
  const bool big = g.M >= 256 && g.N >= 256 && tiles_big >= 192 && g.K > 256;
  if (!g.out_f32 && g.batch == 1 && g.causal == CAUSAL_NONE && !g.delta && g.layout != TN && narrow_tiles_pay(g.M, g.N, g.K))
    return g.layout == NN ? launch_bf16<256, 192, true, false, bf16_t, TBP_NARROW_KD, TBP_NARROW_RING>(p, 1, s)
                          : launch_bf16<256, 192, true, true, bf16_t, TBP_NARROW_KD, TBP_NARROW_RING>(p, 1, s);
  if (g.ws && g.causal == CAUSAL_NONE && !g.delta && reinterpret_cast<uintptr_t>(g.ws) % 256 == 0) {
    const SplitPlan plan = gemm_split_plan(dtype, g.layout, g.M, g.N, g.K, g.out_f32, g.batch);
    if (plan.split > 1 && plan.bytes <= g.ws_bytes)
      return g.layout == NN ? launch_bf16_split<256, 256, true, false, bf16_t, 64>(p, plan.split, g.ws, g.ws_counters_zero, s)
                            : launch_bf16_split<256, 256, true, true, bf16_t, 64>(p, plan.split, g.ws, g.ws_counters_zero, s);
  }
  auto run = [&](const GemmParams& q, bool use_big) -> hipError_t {
    if (!use_big && g.batch == 1 && q.K >= 1024 && (long)((q.M + 127) / 128) * ((q.N + 127) / 128) <= 256)
      return g.out_f32 ? dispatch_small_deep<float>(g.layout, q, s) : dispatch_small_deep<bf16_t>(g.layout, q, s);
    if (g.out_f32)
      return use_big ? dispatch_layout<256, 256, float>(g.layout, q, g.batch, s)
                     : dispatch_layout<128, 128, float>(g.layout, q, g.batch, s);
    return use_big ? dispatch_layout<256, 256, bf16_t>(g.layout, q, g.batch, s)
                   : dispatch_layout<128, 128, bf16_t>(g.layout, q, g.batch, s);
  };
  // Tail quantisation: with nt large tiles on 256 compute units the last round runs nt % 256 workgroups.  When
  // that round would be at most three quarters full, the output is cut along its longer side into a part made of
  // whole rounds of large tiles and a remainder: up to half a round's worth runs on 128 x 128 tiles (four times as
  // many workgroups), more than that on 256 x 192 tiles where that kernel exists for the layout (4/3 as many
  // workgroups: one nearly full round of tiles that take 3/4 of the time).
  const long rem = tiles_big % 256;
  const bool has_narrow = (g.out_f32 && g.layout == TN) || (!g.out_f32 && g.layout != TN && !g.delta);
  auto run_rest = [&](const GemmParams& q) -> hipError_t {
    const long t192 = (long)((q.M + 255) / 256) * ((q.N + 191) / 192);
    if (rem <= 128 || !has_narrow || t192 > 256) return run(q, rem > 128);
    if (g.out_f32) return launch_bf16<256, 192, false, false, float, 32>(q, 1, s);
    return g.layout == NN ? launch_bf16<256, 192, true, false, bf16_t, TBP_NARROW_KD, TBP_NARROW_RING>(q, 1, s)
                          : launch_bf16<256, 192, true, true, bf16_t, TBP_NARROW_KD, TBP_NARROW_RING>(q, 1, s);
  };
  const bool defer = g.defer_rest && g.out_f32 && g.layout == TN && g.alpha == 1.f && !g.a_panel;
  if (g.defer_rest) g.defer_rest->M = 0;
  auto hold_back = [&](const GemmParams& q) {       // the remainder, for the caller's grouped launch
    GroupedProduct& r = *g.defer_rest;
    r.A = q.A; r.B = q.B; r.C = static_cast<float*>(q.C);
    r.M = q.M; r.N = q.N; r.K = q.K;
    r.lda = (int)q.lda; r.ldb = (int)q.ldb; r.ldc = (int)q.ldc;
    r.accumulate = q.accumulate;
  };
  if (big && g.batch == 1 && g.causal == CAUSAL_NONE && tiles_big > 256 && rem != 0 &&
      (defer || rem <= 128 || (has_narrow && rem <= 192))) {
    const long whole = tiles_big - rem;
    const size_t ce = g.out_f32 ? 4 : 2;
    GemmParams a = p, b = p;
    if (tiles_n >= tiles_m) {                       // cut along N
      const int cols = (int)(whole / tiles_m);      // tile columns of the first part
      if (cols > 0 && cols < tiles_n) {
        const long n0 = (long)cols * 256;
        a.N = (int)n0;
        b.N = g.N - (int)n0;
        b.B = (const char*)p.B + (g.layout == NT ? n0 * g.ldb : n0) * 2;
        b.C = (char*)p.C + n0 * ce;
        if (p.R) b.R = (const char*)p.R + n0 * 2;
        hipError_t e = run(a, true);
        if (defer) { hold_back(b); return e; }
        return e != hipSuccess ? e : run_rest(b);
      }
    } else {                                        // cut along M
      const int rows = (int)(whole / tiles_n);
      if (rows > 0 && rows < tiles_m) {
        const long m0 = (long)rows * 256;
        a.M = (int)m0;
        b.M = g.M - (int)m0;
        b.A = (const char*)p.A + (g.layout == TN ? m0 : m0 * g.lda) * 2;
        b.C = (char*)p.C + m0 * g.ldc * ce;
        if (p.R) b.R = (const char*)p.R + m0 * g.ldc * 2;
        hipError_t e = run(a, true);
        if (defer) { hold_back(b); return e; }
        return e != hipSuccess ? e : run_rest(b);
      }
    }
  }
  return run(p, big);
}

}  // namespace tbp
