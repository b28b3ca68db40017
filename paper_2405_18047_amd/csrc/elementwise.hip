// HBM-bound kernels of the stage: RMSNorm, SwiGLU, rotary embedding, softmax (forward and backward-p1).
// All of them move 16 bytes per lane per access, keep a row's values in registers between the
// reduction and the write (one read of every input, one write of every output), do their arithmetic in
// fp32 and reduce over a row with wavefront (64-lane) butterflies.
#include "kernels.h"

namespace tbp {

typedef __bf16 bf16_t;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

// ---- 16-byte vector access, unpacked to fp32 ------------------------------------------------------
template <typename T> struct Vec;
template <> struct Vec<float> {
  static constexpr int N = 4;
  typedef float4 Raw;
  static __device__ __forceinline__ Raw load_raw(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ void unpack(const Raw& r, float* v) { v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w; }
  static __device__ __forceinline__ void load(const float* p, float* v) {
    const float4 r = *reinterpret_cast<const float4*>(p);
    v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
  }
  static __device__ __forceinline__ void store(float* p, const float* v) {
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  }
};
template <> struct Vec<bf16_t> {
  static constexpr int N = 8;
  typedef u32x4 Raw;
  static __device__ __forceinline__ Raw load_raw(const bf16_t* p) { return *reinterpret_cast<const u32x4*>(p); }
  static __device__ __forceinline__ void unpack(const Raw& r, float* v) {
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(r[i] << 16);
      v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float* v) {
    const u32x4 r = *reinterpret_cast<const u32x4*>(p);
#pragma unroll
    for (int i = 0; i < 4; i++) {
      v[2 * i] = __uint_as_float(r[i] << 16);
      v[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float* v) {
    typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
    bf16x8 o;
#pragma unroll
    for (int i = 0; i < 8; i++) o[i] = (bf16_t)v[i];      // round to nearest even
    *reinterpret_cast<bf16x8*>(p) = o;
  }
};

// Wavefront (64-lane) reductions on the data-parallel-primitive path: four in-row steps (quad swaps, half-row and
// row mirrors), then the row totals are chained with row_bcast15 / row_bcast31, which leaves the result in lane 63.
// No LDS traffic and no cross-lane permute unit involved.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_move(float identity, float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, identity),
                                                               __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_move<0xB1, 0xF>(0.f, v);     // quad_perm [1,0,3,2]
  v += dpp_move<0x4E, 0xF>(0.f, v);     // quad_perm [2,3,0,1]
  v += dpp_move<0x141, 0xF>(0.f, v);    // row_half_mirror
  v += dpp_move<0x140, 0xF>(0.f, v);    // row_mirror: every lane of a 16-lane row holds the row total
  v += dpp_move<0x142, 0xA>(0.f, v);    // row_bcast15 into rows 1 and 3
  v += dpp_move<0x143, 0xC>(0.f, v);    // row_bcast31 into rows 2 and 3: lane 63 holds the wave total
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
  const float ninf = -INFINITY;
  v = fmaxf(v, dpp_move<0xB1, 0xF>(ninf, v));
  v = fmaxf(v, dpp_move<0x4E, 0xF>(ninf, v));
  v = fmaxf(v, dpp_move<0x141, 0xF>(ninf, v));
  v = fmaxf(v, dpp_move<0x140, 0xF>(ninf, v));
  v = fmaxf(v, dpp_move<0x142, 0xA>(ninf, v));
  v = fmaxf(v, dpp_move<0x143, 0xC>(ninf, v));
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// ---- RMSNorm forward: one 256-thread workgroup per row ----------------------------------------------
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(int rows, int d, float eps, const T* __restrict__ x,
                                                          const T* __restrict__ g, T* __restrict__ y) {
  constexpr int N = Vec<T>::N;
  __shared__ float red[4];
  const int row = blockIdx.x;
  const int nchunk = d / N;
  const T* xr = x + (long)row * d;
  float xv[MAXC][N];
  float ss = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int ch = threadIdx.x + 256 * c;
    if (ch < nchunk) {
      Vec<T>::load(xr + ch * N, xv[c]);
#pragma unroll
      for (int i = 0; i < N; i++) ss += xv[c][i] * xv[c][i];
    }
  }
  ss = wave_sum(ss);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float r = rsqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int ch = threadIdx.x + 256 * c;
    if (ch < nchunk) {
      float gv[N], o[N];
      Vec<T>::load(g + ch * N, gv);
#pragma unroll
      for (int i = 0; i < N; i++) o[i] = xv[c][i] * r * gv[i];
      Vec<T>::store(y + (long)row * d + ch * N, o);
    }
  }
}

// ---- RMSNorm backward-p1 (+ residual fan-in, + gain-gradient partials) -------------------------------
// dx = resid + r*yhat - x * r^3 * mean(yhat * x), yhat = dy * g;  gain gradient: column sums of dy * x * r.
// 512 threads = 8 waves = 8/WPR row groups of WPR waves; each group owns one row at a time (a row's x and dy are
// fetched in one go and kept packed in registers, at most MAXC 16-byte vectors per lane).  The two row sums are
// wavefront reductions; only when a row is wider than one wave can hold (WPR > 1) do the group's waves meet in
// LDS, with one barrier per row.  Column partials of the gain gradient stay in registers over the rows a group
// sees and are folded over the groups through LDS in group order (fixed order: reproducible) into one partial row
// per workgroup, which colsum_kernel adds up.
// GAIN_ONLY (the gain gradient as a backward-p2 operation): only x and dy are read, and only the partials written.
// partials == nullptr (backward-p1 of a stage that computes the gain gradient in p2): nothing is written for the gain.
template <typename T, int MAXC, int WPR, bool GAIN_ONLY = false, int NW = 8>
__global__ __launch_bounds__(64 * NW) void rmsnorm_p1_kernel(int rows, int d, float eps, const T* __restrict__ dy,
                                                         const T* __restrict__ x, const T* __restrict__ g,
                                                         const T* __restrict__ resid, T* __restrict__ dx,
                                                         float* __restrict__ partials) {
  constexpr int N = Vec<T>::N, G = NW / WPR, TPR = 64 * WPR;     // groups per workgroup, threads per row
  typedef typename Vec<T>::Raw Raw;
  extern __shared__ float lds[];              // [2][NW waves][2 sums] reduction slots, then [d] column buffer
  float* const red = lds;
  float* const colbuf = lds + 4 * NW;
  const int wave = threadIdx.x >> 6, grp = wave / WPR, t = threadIdx.x - grp * TPR;
  const int nchunk = d / N;
  float cacc[MAXC][N];
#pragma unroll
  for (int c = 0; c < MAXC; c++)
#pragma unroll
    for (int i = 0; i < N; i++) cacc[c][i] = 0.f;
  const int stride = G * gridDim.x;
  const int iters = (rows + stride - 1) / stride;
  // rows are double-buffered in registers: the next row's x, dy and residual are requested before the current
  // row is reduced, so a memory latency is paid once per workgroup, not once per row
  Raw xn[MAXC], yn[MAXC], rn[MAXC];
  auto fetch = [&](int it) {
    const int row = (it * (int)gridDim.x + (int)blockIdx.x) * G + grp;
    if (it < iters && row < rows) {
      const long base = (long)row * d;
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (ch < nchunk) {
          xn[c] = Vec<T>::load_raw(x + base + ch * N);
          yn[c] = Vec<T>::load_raw(dy + base + ch * N);
          if (!GAIN_ONLY && resid) rn[c] = Vec<T>::load_raw(resid + base + ch * N);
        }
      }
    }
  };
  fetch(0);
  for (int it = 0; it < iters; it++) {
    const int row = (it * (int)gridDim.x + (int)blockIdx.x) * G + grp;
    const bool live = row < rows;
    const long base = (long)row * d;
    Raw xr[MAXC], yr[MAXC], rr[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; c++) { xr[c] = xn[c]; yr[c] = yn[c]; rr[c] = rn[c]; }
    fetch(it + 1);
    // the gain vector is a few KiB and is re-read from the caches for every row: hiding the pointer from the
    // optimiser keeps it from hoisting MAXC more live vectors per lane out of the row loop
    const T* gp = g;
    asm volatile("" : "+s"(gp));
    float s_xx = 0.f, s_yx = 0.f;
#pragma unroll
    for (int c = 0; c < MAXC; c++) {
      const int ch = t + TPR * c;
      if (live && ch < nchunk) {
        float xv[N], yv[N], gv[N];
        Vec<T>::unpack(xr[c], xv);
        Vec<T>::unpack(yr[c], yv);
        if constexpr (!GAIN_ONLY) Vec<T>::load(gp + ch * N, gv);
#pragma unroll
        for (int i = 0; i < N; i++) {
          s_xx += xv[i] * xv[i];
          if constexpr (!GAIN_ONLY) s_yx += yv[i] * gv[i] * xv[i];
        }
      }
    }
    s_xx = wave_sum(s_xx);
    if constexpr (!GAIN_ONLY) s_yx = wave_sum(s_yx);
    if constexpr (WPR > 1) {                  // two slot sets used alternately: one barrier per row is enough
      float* const slot = red + (it & 1) * 2 * NW;
      if ((threadIdx.x & 63) == 0) {
        slot[wave * 2] = s_xx;
        slot[wave * 2 + 1] = s_yx;
      }
      __syncthreads();
      s_xx = 0.f; s_yx = 0.f;
#pragma unroll
      for (int w = 0; w < WPR; w++) {
        s_xx += slot[(grp * WPR + w) * 2];
        s_yx += slot[(grp * WPR + w) * 2 + 1];
      }
    }
    const float r = rsqrtf(s_xx / (float)d + eps);
    const float coef = r * r * r * (s_yx / (float)d);
#pragma unroll
    for (int c = 0; c < MAXC; c++) {
      const int ch = t + TPR * c;
      if (live && ch < nchunk) {
        float xv[N], yv[N];
        Vec<T>::unpack(xr[c], xv);
        Vec<T>::unpack(yr[c], yv);
#pragma unroll
        for (int i = 0; i < N; i++) cacc[c][i] += yv[i] * xv[i] * r;
        if constexpr (!GAIN_ONLY) {
          float gv[N], o[N];
          Vec<T>::load(gp + ch * N, gv);
          if (resid) Vec<T>::unpack(rr[c], o);
          else {
#pragma unroll
            for (int i = 0; i < N; i++) o[i] = 0.f;
          }
#pragma unroll
          for (int i = 0; i < N; i++) o[i] += r * yv[i] * gv[i] - xv[i] * coef;
          Vec<T>::store(dx + base + ch * N, o);
        }
      }
    }
  }
  if (!partials) return;                      // (uniform over the grid)
  __syncthreads();
  for (int gi = 0; gi < G; gi++) {
    if (grp == gi) {
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (ch < nchunk) {
#pragma unroll
          for (int i = 0; i < N; i++) {
            const int col = ch * N + i;
            colbuf[col] = (gi == 0 ? 0.f : colbuf[col]) + cacc[c][i];
          }
        }
      }
    }
    __syncthreads();
  }
  for (int col = threadIdx.x; col < d; col += 64 * NW) partials[(long)blockIdx.x * d + col] = colbuf[col];
}

// The same operation with a deeper request queue.  WPR waves share a row (64 * WPR lanes, MAXC vectors per lane and
// tensor), G = NW / WPR rows are in work per workgroup, and every lane keeps the x, dy and residual vectors of its
// next PD rows in a register ring: a row's loads are issued PD iterations before the row is reduced, so each compute
// unit has G * PD rows (24 KiB each at d = 4096) in flight at all times instead of G, which is what a memory system
// with several microseconds of loaded latency needs to stay busy.  The lane's slice of the gain vector stays unpacked
// in registers for the whole kernel (a lane owns the same columns in every row).  Reductions and the fold of the gain
// gradient's column partials are those of the kernel above.
template <typename T, int MAXC, int WPR, bool GAIN_ONLY, int NW, int PD>
__global__ __launch_bounds__(64 * NW) void rmsnorm_p1_ring_kernel(int rows, int d, float eps, const T* __restrict__ dy,
                                                                  const T* __restrict__ x, const T* __restrict__ g,
                                                                  const T* __restrict__ resid, T* __restrict__ dx,
                                                                  float* __restrict__ partials) {
  constexpr int N = Vec<T>::N, G = NW / WPR, TPR = 64 * WPR;
  typedef typename Vec<T>::Raw Raw;
  extern __shared__ float lds[];              // [2][NW waves][2 sums] reduction slots, then [d] column buffer
  float* const red = lds;
  float* const colbuf = lds + 4 * NW;
  const int wave = threadIdx.x >> 6, grp = wave / WPR, t = threadIdx.x - grp * TPR;
  const int nchunk = d / N;
  float cacc[MAXC][N], gv[MAXC][N];
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
#pragma unroll
    for (int i = 0; i < N; i++) { cacc[c][i] = 0.f; gv[c][i] = 0.f; }
    if constexpr (!GAIN_ONLY) {
      const int ch = t + TPR * c;
      if (ch < nchunk) Vec<T>::load(g + ch * N, gv[c]);
    }
  }
  const int stride = G * (int)gridDim.x;
  const int iters = (rows + stride - 1) / stride;
  Raw xq[PD][MAXC], yq[PD][MAXC], rq[PD][MAXC];
  auto fetch = [&](int it, Raw* xv, Raw* yv, Raw* rv) {
    const int row = (it * (int)gridDim.x + (int)blockIdx.x) * G + grp;
    if (it < iters && row < rows) {
      const long base = (long)row * d;
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (ch < nchunk) {
          xv[c] = Vec<T>::load_raw(x + base + ch * N);
          yv[c] = Vec<T>::load_raw(dy + base + ch * N);
          if (!GAIN_ONLY && resid) rv[c] = Vec<T>::load_raw(resid + base + ch * N);
        }
      }
    }
  };
#pragma unroll
  for (int p = 0; p < PD; p++) fetch(p, xq[p], yq[p], rq[p]);
  for (int it0 = 0; it0 < iters; it0 += PD) {
#pragma unroll
    for (int p = 0; p < PD; p++) {
      const int it = it0 + p;
      if (it >= iters) break;                 // (uniform over the workgroup)
      const int row = (it * (int)gridDim.x + (int)blockIdx.x) * G + grp;
      const bool live = row < rows;
      const long base = (long)row * d;
      Raw xr[MAXC], yr[MAXC], rr[MAXC];
#pragma unroll
      for (int c = 0; c < MAXC; c++) { xr[c] = xq[p][c]; yr[c] = yq[p][c]; rr[c] = rq[p][c]; }
      fetch(it + PD, xq[p], yq[p], rq[p]);
      float s_xx = 0.f, s_yx = 0.f;
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (live && ch < nchunk) {
          float xv[N], yv[N];
          Vec<T>::unpack(xr[c], xv);
          Vec<T>::unpack(yr[c], yv);
#pragma unroll
          for (int i = 0; i < N; i++) {
            s_xx += xv[i] * xv[i];
            if constexpr (!GAIN_ONLY) s_yx += yv[i] * gv[c][i] * xv[i];
          }
        }
      }
      s_xx = wave_sum(s_xx);
      if constexpr (!GAIN_ONLY) s_yx = wave_sum(s_yx);
      if constexpr (WPR > 1) {                // two slot sets used alternately: one barrier per row is enough
        float* const slot = red + (it & 1) * 2 * NW;
        if ((threadIdx.x & 63) == 0) {
          slot[wave * 2] = s_xx;
          slot[wave * 2 + 1] = s_yx;
        }
        __syncthreads();
        s_xx = 0.f; s_yx = 0.f;
#pragma unroll
        for (int w = 0; w < WPR; w++) {
          s_xx += slot[(grp * WPR + w) * 2];
          s_yx += slot[(grp * WPR + w) * 2 + 1];
        }
      }
      const float r = rsqrtf(s_xx / (float)d + eps);
      const float coef = r * r * r * (s_yx / (float)d);
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (live && ch < nchunk) {
          float xv[N], yv[N];
          Vec<T>::unpack(xr[c], xv);
          Vec<T>::unpack(yr[c], yv);
#pragma unroll
          for (int i = 0; i < N; i++) cacc[c][i] += yv[i] * xv[i] * r;
          if constexpr (!GAIN_ONLY) {
            float o[N];
            if (resid) Vec<T>::unpack(rr[c], o);
            else {
#pragma unroll
              for (int i = 0; i < N; i++) o[i] = 0.f;
            }
#pragma unroll
            for (int i = 0; i < N; i++) o[i] += r * yv[i] * gv[c][i] - xv[i] * coef;
            Vec<T>::store(dx + base + ch * N, o);
          }
        }
      }
    }
  }
  if (!partials) return;                      // (uniform over the grid)
  __syncthreads();
  for (int gi = 0; gi < G; gi++) {
    if (grp == gi) {
#pragma unroll
      for (int c = 0; c < MAXC; c++) {
        const int ch = t + TPR * c;
        if (ch < nchunk) {
#pragma unroll
          for (int i = 0; i < N; i++) {
            const int col = ch * N + i;
            colbuf[col] = (gi == 0 ? 0.f : colbuf[col]) + cacc[c][i];
          }
        }
      }
    }
    __syncthreads();
  }
  for (int col = threadIdx.x; col < d; col += 64 * NW) partials[(long)blockIdx.x * d + col] = colbuf[col];
}

// out[col] (= or +=) sum over the first n_rows rows of parts[row][col].
// A workgroup covers kColsumCols columns with 16 row lanes each (64-byte reads; 16 partial sums folded in LDS in a
// fixed order, so the result is reproducible).
constexpr int kColsumCols = 16;
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ parts, int n_rows, int d, int accumulate,
                                                     float* __restrict__ out) {
  __shared__ float fold[16][kColsumCols + 1];
  const int c = threadIdx.x & (kColsumCols - 1), rlane = threadIdx.x / kColsumCols;
  const int col = blockIdx.x * kColsumCols + c;
  float s = 0.f;
  if (col < d) {
    // four independent chains per lane (rows r, r + 16, r + 32, r + 48 of each group of 64): the loads of a group
    // are in flight together instead of one after the other; the chains are added in a fixed order
    float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
    int r = rlane;
    for (; r + 48 < n_rows; r += 64) {
      const float v0 = parts[(long)r * d + col], v1 = parts[(long)(r + 16) * d + col];
      const float v2 = parts[(long)(r + 32) * d + col], v3 = parts[(long)(r + 48) * d + col];
      a0 += v0; a1 += v1; a2 += v2; a3 += v3;
    }
    for (; r < n_rows; r += 16) a0 += parts[(long)r * d + col];
    s = (a0 + a1) + (a2 + a3);
  }
  fold[rlane][c] = s;
  __syncthreads();
  if (rlane == 0 && col < d) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i++) t += fold[i][c];
    out[col] = accumulate ? out[col] + t : t;
  }
}

// ---- SwiGLU -----------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void swiglu_fwd_kernel(long nvec, int fchunks, int f, const T* __restrict__ gu,
                                                         T* __restrict__ m) {
  constexpr int N = Vec<T>::N;
  for (long v = blockIdx.x * 256L + threadIdx.x; v < nvec; v += 256L * gridDim.x) {
    const long row = v / fchunks;
    const int col = (int)(v - row * fchunks) * N;
    float a[N], b[N], o[N];
    Vec<T>::load(gu + row * 2 * f + col, a);
    Vec<T>::load(gu + row * 2 * f + f + col, b);
#pragma unroll
    for (int i = 0; i < N; i++) o[i] = a[i] / (1.f + __expf(-a[i])) * b[i];
    Vec<T>::store(m + row * f + col, o);
  }
}

template <typename T>
__global__ __launch_bounds__(256) void swiglu_p1_kernel(long nvec, int fchunks, int f, const T* __restrict__ dm,
                                                        const T* __restrict__ gu, T* __restrict__ dgu) {
  constexpr int N = Vec<T>::N;
  for (long v = blockIdx.x * 256L + threadIdx.x; v < nvec; v += 256L * gridDim.x) {
    const long row = v / fchunks;
    const int col = (int)(v - row * fchunks) * N;
    float a[N], b[N], g[N], da[N], db[N];
    Vec<T>::load(gu + row * 2 * f + col, a);
    Vec<T>::load(gu + row * 2 * f + f + col, b);
    Vec<T>::load(dm + row * f + col, g);
#pragma unroll
    for (int i = 0; i < N; i++) {
      const float s = 1.f / (1.f + __expf(-a[i]));
      da[i] = g[i] * b[i] * s * (1.f + a[i] * (1.f - s));
      db[i] = g[i] * a[i] * s;
    }
    Vec<T>::store(dgu + row * 2 * f + col, da);
    Vec<T>::store(dgu + row * 2 * f + f + col, db);
  }
}

// ---- rotary embedding ---------------------------------------------------------------------------------
// table[p][i] = (cos, sin)(p * base^(-2i/dh)), evaluated in fp64 once.
__global__ void rope_table_kernel(int seq, int half, float base, float2* __restrict__ table) {
  const int idx = blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= seq * half) return;
  const int p = idx / half, i = idx - p * half;
  const double theta = pow((double)base, -(double)i / (double)half);
  const double ang = (double)p * theta;
  table[idx] = make_float2((float)cos(ang), (float)sin(ang));
}

// A thread owns one 16-byte column chunk of the rotation table row of its token (cos, sin kept in registers) and
// applies it to kRopeHeads consecutive heads, so the table is read once per 8 heads instead of once per head.
constexpr int kRopeHeads = 8;
template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(long nitems, int seq, int n_heads, int head_dim, long ld,
                                                   const float2* __restrict__ table, float sgn, T* __restrict__ x) {
  constexpr int N = Vec<T>::N;
  const int half = head_dim / 2;
  const int cph = half / N;                   // chunks per head half
  const int ngrp = (n_heads + kRopeHeads - 1) / kRopeHeads;
  for (long v = blockIdx.x * 256L + threadIdx.x; v < nitems; v += 256L * gridDim.x) {
    const int c = (int)(v % cph);
    const long gv = v / cph;
    const int hg = (int)(gv % ngrp);
    const long row = gv / ngrp;
    const int pos = (int)(row % seq);
    float cs[N], sn[N];
    const float2* tb = table + (long)pos * half + c * N;
#pragma unroll
    for (int i = 0; i < N; i++) {
      const float2 t = tb[i];
      cs[i] = t.x;
      sn[i] = t.y * sgn;
    }
    const int h0 = hg * kRopeHeads;
    const int hn = (n_heads - h0) < kRopeHeads ? (n_heads - h0) : kRopeHeads;
    T* base = x + row * ld + (long)h0 * head_dim + c * N;
#pragma unroll 4
    for (int u = 0; u < hn; u++) {
      T* pa = base + (long)u * head_dim;
      T* pb = pa + half;
      float a[N], b[N], oa[N], ob[N];
      Vec<T>::load(pa, a);
      Vec<T>::load(pb, b);
#pragma unroll
      for (int i = 0; i < N; i++) {
        oa[i] = a[i] * cs[i] - b[i] * sn[i];
        ob[i] = a[i] * sn[i] + b[i] * cs[i];
      }
      Vec<T>::store(pa, oa);
      Vec<T>::store(pb, ob);
    }
  }
}

// ---- softmax ------------------------------------------------------------------------------------------
// One wavefront per PAIR of rows (i, S-1-i) of one matrix.  Row i of a causal matrix has i+1 live columns, so the
// two rows of a pair hold S+1 live elements between them whatever i is: every wave does the same amount of work
// and no wave is left with a handful of active lanes.  The pair is walked as one stream of 16-byte chunks, first
// row A's, then row B's; each chunk knows its row, so the two row reductions are two wavefront reductions over
// the same registers.  A written row is zero-filled from the diagonal up to the next multiple of kCausalPad
// columns (the products that consume it skip everything beyond that).
struct RowPair {
  long rowA, rowB;      // global row indices (matrix * seq + row)
  int liveA, liveB;     // live columns
  int nA, nAB;          // chunks (of N elements) written for row A, and for both rows
};
template <int N>
__device__ __forceinline__ RowPair row_pair(long pair, int seq, int causal) {
  const int half = seq / 2;
  const long mat = pair / half;
  const int i = (int)(pair - mat * half);
  RowPair r;
  r.rowA = mat * seq + i;
  r.rowB = mat * seq + (seq - 1 - i);
  r.liveA = causal ? i + 1 : seq;
  r.liveB = causal ? seq - i : seq;
  int fa = (r.liveA + kCausalPad - 1) / kCausalPad * kCausalPad, fb = (r.liveB + kCausalPad - 1) / kCausalPad * kCausalPad;
  if (fa > seq) fa = seq;
  if (fb > seq) fb = seq;
  r.nA = fa / N;
  r.nAB = r.nA + fb / N;
  return r;
}

template <typename T, int MAXC>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(long npairs, int seq, int causal,
                                                          const float* __restrict__ scores, T* __restrict__ P) {
  const long pair = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (pair >= npairs) return;
  const int lane = threadIdx.x & 63;
  const RowPair rp = row_pair<4>(pair, seq, causal);
  float v[MAXC][4];
  float mxA = -INFINITY, mxB = -INFINITY;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int u = lane + 64 * c;
    const bool isB = u >= rp.nA;
    const int col = (isB ? u - rp.nA : u) * 4;
    const int live = isB ? rp.liveB : rp.liveA;
    if (u < rp.nAB && col < live) {
      Vec<float>::load(scores + (isB ? rp.rowB : rp.rowA) * seq + col, v[c]);
      float m = -INFINITY;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        if (col + e >= live) v[c][e] = -INFINITY;
        m = fmaxf(m, v[c][e]);
      }
      if (isB) mxB = fmaxf(mxB, m); else mxA = fmaxf(mxA, m);
    }
  }
  mxA = wave_max(mxA);
  mxB = wave_max(mxB);
  float sumA = 0.f, sumB = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int u = lane + 64 * c;
    const bool isB = u >= rp.nA;
    const int col = (isB ? u - rp.nA : u) * 4;
    const int live = isB ? rp.liveB : rp.liveA;
    if (u < rp.nAB && col < live) {
      const float mx = isB ? mxB : mxA;
      float t = 0.f;
#pragma unroll
      for (int e = 0; e < 4; e++) {
        v[c][e] = __expf(v[c][e] - mx);
        t += v[c][e];
      }
      if (isB) sumB += t; else sumA += t;
    }
  }
  sumA = wave_sum(sumA);
  sumB = wave_sum(sumB);
  const float invA = 1.f / sumA, invB = 1.f / sumB;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int u = lane + 64 * c;
    const bool isB = u >= rp.nA;
    const int col = (isB ? u - rp.nA : u) * 4;
    const int live = isB ? rp.liveB : rp.liveA;
    if (u < rp.nAB) {
      T* o = P + (isB ? rp.rowB : rp.rowA) * seq + col;
      const float inv = isB ? invB : invA;
      if (col < live) {
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (T)(v[c][e] * inv);
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++) o[e] = (T)0.f;
      }
    }
  }
}

// dS = P * (dP - sum_j dP_j P_j), in place over dP; same pairing and zero-fill rule.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void softmax_p1_kernel(long npairs, int seq, int causal, const T* __restrict__ P,
                                                         T* __restrict__ dP) {
  constexpr int N = Vec<T>::N;
  typedef typename Vec<T>::Raw Raw;
  const long pair = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (pair >= npairs) return;
  const int lane = threadIdx.x & 63;
  const RowPair rp = row_pair<N>(pair, seq, causal);
  Raw pr[MAXC], gr[MAXC];
  float dotA = 0.f, dotB = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int u = lane + 64 * c;
    const bool isB = u >= rp.nA;
    const int col = (isB ? u - rp.nA : u) * N;
    const int live = isB ? rp.liveB : rp.liveA;
    if (u < rp.nAB && col < live) {
      const long off = (isB ? rp.rowB : rp.rowA) * seq + col;
      pr[c] = Vec<T>::load_raw(P + off);
      gr[c] = Vec<T>::load_raw(dP + off);
      float pv[N], gv[N];
      Vec<T>::unpack(pr[c], pv);
      Vec<T>::unpack(gr[c], gv);
      float t = 0.f;
#pragma unroll
      for (int e = 0; e < N; e++)
        if (col + e < live) t += pv[e] * gv[e];
      if (isB) dotB += t; else dotA += t;
    }
  }
  dotA = wave_sum(dotA);
  dotB = wave_sum(dotB);
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int u = lane + 64 * c;
    const bool isB = u >= rp.nA;
    const int col = (isB ? u - rp.nA : u) * N;
    const int live = isB ? rp.liveB : rp.liveA;
    if (u < rp.nAB) {
      float o[N];
      if (col < live) {
        const float dot = isB ? dotB : dotA;
        float pv[N], gv[N];
        Vec<T>::unpack(pr[c], pv);
        Vec<T>::unpack(gr[c], gv);
#pragma unroll
        for (int e = 0; e < N; e++) o[e] = (col + e < live) ? pv[e] * (gv[e] - dot) : 0.f;
      } else {
#pragma unroll
        for (int e = 0; e < N; e++) o[e] = 0.f;
      }
      Vec<T>::store(dP + (isB ? rp.rowB : rp.rowA) * seq + col, o);
    }
  }
}

// ---- per-head row dot products: delta[t, h] = sum_c a[t, h*dh + c] * b[t, h*dh + c] -----------------------------
// (the row sums rowsum(dP * P) of the softmax backward equal rowsum(do * o), which needs no S x S tensor).
// One 256-thread workgroup per token row: 16-byte chunk products to LDS, then one thread per head adds its chunks.
template <typename T>
__global__ __launch_bounds__(256) void head_rowdot_kernel(int n_heads, int head_dim, const T* __restrict__ a,
                                                          const T* __restrict__ b, float* __restrict__ delta) {
  constexpr int N = Vec<T>::N;
  extern __shared__ float part[];             // [d / N]
  const long row = blockIdx.x;
  const int d = n_heads * head_dim, nchunk = d / N, cph = head_dim / N;
  for (int ch = threadIdx.x; ch < nchunk; ch += 256) {
    float x[N], y[N];
    Vec<T>::load(a + row * d + ch * N, x);
    Vec<T>::load(b + row * d + ch * N, y);
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < N; i++) t += x[i] * y[i];
    part[ch] = t;
  }
  __syncthreads();
  for (int h = threadIdx.x; h < n_heads; h += 256) {
    float t = 0.f;
    for (int c = 0; c < cph; c++) t += part[h * cph + c];
    delta[row * n_heads + h] = t;
  }
}

// ------------------------------------------------------------------------------------------ host
static inline int chunks_per_thread(int d, int n) { return (d / n + 255) / 256; }

template <typename T>
static hipError_t rmsnorm_fwd_t(int rows, int d, float eps, const void* x, const void* g, void* y, hipStream_t s) {
  const int c = chunks_per_thread(d, Vec<T>::N);
  auto X = (const T*)x; auto G = (const T*)g; auto Y = (T*)y;
  if (c <= 1) hipLaunchKernelGGL((rmsnorm_fwd_kernel<T, 1>), dim3(rows), dim3(256), 0, s, rows, d, eps, X, G, Y);
  else if (c <= 2) hipLaunchKernelGGL((rmsnorm_fwd_kernel<T, 2>), dim3(rows), dim3(256), 0, s, rows, d, eps, X, G, Y);
  else if (c <= 4) hipLaunchKernelGGL((rmsnorm_fwd_kernel<T, 4>), dim3(rows), dim3(256), 0, s, rows, d, eps, X, G, Y);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
hipError_t rmsnorm_fwd(int dtype, int rows, int d, float eps, const void* x, const void* g, void* y, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  return dtype ? rmsnorm_fwd_t<bf16_t>(rows, d, eps, x, g, y, s) : rmsnorm_fwd_t<float>(rows, d, eps, x, g, y, s);
}

// Which kernel a (storage type, width) pair runs on, and how many rows a workgroup has in work at a time.  The number
// of workgroups, which is the number of partial rows of the gain gradient that the row kernel leaves, follows from it.
struct NormPlan { int kind, wpr, rows_per_block; };      // kind 0: rmsnorm_p1_kernel with `wpr` waves per row; 1: ring kernel
#ifndef TBP_RING_NW1
#define TBP_RING_NW1 16
#endif
#ifndef TBP_RING_PD1
#define TBP_RING_PD1 2
#endif
#ifndef TBP_RING_PD2
#define TBP_RING_PD2 2
#endif
static NormPlan norm_plan(int dtype, int d) {
  const int wc = (d / (dtype ? 8 : 4) + 63) / 64;   // vectors per lane if one wave owned a whole row
  if (dtype) {
    // bf16 rows of more than 2048 columns (the 7B and 13B widths among them) run on the ring kernel, 8 waves per row:
    // up to 4096 columns one vector per lane and two rows per 1024-thread workgroup; wider rows two vectors per lane
    // and one row per 512-thread workgroup (two vectors per lane in 1024 threads do not fit the register file)
    if (wc > 4) return NormPlan{1, 8, wc <= 8 ? TBP_RING_NW1 / 8 : 1};
    // 1024 < columns <= 2048: the same kernel with 4 waves per row, four rows per 1024-thread workgroup
    if (wc > 2) return NormPlan{1, 4, 4};
    return NormPlan{0, 1, 8};
  }
  const int wpr = wc <= 4 ? 1 : wc <= 8 ? 2 : wc <= 16 ? 4 : 8;
  return NormPlan{0, wpr, 8 / wpr};
}
int rmsnorm_partial_rows(int dtype, int rows, int d) {
  if (rows <= 0 || d <= 0) return 0;
  const int g = norm_plan(dtype, d).rows_per_block;
  const int nblk = (rows + g - 1) / g;
  return nblk < kNormPartialBlocks ? nblk : kNormPartialBlocks;
}

template <typename T, int WPR, bool GAIN_ONLY>
static hipError_t rmsnorm_p1_w(int rows, int d, float eps, const T* dy, const T* x, const T* g, const T* resid, T* dx,
                               float* partials, int nblk, hipStream_t s) {
  constexpr int NW = 8;
  const int c = (d / Vec<T>::N + 64 * WPR - 1) / (64 * WPR);      // vectors per lane
  const size_t smem = (4 * NW + (size_t)d) * sizeof(float);
  const dim3 grid(nblk), block(64 * NW);
  if (c <= 1) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 1, WPR, GAIN_ONLY, NW>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else if (c <= 2) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 2, WPR, GAIN_ONLY, NW>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else if (c <= 4) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 4, WPR, GAIN_ONLY, NW>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <typename T, bool GAIN_ONLY>
static hipError_t rmsnorm_p1_ring(int rows, int d, float eps, const T* dy, const T* x, const T* g, const T* resid, T* dx,
                                  float* partials, int nblk, int wpr, hipStream_t s) {
  if (wpr == 4) {       // at most 256 vectors per row: one per lane
    const size_t smem4 = (4 * 16 + (size_t)d) * sizeof(float);
    hipLaunchKernelGGL((rmsnorm_p1_ring_kernel<T, 1, 4, GAIN_ONLY, 16, TBP_RING_PD1>), dim3(nblk), dim3(1024), smem4, s, rows, d, eps, dy, x, g, resid, dx, partials);
    return hipGetLastError();
  }
  constexpr int WPR = 8;
  const int c = (d / Vec<T>::N + 64 * WPR - 1) / (64 * WPR);      // vectors per lane
  if (c > 2) return hipErrorInvalidValue;
  const int NW = c == 1 ? TBP_RING_NW1 : 8;
  const size_t smem = (4 * NW + (size_t)d) * sizeof(float);
  const dim3 grid(nblk), block(64 * NW);
  if (c == 1) hipLaunchKernelGGL((rmsnorm_p1_ring_kernel<T, 1, WPR, GAIN_ONLY, TBP_RING_NW1, TBP_RING_PD1>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else hipLaunchKernelGGL((rmsnorm_p1_ring_kernel<T, 2, WPR, GAIN_ONLY, 8, TBP_RING_PD2>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  return hipGetLastError();
}

// The row kernel alone: dx (unless GAIN_ONLY) and, if `partials` is given, rmsnorm_partial_rows(...) partial rows of
// the gain gradient.
template <typename T, bool GAIN_ONLY>
static hipError_t rmsnorm_rows_t(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                                 const void* resid, void* dx, float* partials, hipStream_t s) {
  auto DY = (const T*)dy; auto X = (const T*)x; auto G = (const T*)g; auto RS = (const T*)resid; auto DX = (T*)dx;
  const NormPlan pl = norm_plan(dtype, d);
  const int nblk = rmsnorm_partial_rows(dtype, rows, d);
  if constexpr (sizeof(T) == 2) {
    if (pl.kind == 1) return rmsnorm_p1_ring<T, GAIN_ONLY>(rows, d, eps, DY, X, G, RS, DX, partials, nblk, pl.wpr, s);
  }
  switch (pl.wpr) {
    case 1: return rmsnorm_p1_w<T, 1, GAIN_ONLY>(rows, d, eps, DY, X, G, RS, DX, partials, nblk, s);
    case 2: return rmsnorm_p1_w<T, 2, GAIN_ONLY>(rows, d, eps, DY, X, G, RS, DX, partials, nblk, s);
    case 4: return rmsnorm_p1_w<T, 4, GAIN_ONLY>(rows, d, eps, DY, X, G, RS, DX, partials, nblk, s);
    default: return rmsnorm_p1_w<T, 8, GAIN_ONLY>(rows, d, eps, DY, X, G, RS, DX, partials, nblk, s);
  }
}

hipError_t gain_partials_sum(const float* partials, int n_rows, int d, int accumulate, float* out, hipStream_t s) {
  hipLaunchKernelGGL(colsum_kernel, dim3((d + kColsumCols - 1) / kColsumCols), dim3(256), 0, s, partials, n_rows > 0 ? n_rows : 0, d,
                     accumulate, out);
  return hipGetLastError();
}

hipError_t rmsnorm_p1_rows(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                           const void* resid, void* dx, float* partials, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  return dtype ? rmsnorm_rows_t<bf16_t, false>(dtype, rows, d, eps, dy, x, g, resid, dx, partials, s)
               : rmsnorm_rows_t<float, false>(dtype, rows, d, eps, dy, x, g, resid, dx, partials, s);
}

hipError_t rmsnorm_p1(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                      const void* resid, void* dx, float* dg_out, float* partials, hipStream_t s) {
  hipError_t e = rmsnorm_p1_rows(dtype, rows, d, eps, dy, x, g, resid, dx, dg_out ? partials : nullptr, s);
  if (e != hipSuccess || !dg_out) return e;
  return gain_partials_sum(partials, rmsnorm_partial_rows(dtype, rows, d), d, 0, dg_out, s);     // (no rows: zeros)
}

hipError_t rmsnorm_gain_p2(int dtype, int rows, int d, float eps, const void* dy, const void* x, int accumulate,
                           float* dg_out, float* partials, hipStream_t s) {
  if (rows <= 0) return accumulate ? hipSuccess : gain_partials_sum(partials, 0, d, 0, dg_out, s);
  hipError_t e = dtype ? rmsnorm_rows_t<bf16_t, true>(dtype, rows, d, eps, dy, x, nullptr, nullptr, nullptr, partials, s)
                       : rmsnorm_rows_t<float, true>(dtype, rows, d, eps, dy, x, nullptr, nullptr, nullptr, partials, s);
  if (e != hipSuccess) return e;
  return gain_partials_sum(partials, rmsnorm_partial_rows(dtype, rows, d), d, accumulate, dg_out, s);
}

static inline unsigned grid_for(long nvec) {
  long b = (nvec + 255) / 256;
  const long cap = 256L * 32;               // 32 workgroups per compute unit, then grid-stride
  return (unsigned)(b < cap ? (b > 0 ? b : 1) : cap);
}

hipError_t swiglu_fwd(int dtype, int rows, int f, const void* gu, void* m, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int n = dtype ? 8 : 4;
  const long nvec = (long)rows * (f / n);
  if (dtype) hipLaunchKernelGGL(swiglu_fwd_kernel<bf16_t>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, f / n, f,
                                (const bf16_t*)gu, (bf16_t*)m);
  else hipLaunchKernelGGL(swiglu_fwd_kernel<float>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, f / n, f,
                          (const float*)gu, (float*)m);
  return hipGetLastError();
}
hipError_t swiglu_p1(int dtype, int rows, int f, const void* dm, const void* gu, void* dgu, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int n = dtype ? 8 : 4;
  const long nvec = (long)rows * (f / n);
  if (dtype) hipLaunchKernelGGL(swiglu_p1_kernel<bf16_t>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, f / n, f,
                                (const bf16_t*)dm, (const bf16_t*)gu, (bf16_t*)dgu);
  else hipLaunchKernelGGL(swiglu_p1_kernel<float>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, f / n, f,
                          (const float*)dm, (const float*)gu, (float*)dgu);
  return hipGetLastError();
}

hipError_t rope_table(int seq, int head_dim, float base, float2* table, hipStream_t s) {
  const int n = seq * (head_dim / 2);
  hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, s, seq, head_dim / 2, base, table);
  return hipGetLastError();
}
hipError_t rope(int dtype, int rows, int seq, int n_heads, int head_dim, long ld, const float2* table, int inverse,
                void* x, hipStream_t s) {
  if (rows <= 0 || n_heads <= 0) return hipSuccess;
  const int n = dtype ? 8 : 4;
  const long nvec = (long)rows * ((n_heads + kRopeHeads - 1) / kRopeHeads) * (head_dim / 2 / n);
  const float sgn = inverse ? -1.f : 1.f;
  if (dtype) hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, seq, n_heads,
                                head_dim, ld, table, sgn, (bf16_t*)x);
  else hipLaunchKernelGGL(rope_kernel<float>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, seq, n_heads, head_dim,
                          ld, table, sgn, (float*)x);
  return hipGetLastError();
}

// chunks per lane needed for a row pair: the two zero-filled rows hold at most min(2 S, S + 2 * kCausalPad) elements
static inline int pair_chunks(int seq, int causal, int n) {
  long el = causal ? (long)seq + 2 * kCausalPad : 2L * seq;
  if (el > 2L * seq) el = 2L * seq;
  return (int)((el / n + 63) / 64);
}
#define TBP_PICK_MAXC(KERNEL, ...)                                                                           \
  do {                                                                                                       \
    if (c <= 2) hipLaunchKernelGGL((KERNEL<T, 2>), grid, dim3(256), 0, s, __VA_ARGS__);                       \
    else if (c <= 3) hipLaunchKernelGGL((KERNEL<T, 3>), grid, dim3(256), 0, s, __VA_ARGS__);                  \
    else if (c <= 5) hipLaunchKernelGGL((KERNEL<T, 5>), grid, dim3(256), 0, s, __VA_ARGS__);                  \
    else if (c <= 8) hipLaunchKernelGGL((KERNEL<T, 8>), grid, dim3(256), 0, s, __VA_ARGS__);                  \
    else if (c <= 10) hipLaunchKernelGGL((KERNEL<T, 10>), grid, dim3(256), 0, s, __VA_ARGS__);                \
    else if (c <= 18) hipLaunchKernelGGL((KERNEL<T, 18>), grid, dim3(256), 0, s, __VA_ARGS__);                \
    else if (c <= 32) hipLaunchKernelGGL((KERNEL<T, 32>), grid, dim3(256), 0, s, __VA_ARGS__);                \
    else return hipErrorInvalidValue;                                                                        \
  } while (0)

template <typename T>
static hipError_t softmax_fwd_t(long nrows, int seq, int causal, const float* sc, void* P, hipStream_t s) {
  const int c = pair_chunks(seq, causal, 4);
  const long npairs = nrows / 2;
  const dim3 grid((unsigned)((npairs + 3) / 4));
  TBP_PICK_MAXC(softmax_fwd_kernel, npairs, seq, causal, sc, (T*)P);
  return hipGetLastError();
}
hipError_t softmax_fwd(int dtype, long nrows, int seq, int causal, const float* scores, void* P, hipStream_t s) {
  if (nrows <= 0) return hipSuccess;
  if (seq % 2) return hipErrorInvalidValue;       // rows are processed in pairs (i, seq-1-i)
  return dtype ? softmax_fwd_t<bf16_t>(nrows, seq, causal, scores, P, s)
               : softmax_fwd_t<float>(nrows, seq, causal, scores, P, s);
}

template <typename T>
static hipError_t softmax_p1_t(long nrows, int seq, int causal, const void* P, void* dP, hipStream_t s) {
  const int c = pair_chunks(seq, causal, Vec<T>::N);
  const long npairs = nrows / 2;
  const dim3 grid((unsigned)((npairs + 3) / 4));
  TBP_PICK_MAXC(softmax_p1_kernel, npairs, seq, causal, (const T*)P, (T*)dP);
  return hipGetLastError();
}
#undef TBP_PICK_MAXC
hipError_t softmax_p1(int dtype, long nrows, int seq, int causal, const void* P, void* dP, hipStream_t s) {
  if (nrows <= 0) return hipSuccess;
  if (seq % 2) return hipErrorInvalidValue;
  return dtype ? softmax_p1_t<bf16_t>(nrows, seq, causal, P, dP, s) : softmax_p1_t<float>(nrows, seq, causal, P, dP, s);
}

hipError_t head_rowdot(int dtype, int rows, int n_heads, int head_dim, const void* a, const void* b, float* delta,
                       hipStream_t s) {
  if (rows <= 0 || n_heads <= 0) return hipSuccess;
  const int n = dtype ? 8 : 4;
  const size_t smem = (size_t)(n_heads * head_dim / n) * sizeof(float);
  if (dtype) hipLaunchKernelGGL(head_rowdot_kernel<bf16_t>, dim3(rows), dim3(256), smem, s, n_heads, head_dim,
                                (const bf16_t*)a, (const bf16_t*)b, delta);
  else hipLaunchKernelGGL(head_rowdot_kernel<float>, dim3(rows), dim3(256), smem, s, n_heads, head_dim,
                          (const float*)a, (const float*)b, delta);
  return hipGetLastError();
}

}  // namespace tbp
