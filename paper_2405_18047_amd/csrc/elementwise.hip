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
template <typename T, int MAXC, int WPR>
__global__ __launch_bounds__(512) void rmsnorm_p1_kernel(int rows, int d, float eps, const T* __restrict__ dy,
                                                         const T* __restrict__ x, const T* __restrict__ g,
                                                         const T* __restrict__ resid, T* __restrict__ dx,
                                                         float* __restrict__ partials) {
  constexpr int N = Vec<T>::N, G = 8 / WPR, TPR = 64 * WPR;     // groups per workgroup, threads per row
  typedef typename Vec<T>::Raw Raw;
  extern __shared__ float lds[];              // [2][8 waves][2 sums] reduction slots, then [d] column buffer
  float* const red = lds;
  float* const colbuf = lds + 32;
  const int wave = threadIdx.x >> 6, grp = wave / WPR, t = threadIdx.x - grp * TPR;
  const int nchunk = d / N;
  float cacc[MAXC][N];
#pragma unroll
  for (int c = 0; c < MAXC; c++)
#pragma unroll
    for (int i = 0; i < N; i++) cacc[c][i] = 0.f;
  const int stride = G * gridDim.x;
  const int iters = (rows + stride - 1) / stride;
  for (int it = 0; it < iters; it++) {
    const int row = (it * (int)gridDim.x + (int)blockIdx.x) * G + grp;
    const bool live = row < rows;
    const long base = (long)row * d;
    Raw xr[MAXC], yr[MAXC];
#pragma unroll
    for (int c = 0; c < MAXC; c++) {
      const int ch = t + TPR * c;
      if (live && ch < nchunk) {
        xr[c] = Vec<T>::load_raw(x + base + ch * N);
        yr[c] = Vec<T>::load_raw(dy + base + ch * N);
      }
    }
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
        Vec<T>::load(gp + ch * N, gv);
#pragma unroll
        for (int i = 0; i < N; i++) {
          s_xx += xv[i] * xv[i];
          s_yx += yv[i] * gv[i] * xv[i];
        }
      }
    }
    s_xx = wave_sum(s_xx);
    s_yx = wave_sum(s_yx);
    if constexpr (WPR > 1) {                  // two slot sets used alternately: one barrier per row is enough
      float* const slot = red + (it & 1) * 16;
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
        float xv[N], yv[N], gv[N], o[N];
        Vec<T>::unpack(xr[c], xv);
        Vec<T>::unpack(yr[c], yv);
        Vec<T>::load(gp + ch * N, gv);
        if (resid) Vec<T>::load(resid + base + ch * N, o);
        else {
#pragma unroll
          for (int i = 0; i < N; i++) o[i] = 0.f;
        }
#pragma unroll
        for (int i = 0; i < N; i++) {
          o[i] += r * yv[i] * gv[i] - xv[i] * coef;
          cacc[c][i] += yv[i] * xv[i] * r;
        }
        Vec<T>::store(dx + base + ch * N, o);
      }
    }
  }
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
  for (int col = threadIdx.x; col < d; col += 512) partials[(long)blockIdx.x * d + col] = colbuf[col];
}

// out[col] (= or +=) sum_r parts[row_r][col]; rows given by value (host list) or the first n_first_rows rows.
// A workgroup covers 32 columns with 8 row lanes each (128-byte coalesced reads, 8 partial sums folded in LDS in
// a fixed order, so the result is reproducible).
struct RowList { int n; int idx[64]; };
__global__ __launch_bounds__(256) void colsum_kernel(const float* __restrict__ parts, RowList rl, int n_first_rows,
                                                     int d, int accumulate, float* __restrict__ out) {
  __shared__ float fold[8][33];
  const int c = threadIdx.x & 31, rlane = threadIdx.x >> 5;
  const int col = blockIdx.x * 32 + c;
  float s = 0.f;
  if (col < d) {
    if (n_first_rows > 0) {
      for (int r = rlane; r < n_first_rows; r += 8) s += parts[(long)r * d + col];
    } else {
      for (int r = rlane; r < rl.n; r += 8) s += parts[(long)rl.idx[r] * d + col];
    }
  }
  fold[rlane][c] = s;
  __syncthreads();
  if (rlane == 0 && col < d) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 8; i++) t += fold[i][c];
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

template <typename T>
__global__ __launch_bounds__(256) void rope_kernel(long nvec, int seq, int n_heads, int head_dim, long ld,
                                                   const float2* __restrict__ table, float sgn, T* __restrict__ x) {
  constexpr int N = Vec<T>::N;
  const int half = head_dim / 2;
  const int cph = half / N;                   // chunks per head half
  for (long v = blockIdx.x * 256L + threadIdx.x; v < nvec; v += 256L * gridDim.x) {
    const int c = (int)(v % cph);
    const long hv = v / cph;
    const int h = (int)(hv % n_heads);
    const long row = hv / n_heads;
    const int pos = (int)(row % seq);
    T* pa = x + row * ld + (long)h * head_dim + c * N;
    T* pb = pa + half;
    float a[N], b[N], oa[N], ob[N];
    Vec<T>::load(pa, a);
    Vec<T>::load(pb, b);
    const float2* tb = table + (long)pos * half + c * N;
#pragma unroll
    for (int i = 0; i < N; i++) {
      const float2 cs = tb[i];
      const float sn = cs.y * sgn;
      oa[i] = a[i] * cs.x - b[i] * sn;
      ob[i] = a[i] * sn + b[i] * cs.x;
    }
    Vec<T>::store(pa, oa);
    Vec<T>::store(pb, ob);
  }
}

// ---- softmax ------------------------------------------------------------------------------------------
// One wavefront per row.  Row `i` of a causal matrix has i+1 live columns; the written row is zero-filled
// up to the next multiple of kCausalPad (the products that consume it skip everything beyond that).
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void softmax_fwd_kernel(long nrows, int seq, int causal,
                                                          const float* __restrict__ scores, T* __restrict__ P) {
  const long row = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int i = (int)(row % seq);
  const int live = causal ? i + 1 : seq;
  int fill = (live + kCausalPad - 1) / kCausalPad * kCausalPad;
  if (fill > seq) fill = seq;
  const float* s = scores + row * seq;
  float v[MAXC][4];
  float mx = -INFINITY;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int col = (lane + 64 * c) * 4;
    if (col < live) {
      Vec<float>::load(s + col, v[c]);
#pragma unroll
      for (int e = 0; e < 4; e++) {
        if (col + e >= live) v[c][e] = -INFINITY;
        mx = fmaxf(mx, v[c][e]);
      }
    }
  }
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int col = (lane + 64 * c) * 4;
    if (col < live) {
#pragma unroll
      for (int e = 0; e < 4; e++) {
        v[c][e] = __expf(v[c][e] - mx);
        sum += v[c][e];
      }
    }
  }
  sum = wave_sum(sum);
  const float inv = 1.f / sum;
  T* o = P + row * seq;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int col = (lane + 64 * c) * 4;
    if (col < fill) {
      if (col < live) {
#pragma unroll
        for (int e = 0; e < 4; e++) o[col + e] = (T)(v[c][e] * inv);
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++) o[col + e] = (T)0.f;
      }
    }
  }
}

// dS = P * (dP - sum_j dP_j P_j), in place over dP; same zero-fill rule.
template <typename T, int MAXC>
__global__ __launch_bounds__(256) void softmax_p1_kernel(long nrows, int seq, int causal, const T* __restrict__ P,
                                                         T* __restrict__ dP) {
  constexpr int N = Vec<T>::N;
  const long row = blockIdx.x * 4L + (threadIdx.x >> 6);
  if (row >= nrows) return;
  const int lane = threadIdx.x & 63;
  const int i = (int)(row % seq);
  const int live = causal ? i + 1 : seq;
  int fill = (live + kCausalPad - 1) / kCausalPad * kCausalPad;
  if (fill > seq) fill = seq;
  const T* p = P + row * seq;
  T* g = dP + row * seq;
  float pv[MAXC][N], gv[MAXC][N];
  float dot = 0.f;
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int col = (lane + 64 * c) * N;
    if (col < live) {
      Vec<T>::load(p + col, pv[c]);
      Vec<T>::load(g + col, gv[c]);
#pragma unroll
      for (int e = 0; e < N; e++) {
        if (col + e >= live) { pv[c][e] = 0.f; gv[c][e] = 0.f; }
        dot += pv[c][e] * gv[c][e];
      }
    }
  }
  dot = wave_sum(dot);
#pragma unroll
  for (int c = 0; c < MAXC; c++) {
    const int col = (lane + 64 * c) * N;
    if (col < fill) {
      float o[N];
#pragma unroll
      for (int e = 0; e < N; e++) o[e] = (col < live) ? pv[c][e] * (gv[c][e] - dot) : 0.f;
      Vec<T>::store(g + col, o);
    }
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

template <typename T, int WPR>
static hipError_t rmsnorm_p1_w(int rows, int d, float eps, const T* dy, const T* x, const T* g, const T* resid, T* dx,
                               float* partials, int* nblk_out, hipStream_t s) {
  constexpr int G = 8 / WPR;
  const int c = (d / Vec<T>::N + 64 * WPR - 1) / (64 * WPR);      // vectors per lane
  int nblk = (rows + G - 1) / G;
  if (nblk > kNormPartialBlocks) nblk = kNormPartialBlocks;
  *nblk_out = nblk;
  const size_t smem = (32 + (size_t)d) * sizeof(float);
  const dim3 grid(nblk), block(512);
  if (c <= 1) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 1, WPR>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else if (c <= 2) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 2, WPR>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else if (c <= 4) hipLaunchKernelGGL((rmsnorm_p1_kernel<T, 4, WPR>), grid, block, smem, s, rows, d, eps, dy, x, g, resid, dx, partials);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

template <typename T>
static hipError_t rmsnorm_p1_t(int rows, int d, float eps, const void* dy, const void* x, const void* g,
                               const void* resid, void* dx, float* dg_out, float* partials, hipStream_t s) {
  auto DY = (const T*)dy; auto X = (const T*)x; auto G = (const T*)g; auto RS = (const T*)resid; auto DX = (T*)dx;
  const int wc = (d / Vec<T>::N + 63) / 64;         // vectors per lane if one wave owned a whole row
  int nblk = 0;
  hipError_t e;
  if (wc <= 4) e = rmsnorm_p1_w<T, 1>(rows, d, eps, DY, X, G, RS, DX, partials, &nblk, s);
  else if (wc <= 8) e = rmsnorm_p1_w<T, 2>(rows, d, eps, DY, X, G, RS, DX, partials, &nblk, s);
  else if (wc <= 16) e = rmsnorm_p1_w<T, 4>(rows, d, eps, DY, X, G, RS, DX, partials, &nblk, s);
  else e = rmsnorm_p1_w<T, 8>(rows, d, eps, DY, X, G, RS, DX, partials, &nblk, s);
  if (e != hipSuccess) return e;
  RowList rl{};
  hipLaunchKernelGGL(colsum_kernel, dim3((d + 31) / 32), dim3(256), 0, s, (const float*)partials, rl, nblk, d, 0,
                     dg_out);
  return hipGetLastError();
}
hipError_t rmsnorm_p1(int dtype, int rows, int d, float eps, const void* dy, const void* x, const void* g,
                      const void* resid, void* dx, float* dg_out, float* partials, hipStream_t s) {
  if (rows <= 0) {      // no rows: the gain gradient is zero (written by the same column-sum kernel)
    RowList none{};
    hipLaunchKernelGGL(colsum_kernel, dim3((d + 31) / 32), dim3(256), 0, s, (const float*)partials, none, 0, d, 0,
                       dg_out);
    return hipGetLastError();
  }
  return dtype ? rmsnorm_p1_t<bf16_t>(rows, d, eps, dy, x, g, resid, dx, dg_out, partials, s)
               : rmsnorm_p1_t<float>(rows, d, eps, dy, x, g, resid, dx, dg_out, partials, s);
}

hipError_t gain_grad_sum(const float* parts, const int* rows_host, int n, int d, int accumulate, float* out,
                         hipStream_t s) {
  int done = 0;
  do {
    RowList rl{};
    rl.n = (n - done) < 64 ? (n - done) : 64;
    for (int i = 0; i < rl.n; i++) rl.idx[i] = rows_host[done + i];
    hipLaunchKernelGGL(colsum_kernel, dim3((d + 31) / 32), dim3(256), 0, s, parts, rl, 0, d,
                       (accumulate || done > 0) ? 1 : 0, out);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    done += rl.n;
  } while (done < n);
  return hipSuccess;
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
  const long nvec = (long)rows * n_heads * (head_dim / 2 / n);
  const float sgn = inverse ? -1.f : 1.f;
  if (dtype) hipLaunchKernelGGL(rope_kernel<bf16_t>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, seq, n_heads,
                                head_dim, ld, table, sgn, (bf16_t*)x);
  else hipLaunchKernelGGL(rope_kernel<float>, dim3(grid_for(nvec)), dim3(256), 0, s, nvec, seq, n_heads, head_dim,
                          ld, table, sgn, (float*)x);
  return hipGetLastError();
}

template <typename T>
static hipError_t softmax_fwd_t(long nrows, int seq, int causal, const float* sc, void* P, hipStream_t s) {
  const int c = (seq / 4 + 63) / 64;
  const dim3 grid((unsigned)((nrows + 3) / 4));
  if (c <= 4) hipLaunchKernelGGL((softmax_fwd_kernel<T, 4>), grid, dim3(256), 0, s, nrows, seq, causal, sc, (T*)P);
  else if (c <= 8) hipLaunchKernelGGL((softmax_fwd_kernel<T, 8>), grid, dim3(256), 0, s, nrows, seq, causal, sc, (T*)P);
  else if (c <= 16) hipLaunchKernelGGL((softmax_fwd_kernel<T, 16>), grid, dim3(256), 0, s, nrows, seq, causal, sc, (T*)P);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
hipError_t softmax_fwd(int dtype, long nrows, int seq, int causal, const float* scores, void* P, hipStream_t s) {
  if (nrows <= 0) return hipSuccess;
  return dtype ? softmax_fwd_t<bf16_t>(nrows, seq, causal, scores, P, s)
               : softmax_fwd_t<float>(nrows, seq, causal, scores, P, s);
}

template <typename T>
static hipError_t softmax_p1_t(long nrows, int seq, int causal, const void* P, void* dP, hipStream_t s) {
  const int c = (seq / Vec<T>::N + 63) / 64;
  const dim3 grid((unsigned)((nrows + 3) / 4));
  if (c <= 2) hipLaunchKernelGGL((softmax_p1_kernel<T, 2>), grid, dim3(256), 0, s, nrows, seq, causal, (const T*)P, (T*)dP);
  else if (c <= 4) hipLaunchKernelGGL((softmax_p1_kernel<T, 4>), grid, dim3(256), 0, s, nrows, seq, causal, (const T*)P, (T*)dP);
  else if (c <= 8) hipLaunchKernelGGL((softmax_p1_kernel<T, 8>), grid, dim3(256), 0, s, nrows, seq, causal, (const T*)P, (T*)dP);
  else if (c <= 16) hipLaunchKernelGGL((softmax_p1_kernel<T, 16>), grid, dim3(256), 0, s, nrows, seq, causal, (const T*)P, (T*)dP);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}
hipError_t softmax_p1(int dtype, long nrows, int seq, int causal, const void* P, void* dP, hipStream_t s) {
  if (nrows <= 0) return hipSuccess;
  return dtype ? softmax_p1_t<bf16_t>(nrows, seq, causal, P, dP, s) : softmax_p1_t<float>(nrows, seq, causal, P, dP, s);
}

}  // namespace tbp
