// Row-wise, HBM-bound kernels: LayerNorm forward/backward, GELU backward, softmax
// cross-entropy, embedding forward/backward, dtype conversion.
//
// One 64-lane wave owns one row; lane i holds columns i, i+64, ... in registers, so a
// wave load touches one contiguous run of the row and reductions are wave shuffles.
// Column reductions over rows (LayerNorm's dgamma/dbeta) are two-stage with a row ->
// chunk mapping fixed by the shape, so they are reproducible bit for bit (no atomics).
#include "device_common.h"
#include <initializer_list>

#include "kernels.h"
#include "philox.h"

namespace mk {

constexpr int kRowsPerChunk = 16;   // rows summed by one block of a two-stage column reduction
constexpr int kMaxNPL = 16;         // columns per lane: supports rows up to 1024 wide

// ---------------------------------------------------------------- LayerNorm forward
template <typename T, int NPL>
__device__ __forceinline__ void row_stats(const float (&v)[NPL], int H, int lane, float& mean, float& rstd,
                                          float eps) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NPL; ++i) if (lane + 64 * i < H) s += v[i];
  mean = wave_sum(s) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NPL; ++i) if (lane + 64 * i < H) { float d = v[i] - mean; q += d * d; }
  rstd = rsqrtf(wave_sum(q) / (float)H + eps);
}

template <typename TX, typename T, int NPL>
__global__ __launch_bounds__(256) void ln_fwd_kernel(const TX* __restrict__ x, const T* __restrict__ gamma,
                                                     const T* __restrict__ beta, T* __restrict__ y, int Trows,
                                                     int H, float eps) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Trows) return;
  const TX* xr = x + (int64_t)row * H;
  float v[NPL];
#pragma unroll
  for (int i = 0; i < NPL; ++i) { int c = lane + 64 * i; v[i] = c < H ? ld<TX>(xr + c) : 0.f; }
  float mean, rstd;
  row_stats<T, NPL>(v, H, lane, mean, rstd, eps);
  T* yr = y + (int64_t)row * H;
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    int c = lane + 64 * i;
    if (c < H) st<T>(yr + c, (v[i] - mean) * rstd * ld<T>(gamma + c) + ld<T>(beta + c));
  }
}

// ---------------------------------------------------------------- LayerNorm backward
// Block = 4 waves = kRowsPerChunk rows.  Statistics are recomputed from x; `add` (optional) is a
// residual-path gradient added to the result.  dx may alias dy; add must not alias dx.  Each wave keeps
// per-column sums of dy*xhat and dy over its rows; the four waves are combined through LDS
// in wave order and written as one partial row.
template <typename TD, typename TX, typename T, int NPL>
__global__ __launch_bounds__(256) void ln_bwd_kernel(const TD* __restrict__ dy, const TX* __restrict__ x,
                                                     const T* __restrict__ gamma, T* __restrict__ dx,
                                                     const T* __restrict__ add, float* __restrict__ partial,
                                                     int Trows, int H, float eps) {
  __shared__ float red[4][2][64 * NPL];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float g[NPL], sg[NPL], sb[NPL];
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    int c = lane + 64 * i;
    g[i] = c < H ? ld<T>(gamma + c) : 0.f;
    sg[i] = 0.f; sb[i] = 0.f;
  }
  for (int rr = 0; rr < kRowsPerChunk / 4; ++rr) {
    int row = blockIdx.x * kRowsPerChunk + rr * 4 + wave;
    if (row >= Trows) break;
    const TX* xr = x + (int64_t)row * H;
    const TD* dr = dy + (int64_t)row * H;
    float v[NPL], d[NPL];
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      int c = lane + 64 * i;
      v[i] = c < H ? ld<TX>(xr + c) : 0.f;
      d[i] = c < H ? ld<TD>(dr + c) : 0.f;
    }
    float mean, rstd;
    row_stats<T, NPL>(v, H, lane, mean, rstd, eps);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      float xh = (v[i] - mean) * rstd;
      v[i] = xh;
      sg[i] += d[i] * xh;
      sb[i] += d[i];
      float dxh = d[i] * g[i];
      d[i] = dxh;
      s1 += dxh;
      s2 += dxh * xh;
    }
    s1 = wave_sum(s1) / (float)H;
    s2 = wave_sum(s2) / (float)H;
    T* or_ = dx + (int64_t)row * H;
    const T* ar = add ? add + (int64_t)row * H : nullptr;
#pragma unroll
    for (int i = 0; i < NPL; ++i) {
      int c = lane + 64 * i;
      if (c < H) st<T>(or_ + c, rstd * (d[i] - s1 - v[i] * s2) + (ar ? ld<T>(ar + c) : 0.f));
    }
  }
#pragma unroll
  for (int i = 0; i < NPL; ++i) { red[wave][0][lane + 64 * i] = sg[i]; red[wave][1][lane + 64 * i] = sb[i]; }
  __syncthreads();
  float* prow = partial + (int64_t)blockIdx.x * 2 * H;
  for (int c = threadIdx.x; c < 2 * H; c += 256) {
    int which = c / H, col = c - which * H;
    float s = red[0][which][col];
    s += red[1][which][col];
    s += red[2][which][col];
    s += red[3][which][col];
    prow[c] = s;
  }
}

// out[c] = sum over partial rows, c in [0, ncols): 16 row groups x 16 columns per block,
// each group adds its rows in order, groups are combined in order.  (Fallback for column counts
// or pointers that do not allow 16-byte accesses.)
__global__ __launch_bounds__(256) void reduce_partials_kernel(const float* __restrict__ partial, int P,
                                                              int ncols, float* __restrict__ out0,
                                                              float* __restrict__ out1, int split) {
  __shared__ float red[16][17];
  const int cg = threadIdx.x & 15, rg = threadIdx.x >> 4;
  const int c = blockIdx.x * 16 + cg;
  float s = 0.f;
  if (c < ncols)
    for (int r = rg; r < P; r += 16) s += partial[(int64_t)r * ncols + c];
  red[rg][cg] = s;
  __syncthreads();
  if (rg == 0 && c < ncols) {
    float t = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i][cg];
    if (c < split) out0[c] = t; else out1[c - split] = t;
  }
}

// The same sums with whole 128-byte lines: a block owns 32 columns, 32 row groups x 8 lanes of four
// columns; a group adds rows g, g + 32, ... in order, eight loads in flight at a time (a chain of
// dependent loads costs a memory latency per row), groups are combined in order.
__global__ __launch_bounds__(256) void reduce_partials_vec_kernel(const float* __restrict__ partial, int P,
                                                                  int ncols, float* __restrict__ out0,
                                                                  float* __restrict__ out1, int split) {
  __shared__ float4 red[32][8];
  const int cq = threadIdx.x & 7, rg = threadIdx.x >> 3;
  const int c = blockIdx.x * 32 + cq * 4;
  float4 s = make_float4(0.f, 0.f, 0.f, 0.f);
  if (c < ncols)
    for (int r0 = rg; r0 < P; r0 += 32 * 8) {
      float4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int r = r0 + 32 * u;
        v[u] = r < P ? *(const float4*)(partial + (int64_t)r * ncols + c) : make_float4(0.f, 0.f, 0.f, 0.f);
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) { s.x += v[u].x; s.y += v[u].y; s.z += v[u].z; s.w += v[u].w; }
    }
  red[rg][cq] = s;
  __syncthreads();
  if (rg == 0 && c < ncols) {
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int i = 0; i < 32; ++i) { const float4 q = red[i][cq]; t.x += q.x; t.y += q.y; t.z += q.z; t.w += q.w; }
    const float e[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
    for (int k = 0; k < 4; ++k) { const int cc = c + k; if (cc < split) out0[cc] = e[k]; else out1[cc - split] = e[k]; }
  }
}

// ---------------------------------------------------------------- vectorised row access
// 16-byte chunks: 8 bf16 or 4 fp32 per lane and access; lane l owns chunks l, l+64, ...
template <typename T> struct Chunk;
template <> struct Chunk<bf16_t> {
  static constexpr int N = 8;
  static __device__ __forceinline__ void load(const bf16_t* p, float (&v)[8]) {
    const uint4 u = *(const uint4*)p;
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xFFFF0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xFFFF0000u);
    v[4] = __uint_as_float(u.z << 16); v[5] = __uint_as_float(u.z & 0xFFFF0000u);
    v[6] = __uint_as_float(u.w << 16); v[7] = __uint_as_float(u.w & 0xFFFF0000u);
  }
  static __device__ __forceinline__ void store(bf16_t* p, const float (&v)[8]) {
    uint4 u;
    u.x = pack_bf16x2(v[0], v[1]);
    u.y = pack_bf16x2(v[2], v[3]);
    u.z = pack_bf16x2(v[4], v[5]);
    u.w = pack_bf16x2(v[6], v[7]);
    *(uint4*)p = u;
  }
};
template <> struct Chunk<float> {
  static constexpr int N = 4;
  static __device__ __forceinline__ void load(const float* p, float (&v)[4]) {
    const float4 u = *(const float4*)p;
    v[0] = u.x; v[1] = u.y; v[2] = u.z; v[3] = u.w;
  }
  static __device__ __forceinline__ void store(float* p, const float (&v)[4]) {
    *(float4*)p = make_float4(v[0], v[1], v[2], v[3]);
  }
};

// E consecutive elements of type T as floats (E = Chunk<storage type>::N; fp32 sources of a bf16
// configuration take two 16-byte loads)
template <typename T, int E>
__device__ __forceinline__ void load_elems(const T* p, float (&v)[E]) {
  constexpr int N = Chunk<T>::N;
#pragma unroll
  for (int k = 0; k < E / N; ++k) {
    float t[N];
    Chunk<T>::load(p + k * N, t);
#pragma unroll
    for (int e = 0; e < N; ++e) v[k * N + e] = t[e];
  }
}

// mean and 1/std of a row held as NC chunks per lane (chunks >= nchunks hold zeros)
template <int NC, int E>
__device__ __forceinline__ void chunk_stats(const float (&v)[NC][E], int nchunks, int lane, int H, float eps,
                                            float& mean, float& rstd) {
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int e = 0; e < E; ++e) s += v[i][e];
  mean = wave_sum(s) / (float)H;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < NC; ++i)
    if (lane + 64 * i < nchunks)
#pragma unroll
      for (int e = 0; e < E; ++e) { const float d = v[i][e] - mean; q += d * d; }
  rstd = rsqrtf(wave_sum(q) / (float)H + eps);
}

template <typename TX, typename T, int NC>
__global__ __launch_bounds__(256) void ln_fwd_vec_kernel(const TX* __restrict__ x, const T* __restrict__ gamma,
                                                         const T* __restrict__ beta, T* __restrict__ y, int Trows,
                                                         int H, float eps) {
  constexpr int E = Chunk<T>::N;
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Trows) return;
  const int nchunks = H / E;
  const TX* xr = x + (int64_t)row * H;
  float v[NC][E];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) load_elems<TX, E>(xr + c * E, v[i]);
    else
#pragma unroll
      for (int e = 0; e < E; ++e) v[i][e] = 0.f;
  }
  float mean, rstd;
  chunk_stats<NC, E>(v, nchunks, lane, H, eps, mean, rstd);
  T* yr = y + (int64_t)row * H;
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) {
      float g[E], b[E], o[E];
      Chunk<T>::load(gamma + c * E, g);
      Chunk<T>::load(beta + c * E, b);
#pragma unroll
      for (int e = 0; e < E; ++e) o[e] = (v[i][e] - mean) * rstd * g[e] + b[e];
      Chunk<T>::store(yr + c * E, o);
    }
  }
}

// Backward: block = 4 waves = kRowsPerChunk rows, every wave takes 4 rows and issues all their
// loads before any arithmetic.  Same outputs and the same summation order as ln_bwd_kernel.
template <typename TD, typename TX, typename T, int NC>
__global__ __launch_bounds__(256) void ln_bwd_vec_kernel(const TD* __restrict__ dy, const TX* __restrict__ x,
                                                         const T* __restrict__ gamma, T* __restrict__ dx,
                                                         const T* __restrict__ add, float* __restrict__ partial,
                                                         int Trows, int H, float eps) {
  constexpr int E = Chunk<T>::N;
  constexpr int R = kRowsPerChunk / 4;
  __shared__ float red[4][2][64 * NC * E];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int nchunks = H / E;
  float g[NC][E], sg[NC][E], sb[NC][E];
#pragma unroll
  for (int i = 0; i < NC; ++i) {
    const int c = lane + 64 * i;
    if (c < nchunks) Chunk<T>::load(gamma + c * E, g[i]);
#pragma unroll
    for (int e = 0; e < E; ++e) { if (c >= nchunks) g[i][e] = 0.f; sg[i][e] = 0.f; sb[i][e] = 0.f; }
  }
  float v[R][NC][E], d[R][NC][E];
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const int row = blockIdx.x * kRowsPerChunk + rr * 4 + wave;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      if (row < Trows && c < nchunks) {
        load_elems<TX, E>(x + (int64_t)row * H + c * E, v[rr][i]);
        load_elems<TD, E>(dy + (int64_t)row * H + c * E, d[rr][i]);
      } else {
#pragma unroll
        for (int e = 0; e < E; ++e) { v[rr][i][e] = 0.f; d[rr][i][e] = 0.f; }
      }
    }
  }
#pragma unroll
  for (int rr = 0; rr < R; ++rr) {
    const int row = blockIdx.x * kRowsPerChunk + rr * 4 + wave;
    if (row >= Trows) break;
    float mean, rstd;
    chunk_stats<NC, E>(v[rr], nchunks, lane, H, eps, mean, rstd);
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int i = 0; i < NC; ++i)
      if (lane + 64 * i < nchunks)
#pragma unroll
        for (int e = 0; e < E; ++e) {
          const float xh = (v[rr][i][e] - mean) * rstd;
          v[rr][i][e] = xh;
          sg[i][e] += d[rr][i][e] * xh;
          sb[i][e] += d[rr][i][e];
          const float dxh = d[rr][i][e] * g[i][e];
          d[rr][i][e] = dxh;
          s1 += dxh;
          s2 += dxh * xh;
        }
    s1 = wave_sum(s1) / (float)H;
    s2 = wave_sum(s2) / (float)H;
#pragma unroll
    for (int i = 0; i < NC; ++i) {
      const int c = lane + 64 * i;
      if (c < nchunks) {
        float o[E];
#pragma unroll
        for (int e = 0; e < E; ++e) o[e] = rstd * (d[rr][i][e] - s1 - v[rr][i][e] * s2);
        if (add) {
          float a[E];
          Chunk<T>::load(add + (int64_t)row * H + c * E, a);
#pragma unroll
          for (int e = 0; e < E; ++e) o[e] += a[e];
        }
        Chunk<T>::store(dx + (int64_t)row * H + c * E, o);
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int e = 0; e < E; ++e) {
      red[wave][0][(lane + 64 * i) * E + e] = sg[i][e];
      red[wave][1][(lane + 64 * i) * E + e] = sb[i][e];
    }
  __syncthreads();
  float* prow = partial + (int64_t)blockIdx.x * 2 * H;
  for (int c = threadIdx.x; c < 2 * H; c += 256) {
    const int which = c / H, col = c - which * H;
    float s = red[0][which][col];
    s += red[1][which][col];
    s += red[2][which][col];
    s += red[3][which][col];
    prow[c] = s;
  }
}

// ---------------------------------------------------------------- GELU backward (in place)
template <typename T>
__global__ __launch_bounds__(256) void gelu_bwd_scalar_kernel(T* __restrict__ d, const T* __restrict__ pre,
                                                              int64_t n, int tanh_form) {
  int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (i + e < n) {
      float x = ld<T>(pre + i + e);
      float gp = tanh_form ? gelu_tanh_grad(x) : gelu_erf_grad(x);
      st<T>(d + i + e, ld<T>(d + i + e) * gp);
    }
  }
}
__global__ __launch_bounds__(256) void gelu_bwd_bf16_kernel(bf16_t* __restrict__ d,
                                                            const bf16_t* __restrict__ pre, int64_t n,
                                                            int tanh_form) {
  int64_t i = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 8;
  if (i >= n) return;
  if (i + 8 <= n) {
    uint4 dv = *(const uint4*)(d + i), pv = *(const uint4*)(pre + i);
    bf16_t* dp = (bf16_t*)&dv;
    const bf16_t* pp = (const bf16_t*)&pv;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = bf16_to_f32(pp[e]);
      float gp = tanh_form ? gelu_tanh_grad(x) : gelu_erf_grad_bf16(x);
      dp[e] = f32_to_bf16(bf16_to_f32(dp[e]) * gp);
    }
    *(uint4*)(d + i) = dv;
  } else {
    for (int e = 0; i + e < n; ++e) {
      float x = bf16_to_f32(pre[i + e]);
      float gp = tanh_form ? gelu_tanh_grad(x) : gelu_erf_grad_bf16(x);
      d[i + e] = f32_to_bf16(bf16_to_f32(d[i + e]) * gp);
    }
  }
}

// ---------------------------------------------------------------- softmax cross-entropy
// One block per row.  Pass 1: running (max, sum of exp) per thread, merged in a fixed tree.
// Pass 2: the row is overwritten with (softmax - onehot)/n_valid, zero for unscored rows and
// for the padding columns [V, ld).
template <typename T>
__global__ __launch_bounds__(256) void xent_kernel(T* __restrict__ logits, int64_t ldl,
                                                   const int32_t* __restrict__ labels,
                                                   float* __restrict__ row_loss, int V, float inv_n) {
  __shared__ float sm[4], ss[4];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  T* lr = logits + (int64_t)row * ldl;
  const int label = labels[row];
  float m = -INFINITY, s = 0.f;
  for (int c = tid; c < V; c += 256) {
    float v = ld<T>(lr + c);
    if (v > m) { s = s * __expf(m - v) + 1.f; m = v; } else { s += __expf(v - m); }
  }
  float wm = wave_max(m);
  s = wave_sum(m == -INFINITY ? 0.f : s * __expf(m - wm));   // threads or waves past a short row hold nothing
  if (lane == 0) { sm[wave] = wm; ss[wave] = s; }
  __syncthreads();
  float bm = fmaxf(fmaxf(sm[0], sm[1]), fmaxf(sm[2], sm[3]));
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < 4; ++w) bs += sm[w] == -INFINITY ? 0.f : ss[w] * __expf(sm[w] - bm);
  const float lse = bm + __logf(bs);
  if (tid == 0) row_loss[row] = label >= 0 ? lse - ld<T>(lr + label) : 0.f;
  __syncthreads();   // the label's logit is read before the row is overwritten
  const float scale = label >= 0 ? inv_n : 0.f;
  for (int c = tid; c < ldl; c += 256) {
    float g = 0.f;
    if (c < V) g = (__expf(ld<T>(lr + c) - lse) - (c == label ? 1.f : 0.f)) * scale;
    st<T>(lr + c, g);
  }
}

// bf16 rows of up to NCH * THREADS 16-byte chunks: the row is read once, kept in registers as
// fp32, and written once.
template <int THREADS, int NCH>
__global__ __launch_bounds__(THREADS) void xent_bf16_kernel(bf16_t* __restrict__ logits, int64_t ldl,
                                                            const int32_t* __restrict__ labels,
                                                            float* __restrict__ row_loss, int V, float inv_n) {
  constexpr int NW = THREADS / 64;
  __shared__ float sm[NW], ss[NW];
  const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  bf16_t* lr = logits + (int64_t)row * ldl;
  const int label = labels[row];
  const float picked = (tid == 0 && label >= 0) ? bf16_to_f32(lr[label]) : 0.f;
  const int nchunks = (int)(ldl / 8);
  float v[NCH][8];
  float m = -INFINITY;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = tid + THREADS * i;
    if (c < nchunks) {
      Chunk<bf16_t>::load(lr + c * 8, v[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (c * 8 + e >= V) v[i][e] = -INFINITY;
        m = fmaxf(m, v[i][e]);
      }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) v[i][e] = -INFINITY;
    }
  }
  m = wave_max(m);
  if (lane == 0) sm[wave] = m;
  __syncthreads();
  float bm = sm[0];
#pragma unroll
  for (int w = 1; w < NW; ++w) bm = fmaxf(bm, sm[w]);
  // the exponentials are kept (in place of the logits): the gradient is made from them, so each
  // element costs one exponential, not two
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i)
#pragma unroll
    for (int e = 0; e < 8; ++e) { v[i][e] = __expf(v[i][e] - bm); s += v[i][e]; }
  s = wave_sum(s);
  if (lane == 0) ss[wave] = s;
  __syncthreads();
  float bs = 0.f;
#pragma unroll
  for (int w = 0; w < NW; ++w) bs += ss[w];
  const float lse = bm + __logf(bs);
  if (tid == 0) row_loss[row] = label >= 0 ? lse - picked : 0.f;
  const float scale = label >= 0 ? inv_n : 0.f;
  const float pscale = scale / bs;                    // softmax = exp(v - max) / sum
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = tid + THREADS * i;
    if (c < nchunks) {
      float g[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int col = c * 8 + e;
        g[e] = v[i][e] * pscale - (col == label ? scale : 0.f);   // columns >= V hold exp(-inf) = 0
      }
      Chunk<bf16_t>::store(lr + c * 8, g);
    }
  }
}

__global__ __launch_bounds__(256) void loss_reduce_kernel(const float* __restrict__ row_loss, int n, float inv_n,
                                                          float* __restrict__ loss) {
  __shared__ float red[256];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += 256) s += row_loss[i];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) red[threadIdx.x] += red[threadIdx.x + o];
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss = red[0] * inv_n;
}

// ---------------------------------------------------------------- embedding
template <typename T, int NPL>
__global__ __launch_bounds__(256) void embed_fwd_kernel(const int32_t* __restrict__ ids, const T* __restrict__ tok,
                                                        const T* __restrict__ pos, const T* __restrict__ gamma,
                                                        const T* __restrict__ beta, T* __restrict__ sum_out,
                                                        T* __restrict__ y, int Trows, int L, int H, float eps,
                                                        int has_ln) {
  const int lane = threadIdx.x & 63, row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= Trows) return;
  const T* tr = tok + (int64_t)ids[row] * H;
  const T* pr = pos + (int64_t)(row % L) * H;
  float v[NPL];
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    int c = lane + 64 * i;
    // the sum is formed in the storage type so LayerNorm sees exactly what is saved
    v[i] = c < H ? rnd<T>(ld<T>(tr + c) + ld<T>(pr + c)) : 0.f;
  }
  if (sum_out) {
    T* sr = sum_out + (int64_t)row * H;
#pragma unroll
    for (int i = 0; i < NPL; ++i) { int c = lane + 64 * i; if (c < H) st<T>(sr + c, v[i]); }
  }
  T* yr = y + (int64_t)row * H;
  if (!has_ln) {
#pragma unroll
    for (int i = 0; i < NPL; ++i) { int c = lane + 64 * i; if (c < H) st<T>(yr + c, v[i]); }
    return;
  }
  float mean, rstd;
  row_stats<T, NPL>(v, H, lane, mean, rstd, eps);
#pragma unroll
  for (int i = 0; i < NPL; ++i) {
    int c = lane + 64 * i;
    if (c < H) st<T>(yr + c, (v[i] - mean) * rstd * ld<T>(gamma + c) + ld<T>(beta + c));
  }
}

// dpos[p][c] = sum over samples b (in order) of d[b*L+p][c]; rows p >= L are cleared.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_pos_kernel(const T* __restrict__ d, float* __restrict__ dpos,
                                                            int B, int L, int H, int max_seq) {
  int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (int64_t)max_seq * H) return;
  int p = (int)(idx / H), c = (int)(idx - (int64_t)p * H);
  float s = 0.f;
  if (p < L)
    for (int b = 0; b < B; ++b) s += ld<T>(d + ((int64_t)b * L + p) * H + c);
  dpos[idx] = s;
}

// One wave per distinct token id: rows of d at that id's positions (ascending) are summed
// and added onto the id's gradient row.
template <typename T>
__global__ __launch_bounds__(256) void embed_bwd_tok_kernel(const T* __restrict__ d, const int32_t* __restrict__ ids,
                                                            const int32_t* __restrict__ order,
                                                            const int32_t* __restrict__ seg, int n_seg,
                                                            float* __restrict__ dtok, int H) {
  const int lane = threadIdx.x & 63, sidx = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (sidx >= n_seg) return;
  const int beg = seg[sidx], end = seg[sidx + 1];
  const int id = ids[order[beg]];
  float* out = dtok + (int64_t)id * H;
  for (int c = lane; c < H; c += 64) {
    float s = 0.f;
    for (int k = beg; k < end; ++k) s += ld<T>(d + (int64_t)order[k] * H + c);
    out[c] += s;
  }
}

template <typename T>
__global__ __launch_bounds__(256) void convert_kernel(const float* __restrict__ src, T* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) st<T>(dst + i, src[i]);
}

template <typename T>
__global__ __launch_bounds__(256) void widen_kernel(const T* __restrict__ src, float* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = ld<T>(src + i);
}

// dst[i] = (resid ? resid[i] : 0) + keep(i) * scale * src[i]; element i reads word i % 4 of block
// i / 4.  Four elements per thread; dst may be src.
template <typename TIO, typename TR>
__global__ __launch_bounds__(256) void dropout_kernel(TIO* __restrict__ dst, const TIO* src, const TR* __restrict__ resid,
                                                      int64_t n, DropDesc d) {
  const int64_t blk = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t i0 = 4 * blk;
  if (i0 >= n) return;
  const uint4 w4 = drop_words(d, (uint64_t)blk);
  const uint32_t w[4] = {w4.x, w4.y, w4.z, w4.w};
  const int cnt = (int)min((int64_t)4, n - i0);
  for (int e = 0; e < cnt; ++e) {
    float v = w[e] >= d.thr ? ld<TIO>(src + i0 + e) * d.scale : 0.f;
    if (resid) v += ld<TR>(resid + i0 + e);
    st<TIO>(dst + i0 + e, v);
  }
}

// One block per chunk of kAdamChunk elements of one tensor; element-wise, fp32 arithmetic:
//   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2
//   p = p - lr * ( (m / c1) / (sqrt(v / c2) + eps) + wd p )      (decoupled weight decay)
// The low-precision copy, when there is one, is the new master value rounded to nearest-even.
__global__ __launch_bounds__(256) void adamw_kernel(const AdamTensor* __restrict__ tensors,
                                                    const AdamChunk* __restrict__ chunks, AdamHyper h) {
  const AdamChunk ck = chunks[blockIdx.x];
  const AdamTensor t = tensors[ck.tensor];
  const float wd = t.decay ? h.weight_decay : 0.f;
  const int64_t end = min(t.n, ck.start + (int64_t)kAdamChunk);
  bf16_t* lowp = (bf16_t*)t.lowp;
  // 4 elements per thread and pass while the chunk allows (tensor starts are 256-byte aligned)
  for (int64_t i = ck.start + 4 * (int64_t)threadIdx.x; i < end; i += 4 * 256) {
    if (i + 4 <= end) {
      const float4 g = *(const float4*)(t.grad + i);
      float4 m = *(const float4*)(t.m + i), v = *(const float4*)(t.v + i), p = *(const float4*)(t.master + i);
      const float gs[4] = {g.x, g.y, g.z, g.w};
      float ms[4] = {m.x, m.y, m.z, m.w}, vs[4] = {v.x, v.y, v.z, v.w}, ps[4] = {p.x, p.y, p.z, p.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        ms[e] = h.beta1 * ms[e] + (1.f - h.beta1) * gs[e];
        vs[e] = h.beta2 * vs[e] + (1.f - h.beta2) * gs[e] * gs[e];
        ps[e] -= h.lr * ((ms[e] * h.inv_c1) / (sqrtf(vs[e] * h.inv_c2) + h.eps) + wd * ps[e]);
      }
      *(float4*)(t.m + i) = make_float4(ms[0], ms[1], ms[2], ms[3]);
      *(float4*)(t.v + i) = make_float4(vs[0], vs[1], vs[2], vs[3]);
      *(float4*)(t.master + i) = make_float4(ps[0], ps[1], ps[2], ps[3]);
      if (lowp) {
        uint2 w;
        w.x = pack_bf16x2(ps[0], ps[1]);
        w.y = pack_bf16x2(ps[2], ps[3]);
        *(uint2*)(lowp + i) = w;
      }
    } else {
      for (int64_t j = i; j < end; ++j) {
        const float g = t.grad[j];
        const float m = h.beta1 * t.m[j] + (1.f - h.beta1) * g;
        const float v = h.beta2 * t.v[j] + (1.f - h.beta2) * g * g;
        float pv = t.master[j];
        pv -= h.lr * ((m * h.inv_c1) / (sqrtf(v * h.inv_c2) + h.eps) + wd * pv);
        t.m[j] = m; t.v[j] = v; t.master[j] = pv;
        if (lowp) lowp[j] = f32_to_bf16(pv);
      }
    }
  }
}

__global__ __launch_bounds__(256) void fill_zero_kernel(uint32_t* __restrict__ p, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---------------------------------------------------------------- launchers
#define DISPATCH_NPL(H, M)                      \
  do {                                          \
    int npl_ = ((H) + 63) / 64;                 \
    if (npl_ <= 1) { M(1); }                    \
    else if (npl_ <= 2) { M(2); }               \
    else if (npl_ <= 4) { M(4); }               \
    else if (npl_ <= 8) { M(8); }               \
    else if (npl_ <= 12) { M(12); }             \
    else { M(16); }                             \
  } while (0)

// rows whose length is a whole number of 16-byte chunks and whose storage is 16-byte aligned
template <typename T>
static bool vec_ok(int H, std::initializer_list<const void*> ptrs) {
  if (H % Chunk<T>::N) return false;
  for (const void* p : ptrs) if (p && (((uintptr_t)p) & 15)) return false;
  return true;
}

template <typename TX, typename T>
static void ln_fwd_t(const void* x, const void* g, const void* b, void* y, int T_, int H, float eps,
                     hipStream_t st) {
  dim3 grid((T_ + 3) / 4);
  if (vec_ok<T>(H, {x, g, b, y})) {
    const int nc = (H / Chunk<T>::N + 63) / 64;
#define V_(NC) hipLaunchKernelGGL((ln_fwd_vec_kernel<TX, T, NC>), grid, dim3(256), 0, st, (const TX*)x, (const T*)g, \
                                   (const T*)b, (T*)y, T_, H, eps)
    if (nc <= 1) { V_(1); return; }
    if (nc <= 2) { V_(2); return; }
    if (nc <= 4) { V_(4); return; }
#undef V_
  }
#define M_(NPL) hipLaunchKernelGGL((ln_fwd_kernel<TX, T, NPL>), grid, dim3(256), 0, st, (const TX*)x, (const T*)g, \
                                   (const T*)b, (T*)y, T_, H, eps)
  DISPATCH_NPL(H, M_);
#undef M_
}
void layernorm_fwd(int dtype, const void* x, bool x_f32, const void* gamma, const void* beta, void* y, int T_,
                   int H, float eps, hipStream_t st) {
  if (T_ <= 0) return;
  if (dtype != BF16) ln_fwd_t<float, float>(x, gamma, beta, y, T_, H, eps, st);
  else if (x_f32) ln_fwd_t<float, bf16_t>(x, gamma, beta, y, T_, H, eps, st);
  else ln_fwd_t<bf16_t, bf16_t>(x, gamma, beta, y, T_, H, eps, st);
}

template <typename TD, typename TX, typename T>
static void ln_bwd_t(const void* dy, const void* x, const void* g, void* dx, const void* add, float* partial,
                     int T_, int H, float eps, hipStream_t st) {
  dim3 grid((T_ + kRowsPerChunk - 1) / kRowsPerChunk);
  if (vec_ok<T>(H, {dy, x, g, dx, add})) {
    const int nc = (H / Chunk<T>::N + 63) / 64;
#define V_(NC) hipLaunchKernelGGL((ln_bwd_vec_kernel<TD, TX, T, NC>), grid, dim3(256), 0, st, (const TD*)dy, \
                                   (const TX*)x, (const T*)g, (T*)dx, (const T*)add, partial, T_, H, eps)
    if (nc <= 1) { V_(1); return; }
    if (nc <= 2) { V_(2); return; }
#undef V_
  }
#define M_(NPL) hipLaunchKernelGGL((ln_bwd_kernel<TD, TX, T, NPL>), grid, dim3(256), 0, st, (const TD*)dy,    \
                                   (const TX*)x, (const T*)g, (T*)dx, (const T*)add, partial, T_, H, eps)
  DISPATCH_NPL(H, M_);
#undef M_
}
void layernorm_bwd_rows(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32, const void* gamma, void* dx,
                        const void* add, float* partial, int T_, int H, float eps, hipStream_t st) {
  if (T_ <= 0) return;
  if (dtype != BF16) ln_bwd_t<float, float, float>(dy, x, gamma, dx, add, partial, T_, H, eps, st);
  else if (dy_f32 && x_f32) ln_bwd_t<float, float, bf16_t>(dy, x, gamma, dx, add, partial, T_, H, eps, st);
  else if (dy_f32) ln_bwd_t<float, bf16_t, bf16_t>(dy, x, gamma, dx, add, partial, T_, H, eps, st);
  else if (x_f32) ln_bwd_t<bf16_t, float, bf16_t>(dy, x, gamma, dx, add, partial, T_, H, eps, st);
  else ln_bwd_t<bf16_t, bf16_t, bf16_t>(dy, x, gamma, dx, add, partial, T_, H, eps, st);
}
void layernorm_bwd_reduce(const float* partial, float* dgamma, float* dbeta, int T_, int H, hipStream_t st) {
  if (T_ <= 0) return;
  int P = (T_ + kRowsPerChunk - 1) / kRowsPerChunk;
  if ((H & 1) == 0 && (((uintptr_t)partial) & 15) == 0)      // rows of 2H floats: every float4 inside a row, lines aligned
    hipLaunchKernelGGL(reduce_partials_vec_kernel, dim3((2 * H + 31) / 32), dim3(256), 0, st, partial, P, 2 * H, dgamma,
                       dbeta, H);
  else
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((2 * H + 15) / 16), dim3(256), 0, st, partial, P, 2 * H, dgamma,
                       dbeta, H);
}
void layernorm_bwd(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32, const void* gamma, void* dx,
                   const void* add, float* dgamma, float* dbeta, float* partial, int T_, int H, float eps,
                   hipStream_t st) {
  layernorm_bwd_rows(dtype, dy, dy_f32, x, x_f32, gamma, dx, add, partial, T_, H, eps, st);
  layernorm_bwd_reduce(partial, dgamma, dbeta, T_, H, st);
}
int partial_rows(int T_) { return (T_ + kRowsPerChunk - 1) / kRowsPerChunk; }

// Scratch of the entry point that allocates nothing: the per-chunk partial sums of the LayerNorm
// backward.  Each device the library runs on holds its own copy until the process ends; host code
// never uses the array's name as an address, only what hipGetSymbolAddress returned for the
// device that was current.
static __device__ __align__(256) float scratch[kStaticPartialFloats];
static float* g_scratch_of_device[64];

int layernorm_bwd_static(int dtype, const void* dy, bool dy_f32, const void* x, bool x_f32, const void* gamma,
                         void* dx, const void* add, float* dgamma, float* dbeta, int T_, int H, float eps,
                         hipStream_t st) {
  if ((size_t)partial_rows(T_) * 2 * (size_t)H > kStaticPartialFloats) return -1;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return -2;
  float* ptr = g_scratch_of_device[dev];
  if (!ptr) {
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return -2;
    g_scratch_of_device[dev] = ptr;
  }
  // every partial row that the reduction reads is written by the row pass first: nothing to clear
  layernorm_bwd(dtype, dy, dy_f32, x, x_f32, gamma, dx, add, dgamma, dbeta, ptr, T_, H, eps, st);
  return 0;
}

void gelu_bwd(int dtype, void* d, const void* pre, int64_t n, int tanh_form, hipStream_t st) {
  if (n <= 0) return;
  dim3 grid((unsigned)((n + 2047) / 2048));
  if (dtype == BF16) hipLaunchKernelGGL(gelu_bwd_bf16_kernel, grid, dim3(256), 0, st, (bf16_t*)d, (const bf16_t*)pre, n, tanh_form);
  else hipLaunchKernelGGL(gelu_bwd_scalar_kernel<float>, grid, dim3(256), 0, st, (float*)d, (const float*)pre, n, tanh_form);
}

void softmax_xent(int dtype, void* logits, int64_t ldl, const int32_t* labels, float* row_loss, float* loss,
                  int T_, int V, int n_valid, hipStream_t st) {
  if (T_ <= 0) return;
  float inv_n = 1.0f / (float)(n_valid > 0 ? n_valid : 1);
  const int64_t nch = ldl / 8;
  if (dtype == BF16 && ldl % 8 == 0 && ((((uintptr_t)logits) & 15) == 0) && nch <= 16 * 1024) {
    bf16_t* lg = (bf16_t*)logits;
    // threads x chunks per thread: the fewest registers per thread that hold the row (more waves per SIMD)
#define X_(TH, NC) hipLaunchKernelGGL((xent_bf16_kernel<TH, NC>), dim3(T_), dim3(TH), 0, st, lg, ldl, labels, row_loss, V, inv_n)
    if (nch <= 4 * 256) X_(256, 4);
    else if (nch <= 8 * 256) X_(256, 8);
    else if (nch <= 4 * 1024) X_(1024, 4);
    else if (nch <= 8 * 512) X_(512, 8);
    else if (nch <= 8 * 1024) X_(1024, 8);
    else X_(1024, 16);
#undef X_
  } else if (dtype == BF16) hipLaunchKernelGGL(xent_kernel<bf16_t>, dim3(T_), dim3(256), 0, st, (bf16_t*)logits, ldl, labels, row_loss, V, inv_n);
  else hipLaunchKernelGGL(xent_kernel<float>, dim3(T_), dim3(256), 0, st, (float*)logits, ldl, labels, row_loss, V, inv_n);
  hipLaunchKernelGGL(loss_reduce_kernel, dim3(1), dim3(256), 0, st, row_loss, T_, inv_n, loss);
}

template <typename T>
static void embed_fwd_t(const int32_t* ids, const void* tok, const void* pos, const void* g, const void* b,
                        void* sum_out, void* y, int B, int L, int H, float eps, int has_ln, hipStream_t st) {
  int T_ = B * L;
  dim3 grid((T_ + 3) / 4);
#define M_(NPL) hipLaunchKernelGGL((embed_fwd_kernel<T, NPL>), grid, dim3(256), 0, st, ids, (const T*)tok,     \
                                   (const T*)pos, (const T*)g, (const T*)b, (T*)sum_out, (T*)y, T_, L, H, eps, \
                                   has_ln)
  DISPATCH_NPL(H, M_);
#undef M_
}
void embed_fwd(int dtype, const int32_t* ids, const void* tok, const void* pos, const void* gamma,
               const void* beta, void* sum_out, void* y, int B, int L, int H, float eps, int has_ln,
               hipStream_t st) {
  if (B * L <= 0) return;
  if (dtype == BF16) embed_fwd_t<bf16_t>(ids, tok, pos, gamma, beta, sum_out, y, B, L, H, eps, has_ln, st);
  else embed_fwd_t<float>(ids, tok, pos, gamma, beta, sum_out, y, B, L, H, eps, has_ln, st);
}

void embed_bwd(int dtype, const void* d, const int32_t* ids, const int32_t* order, const int32_t* seg,
               int n_seg, float* dtok, float* dpos, int B, int L, int H, int max_seq, hipStream_t st) {
  if (B * L <= 0) return;
  dim3 gp((unsigned)(((int64_t)max_seq * H + 255) / 256)), gt((n_seg + 3) / 4);
  if (dtype == BF16) {
    hipLaunchKernelGGL(embed_bwd_pos_kernel<bf16_t>, gp, dim3(256), 0, st, (const bf16_t*)d, dpos, B, L, H, max_seq);
    hipLaunchKernelGGL(embed_bwd_tok_kernel<bf16_t>, gt, dim3(256), 0, st, (const bf16_t*)d, ids, order, seg, n_seg, dtok, H);
  } else {
    hipLaunchKernelGGL(embed_bwd_pos_kernel<float>, gp, dim3(256), 0, st, (const float*)d, dpos, B, L, H, max_seq);
    hipLaunchKernelGGL(embed_bwd_tok_kernel<float>, gt, dim3(256), 0, st, (const float*)d, ids, order, seg, n_seg, dtok, H);
  }
}

void convert_from_f32(int dtype, const float* src, void* dst, int64_t n, hipStream_t st) {
  if (n <= 0) return;
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == BF16) hipLaunchKernelGGL(convert_kernel<bf16_t>, grid, dim3(256), 0, st, src, (bf16_t*)dst, n);
  else hipLaunchKernelGGL(convert_kernel<float>, grid, dim3(256), 0, st, src, (float*)dst, n);
}

void convert_to_f32(int dtype, const void* src, float* dst, int64_t n, hipStream_t st) {
  if (n <= 0) return;
  dim3 grid((unsigned)((n + 255) / 256));
  if (dtype == BF16) hipLaunchKernelGGL(widen_kernel<bf16_t>, grid, dim3(256), 0, st, (const bf16_t*)src, dst, n);
  else hipLaunchKernelGGL(widen_kernel<float>, grid, dim3(256), 0, st, (const float*)src, dst, n);
}

void dropout_apply(int dtype, void* dst, const void* src, bool io_f32, const void* resid, int64_t n, const DropDesc& d,
                   hipStream_t st) {
  if (n <= 0) return;
  dim3 grid((unsigned)(((n + 3) / 4 + 255) / 256));
  if (dtype == BF16 && !io_f32)
    hipLaunchKernelGGL((dropout_kernel<bf16_t, bf16_t>), grid, dim3(256), 0, st, (bf16_t*)dst, (const bf16_t*)src,
                       (const bf16_t*)resid, n, d);
  else if (dtype == BF16)
    hipLaunchKernelGGL((dropout_kernel<float, bf16_t>), grid, dim3(256), 0, st, (float*)dst, (const float*)src,
                       (const bf16_t*)resid, n, d);
  else
    hipLaunchKernelGGL((dropout_kernel<float, float>), grid, dim3(256), 0, st, (float*)dst, (const float*)src,
                       (const float*)resid, n, d);
}

void adamw_update(int lowp_dtype, const AdamTensor* tensors, const AdamChunk* chunks, int n_chunks, AdamHyper h,
                  hipStream_t st) {
  (void)lowp_dtype;                                  // the only low-precision storage type is bf16
  if (n_chunks <= 0) return;
  hipLaunchKernelGGL(adamw_kernel, dim3((unsigned)n_chunks), dim3(256), 0, st, tensors, chunks, h);
}

void fill_zero(void* p, int64_t bytes, hipStream_t st) {
  int64_t n = bytes / 4;
  if (n <= 0) return;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (uint32_t*)p, n);
}

}  // namespace mk
