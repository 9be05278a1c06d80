// Fused attention, forward and backward, without materialising the L x L matrices.
//
// Wave-per-row kernels in fp32 arithmetic for head sizes 32 and 64 (the fp32 configuration and
// bf16 with head size 32; bf16 with head size 64 runs on the MFMA kernels of attention_mfma.hip).  One wave owns one
// query row (forward, dQ) or one key row (dK/dV): its 64 lanes first each take one
// opposite-side row to form a score, then each take one head-dimension column to
// accumulate the output, with the scores broadcast lane by lane.  Every output element is
// produced by exactly one wave in a fixed order, so results are reproducible bit for bit
// (no atomics, in particular none on dQ).
//
//   forward   O_i = sum_j softmax_j(q_i k_j / sqrt(d)) v_j,   lse_i = log sum_j exp(s_ij)
//   backward  P_ij = exp(s_ij - lse_i), dP_ij = dO_i v_j, dS_ij = P_ij (dP_ij - delta_i),
//             delta_i = dO_i O_i;  dQ = dS K / sqrt(d), dK = dS^T Q / sqrt(d), dV = P^T dO
#include "device_common.h"
#include "kernels.h"
#include "philox.h"

namespace mk {

template <int D>
__device__ __forceinline__ void load_row(const bf16_t* p, float (&r)[D]) {
#pragma unroll
  for (int c = 0; c < D; c += 8) {
    uint4 v = *(const uint4*)(p + c);
    const bf16_t* h = (const bf16_t*)&v;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[c + e] = bf16_to_f32(h[e]);
  }
}
template <int D>
__device__ __forceinline__ void load_row(const float* p, float (&r)[D]) {
#pragma unroll
  for (int c = 0; c < D; c += 4) {
    float4 v = *(const float4*)(p + c);
    r[c] = v.x; r[c + 1] = v.y; r[c + 2] = v.z; r[c + 3] = v.w;
  }
}
template <typename T, int D>
__device__ __forceinline__ float dot_row(const T* p, const float (&q)[D]) {
  float r[D];
  load_row<D>(p, r);
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < D; ++c) s = fmaf(q[c], r[c], s);
  return s;
}

constexpr int kRowsPerBlock = 16;   // 4 waves x 4 rows

// bf16, head size 64: MFMA kernels
void attention_fwd_mfma(const void* qkv, void* ctx, float* lse, const int32_t* lens, int B, int L, int nh, int causal,
                        const DropDesc& drop, hipStream_t st);
void attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse, float* delta, void* dqkv,
                        const int32_t* lens, int B, int L, int nh, int causal, const DropDesc& drop, hipStream_t st);

// qkv row stride is 3*H; head hh of token t: q at t*3H + hh*D, k at +H, v at +2H.
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const T* __restrict__ qkv, T* __restrict__ ctx,
                                                       float* __restrict__ lse, const int32_t* __restrict__ lens,
                                                       int L, int nh, int causal, DropDesc drop) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const float scale = rsqrtf((float)D);
  for (int rr = 0; rr < kRowsPerBlock / 4; ++rr) {
    const int i = blockIdx.x * kRowsPerBlock + wave * (kRowsPerBlock / 4) + rr;
    if (i >= L) break;
    float q[D];
    load_row<D>(base + (int64_t)i * ld3, q);
    const int Lb = lens ? lens[b] : L;                 // keys from Lb on are padding
    const int jmax = min(causal ? i + 1 : L, Lb);
    float m = -INFINITY, l = 0.f, o = 0.f;
    for (int j0 = 0; j0 < jmax; j0 += 64) {
      const int j = j0 + lane;
      float s = -INFINITY;
      if (j < jmax) s = scale * dot_row<T, D>(base + (int64_t)j * ld3 + H, q);
      const float mnew = fmaxf(m, wave_max(s));
      const float p = j < jmax ? expf(s - mnew) : 0.f;
      const float alpha = expf(m - mnew);
      l = l * alpha + wave_sum(p);                  // the normaliser counts every probability
      o *= alpha;
      const float pd = drop.thr && j < jmax && !attn_keep(drop, (int64_t)bh * L + i, (L + 3) >> 2, j) ? 0.f : p;
      const int cnt = min(64, jmax - j0);
      const T* vcol = base + (int64_t)j0 * ld3 + 2 * H + (lane < D ? lane : 0);
      for (int jj = 0; jj < cnt; ++jj) {
        const float pj = __shfl(pd, jj, 64);
        o = fmaf(pj, ld<T>(vcol + (int64_t)jj * ld3), o);
      }
      m = mnew;
    }
    if (lane < D) st<T>(ctx + ((int64_t)b * L + i) * H + hh * D + lane, o * (drop.scale / l));
    if (lane == 0) lse[(int64_t)bh * L + i] = m + logf(l);
  }
}

// delta[b,h,i] = sum_c dO[i,c] * O[i,c]
template <typename T, int D>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ ctx, const T* __restrict__ dctx,
                                                         float* __restrict__ delta, int B, int L, int nh) {
  const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;      // (b, i, hh) fastest hh
  if (idx >= (int64_t)B * L * nh) return;
  const int hh = (int)(idx % nh);
  const int64_t t = idx / nh;
  const int b = (int)(t / L), i = (int)(t - (int64_t)b * L);
  float o[D];
  load_row<D>(ctx + t * nh * D + hh * D, o);
  float s = dot_row<T, D>(dctx + t * nh * D + hh * D, o);
  delta[((int64_t)b * nh + hh) * L + i] = s;
}

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const T* __restrict__ qkv, const T* __restrict__ dctx,
                                                          const float* __restrict__ lse,
                                                          const float* __restrict__ delta, T* __restrict__ dqkv,
                                                          const int32_t* __restrict__ lens, int L, int nh, int causal,
                                                          DropDesc drop) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const float scale = rsqrtf((float)D);
  const int Lb = lens ? lens[b] : L;
  for (int rr = 0; rr < kRowsPerBlock / 4; ++rr) {
    const int i = blockIdx.x * kRowsPerBlock + wave * (kRowsPerBlock / 4) + rr;
    if (i >= L) break;
    float q[D], go[D];
    load_row<D>(base + (int64_t)i * ld3, q);
    load_row<D>(dctx + ((int64_t)b * L + i) * H + hh * D, go);
    const float lse_i = lse[(int64_t)bh * L + i], delta_i = delta[(int64_t)bh * L + i];
    const int jmax = min(causal ? i + 1 : L, Lb);
    float dq = 0.f;
    for (int j0 = 0; j0 < jmax; j0 += 64) {
      const int j = j0 + lane;
      float ds = 0.f;
      if (j < jmax) {
        const float s = scale * dot_row<T, D>(base + (int64_t)j * ld3 + H, q);
        const float p = expf(s - lse_i);
        float dp = dot_row<T, D>(base + (int64_t)j * ld3 + 2 * H, go);
        if (drop.thr) dp = attn_keep(drop, (int64_t)bh * L + i, (L + 3) >> 2, j) ? dp * drop.scale : 0.f;
        ds = p * (dp - delta_i);
      }
      const int cnt = min(64, jmax - j0);
      const T* kcol = base + (int64_t)j0 * ld3 + H + (lane < D ? lane : 0);
      for (int jj = 0; jj < cnt; ++jj) dq = fmaf(__shfl(ds, jj, 64), ld<T>(kcol + (int64_t)jj * ld3), dq);
    }
    if (lane < D) st<T>(dqkv + ((int64_t)b * L + i) * ld3 + hh * D + lane, dq * scale);
  }
}

template <typename T, int D>
__global__ __launch_bounds__(256) void attn_bwd_dkv_kernel(const T* __restrict__ qkv, const T* __restrict__ dctx,
                                                           const float* __restrict__ lse,
                                                           const float* __restrict__ delta, T* __restrict__ dqkv,
                                                           const int32_t* __restrict__ lens, int L, int nh, int causal,
                                                           DropDesc drop) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const T* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const T* gobase = dctx + (int64_t)b * L * H + hh * D;
  const float scale = rsqrtf((float)D);
  for (int rr = 0; rr < kRowsPerBlock / 4; ++rr) {
    const int j = blockIdx.x * kRowsPerBlock + wave * (kRowsPerBlock / 4) + rr;
    if (j >= L) break;
    float k[D], v[D];
    load_row<D>(base + (int64_t)j * ld3 + H, k);
    load_row<D>(base + (int64_t)j * ld3 + 2 * H, v);
    float dk = 0.f, dv = 0.f;
    const int istart = causal ? j : 0;
    const int iend = (lens && j >= lens[b]) ? 0 : L;     // a padded key gets no weight from any query
    for (int i0 = istart; i0 < iend; i0 += 64) {
      const int i = i0 + lane;
      float p = 0.f, ds = 0.f;
      if (i < L) {
        const float s = scale * dot_row<T, D>(base + (int64_t)i * ld3, k);
        p = expf(s - lse[(int64_t)bh * L + i]);
        float dp = dot_row<T, D>(gobase + (int64_t)i * H, v);
        float pd = p;                                   // what multiplied V in the forward
        if (drop.thr) {
          const bool keep = attn_keep(drop, (int64_t)bh * L + i, (L + 3) >> 2, j);
          dp = keep ? dp * drop.scale : 0.f;
          pd = keep ? p * drop.scale : 0.f;
        }
        ds = p * (dp - delta[(int64_t)bh * L + i]);
        p = pd;
      }
      const int cnt = min(64, L - i0);
      const int cl = lane < D ? lane : 0;
      const T* qcol = base + (int64_t)i0 * ld3 + cl;
      const T* gcol = gobase + (int64_t)i0 * H + cl;
      for (int ii = 0; ii < cnt; ++ii) {
        dv = fmaf(__shfl(p, ii, 64), ld<T>(gcol + (int64_t)ii * H), dv);
        dk = fmaf(__shfl(ds, ii, 64), ld<T>(qcol + (int64_t)ii * ld3), dk);
      }
    }
    if (lane < D) {
      T* out = dqkv + ((int64_t)b * L + j) * ld3 + hh * D + lane;
      st<T>(out + H, dk * scale);
      st<T>(out + 2 * H, dv);
    }
  }
}

template <typename T, int D>
static void fwd_t(const void* qkv, void* ctx, float* lse, const int32_t* lens, int B, int L, int nh, int causal,
                  const DropDesc& drop, hipStream_t st) {
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, B * nh);
  hipLaunchKernelGGL((attn_fwd_kernel<T, D>), grid, dim3(256), 0, st, (const T*)qkv, (T*)ctx, lse, lens, L, nh, causal,
                     drop);
}
template <typename T, int D>
static void bwd_t(const void* qkv, const void* ctx, const void* dctx, const float* lse, float* delta, void* dqkv,
                  const int32_t* lens, int B, int L, int nh, int causal, const DropDesc& drop, hipStream_t st) {
  int64_t n = (int64_t)B * L * nh;
  hipLaunchKernelGGL((attn_delta_kernel<T, D>), dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st,
                     (const T*)ctx, (const T*)dctx, delta, B, L, nh);
  dim3 grid((L + kRowsPerBlock - 1) / kRowsPerBlock, B * nh);
  hipLaunchKernelGGL((attn_bwd_dq_kernel<T, D>), grid, dim3(256), 0, st, (const T*)qkv, (const T*)dctx, lse,
                     delta, (T*)dqkv, lens, L, nh, causal, drop);
  hipLaunchKernelGGL((attn_bwd_dkv_kernel<T, D>), grid, dim3(256), 0, st, (const T*)qkv, (const T*)dctx, lse,
                     delta, (T*)dqkv, lens, L, nh, causal, drop);
}

#define DISPATCH_TD(CALL_F32, CALL_BF16)                         \
  if (dtype == BF16) {                                           \
    if (d == 32) { CALL_BF16(32); } else { CALL_BF16(64); } \
  } else {                                                       \
    if (d == 32) { CALL_F32(32); } else { CALL_F32(64); } \
  }

void attention_fwd(int dtype, const void* qkv, void* ctx, float* lse, const int32_t* lens, int B, int L, int nh, int d,
                   int causal, const DropDesc& drop, hipStream_t st) {
  if (B * L <= 0) return;
  if (dtype == BF16 && d == 64) { attention_fwd_mfma(qkv, ctx, lse, lens, B, L, nh, causal, drop, st); return; }
#define F32_(DD) fwd_t<float, DD>(qkv, ctx, lse, lens, B, L, nh, causal, drop, st)
#define BF_(DD) fwd_t<bf16_t, DD>(qkv, ctx, lse, lens, B, L, nh, causal, drop, st)
  DISPATCH_TD(F32_, BF_)
#undef F32_
#undef BF_
}

void attention_bwd(int dtype, const void* qkv, const void* ctx, const void* dctx, const float* lse, float* delta,
                   void* dqkv, const int32_t* lens, int B, int L, int nh, int d, int causal, const DropDesc& drop,
                   hipStream_t st) {
  if (B * L <= 0) return;
  if (dtype == BF16 && d == 64) {        // delta is made inside the dQ kernel
    attention_bwd_mfma(qkv, ctx, dctx, lse, delta, dqkv, lens, B, L, nh, causal, drop, st);
    return;
  }
#define F32_(DD) bwd_t<float, DD>(qkv, ctx, dctx, lse, delta, dqkv, lens, B, L, nh, causal, drop, st)
#define BF_(DD) bwd_t<bf16_t, DD>(qkv, ctx, dctx, lse, delta, dqkv, lens, B, L, nh, causal, drop, st)
  DISPATCH_TD(F32_, BF_)
#undef F32_
#undef BF_
}

}  // namespace mk
