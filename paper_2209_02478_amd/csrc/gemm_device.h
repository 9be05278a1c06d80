// Device-side pieces shared by the GEMM kernels: argument block and fused epilogues.
#pragma once
#include "device_common.h"
#include "kernels.h"

namespace mk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));   // native vector: stays in registers


struct GemmDev {
  const void* A; const void* B; void* C;
  const void* bias; const void* resid; void* gelu_out; float* a_rowsum;
  int64_t lda, ldb, ldc, ldr;
  int M, N, K;
  int a_k, b_k, c_f32, gelu;
  int splits;            // > 1: k range cut in `splits` parts, raw fp32 tiles go to `partial`
  float* partial;        // [splits][M][N] followed by [splits][M] row sums
};

template <typename T>
__device__ __forceinline__ void epilogue(const GemmDev& p, int m, int n, float v) {
  if (m >= p.M || n >= p.N) return;
  if (p.bias) v += ld<T>((const T*)p.bias + n);
  if (p.resid) v += ld<T>((const T*)p.resid + (int64_t)m * p.ldr + n);
  int64_t o = (int64_t)m * p.ldc + n;
  if (p.c_f32) {
    ((float*)p.C)[o] = v;
  } else {
    st<T>((T*)p.C + o, v);
    if (p.gelu) st<T>((T*)p.gelu_out + o, p.gelu == GELU_TANH ? gelu_tanh(v) : gelu_erf(v));
  }
}

__device__ __forceinline__ void epilogue4_edge(const GemmDev& p, int m, int n, float v0, float v1, float v2, float v3) {
  epilogue<bf16_t>(p, m, n, v0); epilogue<bf16_t>(p, m, n + 1, v1);
  epilogue<bf16_t>(p, m, n + 2, v2); epilogue<bf16_t>(p, m, n + 3, v3);
}

// epilogue for 4 consecutive columns n..n+3 of row m
template <bool VEC>
__device__ __forceinline__ void epilogue4(const GemmDev& p, int m, int n, float v0, float v1, float v2, float v3) {
  if (m >= p.M || n >= p.N) return;
  if (!VEC || n + 4 > p.N) { epilogue4_edge(p, m, n, v0, v1, v2, v3); return; }
  float v[4] = {v0, v1, v2, v3};
  if (p.bias) {
    const uint2 b = *(const uint2*)((const bf16_t*)p.bias + n);
    v[0] += __uint_as_float(b.x << 16); v[1] += __uint_as_float(b.x & 0xFFFF0000u);
    v[2] += __uint_as_float(b.y << 16); v[3] += __uint_as_float(b.y & 0xFFFF0000u);
  }
  if (p.resid) {
    const uint2 b = *(const uint2*)((const bf16_t*)p.resid + (int64_t)m * p.ldr + n);
    v[0] += __uint_as_float(b.x << 16); v[1] += __uint_as_float(b.x & 0xFFFF0000u);
    v[2] += __uint_as_float(b.y << 16); v[3] += __uint_as_float(b.y & 0xFFFF0000u);
  }
  const int64_t o = (int64_t)m * p.ldc + n;
  if (p.c_f32) {
    *(float4*)((float*)p.C + o) = make_float4(v[0], v[1], v[2], v[3]);
    return;
  }
  uint2 w;
  w.x = pack_bf16x2(v[0], v[1]);
  w.y = pack_bf16x2(v[2], v[3]);
  *(uint2*)((bf16_t*)p.C + o) = w;
  if (p.gelu) {
    float g[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) g[e] = p.gelu == GELU_TANH ? gelu_tanh(v[e]) : gelu_erf_bf16(v[e]);
    w.x = pack_bf16x2(g[0], g[1]);
    w.y = pack_bf16x2(g[2], g[3]);
    *(uint2*)((bf16_t*)p.gelu_out + o) = w;
  }
}

}  // namespace mk
