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
  int vec;               // C, bias, residual and GELU output allow 16-byte accesses at columns n % 8 == 0
  int a_tail_zero;       // A k-major, K % 8 != 0: the columns up to the next multiple of 8 exist and are zero
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

// ---- block tile -> C for the bf16 kernels -----------------------------------------------------
// A 128 x 128 block tile held by 4 waves (wave (wm, wn): rows wm*64.., columns wn*64..) as 2 x 2
// MFMA 32x32 accumulators with the operand roles swapped: accumulator (i, j), register r of a
// lane is row i*32 + lane%32, column j*32 + 8*(r/4) + 4*(lane/32) + r%4 of the wave's 64 x 64.
//
// In that layout a store instruction would touch 32 rows with 16 bytes each.  The tile is turned
// through LDS instead (the operand tiles are dead by then): every wave parks its 64 x 64 floats in
// 16 KB of its own, then walks them 8 rows at a time, 8 lanes per row with 8 consecutive columns
// each, so bias / residual loads and the C / GELU stores are whole 128-byte lines.  The walk is a
// rolled loop, which also keeps the kernel's code small.  Float4 chunk c of row r sits at chunk
// position c ^ (r & 15): conflict-free for the accumulator writes (16 rows, one chunk) and for
// the row reads (two rows, all even or all odd chunks).

__device__ __forceinline__ void unpack_bf16x8(const u32x4 w, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = __uint_as_float(w[e] << 16);
    f[2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
  }
}
__device__ __forceinline__ u32x4 pack_bf16x8(const float (&f)[8]) {
  u32x4 w;
#pragma unroll
  for (int e = 0; e < 4; ++e) w[e] = pack_bf16x2(f[2 * e], f[2 * e + 1]);
  return w;
}

// m0w, n0w: first row / column of this wave's 64 x 64 part; wstage: 16 KB / HALVES of LDS owned
// by this wave (HALVES == 2: the two 32-column halves take turns in 8 KB).  Every thread of the
// block must call it.
template <int HALVES>
__device__ __forceinline__ void store_tile(const GemmDev& p, const f32x16 (&acc)[2][2], int m0w, int n0w, int lane,
                                           float* wstage) {
  constexpr int COLS = 64 / HALVES, CHUNKS = COLS / 4, LPR = COLS / 8;   // staged columns, float4 chunks, lanes per row
  constexpr int RPI = 64 / LPR;                                          // rows per loop iteration
#pragma unroll
  for (int h = 0; h < HALVES; ++h) {
    __syncthreads();                                            // operand tiles / the previous half are dead
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int jj = 0; jj < 2 / HALVES; ++jj)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int j = HALVES == 2 ? h : jj;
          const int row = i * 32 + (lane & 31), c = jj * 8 + 2 * g + (lane >> 5);
          *(float4*)&wstage[row * COLS + ((c ^ (row & (CHUNKS - 1))) << 2)] =
              make_float4(acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2], acc[i][j][4 * g + 3]);
        }
    __syncthreads();
    const int nh = n0w + h * COLS;
    if (!p.vec) {                                               // unaligned operands: one element at a time
      for (int idx = lane; idx < 64 * COLS; idx += 64) {
        const int row = idx / COLS, col = idx % COLS;
        epilogue<bf16_t>(p, m0w + row, nh + col,
                         wstage[row * COLS + ((((col >> 2) ^ (row & (CHUNKS - 1))) << 2) | (col & 3))]);
      }
      continue;
    }
    const int n = nh + (lane % LPR) * 8, c0 = 2 * (lane % LPR);
    for (int it = 0; it < 64 / RPI; ++it) {
      const int row = it * RPI + lane / LPR, m = m0w + row;
      if (m >= p.M || n >= p.N) continue;
      const float4 lo = *(const float4*)&wstage[row * COLS + ((c0 ^ (row & (CHUNKS - 1))) << 2)];
      const float4 hi = *(const float4*)&wstage[row * COLS + (((c0 + 1) ^ (row & (CHUNKS - 1))) << 2)];
      float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
      if (n + 8 > p.N) {                                        // ragged end of the row
        for (int e = 0; e < 8; ++e) epilogue<bf16_t>(p, m, n + e, v[e]);
        continue;
      }
      float f[8];
      if (p.bias) {
        unpack_bf16x8(*(const u32x4*)((const bf16_t*)p.bias + n), f);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += f[e];
      }
      if (p.resid) {
        unpack_bf16x8(*(const u32x4*)((const bf16_t*)p.resid + (int64_t)m * p.ldr + n), f);
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] += f[e];
      }
      const int64_t o = (int64_t)m * p.ldc + n;
      if (p.c_f32) {
        *(float4*)((float*)p.C + o) = make_float4(v[0], v[1], v[2], v[3]);
        *(float4*)((float*)p.C + o + 4) = make_float4(v[4], v[5], v[6], v[7]);
        continue;
      }
      *(u32x4*)((bf16_t*)p.C + o) = pack_bf16x8(v);
      if (p.gelu == GELU_ERF) {
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = gelu_erf_bf16(v[e]);
        *(u32x4*)((bf16_t*)p.gelu_out + o) = pack_bf16x8(f);
      } else if (p.gelu == GELU_TANH) {
#pragma unroll
        for (int e = 0; e < 8; ++e) f[e] = gelu_tanh_bf16(v[e]);
        *(u32x4*)((bf16_t*)p.gelu_out + o) = pack_bf16x8(f);
      }
    }
  }
}

}  // namespace mk
