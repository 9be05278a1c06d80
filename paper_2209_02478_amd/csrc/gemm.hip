// GEMM kernels: C[M,N] = sum_k A(m,k) B(n,k) with fused epilogues.
//
// One operand description serves the three products of a linear layer:
//   forward   Y[T,out]  = X[T,in]   W[out,in]^T     A k-major, B k-major
//   dgrad     dX[T,in]  = dY[T,out] W[out,in]       A k-major, B m-major
//   wgrad     dW[out,in]= dY[T,out]^T X[T,in]       A m-major, B m-major
// "k-major": the reduction index is the contiguous one in memory.
//
// bf16: 128x128x32 tiles, 4 waves (2x2), each wave 64x64 as 2x2 MFMA 32x32x16
// tiles with fp32 accumulators.  Both operands are staged in LDS k-contiguous;
// m-major operands are transposed in registers on the way in, so the MFMA inner
// loop is the same for all three products.  The reduction order over k is fixed
// by the shape alone, so results are reproducible bit for bit.
// fp32: a plain 64x64x16 LDS-tiled kernel (small-model configuration only).
#include "device_common.h"
#include "kernels.h"

namespace mk {

struct GemmDev {
  const void* A; const void* B; void* C;
  const void* bias; const void* resid; void* gelu_out; float* a_rowsum;
  int64_t lda, ldb, ldc, ldr;
  int M, N, K;
  int a_k, b_k, c_f32, gelu;
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

// ------------------------------------------------------------------ fp32
__global__ __launch_bounds__(256) void sgemm_kernel(GemmDev p) {
  __shared__ float As[16][68];
  __shared__ float Bs[16][68];
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const float* A = (const float*)p.A;
  const float* B = (const float*)p.B;
  float acc[4][4] = {};
  const bool do_rowsum = p.a_rowsum && blockIdx.x == 0 && tid < 64;
  float rs = 0.f;
  for (int k0 = 0; k0 < p.K; k0 += 16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      int idx = tid + i * 256;
      int r, k;
      if (p.a_k) { r = idx >> 4; k = idx & 15; } else { r = idx & 63; k = idx >> 6; }
      int gm = m0 + r, gk = k0 + k;
      float v = 0.f;
      if (gm < p.M && gk < p.K) v = p.a_k ? A[(int64_t)gm * p.lda + gk] : A[(int64_t)gk * p.lda + gm];
      As[k][r] = v;
      if (p.b_k) { r = idx >> 4; k = idx & 15; } else { r = idx & 63; k = idx >> 6; }
      int gn = n0 + r;
      gk = k0 + k;
      v = 0.f;
      if (gn < p.N && gk < p.K) v = p.b_k ? B[(int64_t)gn * p.ldb + gk] : B[(int64_t)gk * p.ldb + gn];
      Bs[k][r] = v;
    }
    __syncthreads();
    if (do_rowsum)
#pragma unroll
      for (int k = 0; k < 16; ++k) rs += As[k][tid];
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) { a[i] = As[k][ty * 4 + i]; b[i] = Bs[k][tx * 4 + i]; }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) epilogue<float>(p, m0 + ty * 4 + i, n0 + tx * 4 + j, acc[i][j]);
  if (do_rowsum && m0 + tid < p.M) p.a_rowsum[m0 + tid] = rs;
}

// ------------------------------------------------------------------ bf16 MFMA
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int BM = 128, BN = 128, BK = 32, LDSK = BK + 8;

// Stage registers for one operand tile (128 rows x 32 k).
struct Stage { uint4 v[4]; };

// k-major source: elem(r,k) = X[r*ld + k]; two 16-byte chunks per thread.
__device__ __forceinline__ void load_kmajor(Stage& s, const bf16_t* X, int64_t ldx, int R, int K,
                                            int r0, int k0, int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = tid + i * 256;
    int gr = r0 + (c >> 2), gk = k0 + (c & 3) * 8;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (gr < R) {
      const bf16_t* src = X + (int64_t)gr * ldx + gk;
      if (gk + 8 <= K) {
        v = *(const uint4*)src;
      } else if (gk < K) {
        bf16_t t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = (gk + e < K) ? src[e] : (bf16_t)0;
        v = *(uint4*)t;
      }
    }
    s.v[i] = v;
  }
}
__device__ __forceinline__ void store_kmajor(const Stage& s, bf16_t (*tile)[LDSK], int tid) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    int c = tid + i * 256;
    *(uint4*)&tile[c >> 2][(c & 3) * 8] = s.v[i];
  }
}

// m-major source: elem(r,k) = X[k*ld + r]; threads 0..127 each take a 4(k) x 8(r) block.
__device__ __forceinline__ void load_mmajor(Stage& s, const bf16_t* X, int64_t ldx, int R, int K,
                                            int r0, int k0, int tid) {
  if (tid >= 128) return;
  int kq = tid >> 4, rb = tid & 15;
  int gr = r0 + rb * 8;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int gk = k0 + kq * 4 + j;
    uint4 v = make_uint4(0, 0, 0, 0);
    if (gk < K) {
      const bf16_t* src = X + (int64_t)gk * ldx + gr;
      if (gr + 8 <= R) {
        v = *(const uint4*)src;
      } else if (gr < R) {
        bf16_t t[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) t[e] = (gr + e < R) ? src[e] : (bf16_t)0;
        v = *(uint4*)t;
      }
    }
    s.v[j] = v;
  }
}
__device__ __forceinline__ uint32_t pick(const uint4& v, int d) {
  return d == 0 ? v.x : d == 1 ? v.y : d == 2 ? v.z : v.w;
}
__device__ __forceinline__ void store_mmajor(const Stage& s, bf16_t (*tile)[LDSK], int tid) {
  if (tid >= 128) return;
  int kq = tid >> 4, rb = tid & 15;
#pragma unroll
  for (int mm = 0; mm < 8; ++mm) {
    const int d = mm >> 1;
    uint32_t a0 = pick(s.v[0], d), a1 = pick(s.v[1], d), a2 = pick(s.v[2], d), a3 = pick(s.v[3], d);
    uint2 o;
    if (mm & 1) {
      o.x = (a0 >> 16) | (a1 & 0xFFFF0000u);
      o.y = (a2 >> 16) | (a3 & 0xFFFF0000u);
    } else {
      o.x = (a0 & 0xFFFFu) | (a1 << 16);
      o.y = (a2 & 0xFFFFu) | (a3 << 16);
    }
    *(uint2*)&tile[rb * 8 + mm][kq * 4] = o;
  }
}

template <bool AK, bool BKM>
__global__ __launch_bounds__(256) void bgemm_kernel(GemmDev p) {
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM][LDSK];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN][LDSK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const bf16_t* A = (const bf16_t*)p.A;
  const bf16_t* B = (const bf16_t*)p.B;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  Stage sa, sb;
  const int nk = (p.K + BK - 1) / BK;
  // bias gradient: blocks of the first column tile also sum their A rows (2 threads per row)
  const bool do_rowsum = p.a_rowsum && blockIdx.x == 0;
  float rs = 0.f;
  if (AK) load_kmajor(sa, A, p.lda, p.M, p.K, m0, 0, tid); else load_mmajor(sa, A, p.lda, p.M, p.K, m0, 0, tid);
  if (BKM) load_kmajor(sb, B, p.ldb, p.N, p.K, n0, 0, tid); else load_mmajor(sb, B, p.ldb, p.N, p.K, n0, 0, tid);
  if (AK) store_kmajor(sa, As[0], tid); else store_mmajor(sa, As[0], tid);
  if (BKM) store_kmajor(sb, Bs[0], tid); else store_mmajor(sb, Bs[0], tid);
  __syncthreads();

  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < nk;
    if (more) {
      const int k0 = (kt + 1) * BK;
      if (AK) load_kmajor(sa, A, p.lda, p.M, p.K, m0, k0, tid); else load_mmajor(sa, A, p.lda, p.M, p.K, m0, k0, tid);
      if (BKM) load_kmajor(sb, B, p.ldb, p.N, p.K, n0, k0, tid); else load_mmajor(sb, B, p.ldb, p.N, p.K, n0, k0, tid);
    }
    if (do_rowsum) {
      const bf16_t* src = &As[cur][tid >> 1][(tid & 1) * 16];
#pragma unroll
      for (int e = 0; e < 16; ++e) rs += bf16_to_f32(src[e]);
    }
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[2], bfr[2];
      const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = *(const bf16x8*)&As[cur][wm * 64 + i * 32 + (lane & 31)][kk];
        bfr[i] = *(const bf16x8*)&Bs[cur][wn * 64 + i * 32 + (lane & 31)][kk];
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (more) {
      if (AK) store_kmajor(sa, As[cur ^ 1], tid); else store_mmajor(sa, As[cur ^ 1], tid);
      if (BKM) store_kmajor(sb, Bs[cur ^ 1], tid); else store_mmajor(sb, Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  if (do_rowsum) {
    float tot = rs + __shfl_xor(rs, 1, 64);
    int m = m0 + (tid >> 1);
    if ((tid & 1) == 0 && m < p.M) p.a_rowsum[m] = tot;
  }
  // accumulator layout of the 32x32 MFMA: lane%32 is the column, register r holds
  // row 8*(r/4) + 4*(lane/32) + r%4
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        int m = m0 + wm * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        int n = n0 + wn * 64 + j * 32 + (lane & 31);
        epilogue<bf16_t>(p, m, n, acc[i][j][r]);
      }
}

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

bool gemm(int dtype, const GemmArgs& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return true;
  GemmDev p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.bias = g.bias; p.resid = g.resid; p.gelu_out = g.gelu_out; p.a_rowsum = g.a_rowsum;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldr = g.ldr;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.a_k = g.a_kmajor; p.b_k = g.b_kmajor; p.c_f32 = g.c_f32; p.gelu = g.gelu;
  if (p.gelu && (p.c_f32 || !p.gelu_out)) return false;
  if (dtype == F32) {
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
    hipLaunchKernelGGL(sgemm_kernel, grid, dim3(256), 0, st, p);
    return true;
  }
  if ((g.lda & 7) || (g.ldb & 7) || !aligned16(g.A) || !aligned16(g.B)) return false;
  dim3 grid((g.N + BN - 1) / BN, (g.M + BM - 1) / BM);
  if (g.a_kmajor && g.b_kmajor) hipLaunchKernelGGL((bgemm_kernel<true, true>), grid, dim3(256), 0, st, p);
  else if (g.a_kmajor && !g.b_kmajor) hipLaunchKernelGGL((bgemm_kernel<true, false>), grid, dim3(256), 0, st, p);
  else if (!g.a_kmajor && g.b_kmajor) hipLaunchKernelGGL((bgemm_kernel<false, true>), grid, dim3(256), 0, st, p);
  else hipLaunchKernelGGL((bgemm_kernel<false, false>), grid, dim3(256), 0, st, p);
  return true;
}

}  // namespace mk
