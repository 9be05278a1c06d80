// GEMM kernels: C[M,N] = sum_k A(m,k) B(n,k) with fused epilogues.
//
// One operand description serves the three products of a linear layer:
//   forward   Y[T,out]  = X[T,in]   W[out,in]^T     A k-major, B k-major
//   dgrad     dX[T,in]  = dY[T,out] W[out,in]       A k-major, B m-major
//   wgrad     dW[out,in]= dY[T,out]^T X[T,in]       A m-major, B m-major
// "k-major": the reduction index is the contiguous one in memory.
//
// bf16: 128x128x64 tiles, 4 waves (2x2), each wave 64x64 as 2x2 MFMA 32x32x16
// tiles with fp32 accumulators, LDS double-buffered through registers.  k-major
// operands are staged [row][k] and read 16 bytes per lane; m-major operands are
// staged as they come, [k][row], and read with the transposing LDS loads of
// gfx950, so no operand is ever transposed in memory or in registers.  The
// reduction order over k is fixed by the shape alone: results are reproducible
// bit for bit.
// fp32: a plain 64x64x16 LDS-tiled kernel (small-model configuration only).
#include "device_common.h"
#include "gemm_device.h"

#include <hip/hip_ext.h>

#include <algorithm>

#include "kernels.h"

namespace mk {

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
constexpr int BM = 128, BN = 128, BK = 64;
constexpr int GROUP_M = 4;                      // row panels per tile group (4-6 measured best in the step, 8 and 1 about 0.5 % behind, 64 3 % behind)
constexpr int NCH = BK / 16;                    // 16-byte chunks per thread and operand tile
constexpr int KCH = BK / 8;                     // chunks along k of a k-major row
constexpr int LDK = BK + 8;        // row stride of a k-major tile [128 rows][64 k] (144 B: conflict-free 16 B reads)
constexpr int LDM = 128 + 32;      // row stride of an m-major tile [64 k][128 rows] (320 B: conflict-free transposing reads)
constexpr int TILE_K_ELEMS = 128 * LDK, TILE_M_ELEMS = BK * LDM;

// One operand tile: global -> registers -> LDS -> MFMA fragments.
//   k-major source (elem(r,k) = X[r*ld+k]) is stored [row][k]; a fragment is one 16-byte read.
//   m-major source (elem(r,k) = X[k*ld+r]) is stored as it comes, [k][row]; a fragment is two
//   transposing 8-byte reads (ds_read_b64_tr_b16: within 16 lanes, lane i receives element i%4
//   of the four lanes 4k + i/4, i.e. a 4(k) x 16(row) block is handed out one row index per lane).
template <bool KM>
struct Tile {
  static constexpr int ELEMS = KM ? TILE_K_ELEMS : TILE_M_ELEMS;

  static __device__ __forceinline__ void addr(int c, int r0, int k0, int& gr, int& gk) {
    const int a = KM ? (c / KCH) : (c >> 4);         // slow index within the tile
    const int f = KM ? (c % KCH) * 8 : (c & 15) * 8; // fast (contiguous) index
    gr = KM ? r0 + a : r0 + f;                       // row (m or n) of the first element
    gk = KM ? k0 + f : k0 + a;                       // reduction index of the first element
  }
  // tile fully inside the matrix: plain 16-byte loads
  static __device__ __forceinline__ void load(u32x4 (&v)[NCH], const bf16_t* __restrict__ X, int64_t ldx, int r0, int k0,
                                              int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int gr, gk;
      addr(tid + i * 256, r0, k0, gr, gk);
      v[i] = *(const u32x4*)(KM ? X + (int64_t)gr * ldx + gk : X + (int64_t)gk * ldx + gr);
    }
  }
  // tile crossing an edge: out-of-range elements read as zero
  struct Regs { u32x4 v[NCH]; };
  static __device__ __forceinline__ Regs load_edge(const bf16_t* __restrict__ X, int64_t ldx, int R, int K, int r0,
                                                int k0, int tid) {
    Regs out;
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      int gr, gk;
      addr(tid + i * 256, r0, k0, gr, gk);
      const bf16_t* src = KM ? X + (int64_t)gr * ldx + gk : X + (int64_t)gk * ldx + gr;
      u32x4 t = {0u, 0u, 0u, 0u};
      const bool slow_ok = KM ? gr < R : gk < K;
      const int fast_pos = KM ? gk : gr, fast_end = KM ? K : R;
      if (slow_ok) {
        if (fast_pos + 8 <= fast_end) {
          t = *(const u32x4*)src;
        } else if (fast_pos < fast_end) {
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const uint32_t e = fast_pos + q < fast_end ? (uint32_t)src[q] : 0u;
            t[q >> 1] |= e << (16 * (q & 1));
          }
        }
      }
      out.v[i] = t;
    }
    return out;
  }
  static __device__ __forceinline__ void store(const u32x4 (&v)[NCH], bf16_t* tile, int tid) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = tid + i * 256;
      if (KM) *(u32x4*)&tile[(c / KCH) * LDK + (c % KCH) * 8] = v[i];
      else *(u32x4*)&tile[(c >> 4) * LDM + (c & 15) * 8] = v[i];
    }
  }
  // fragment for rows rbase + lane%32, reduction indices 16*ks + 8*(lane/32) .. +7
  static __device__ __forceinline__ bf16x8 frag(const bf16_t* tile, int rbase, int ks, int lane) {
    if (KM) return *(const bf16x8*)&tile[(rbase + (lane & 31)) * LDK + ks * 16 + (lane >> 5) * 8];
    const int krow = ks * 16 + 8 * (lane >> 5) + ((lane & 15) >> 2);
    const int col = rbase + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    struct { s16x4 lo, hi; } r;
    r.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)&tile[krow * LDM + col]);
    r.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)&tile[(krow + 4) * LDM + col]);
    return __builtin_bit_cast(bf16x8, r);
  }
  // sum over the tile's 64 reduction indices of row `row` (partial, see caller)
  static __device__ __forceinline__ float rowsum_part(const bf16_t* tile, int tid) {
    float s = 0.f;
    if (KM) {                       // two threads per row, half of the k range each
      const bf16_t* src = &tile[(tid >> 1) * LDK + (tid & 1) * (BK / 2)];
#pragma unroll
      for (int e = 0; e < BK / 2; ++e) s += bf16_to_f32(src[e]);
    } else {                        // two threads per row: lower / upper half of the k rows
      const bf16_t* src = &tile[(tid & 1) * (BK / 2) * LDM + (tid >> 1)];
#pragma unroll
      for (int e = 0; e < BK / 2; ++e) s += bf16_to_f32(src[e * LDM]);
    }
    return s;
  }
};

// k loop of one block.  Global loads run two k tiles ahead of the MFMAs (two register sets), LDS
// holds two tiles, one barrier per k tile.  EDGE: tile crosses a matrix edge or K has a tail.
template <bool AK, bool BKM, bool EDGE>
__device__ __forceinline__ void mainloop(const GemmDev& p, bf16_t* As, bf16_t* Bs, int m0, int n0, int kt_begin, int nk,
                                         int tid, int lane, int wm, int wn, bool do_rowsum, f32x16 (&acc)[2][2],
                                         float& rs) {
  typedef Tile<AK> TA;
  typedef Tile<BKM> TB;
  const bf16_t* A = (const bf16_t*)p.A;
  const bf16_t* B = (const bf16_t*)p.B;
  // two register sets (named, never indexed at run time, so they stay in registers)
  u32x4 ra0[NCH], rb0[NCH], ra1[NCH], rb1[NCH];
  auto fetch = [&](u32x4 (&xa)[NCH], u32x4 (&xb)[NCH], int kt) {      // k tile kt (relative) -> register set
    const int k0 = (kt_begin + kt) * BK;
    if (!EDGE) {
      TA::load(xa, A, p.lda, m0, k0, tid);
      TB::load(xb, B, p.ldb, n0, k0, tid);
    } else {
      const typename TA::Regs ea = TA::load_edge(A, p.lda, p.M, p.K, m0, k0, tid);
      const typename TB::Regs eb = TB::load_edge(B, p.ldb, p.N, p.K, n0, k0, tid);
#pragma unroll
      for (int i = 0; i < NCH; ++i) { xa[i] = ea.v[i]; xb[i] = eb.v[i]; }
    }
  };
  auto stash = [&](const u32x4 (&xa)[NCH], const u32x4 (&xb)[NCH], int buf) {
    TA::store(xa, As + buf * TA::ELEMS, tid);
    TB::store(xb, Bs + buf * TB::ELEMS, tid);
  };
  auto compute = [&](int buf) {
    const bf16_t* at = As + buf * TA::ELEMS;
    const bf16_t* bt = Bs + buf * TB::ELEMS;
    if (do_rowsum) rs += TA::rowsum_part(at, tid);
    __builtin_amdgcn_iglp_opt(0);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[2], bfr[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        af[i] = TA::frag(at, wm * 64 + i * 32, ks, lane);
        bfr[i] = TB::frag(bt, wn * 64 + i * 32, ks, lane);
      }
      // roles swapped (B tile rows feed the MFMA's A side): a lane then owns one output row m
      // and, per register group, four consecutive columns n
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
    }
  };
  if (nk <= 0) return;
  fetch(ra0, rb0, 0);
  stash(ra0, rb0, 0);
  if (nk > 1) fetch(ra1, rb1, 1);
  __syncthreads();
  int kt = 0;
  // steady state: every fetch is unconditional, so the wait before a stash only covers the
  // older register set and the newer loads stay in flight across the MFMAs
  for (; kt + 3 < nk; kt += 2) {
    fetch(ra0, rb0, kt + 2);
    compute(0);
    stash(ra1, rb1, 1);
    __syncthreads();
    fetch(ra1, rb1, kt + 3);
    compute(1);
    stash(ra0, rb0, 0);
    __syncthreads();
  }
  // one to three tiles left: buffer 0 holds tile kt, set 1 holds tile kt+1 (if any)
  if (kt + 2 < nk) fetch(ra0, rb0, kt + 2);
  compute(0);
  if (kt + 1 < nk) {
    stash(ra1, rb1, 1);
    __syncthreads();
    compute(1);
    if (kt + 2 < nk) {
      stash(ra0, rb0, 0);
      __syncthreads();
      compute(0);
    }
  }
}

// Grid: one-dimensional, 8 * ceil(units/8) blocks, a unit being (tile, k split).  Hardware hands
// consecutive block ids to the 8 XCDs in turn, so block id -> (xcd, slot) -> unit xcd*per + slot
// gives every XCD (and its L2) a contiguous run of tiles that share A row panels.
//
// Pipeline: global loads run two k tiles ahead of the MFMAs (two register sets), LDS holds two
// tiles; one barrier per k tile.
template <bool AK, bool BKM>
__global__ __launch_bounds__(256, 2) void bgemm_kernel(GemmDev p, int tiles_n, int total, int per_xcd) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  typedef Tile<AK> TA;
  typedef Tile<BKM> TB;
  bf16_t* As = (bf16_t*)smem_raw;                    // two buffers of TA::ELEMS
  bf16_t* Bs = As + 2 * TA::ELEMS;                   // two buffers of TB::ELEMS
  const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (unit >= total) return;
  // units run part by part (all tiles of the first k range, then of the second, ...): an XCD's
  // contiguous run of units then shares one k range of both operands in its L2
  const int n_tiles = total / p.splits;
  const int split = unit / n_tiles, t = unit - split * n_tiles;
  // tiles run down groups of GROUP_M row panels, so the tiles in flight on one XCD cover a
  // squarish patch of C and share both A and B panels in its L2
  const int tiles_m = (p.M + BM - 1) / BM;
  const int group = t / (GROUP_M * tiles_n), first_m = group * GROUP_M;
  const int gsize = min(tiles_m - first_m, GROUP_M);
  const int in_group = t - group * GROUP_M * tiles_n;
  const int tile_m = first_m + in_group % gsize, tile_n = in_group / gsize;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = tile_m * BM, n0 = tile_n * BN;
  const bf16_t* A = (const bf16_t*)p.A;
  const bf16_t* B = (const bf16_t*)p.B;
  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // this block's k tiles: [kt_begin, kt_begin + nk)
  const int nk_all = (p.K + BK - 1) / BK;
  const int per_split = (nk_all + p.splits - 1) / p.splits;
  const int kt_begin = split * per_split;
  const int nk = max(0, min(nk_all, kt_begin + per_split) - kt_begin);
  const bool do_rowsum = p.a_rowsum && tile_n == 0;
  float rs = 0.f;
  // tiles fully inside the matrices take the loop without any bounds logic
  if (m0 + BM <= p.M && n0 + BN <= p.N && p.K % BK == 0)
    mainloop<AK, BKM, false>(p, As, Bs, m0, n0, kt_begin, nk, tid, lane, wm, wn, do_rowsum, acc, rs);
  else
    mainloop<AK, BKM, true>(p, As, Bs, m0, n0, kt_begin, nk, tid, lane, wm, wn, do_rowsum, acc, rs);

  GemmDev q = p;
  float* rowsum = p.a_rowsum;
  if (p.splits > 1) {
    // raw fp32 tile and row sums of this k range, as a plain matrix [M][N] in the workspace (which
    // is 16-byte aligned); a second kernel adds the parts in order
    q.C = p.partial + (int64_t)split * p.M * p.N;
    q.ldc = p.N; q.c_f32 = 1; q.bias = nullptr; q.resid = nullptr; q.gelu = GELU_NONE;
    q.vec = (p.N & 3) == 0;
    rowsum = p.partial + (int64_t)p.splits * p.M * p.N + (int64_t)split * p.M;
  }
  if (do_rowsum) {
    const float tot = rs + __shfl_xor(rs, 1, 64);
    const int m = m0 + (tid >> 1);
    if ((tid & 1) == 0 && m < p.M) rowsum[m] = tot;
  }
  static_assert(2 * (TA::ELEMS + TB::ELEMS) * sizeof(bf16_t) >= 4 * 64 * 64 * sizeof(float), "staging needs 16 KB per wave");
  store_tile<1>(q, acc, m0 + wm * 64, n0 + wn * 64, lane, (float*)smem_raw + wave * 4096);
}

// C[m][n] = sum over splits (in order) of partial tiles; row sums likewise.  C is fp32, or bf16
// (the sum rounded once) when OUT_BF16.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float* __restrict__ partial, void* __restrict__ Cv,
                                                            int64_t ldc, float* __restrict__ rowsum, int M, int N,
                                                            int splits) {
  const int64_t MN = (int64_t)M * N;
  const int64_t idx = ((int64_t)blockIdx.x * 256 + threadIdx.x) * 4;
  auto put = [&](int64_t o, float v) {
    if (OUT_BF16) ((bf16_t*)Cv)[o] = f32_to_bf16(v); else ((float*)Cv)[o] = v;
  };
  if (idx < MN) {
    const int m = (int)(idx / N), n = (int)(idx - (int64_t)m * N);
    if ((N & 3) == 0) {
      float4 s = *(const float4*)(partial + idx);
      for (int k = 1; k < splits; ++k) {
        const float4 v = *(const float4*)(partial + k * MN + idx);
        s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
      }
      const int64_t o = (int64_t)m * ldc + n;
      if (OUT_BF16 && (ldc & 3) == 0) {
        uint2 w;
        w.x = pack_bf16x2(s.x, s.y); w.y = pack_bf16x2(s.z, s.w);
        *(uint2*)((bf16_t*)Cv + o) = w;
      } else {
        put(o, s.x); put(o + 1, s.y); put(o + 2, s.z); put(o + 3, s.w);
      }
    } else {
      for (int e = 0; e < 4 && idx + e < MN; ++e) {
        const int64_t q = idx + e;
        float s2 = partial[q];
        for (int k = 1; k < splits; ++k) s2 += partial[k * MN + q];
        const int mm = (int)(q / N), nn = (int)(q - (int64_t)mm * N);
        put((int64_t)mm * ldc + nn, s2);
      }
    }
  }
  if (rowsum && idx < M) {       // the first M/4 threads also finish the row sums
    const float* rp = partial + (int64_t)splits * MN;
    for (int e = 0; e < 4 && idx + e < M; ++e) {
      float s2 = rp[idx + e];
      for (int k = 1; k < splits; ++k) s2 += rp[(int64_t)k * M + idx + e];
      rowsum[idx + e] = s2;
    }
  }
}

int gemm_splits(int M, int N) {
  const int tiles = ((M + BM - 1) / BM) * ((N + BN - 1) / BN);
  int s = (256 + tiles - 1) / tiles;
  return s < 1 ? 1 : (s > 8 ? 8 : s);
}

// the kernel with 256 x 256 tiles (gemm_pp.hip) and its tile count
bool launch_bgemm_pp(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1);
int bgemm_pp_tiles(int M, int N);
// Which products go to the large-tile kernel: it runs one block per compute unit, so its time is
// a whole number of rounds of 256 tiles, and it pays where those rounds are well filled.  Measured
// against the 128 x 128 kernels with K = 768 and 2304 or 3072 columns over row counts from 4608
// to 9984 (same box, same run): ahead by 25-34 % when the last round is filled to 0.77 or more,
// by 2-9 % between 0.63 and 0.70, behind by 2-15 % from 0.61 down.  Products that cut their
// reduction in parts stay with the small tiles: with few large output tiles they need more
// parts, and the fp32 parts written and read again cost more than the large tile saves.
static bool use_pp(int M, int N, int K) {
  if (M < 256 || N < 256 || K < 512) return false;
  const int units = bgemm_pp_tiles(M, N), rounds = (units + 255) / 256;
  const double fill = (double)units / (256.0 * rounds);
  return fill >= 0.62;
}

// Data-gradient products with a very long reduction and few output tiles (the head's, whose
// reduction runs over the vocabulary): on the large tiles, the reduction cut in parts so that
// about 200 units exist; with K in the tens of thousands a tile's start and end vanish and the
// parts are small against the operands (T = 6400, K = 30528: 330 us in three parts, 535 us on
// 128 x 128 tiles; T = 2048: 117 against 341 us).  The parts' rows are capped so that the scratch
// is a constant of the model, not a function of the batch.
constexpr int kLongK = 8192;
constexpr int64_t kLongKRows = 24576;            // parts x M at most
size_t gemm_long_k_workspace_bytes(int N) { return (size_t)kLongKRows * N * 4; }
static int long_k_splits(int M, int N) {
  const int tiles = bgemm_pp_tiles(M, N);
  int s = (205 + tiles - 1) / tiles;
  const int cap = (int)(kLongKRows / M);
  if (s > cap) s = cap;
  return s < 1 ? 1 : (s > 8 ? 8 : s);
}

size_t gemm_workspace_bytes(int M, int N) {
  const int s = gemm_splits(M, N);
  return s > 1 ? ((size_t)s * M * N + (size_t)s * M) * 4 : 0;
}

// t1 (optional): event bound to the end of this kernel, which ends the product it belongs to
static void launch_splitk_reduce(const GemmDev& p, hipStream_t st, hipEvent_t t1) {
  const int64_t MN = (int64_t)p.M * p.N;
  const dim3 grid((unsigned)((MN / 4 + 256) / 256));
  if (p.c_f32)
    hipExtLaunchKernelGGL(splitk_reduce_kernel<false>, grid, dim3(256), 0, st, nullptr, t1, 0, p.partial, p.C, p.ldc,
                          p.a_rowsum, p.M, p.N, p.splits);
  else
    hipExtLaunchKernelGGL(splitk_reduce_kernel<true>, grid, dim3(256), 0, st, nullptr, t1, 0, p.partial, p.C, p.ldc,
                          p.a_rowsum, p.M, p.N, p.splits);
}

template <bool AK, bool BKM>
static void launch_bgemm(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1) {
  constexpr int smem = 2 * (Tile<AK>::ELEMS + Tile<BKM>::ELEMS) * 2;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)bgemm_kernel<AK, BKM>, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    configured = true;
  }
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n * p.splits, per = (total + 7) / 8;
  hipExtLaunchKernelGGL((bgemm_kernel<AK, BKM>), dim3(per * 8), dim3(256), smem, st, t0, p.splits > 1 ? nullptr : t1, 0, p,
                        tiles_n, total, per);
  if (p.splits > 1) launch_splitk_reduce(p, st, t1);
}

// direct-to-LDS pipeline (gemm_dma.hip); false when the operands do not meet its alignment rules
bool launch_bgemm_dma(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1);

static bool aligned16(const void* p) { return (((uintptr_t)p) & 15) == 0; }

bool gemm(int dtype, const GemmArgs& g, hipStream_t st) {
  if (g.M <= 0 || g.N <= 0 || g.K <= 0) return true;
  GemmDev p;
  p.A = g.A; p.B = g.B; p.C = g.C; p.bias = g.bias; p.resid = g.resid; p.gelu_out = g.gelu_out; p.a_rowsum = g.a_rowsum;
  p.lda = g.lda; p.ldb = g.ldb; p.ldc = g.ldc; p.ldr = g.ldr;
  p.M = g.M; p.N = g.N; p.K = g.K;
  p.a_k = g.a_kmajor; p.b_k = g.b_kmajor; p.c_f32 = g.c_f32; p.gelu = g.gelu;
  p.splits = 1; p.partial = nullptr;
  p.a_tail_zero = g.a_tail_zero ? 1 : 0;
  if (p.gelu && (p.c_f32 || !p.gelu_out)) return false;
  if (dtype == F32) {
    dim3 grid((g.N + 63) / 64, (g.M + 63) / 64);
    hipExtLaunchKernelGGL(sgemm_kernel, grid, dim3(256), 0, st, g.time_start, g.time_stop, 0, p);
    return true;
  }
  if ((g.lda & 7) || (g.ldb & 7) || !aligned16(g.A) || !aligned16(g.B)) return false;
  const bool may_split = g.workspace && g.c_f32 && !g.bias && !g.resid && !g.gelu && aligned16(g.workspace);
  auto splits_for = [&](int want) {
    const int by_k = (g.K + 255) / 256;                                   // >= 256 reduction indices per part
    const int sp = want < by_k ? want : by_k;
    return may_split && sp > 1 && g.workspace_bytes >= ((size_t)sp * g.M * g.N + (size_t)sp * g.M) * 4 ? sp : 1;
  };
  // vector epilogue: eight consecutive columns (16 bytes of bf16, 32 of fp32) per access
  const bool vec = (g.ldc & (g.c_f32 ? 3 : 7)) == 0 && aligned16(g.C) &&
                   (!g.resid || ((g.ldr & 7) == 0 && aligned16(g.resid))) && (!g.bias || aligned16(g.bias)) &&
                   (!g.gelu_out || aligned16(g.gelu_out));
  p.vec = vec ? 1 : 0;
  // a very long reduction behind a k-major A and an m-major B (the head's data gradient)
  if (g.a_kmajor && !g.b_kmajor && g.K >= kLongK && g.M >= 256 && g.N >= 256 && !g.bias && !g.resid && !g.gelu &&
      !g.a_rowsum && g.M <= kLongKRows) {
    int sp = long_k_splits(g.M, g.N);
    if (sp > 1 && !(g.workspace && aligned16(g.workspace) && g.workspace_bytes >= (size_t)sp * g.M * g.N * 4)) sp = 1;
    p.splits = sp;
    p.partial = sp > 1 ? (float*)g.workspace : nullptr;
    if (launch_bgemm_pp(p, st, g.time_start, sp > 1 ? nullptr : g.time_stop)) {
      if (sp > 1) launch_splitk_reduce(p, st, g.time_stop);
      return true;
    }
    p.splits = 1; p.partial = nullptr;
  }
  // few output tiles and a long reduction (weight gradients): cut k so the whole chip works
  {
    const int sp = splits_for(gemm_splits(g.M, g.N));
    if (sp > 1) { p.splits = sp; p.partial = (float*)g.workspace; }
  }
  // large tiles where their rounds are well filled (a choice made from the shape alone)
  if (p.splits == 1 && use_pp(g.M, g.N, g.K) && launch_bgemm_pp(p, st, g.time_start, g.time_stop)) return true;
  // B m-major (weight gradients, data gradients): the direct-to-LDS pipeline measures faster there;
  // the register-staged kernel below is ahead when both operands are k-major (forward)
  if (!g.b_kmajor && launch_bgemm_dma(p, st, g.time_start, p.splits > 1 ? nullptr : g.time_stop)) {
    if (p.splits > 1) launch_splitk_reduce(p, st, g.time_stop);
    return true;
  }
#define LAUNCH_(AKV, BKV) launch_bgemm<AKV, BKV>(p, st, g.time_start, g.time_stop)
  if (g.a_kmajor && g.b_kmajor) LAUNCH_(true, true);
  else if (g.a_kmajor && !g.b_kmajor) LAUNCH_(true, false);
  else if (!g.a_kmajor && g.b_kmajor) LAUNCH_(false, true);
  else LAUNCH_(false, false);
#undef LAUNCH_
  return true;
}

}  // namespace mk
