// bf16 GEMM with a direct global -> LDS pipeline (gfx950 global_load_lds_dwordx4).
//
// C[M,N] = sum_k A(m,k) B(n,k), 128 x 128 x 32 tiles, 4 waves (2 x 2), each wave 64 x 64 as 2 x 2
// MFMA 32x32x16 tiles.  Operand tiles never pass through registers: every lane asks the memory
// pipe to drop 16 bytes straight into LDS, into a ring of three stages (two tiles in flight while
// one is multiplied).  The kernel needs ~140 registers and 48 KB of LDS, so three blocks share a
// CU and fill each other's waits.
//
// A wave-level direct load writes 64 x 16 bytes contiguously, so tiles are stored unpadded and
// bank conflicts are avoided by permuting 16-byte chunks inside a row (the lane -> global
// address map is free, so the permutation costs nothing on the way in):
//   k-major tile [128 rows][32 k], 64 B rows : chunk kc of row r sits at kc ^ ((r >> 2) & 3)
//   m-major tile [32 k][128 rows], 256 B rows: chunk mc of k row q sits at mc ^ (4 * (q & 3))
// k-major fragments are one 16-byte read, m-major fragments two transposing 8-byte reads
// (ds_read_b64_tr_b16).  Elements outside the matrices are fetched from a 16-byte block of
// zeros, so edge tiles need no special loop.
//
// Synchronisation is explicit (no fences): before the barrier of k tile t every wave waits until
// its own loads of tile t have landed (s_waitcnt vmcnt leaves the newer tile in flight); after
// the barrier all waves have also finished reading the stage of tile t-1, which is then refilled
// with tile t+2.  The reduction order over k is fixed by the shape alone.
#include "gemm_device.h"

#include <hip/hip_ext.h>

namespace mk {

namespace {

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int STAGES = 3;
constexpr int TILE_ELEMS = 128 * BK;             // either layout: 8 KB
constexpr int GROUP_M = 4;
constexpr int DMA_PER_WAVE = TILE_ELEMS * 2 / 1024 / 4;   // 1 KB direct loads per wave and operand tile: 2

__device__ __attribute__((aligned(16))) uint32_t g_zero_chunk[4] = {0u, 0u, 0u, 0u};

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

// One wave-level direct load: every lane's 16 bytes at `g` land at lds + 16 * lane.  Written as
// inline assembly so that the compiler does not track it: the ring's waits are placed by hand
// below (the compiler's own tracking drains the whole ring once per turn).
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"      // m0 is a reserved register: named as clobbered on purpose
__device__ __forceinline__ void direct_load(const bf16_t* g, uint32_t lds_byte_address) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_byte_address) : "memory", "m0");
}
#pragma clang diagnostic pop

// s_waitcnt immediate: at most n vector-memory loads outstanding and no LDS operation pending
// (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14)
constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (0 << 8) | ((n >> 4) << 14); }

// Per-thread source of one direct load: where its 16 bytes of k tile 0 live, how far to move
// per k tile, and up to which k tile the address stays inside the matrix.
struct Src {
  const bf16_t* p;     // nullptr-free: points at zeros when the row is outside
  int64_t step;        // elements per k tile (0 for the zero block)
  int k_first;         // reduction index of this chunk in k tile 0 (for the tail test)
};

template <bool KM>
__device__ __forceinline__ Src make_src(const bf16_t* X, int64_t ldx, int R, int r0, int k_begin, int slot) {
  Src s;
  int row, kk;      // row index (m or n) and reduction offset inside the tile of this chunk
  if (KM) {
    const int r = slot >> 2, pc = slot & 3;
    row = r0 + r;
    kk = (pc ^ ((r >> 2) & 3)) * 8;
    s.p = X + (int64_t)row * ldx + k_begin + kk;
    s.step = BK;
  } else {
    const int q = slot >> 4, pc = slot & 15;
    row = r0 + (pc ^ (4 * (q & 3))) * 8;
    kk = q;
    s.p = X + (int64_t)(k_begin + kk) * ldx + row;
    s.step = (int64_t)BK * ldx;
  }
  s.k_first = k_begin + kk;
  if (row >= R) { s.p = (const bf16_t*)g_zero_chunk; s.step = 0; s.k_first = -(1 << 30); }
  return s;
}

// Fragment for tile rows rbase + lane%32, reduction indices 16*ks + 8*(lane/32) .. +7: element
// offset of its first read inside the tile (computed once per thread; the stage base and, for
// the second read of an m-major fragment, a constant are added at the read), then the read.
template <bool KM>
__device__ __forceinline__ int frag_offset(int rbase, int ks, int lane) {
  if (KM) {
    const int r = rbase + (lane & 31);
    const int pc = (2 * ks + (lane >> 5)) ^ ((lane >> 2) & 3);     // (r >> 2) & 3 == (lane >> 2) & 3: rbase % 32 == 0
    return r * BK + pc * 8;
  }
  const int kq = (lane & 15) >> 2;                                  // k row & 3 of this lane's source rows
  const int q = ks * 16 + 8 * (lane >> 5) + kq;
  const int mc = (rbase >> 3) + 2 * ((lane >> 4) & 1) + ((lane & 3) >> 1);
  return q * 128 + (mc ^ (4 * kq)) * 8 + (lane & 1) * 4;
}
template <bool KM>
__device__ __forceinline__ bf16x8 frag_read(const bf16_t* at) {
  if (KM) return *(const bf16x8*)at;
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)at);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(at + 4 * 128));
  typedef short s16x8 __attribute__((ext_vector_type(8)));
  return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// Row sums of the A tile over its reduction indices (the bias gradient riding on a
// weight-gradient product), accumulated per thread over the k tiles and reduced once at the end.
// k-major tile: thread = (row tid/2, half of the 32 indices), one float.
// m-major tile (the layout weight gradients have): a thread owns one 16-byte chunk = 8 consecutive
// rows, for reduction indices tid/16 and tid/16 + 16: two 16-byte reads per tile, eight floats.
template <bool KM>
__device__ __forceinline__ void rowsum_acc(const bf16_t* tile, int tid, float (&rs)[8]) {
  if (KM) {
    const int r = tid >> 1, half = tid & 1;
    const bf16_t* src = &tile[r * BK + half * (BK / 2)];              // chunk order inside a row is immaterial
#pragma unroll
    for (int e = 0; e < BK / 2; ++e) rs[0] += bf16_to_f32(src[e]);
  } else {
    const int c = tid & 15;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int q = (tid >> 4) + 16 * j;
      const bf16x8 v = *(const bf16x8*)&tile[q * 128 + ((c ^ (4 * (q & 3))) * 8)];
#pragma unroll
      for (int e = 0; e < 8; ++e) rs[e] += (float)v[e];
    }
  }
}

}  // namespace

template <bool AK, bool BKM, bool KTAIL>
__global__ __launch_bounds__(256, 3) void bgemm_dma_kernel(GemmDev p, int tiles_n, int total, int per_xcd) {
  // ring of STAGES stages, each an A tile followed by a B tile; the stage of a k tile is chosen at
  // run time, so fragment addresses are a per-thread offset plus the stage base (few registers)
  constexpr int STAGE_ELEMS = 2 * TILE_ELEMS;
  __shared__ __attribute__((aligned(1024))) bf16_t ring[STAGES * STAGE_ELEMS];
  const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (unit >= total) return;
  // units run part by part (all tiles of the first k range, then of the second, ...): an XCD's
  // contiguous run of units then shares one k range of both operands in its L2
  const int n_tiles = total / p.splits;
  const int split = unit / n_tiles, t = unit - split * n_tiles;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int group = t / (GROUP_M * tiles_n), first_m = group * GROUP_M;
  const int gsize = min(tiles_m - first_m, GROUP_M);
  const int in_group = t - group * GROUP_M * tiles_n;
  const int tile_m = first_m + in_group % gsize, tile_n = in_group / gsize;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave-uniform: LDS addresses of the loads stay scalar
  const int wm = wave >> 1, wn = wave & 1;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk_all = (p.K + BK - 1) / BK;
  const int per_split = (nk_all + p.splits - 1) / p.splits;
  const int kt_begin = split * per_split;
  const int nk = max(0, min(nk_all, kt_begin + per_split) - kt_begin);
  const bool do_rowsum = p.a_rowsum && tile_n == 0;
  float rs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // this thread's direct loads: wave w issues loads 2w, 2w+1 of each operand tile, lane = slot
  Src srcA[DMA_PER_WAVE], srcB[DMA_PER_WAVE];
#pragma unroll
  for (int j = 0; j < DMA_PER_WAVE; ++j) {
    const int slot = (wave * DMA_PER_WAVE + j) * 64 + lane;
    srcA[j] = make_src<AK>((const bf16_t*)p.A, p.lda, p.M, m0, kt_begin * BK, slot);
    srcB[j] = make_src<BKM>((const bf16_t*)p.B, p.ldb, p.N, n0, kt_begin * BK, slot);
  }
  // LDS side of a load: byte address of the ring + stage + this wave's share, all scalar, so that
  // issuing a load is an M0 write, the load itself and a pointer increment
  const uint32_t ring_lds = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void*)ring) +
                            (uint32_t)wave * DMA_PER_WAVE * 1024u;
  int k_issue = 0;                                                    // reduction offset of the next tile to issue
  auto issue = [&](int stage_index) {                                 // the next k tile -> ring stage
    const uint32_t a_lds = ring_lds + (uint32_t)stage_index * (STAGE_ELEMS * 2u);
    const uint32_t b_lds = a_lds + TILE_ELEMS * 2u;
#pragma unroll
    for (int j = 0; j < DMA_PER_WAVE; ++j) {
      const bf16_t* ga = srcA[j].p;
      const bf16_t* gb = srcB[j].p;
      if (KTAIL) {                                                    // chunks past K read zeros
        if (srcA[j].k_first + k_issue >= p.K) ga = (const bf16_t*)g_zero_chunk;
        if (srcB[j].k_first + k_issue >= p.K) gb = (const bf16_t*)g_zero_chunk;
      }
      direct_load(ga, a_lds + (uint32_t)j * 1024u);
      direct_load(gb, b_lds + (uint32_t)j * 1024u);
      srcA[j].p += srcA[j].step;
      srcB[j].p += srcB[j].step;
    }
    k_issue += BK;
  };
  // The MFMAs of a tile's second k half are held back until the next tile's first fragments have
  // been requested (after that tile's barrier), so the matrix pipe has work while they travel.
  bf16x8 pa[2], pb[2];                                                // fragments of the pending half
#pragma unroll
  for (int i = 0; i < 2; ++i) { pa[i] = bf16x8{}; pb[i] = bf16x8{}; } // zeros: the first round adds nothing
  auto mfma4 = [&](const bf16x8 (&af)[2], const bf16x8 (&bfr)[2]) {
    // roles swapped (B tile rows feed the MFMA's A side): a lane then owns one output row m
    // and, per register group, four consecutive columns n
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[j], af[i], acc[i][j], 0, 0, 0);
  };
  int a_off[2][2], b_off[2][2];                                       // [k half][32-row block]
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      a_off[ks][i] = frag_offset<AK>(wm * 64 + i * 32, ks, lane);
      b_off[ks][i] = TILE_ELEMS + frag_offset<BKM>(wn * 64 + i * 32, ks, lane);
    }
  auto compute = [&](const bf16_t* stage) {
    static_assert(BK == 32, "two k halves per tile");
    if (do_rowsum) rowsum_acc<AK>(stage, tid, rs);
    __builtin_amdgcn_iglp_opt(0);
    bf16x8 af[2], bfr[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      af[i] = frag_read<AK>(stage + a_off[0][i]);
      bfr[i] = frag_read<BKM>(stage + b_off[0][i]);
    }
    mfma4(pa, pb);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      pa[i] = frag_read<AK>(stage + a_off[1][i]);
      pb[i] = frag_read<BKM>(stage + b_off[1][i]);
    }
    mfma4(af, bfr);
  };
  // One k tile: wait for own loads of tile kt (leaving the newer tile in flight), meet the other
  // waves, refill the stage that was multiplied last, multiply.
  constexpr int PER_TILE = 2 * DMA_PER_WAVE;                          // direct loads per thread and k tile
  static_assert(STAGES == 3, "one newer tile in flight while a tile is multiplied");
  if (nk > 0) {
    issue(0);
    if (nk > 1) issue(1);
    int cur = 0;                                                      // stage of tile kt
    for (int kt = 0; kt < nk; ++kt) {
      if (kt + 1 < nk) __builtin_amdgcn_s_waitcnt(vmcnt_imm(PER_TILE));
      else __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
      __builtin_amdgcn_s_barrier();
      const int fill = cur == 0 ? 2 : cur - 1;                        // stage of tile kt - 1 == stage of tile kt + 2
      if (kt + 2 < nk) issue(fill);
      compute(ring + cur * STAGE_ELEMS);
      cur = cur == 2 ? 0 : cur + 1;
    }
    mfma4(pa, pb);
  }

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
    if (AK) {
      const float tot = rs[0] + __shfl_xor(rs[0], 1, 64);
      const int m = m0 + (tid >> 1);
      if ((tid & 1) == 0 && m < p.M) rowsum[m] = tot;
    } else {
      // sixteen threads hold parts of every row: through the (now dead) ring, summed in a fixed order
      float* red = (float*)ring;                                      // [16 index groups][128 rows]
      __syncthreads();
#pragma unroll
      for (int e = 0; e < 8; ++e) red[(tid >> 4) * 128 + (tid & 15) * 8 + e] = rs[e];
      __syncthreads();
      if (tid < 128) {
        float tot = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) tot += red[g * 128 + tid];
        if (m0 + tid < p.M) rowsum[m0 + tid] = tot;
      }
    }
  }
  static_assert(sizeof(ring) >= 4 * 64 * 32 * sizeof(float), "staging needs 8 KB per wave");
  float* wstage = (float*)ring + wave * 64 * 32;
  store_tile<2>(q, acc, m0 + wm * 64, n0 + wn * 64, lane, wstage);
}

template <bool AK, bool BKM>
static void launch_t(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1) {
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n * p.splits, per = (total + 7) / 8;
  const bool ktail = p.K % BK != 0;
  dim3 grid(per * 8), block(256);
  // t0, t1 (optional): events bound to this kernel's own start and end
  if (ktail) hipExtLaunchKernelGGL((bgemm_dma_kernel<AK, BKM, true>), grid, block, 0, st, t0, t1, 0, p, tiles_n, total, per);
  else hipExtLaunchKernelGGL((bgemm_dma_kernel<AK, BKM, false>), grid, block, 0, st, t0, t1, 0, p, tiles_n, total, per);
}

// Requirements: 16-byte chunks must be wholly inside or wholly outside the matrix along the
// reduction index of a k-major operand (K % 8 == 0), and physically present along the rows of an
// m-major operand (its leading dimension covers the row count rounded up to 8).
bool launch_bgemm_dma(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1) {
  auto up8 = [](int64_t v) { return (v + 7) / 8 * 8; };
  if ((p.a_k || p.b_k) && (p.K & 7)) return false;
  if (!p.a_k && p.lda < up8(p.M)) return false;
  if (!p.b_k && p.ldb < up8(p.N)) return false;
  if (p.a_k && p.b_k) launch_t<true, true>(p, st, t0, t1);
  else if (p.a_k && !p.b_k) launch_t<true, false>(p, st, t0, t1);
  else if (!p.a_k && p.b_k) launch_t<false, true>(p, st, t0, t1);
  else launch_t<false, false>(p, st, t0, t1);
  return true;
}

}  // namespace mk
