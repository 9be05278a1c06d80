// bf16 GEMM, large block tiles, two wave groups taking turns ("ping-pong").
//
// C[M,N] = sum_k A(m,k) B(n,k).  One block of 8 waves per compute unit owns a BM x BN tile of C
// (256 x 256 in the main variant) and walks the reduction in steps of 64.  Why this shape on
// gfx950: a compute unit draws at most 64 bytes per clock from the L2, and a 128 x 128 tile needs
// exactly that at full matrix rate, so the tile has to be larger for the matrix pipes to be the
// limit; 256 x 256 needs 32.  The wave tile (128 x 64) halves the LDS bytes read per MFMA as well.
//
// Operand tiles go global -> LDS directly (global_load_lds_dwordx4) into a ring of NA slots for A
// tiles and NB slots for B tiles (256 x 256: 3 + 2 slots of 32 KB, the whole 160 KB of LDS).
// The eight waves form two groups of four (waves w and w + 4 share a SIMD).  Time is cut into
// intervals by s_barrier; in every interval one group reads MFMA fragments from LDS (and does
// nothing else that needs the matrix pipe) while the other issues the 16 MFMAs of half a k tile
// at raised priority, then they swap.  Each SIMD therefore always has one wave feeding its matrix
// pipe while the LDS latency of the other is hidden behind it.  Group 1 runs one interval behind
// group 0.  Interval n, k tile t, half h:
//     group 0:  fragments(t,h) at n = 4t+2h,    MFMAs(t,h) at n = 4t+2h+1
//     group 1:  fragments(t,h) at n = 4t+2h+1,  MFMAs(t,h) at n = 4t+2h+2
// The slot of tile t-1 is last read in interval 4t-1, so while it multiplies tile t every wave
// issues its share of B tile t+NB-1 and then of A tile t+NA-1, one load at a time between the
// MFMAs (a burst of loads blocks the wave until the memory pipe has accepted all of it; the
// fragment intervals carry no loads, so they stay shorter than the MFMA intervals), and at the
// end of interval 4t+3 it waits (vmcnt, loads complete in order) until tile t+1 has landed,
// leaving the newer tile in flight.  A miss in the L2 costs more than a microsecond here and a k tile of MFMAs about one, so
// the operand that streams from memory (A: activations, gradients) is requested two tiles ahead;
// B (weights in two of the three products) comes from the L2 and one tile ahead is enough.
//
// LDS layouts (16-byte chunks permuted so that fragment reads are conflict-free although a
// direct load can only write 1 KB contiguously):
//   k-major tile [rows][64 k], 128-byte rows : chunk kc of row r sits at kc ^ ((r >> 1) & 7)
//   m-major tile [64 k][rows]               : chunk mc of k row q sits at mc ^ (4 * (q & 3))
// k-major fragments are one 16-byte read, m-major fragments two transposing 8-byte reads.
// The reduction order over k is fixed by the shape alone (results reproducible bit for bit).
#include "gemm_device.h"

#include <hip/hip_ext.h>

namespace mk {

namespace {

constexpr int PBK = 64;                          // reduction indices per stage
constexpr int PGROUP_M = 4;                      // row panels per tile group (L2 reuse)

__device__ __attribute__((aligned(16))) uint32_t g_zero16[4] = {0u, 0u, 0u, 0u};

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4_t;

// One wave-level direct load: lane i's 16 bytes at g land at lds + 16 * i.  Inline assembly, so
// the compiler does not track it: the waits are placed by hand in the loop.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"      // m0 is a reserved register: named as clobbered on purpose
__device__ __forceinline__ void pp_direct_load(const bf16_t* g, uint32_t lds_byte_address) {
  asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(g), "s"(lds_byte_address) : "memory", "m0");
}
// LDS byte address of a pointer into the block's shared memory, as a wave-uniform scalar
__device__ __forceinline__ uint32_t pp_lds_address(const void* p) {
  return __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)(lds_void_t*)p);
}
#pragma clang diagnostic pop

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] << 14)
constexpr int kWaitLds = 15 | (7 << 4) | (0 << 8) | (3 << 14);      // LDS operations done, vector memory untouched
constexpr int wait_vmem(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }   // at most n loads in flight

__device__ __forceinline__ void pp_barrier() {
  // nothing may be scheduled across: the intervals are the synchronisation
  __builtin_amdgcn_sched_barrier(0);
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
  __builtin_amdgcn_sched_barrier(0);
}

// Geometry of one variant: WM x WN waves (WM * WN == 8), each wave TM x TN MFMA tiles of 32 x 32.
template <int WM, int WN, int TM, int TN, int NA, int NB>
struct Geo {
  static_assert(WM * WN == 8, "eight waves");
  static_assert((NA == 2 || NA == 3) && (NB == 2 || NB == 3) && NB <= NA, "ring depths");
  static_assert(TM % 2 == 0 && TN % 2 == 0, "the tile store works on 64 x 64 pieces");
  static constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  static constexpr int A_ELEMS = BM * PBK, B_ELEMS = BN * PBK;
  static constexpr int A_LOADS = BM / 64, B_LOADS = BN / 64;     // 1 KB direct loads per wave and k tile
  static constexpr int SMEM = (NA * A_ELEMS + NB * B_ELEMS) * 2;  // bytes
  // loads a wave may leave in flight when it needs tile t+1: those of tiles t+2 issued after it
  static constexpr int AHEAD = (NA == 3 ? A_LOADS : 0) + (NB == 3 ? B_LOADS : 0);
};

// Source of direct load number j (of R / 8) of a tile with R rows whose first row is r0, for k
// tile 0 of this block: address of the lane's 16 bytes and the chunk's reduction offset in the tile.
template <bool KM, int R>
__device__ __forceinline__ const bf16_t* pp_src(const bf16_t* X, int64_t ldx, int rows_total, int r0, int k_begin,
                                                int j, int lane, int& k_in_tile) {
  if (KM) {
    const int r = 8 * j + (lane >> 3), pc = lane & 7;
    const int kc = pc ^ ((r >> 1) & 7);
    int row = r0 + r;
    if (row >= rows_total) row = r0;                 // rows outside the matrix: any valid row (never stored)
    k_in_tile = kc * 8;
    return X + (int64_t)row * ldx + k_begin + kc * 8;
  }
  constexpr int RC = R / 8;                          // chunks per k row
  const int q = j * (64 / RC) + lane / RC, pos = lane % RC;
  const int mc = pos ^ (4 * (q & 3));
  int row = r0 + mc * 8;
  if (row >= rows_total) row = r0;
  k_in_tile = q;
  return X + (int64_t)(k_begin + q) * ldx + row;
}

// Per-lane fragment offsets (elements inside the tile).  k-major: one per 16-deep k step, the
// 32-row block is an immediate; m-major: one per 32-row block, the k step is an immediate.
template <bool KM, int R, int T>
struct FragOff {
  int v[4];
  __device__ __forceinline__ void init(int first_block, int lane) {
    if (KM) {
      const int sw = (lane >> 1) & 7, hi = lane >> 5;
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) v[ks] = (first_block * 32 + (lane & 31)) * PBK + (((2 * ks + hi) ^ sw) << 3);
    } else {
      const int kq = (lane & 15) >> 2;
      const int lane_base = (8 * (lane >> 5) + kq) * R + (lane & 1) * 4 + (2 * ((lane >> 4) & 1) + ((lane & 3) >> 1)) * 8;
#pragma unroll
      for (int i = 0; i < 4; ++i) v[i] = lane_base + (((4 * (first_block + i)) ^ (4 * kq)) << 3);
    }
  }
  // fragment of 32-row block i (of this wave), k step ks (both compile-time after unrolling)
  __device__ __forceinline__ bf16x8 read(const bf16_t* tile, int i, int ks) const {
    if (KM) return *(const bf16x8*)(tile + v[ks] + i * 32 * PBK);
    const bf16_t* at = tile + v[i] + ks * 16 * R;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)at);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t*)(at + 4 * R));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
};

}  // namespace

template <bool AK, bool BKM, bool KTAIL, int WM, int WN, int TM, int TN, int NA, int NB>
__global__ __launch_bounds__(512) void bgemm_pp_kernel(GemmDev p, int tiles_n, int total, int per_xcd) {
  typedef Geo<WM, WN, TM, TN, NA, NB> G;
  constexpr int BM = G::BM, BN = G::BN;
  extern __shared__ __attribute__((aligned(1024))) unsigned char pp_smem[];
  bf16_t* ring = (bf16_t*)pp_smem;
  const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (unit >= total) return;
  // units run part by part (all tiles of the first k range, then of the second, ...): an XCD's
  // contiguous run of units then shares one k range of both operands in its L2
  const int n_tiles = total / p.splits;
  const int split = unit / n_tiles, t = unit - split * n_tiles;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int group = t / (PGROUP_M * tiles_n), first_m = group * PGROUP_M;
  const int gsize = min(tiles_m - first_m, PGROUP_M);
  const int in_group = t - group * PGROUP_M * tiles_n;
  const int tile_m = first_m + in_group % gsize, tile_n = in_group / gsize;
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform: address arithmetic on it stays scalar
  const int grp = wave >> 2;                          // ping-pong group: waves w and w + 4 share a SIMD
  const int wm = wave / WN, wn = wave % WN;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  f32x16 acc[TM / 2][TN / 2][2][2];                   // [64-row piece][64-column piece][32-row block][32-column block]
#pragma unroll
  for (int a = 0; a < TM / 2; ++a)
#pragma unroll
    for (int b = 0; b < TN / 2; ++b)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[a][b][i][j][r] = 0.f;

  const int nk_all = (p.K + PBK - 1) / PBK;
  const int per_split = (nk_all + p.splits - 1) / p.splits;
  const int kt_begin = split * per_split;
  const int nk = max(0, min(nk_all, kt_begin + per_split) - kt_begin);
  const bool do_rowsum = p.a_rowsum && tile_n == 0;   // A m-major only (the launcher sees to it)
  float rs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // this thread's direct loads
  const bf16_t* pa[G::A_LOADS];
  const bf16_t* pb[G::B_LOADS];
  int ka[G::A_LOADS], kb[G::B_LOADS];
#pragma unroll
  for (int jj = 0; jj < G::A_LOADS; ++jj)
    pa[jj] = pp_src<AK, BM>((const bf16_t*)p.A, p.lda, p.M, m0, kt_begin * PBK, wave * G::A_LOADS + jj, lane, ka[jj]);
#pragma unroll
  for (int jj = 0; jj < G::B_LOADS; ++jj)
    pb[jj] = pp_src<BKM, BN>((const bf16_t*)p.B, p.ldb, p.N, n0, kt_begin * PBK, wave * G::B_LOADS + jj, lane, kb[jj]);
  const int64_t step_a = AK ? PBK : (int64_t)PBK * p.lda, step_b = BKM ? PBK : (int64_t)PBK * p.ldb;
  bf16_t* const ring_b = ring + NA * G::A_ELEMS;
  // the next tile to request of each operand: its first reduction index and its slot
  int ka_next = kt_begin * PBK, kb_next = kt_begin * PBK, slot_a_next = 0, slot_b_next = 0;
  // one direct load of the next A (B) tile, and the bookkeeping once all of a tile's are out
  // (the LDS side is scalar arithmetic on byte addresses: slot base + this wave's share)
  const uint32_t lds_a0 = pp_lds_address(ring) + (uint32_t)wave * G::A_LOADS * 1024u;
  const uint32_t lds_b0 = pp_lds_address(ring_b) + (uint32_t)wave * G::B_LOADS * 1024u;
  auto load_a = [&](int jj) {
    const bf16_t* ga = pa[jj];
    if (KTAIL && ka_next + ka[jj] >= p.K) ga = (const bf16_t*)g_zero16;        // chunks past K read zeros
    pp_direct_load(ga, lds_a0 + (uint32_t)slot_a_next * (G::A_ELEMS * 2u) + (uint32_t)jj * 1024u);
    pa[jj] += step_a;
  };
  auto done_a = [&]() {
    ka_next += PBK;
    slot_a_next = slot_a_next == NA - 1 ? 0 : slot_a_next + 1;
  };
  auto load_b = [&](int jj) {
    const bf16_t* gb = pb[jj];
    if (KTAIL && kb_next + kb[jj] >= p.K) gb = (const bf16_t*)g_zero16;
    pp_direct_load(gb, lds_b0 + (uint32_t)slot_b_next * (G::B_ELEMS * 2u) + (uint32_t)jj * 1024u);
    pb[jj] += step_b;
  };
  auto done_b = [&]() {
    kb_next += PBK;
    slot_b_next = slot_b_next == NB - 1 ? 0 : slot_b_next + 1;
  };
  auto issue_a = [&]() {
#pragma unroll
    for (int jj = 0; jj < G::A_LOADS; ++jj) load_a(jj);
    done_a();
  };
  auto issue_b = [&]() {
#pragma unroll
    for (int jj = 0; jj < G::B_LOADS; ++jj) load_b(jj);
    done_b();
  };
  // end of interval 4t+3 (and of the prologue, t = -1): tile t+1 has landed
  auto wait_tile = [&](int t_) {
    if (G::AHEAD > 0 && t_ + 2 < nk) __builtin_amdgcn_s_waitcnt(wait_vmem(G::AHEAD));
    else __builtin_amdgcn_s_waitcnt(wait_vmem(0));
  };

  FragOff<AK, BM, TM> fa;
  FragOff<BKM, BN, TN> fb;
  fa.init(wm * TM, lane);
  fb.init(wn * TN, lane);
  bf16x8 af[2][TM], bfr[2][TN];                       // fragments of half a k tile
  int slot_a = 0, slot_b = 0;                         // slots of the tile being multiplied
  auto next_tile = [&]() {
    slot_a = slot_a == NA - 1 ? 0 : slot_a + 1;
    slot_b = slot_b == NB - 1 ? 0 : slot_b + 1;
  };
  auto fragments = [&](int h) {
    const bf16_t* sa = ring + slot_a * G::A_ELEMS;
    const bf16_t* sb = ring_b + slot_b * G::B_ELEMS;
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
#pragma unroll
      for (int i = 0; i < TM; ++i) af[s2][i] = fa.read(sa, i, 2 * h + s2);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[s2][j] = fb.read(sb, j, 2 * h + s2);
    }
  };
  // row sums of the A tile (bias gradient riding on a weight-gradient product): a thread owns one
  // chunk position, i.e. 8 consecutive rows, and every (512 / (BM/8))-th k row
  auto rowsum_acc = [&]() {
    constexpr int RC = BM / 8, QSTEP = 512 / RC;
    const bf16_t* sa = ring + slot_a * G::A_ELEMS;
#pragma unroll
    for (int jj = 0; jj < PBK / QSTEP; ++jj) {
      const int q = tid / RC + QSTEP * jj;
      const bf16x8 v = *(const bf16x8*)(sa + q * BM + (tid % RC) * 8);
#pragma unroll
      for (int e = 0; e < 8; ++e) rs[e] += (float)v[e];
    }
  };
  // The 2 * TM * TN MFMAs of half a k tile.  which = 1 (2): the loads of the next B (A) tile are
  // issued between them, evenly spaced, so that the memory pipe takes them one at a time and the
  // matrix pipe never waits for a burst of loads to be accepted (the LDS side of a load is scalar
  // arithmetic, so issuing one is an M0 write, the load and a pointer increment; measured against
  // issuing them behind the fragment reads instead: 3 % ahead).
  auto mfmas = [&](int which, bool go) {
    constexpr int NM = 2 * TM * TN;
    __builtin_amdgcn_s_setprio(1);
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          // roles swapped (B tile rows feed the MFMA's A side): a lane then owns one output row m
          // and, per register group, four consecutive columns n
          acc[i >> 1][j >> 1][i & 1][j & 1] =
              __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s2][j], af[s2][i], acc[i >> 1][j >> 1][i & 1][j & 1], 0, 0, 0);
          const int idx = (s2 * TM + i) * TN + j;
          if (which == 1) {
            constexpr int SP = NM / G::B_LOADS;
            if (idx % SP == 1) { __builtin_amdgcn_sched_barrier(0); if (go) load_b(idx / SP); __builtin_amdgcn_sched_barrier(0); }
          } else if (which == 2) {
            constexpr int SP = NM / G::A_LOADS;
            if (idx % SP == 1) { __builtin_amdgcn_sched_barrier(0); if (go) load_a(idx / SP); __builtin_amdgcn_sched_barrier(0); }
          }
        }
    if (which == 1 && go) done_b();
    if (which == 2 && go) done_a();
    __builtin_amdgcn_s_setprio(0);
  };

  if (nk > 0) {
    // tiles 0 .. N-2 of each ring, tile 0 of both first
    issue_b(); issue_a();
    if (NB > 2 && nk > 1) issue_b();
    if (NA > 2 && nk > 1) issue_a();
    wait_tile(-1);
    pp_barrier();
    if (grp == 0) {
      for (int kt = 0; kt < nk; ++kt) {
        fragments(0);                                 // interval 4kt
        if (do_rowsum) rowsum_acc();
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        pp_barrier();
        mfmas(1, kt + NB - 1 < nk);                   // interval 4kt+1
        pp_barrier();
        fragments(1);                                 // interval 4kt+2
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        pp_barrier();
        mfmas(2, kt + NA - 1 < nk);                   // interval 4kt+3
        wait_tile(kt);
        pp_barrier();
        next_tile();
      }
      pp_barrier();                                   // group 1's last interval
    } else {
      if (NB - 1 < nk) issue_b();                     // interval 0 belongs to group 0
      pp_barrier();
      for (int kt = 0; kt < nk; ++kt) {
        fragments(0);                                 // interval 4kt+1
        if (do_rowsum) rowsum_acc();
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        pp_barrier();
        mfmas(2, kt + NA - 1 < nk);                   // interval 4kt+2
        pp_barrier();
        fragments(1);                                 // interval 4kt+3
        __builtin_amdgcn_s_waitcnt(kWaitLds);
        wait_tile(kt);
        pp_barrier();
        next_tile();
        mfmas(1, kt + NB < nk);                       // interval 4kt+4
        pp_barrier();
      }
    }
  }

  GemmDev q = p;
  float* rowsum = p.a_rowsum;
  if (p.splits > 1) {
    // raw fp32 tile and row sums of this k range, as a plain matrix [M][N] in the workspace; a
    // second kernel adds the parts in order
    q.C = p.partial + (int64_t)split * p.M * p.N;
    q.ldc = p.N; q.c_f32 = 1; q.bias = nullptr; q.resid = nullptr; q.gelu = GELU_NONE;
    q.vec = (p.N & 3) == 0;
    rowsum = p.partial + (int64_t)p.splits * p.M * p.N + (int64_t)split * p.M;
  }
  if (do_rowsum) {
    // RC threads hold parts of every row: through the (now dead) ring, summed in a fixed order
    constexpr int RC = BM / 8, NG = 512 / RC;
    float* red = (float*)ring;                        // [NG k groups][BM rows]
    __syncthreads();
    const int mc = (tid % RC) ^ (4 * ((tid / RC) & 3));
#pragma unroll
    for (int e = 0; e < 8; ++e) red[(tid / RC) * BM + mc * 8 + e] = rs[e];
    __syncthreads();
    if (tid < BM) {
      float tot = 0.f;
#pragma unroll
      for (int g = 0; g < NG; ++g) tot += red[g * BM + tid];
      if (m0 + tid < p.M) rowsum[m0 + tid] = tot;
    }
  }
  // 64 x 64 pieces through LDS: 16 KB per wave when the ring has 128 KB, else two 8 KB halves
  __syncthreads();
  constexpr int HALVES = G::SMEM >= 8 * 16384 ? 1 : 2;
  static_assert(G::SMEM >= 8 * 16384 / HALVES, "staging space");
  float* wstage = (float*)ring + wave * (4096 / HALVES);
#pragma unroll
  for (int a = 0; a < TM / 2; ++a)
#pragma unroll
    for (int b = 0; b < TN / 2; ++b)
      store_tile<HALVES>(q, acc[a][b], m0 + wm * TM * 32 + a * 64, n0 + wn * TN * 32 + b * 64, lane, wstage);
}

template <bool AK, bool BKM, int WM, int WN, int TM, int TN, int NA, int NB>
static void launch_pp(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1) {
  typedef Geo<WM, WN, TM, TN, NA, NB> G;
  static bool configured = false;
  if (!configured) {
    (void)hipFuncSetAttribute((const void*)bgemm_pp_kernel<AK, BKM, false, WM, WN, TM, TN, NA, NB>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, G::SMEM);
    (void)hipFuncSetAttribute((const void*)bgemm_pp_kernel<AK, BKM, true, WM, WN, TM, TN, NA, NB>,
                              hipFuncAttributeMaxDynamicSharedMemorySize, G::SMEM);
    configured = true;
  }
  const int tiles_m = (p.M + G::BM - 1) / G::BM, tiles_n = (p.N + G::BN - 1) / G::BN;
  const int total = tiles_m * tiles_n * p.splits, per = (total + 7) / 8;
  dim3 grid(per * 8), block(512);
  if (p.K % PBK)
    hipExtLaunchKernelGGL((bgemm_pp_kernel<AK, BKM, true, WM, WN, TM, TN, NA, NB>), grid, block, G::SMEM, st, t0, t1, 0, p, tiles_n, total, per);
  else
    hipExtLaunchKernelGGL((bgemm_pp_kernel<AK, BKM, false, WM, WN, TM, TN, NA, NB>), grid, block, G::SMEM, st, t0, t1, 0, p, tiles_n, total, per);
}

// 256 x 256 block tiles, 2 x 4 waves of 128 x 64, rings of 3 A and 2 B tiles.
// Requirements as for the other direct-load kernel: K % 8 == 0 when an operand is k-major (or
// zeros vouched for behind a k-major A's last column, with B m-major), the
// leading dimension of an m-major operand covers its row count rounded up to 8; row sums only
// with an m-major A.
bool launch_bgemm_pp(const GemmDev& p, hipStream_t st, hipEvent_t t0, hipEvent_t t1) {
  auto up8 = [](int64_t v) { return (v + 7) / 8 * 8; };
  // a chunk of a k-major operand that straddles K is moved whole: allowed only where the caller
  // vouches for zeros behind A's last column while B (m-major) reads zeros from row K on
  if ((p.a_k || p.b_k) && (p.K & 7) && !(p.a_tail_zero && p.a_k && !p.b_k && p.lda >= up8(p.K))) return false;
  if (!p.a_k && p.lda < up8(p.M)) return false;
  if (!p.b_k && p.ldb < up8(p.N)) return false;
  if (p.a_rowsum && p.a_k) return false;
  if (p.a_k && p.b_k) launch_pp<true, true, 2, 4, 4, 2, 3, 2>(p, st, t0, t1);
  else if (p.a_k) launch_pp<true, false, 2, 4, 4, 2, 3, 2>(p, st, t0, t1);
  else if (p.b_k) launch_pp<false, true, 2, 4, 4, 2, 3, 2>(p, st, t0, t1);
  else launch_pp<false, false, 2, 4, 4, 2, 3, 2>(p, st, t0, t1);
  return true;
}

// Units of 256 x 256 tiles a product of this shape has, and how well they fill the 256 compute
// units round by round (one block per compute unit).
int bgemm_pp_tiles(int M, int N) { return ((M + 255) / 256) * ((N + 255) / 256); }

}  // namespace mk
