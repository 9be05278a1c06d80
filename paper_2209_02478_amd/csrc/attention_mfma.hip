// Fused attention for bf16, head size 64, on the MFMA units (v_mfma_f32_32x32x16_bf16).
//
// All three kernels compute score tiles transposed, S^T = K Q^T, so that a lane's 32x32
// accumulator registers belong to ONE query (forward, dQ) or ONE key (dK/dV): the softmax
// statistics of a row are then reductions over a lane's own registers plus one exchange with
// lane^32, and a lane's probabilities, converted to bf16, are directly the B operand of the
// next product (P V, dS K, P^T dO, dS^T Q) without passing through LDS.  The operand that
// multiplies them must be contiguous along the reduction index, so K / V / Q / dO tiles are
// also stored transposed in LDS (register transpose of 4x8 blocks on the way in).
//
// MFMA 32x32x16 register layout used below (A: 32 x 16, B: 16 x 32, D: 32 x 32):
//   A, B: lane holds row/column lane%32 and reduction indices 8*(lane/32) .. +7
//   D:    lane holds column lane%32; register r holds row 8*(r/4) + 4*(lane/32) + r%4
// Feeding D registers 8c..8c+7 as a B operand therefore assigns reduction slot (lane/32, e) the
// row 16c + 8*(e/4) + 4*(lane/32) + e%4, and the A operand is gathered with the same map: two
// runs of 4 consecutive indices.
//
// No atomics: dQ comes from a kernel that owns query rows, dK/dV from one that owns key rows.
#include "device_common.h"
#include "kernels.h"
#include "philox.h"

namespace mk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int D = 64;          // head size
constexpr int TK = 64;         // rows of a streamed tile
constexpr int LDT = 72;        // LDS row stride in elements of the tiles read 16 bytes at a time (144 bytes)
// Row stride of the transposed tiles, which are written and read 8 bytes at a time: 34 dwords, an
// odd multiple of two, so that the 8-byte reads of lanes 0..31 (one row each) fall in all different
// banks; with 36 dwords rows r and r + 16 met in the same banks (half of those reads conflicted).
constexpr int LDTT = 68;
constexpr int ROWS_PER_BLOCK = 128;

constexpr float LOG2E = 1.44269504088896340736f;
// 2^x on the transcendental unit (v_exp_f32), no range fix-ups: arguments here are <= ~0 or the
// result is multiplied by zero-gradient terms; -inf gives 0
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ bf16x8 ld_frag(const bf16_t* p) { return *(const bf16x8*)p; }

__device__ __forceinline__ uint32_t pack2(float a, float b) {
  return pack_bf16x2(a, b);
}
// registers 8c .. 8c+7 of an accumulator as a bf16 operand
__device__ __forceinline__ bf16x8 regs_to_frag(const f32x16& v, int c) {
  uint4 u;
  u.x = pack2(v[8 * c + 0], v[8 * c + 1]);
  u.y = pack2(v[8 * c + 2], v[8 * c + 3]);
  u.z = pack2(v[8 * c + 4], v[8 * c + 5]);
  u.w = pack2(v[8 * c + 6], v[8 * c + 7]);
  return __builtin_bit_cast(bf16x8, u);
}
// A operand from a transposed tile: row `row`, reduction indices base+4h+{0..3}, base+8+4h+{0..3}
__device__ __forceinline__ bf16x8 ld_frag_t(const bf16_t (*tile)[LDTT], int row, int base, int h) {
  uint2 lo = *(const uint2*)&tile[row][base + 4 * h];
  uint2 hi = *(const uint2*)&tile[row][base + 8 + 4 * h];
  uint4 u = make_uint4(lo.x, lo.y, hi.x, hi.y);
  return __builtin_bit_cast(bf16x8, u);
}

// 128 threads bring one 64 x 64 tile (rows r0.., row stride ld, rows clamped to last) into LDS,
// as is ([row][d]) and / or transposed ([d][row]).  t in [0,128): 4 rows x 8 columns each.
// Two steps, so that the loads of the next tile can fly while the current one is multiplied.
__device__ __forceinline__ void fetch_tile(const bf16_t* src, int64_t ld, int r0, int last, int t, uint4 (&v)[4]) {
  const int rq = t >> 3, cb = t & 7;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    int r = min(r0 + 4 * rq + j, last);
    v[j] = *(const uint4*)(src + (int64_t)r * ld + 8 * cb);
  }
}
template <bool NORMAL, bool TRANSPOSED>
__device__ __forceinline__ void stash_tile(const uint4 (&v)[4], int t, bf16_t (*normal)[LDT], bf16_t (*transposed)[LDTT]) {
  const int rq = t >> 3, cb = t & 7;
  if (NORMAL) {
#pragma unroll
    for (int j = 0; j < 4; ++j) *(uint4*)&normal[4 * rq + j][8 * cb] = v[j];
  }
  if (TRANSPOSED) {
    const uint32_t* w0 = (const uint32_t*)&v[0];
    const uint32_t* w1 = (const uint32_t*)&v[1];
    const uint32_t* w2 = (const uint32_t*)&v[2];
    const uint32_t* w3 = (const uint32_t*)&v[3];
#pragma unroll
    for (int mm = 0; mm < 8; ++mm) {
      const int d = mm >> 1;
      uint2 o;
      if (mm & 1) {
        o.x = (w0[d] >> 16) | (w1[d] & 0xFFFF0000u);
        o.y = (w2[d] >> 16) | (w3[d] & 0xFFFF0000u);
      } else {
        o.x = (w0[d] & 0xFFFFu) | (w1[d] << 16);
        o.y = (w2[d] & 0xFFFFu) | (w3[d] << 16);
      }
      *(uint2*)&transposed[8 * cb + mm][4 * rq] = o;
    }
  }
}

__device__ __forceinline__ void zero(f32x16& v) {
#pragma unroll
  for (int r = 0; r < 16; ++r) v[r] = 0.f;
}

// store a transposed accumulator pair (rows = head columns, lane column = token) as bf16
__device__ __forceinline__ void store_rows(bf16_t* dst, const f32x16 (&acc)[2], int h, float mul) {
#pragma unroll
  for (int db = 0; db < 2; ++db)
#pragma unroll
    for (int g = 0; g < 4; ++g) {
      uint2 o;
      o.x = pack2(acc[db][4 * g] * mul, acc[db][4 * g + 1] * mul);
      o.y = pack2(acc[db][4 * g + 2] * mul, acc[db][4 * g + 3] * mul);
      *(uint2*)(dst + 32 * db + 8 * g + 4 * h) = o;
    }
}

}  // namespace

// ------------------------------------------------------------------ forward
template <bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void fa_fwd_kernel(const bf16_t* __restrict__ qkv, bf16_t* __restrict__ ctx,
                                                     float* __restrict__ lse, const int32_t* __restrict__ lens,
                                                     int L, int nh, DropDesc drop) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[TK][LDT];   // [key][d]
  __shared__ __attribute__((aligned(16))) bf16_t Vt[D][LDTT];   // [d][key]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ql = lane & 31, h = lane >> 5;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const int qi = blockIdx.x * ROWS_PER_BLOCK + wave * 32 + ql;
  const int qc = min(qi, L - 1);
  const float scale = 0.125f, c2 = scale * LOG2E;    // exp(scale * s - x) == exp2(c2 * s - LOG2E * x)

  bf16x8 qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) qf[kk] = ld_frag(base + (int64_t)qc * ld3 + 16 * kk + 8 * h);
  f32x16 o[2];
  zero(o[0]); zero(o[1]);
  float m = -INFINITY, l = 0.f;                       // running maximum of the raw (unscaled) scores, sum of exps
  const int Lk = lens ? lens[b] : L;                  // keys from Lk on are padding (1 <= Lk <= L)
  const int kend = CAUSAL ? min(Lk, (int)(blockIdx.x + 1) * ROWS_PER_BLOCK) : Lk;

  // threads 0..127 stage K, the others V; the next tile's loads are in flight during the MFMAs
  const bf16_t* mine = tid < 128 ? base + H : base + 2 * H;
  const int t128 = tid & 127;
  uint4 pre[4];
  fetch_tile(mine, ld3, 0, L - 1, t128, pre);
  for (int k0 = 0; k0 < kend; k0 += TK) {
    __syncthreads();
    if (tid < 128) stash_tile<true, false>(pre, t128, Ks, nullptr);
    else stash_tile<false, true>(pre, t128, nullptr, Vt);
    __syncthreads();
    if (k0 + TK < kend) fetch_tile(mine, ld3, k0 + TK, L - 1, t128, pre);
    f32x16 s[2];
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      zero(s[kb]);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk)
        s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(&Ks[32 * kb + ql][16 * kk + 8 * h]), qf[kk], s[kb], 0, 0, 0);
      if (CAUSAL || k0 + TK > Lk) {                   // only tiles that touch the mask pay for it
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key >= Lk || (CAUSAL && key > qi)) s[kb][r] = -INFINITY;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float mnew = fmaxf(m, mx);                  // finite: key 0 is visible to every query
    const float alpha = fast_exp2((m - mnew) * c2);
    const float off = -mnew * c2;
    float rs = 0.f;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float p = fast_exp2(fmaf(s[kb][r], c2, off));
        s[kb][r] = p;
        rs += p;
      }
    rs += __shfl_xor(rs, 32, 64);
    l = l * alpha + rs;                               // the normaliser counts every probability
    m = mnew;
    if (DROP) {                                       // dropped ones leave the P V product; the scale waits for the end
      const int64_t row = (int64_t)bh * L + qc;
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint4 w = attn_drop_words(drop, row, (L + 3) >> 2, k0 + 32 * kb + 8 * g + 4 * h);
          if (w.x < drop.thr) s[kb][4 * g] = 0.f;
          if (w.y < drop.thr) s[kb][4 * g + 1] = 0.f;
          if (w.z < drop.thr) s[kb][4 * g + 2] = 0.f;
          if (w.w < drop.thr) s[kb][4 * g + 3] = 0.f;
        }
    }
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[db][r] *= alpha;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16x8 pf = regs_to_frag(s[kb], c);
#pragma unroll
        for (int db = 0; db < 2; ++db)
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_t(Vt, 32 * db + ql, 32 * kb + 16 * c, h), pf, o[db], 0, 0, 0);
      }
  }
  if (qi < L) {
    store_rows(ctx + ((int64_t)b * L + qi) * H + hh * D, o, h, (DROP ? drop.scale : 1.f) / l);
    if (h == 0) lse[(int64_t)bh * L + qi] = m * scale + __logf(l);
  }
}

// ------------------------------------------------------------------ dQ
template <bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void fa_bwd_dq_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ ctx,
                                                        const bf16_t* __restrict__ dctx,
                                                        const float* __restrict__ lse, float* __restrict__ delta,
                                                        bf16_t* __restrict__ dqkv, const int32_t* __restrict__ lens, int L,
                                                        int nh, DropDesc drop) {
  __shared__ __attribute__((aligned(16))) bf16_t Ks[TK][LDT];   // [key][d]
  __shared__ __attribute__((aligned(16))) bf16_t Kt[D][LDTT];   // [d][key]
  __shared__ __attribute__((aligned(16))) bf16_t Vs[TK][LDT];   // [key][d]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, ql = lane & 31, h = lane >> 5;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const int qi = blockIdx.x * ROWS_PER_BLOCK + wave * 32 + ql;
  const int qc = min(qi, L - 1);
  const float scale = 0.125f;

  // delta = sum over the head's columns of dO * O for this query: each half of the wave holds 32
  // of the 64 columns.  Written out for the dK/dV kernel, which runs after this one.
  bf16x8 qf[4], gf[4];
  float delta_q = 0.f;
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    qf[kk] = ld_frag(base + (int64_t)qc * ld3 + 16 * kk + 8 * h);
    gf[kk] = ld_frag(dctx + ((int64_t)b * L + qc) * H + hh * D + 16 * kk + 8 * h);
    const bf16x8 of = ld_frag(ctx + ((int64_t)b * L + qc) * H + hh * D + 16 * kk + 8 * h);
#pragma unroll
    for (int e = 0; e < 8; ++e) delta_q = fmaf((float)of[e], (float)gf[kk][e], delta_q);
  }
  delta_q += __shfl_xor(delta_q, 32, 64);
  if (h == 0 && qi < L) delta[(int64_t)bh * L + qi] = delta_q;
  const float c2 = scale * LOG2E;
  const float nlse_q = -LOG2E * lse[(int64_t)bh * L + qc];
  f32x16 dq[2];
  zero(dq[0]); zero(dq[1]);
  const int Lk = lens ? lens[b] : L;                  // keys from Lk on are padding (1 <= Lk <= L)
  const int kend = CAUSAL ? min(Lk, (int)(blockIdx.x + 1) * ROWS_PER_BLOCK) : Lk;

  const bf16_t* mine = tid < 128 ? base + H : base + 2 * H;     // threads 0..127 stage K, the others V
  const int t128 = tid & 127;
  uint4 pre[4];
  fetch_tile(mine, ld3, 0, L - 1, t128, pre);
  for (int k0 = 0; k0 < kend; k0 += TK) {
    __syncthreads();
    if (tid < 128) stash_tile<true, true>(pre, t128, Ks, Kt);
    else stash_tile<true, false>(pre, t128, Vs, nullptr);
    __syncthreads();
    if (k0 + TK < kend) fetch_tile(mine, ld3, k0 + TK, L - 1, t128, pre);
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      f32x16 s, dp;
      zero(s); zero(dp);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(&Ks[32 * kb + ql][16 * kk + 8 * h]), qf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(&Vs[32 * kb + ql][16 * kk + 8 * h]), gf[kk], dp, 0, 0, 0);
      }
      if (DROP) {                                     // d(P) of a dropped probability is zero, of a kept one scaled
        const int64_t row = (int64_t)bh * L + qc;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint4 w = attn_drop_words(drop, row, (L + 3) >> 2, k0 + 32 * kb + 8 * g + 4 * h);
          dp[4 * g] = w.x < drop.thr ? 0.f : dp[4 * g] * drop.scale;
          dp[4 * g + 1] = w.y < drop.thr ? 0.f : dp[4 * g + 1] * drop.scale;
          dp[4 * g + 2] = w.z < drop.thr ? 0.f : dp[4 * g + 2] * drop.scale;
          dp[4 * g + 3] = w.w < drop.thr ? 0.f : dp[4 * g + 3] * drop.scale;
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) s[r] = fast_exp2(fmaf(s[r], c2, nlse_q)) * (dp[r] - delta_q);
      if (CAUSAL || k0 + TK > Lk) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = k0 + 32 * kb + 8 * (r >> 2) + 4 * h + (r & 3);
          if (key >= Lk || (CAUSAL && key > qi)) s[r] = 0.f;
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16x8 dsf = regs_to_frag(s, c);
#pragma unroll
        for (int db = 0; db < 2; ++db)
          dq[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_t(Kt, 32 * db + ql, 32 * kb + 16 * c, h), dsf, dq[db], 0, 0, 0);
      }
    }
  }
  if (qi < L) store_rows(dqkv + ((int64_t)b * L + qi) * ld3 + hh * D, dq, h, scale);
}

// ------------------------------------------------------------------ dK, dV
template <bool CAUSAL, bool DROP>
__global__ __launch_bounds__(256, 2) void fa_bwd_dkv_kernel(const bf16_t* __restrict__ qkv, const bf16_t* __restrict__ dctx,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16_t* __restrict__ dqkv, const int32_t* __restrict__ lens, int L,
                                                        int nh, DropDesc drop) {
  __shared__ __attribute__((aligned(16))) bf16_t Qs[TK][LDT];   // [query][d]
  __shared__ __attribute__((aligned(16))) bf16_t Qt[D][LDTT];   // [d][query]
  __shared__ __attribute__((aligned(16))) bf16_t Gs[TK][LDT];   // dO [query][d]
  __shared__ __attribute__((aligned(16))) bf16_t Gt[D][LDTT];   // dO [d][query]
  __shared__ __attribute__((aligned(16))) float lse_s[TK], delta_s[TK];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, kl = lane & 31, h = lane >> 5;
  const int bh = blockIdx.y, b = bh / nh, hh = bh - b * nh;
  const int H = nh * D;
  const int64_t ld3 = 3 * (int64_t)H;
  const bf16_t* base = qkv + (int64_t)b * L * ld3 + hh * D;
  const bf16_t* gbase = dctx + (int64_t)b * L * H + hh * D;
  const int ki = blockIdx.x * ROWS_PER_BLOCK + wave * 32 + kl;
  const int kc = min(ki, L - 1);
  const float scale = 0.125f, c2 = scale * LOG2E;

  bf16x8 kf[4], vf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    kf[kk] = ld_frag(base + (int64_t)kc * ld3 + H + 16 * kk + 8 * h);
    vf[kk] = ld_frag(base + (int64_t)kc * ld3 + 2 * H + 16 * kk + 8 * h);
  }
  f32x16 dk[2], dv[2];
  zero(dk[0]); zero(dk[1]); zero(dv[0]); zero(dv[1]);
  const int qstart = CAUSAL ? blockIdx.x * ROWS_PER_BLOCK : 0;     // earlier queries never see these keys
  const int Lk = lens ? lens[b] : L;                               // keys from Lk on are padding: their dK, dV are zero
  const int qend = (int)blockIdx.x * ROWS_PER_BLOCK >= Lk ? 0 : L; // a block of padded keys only writes zeros

  const bf16_t* mine = tid < 128 ? base : gbase;                 // threads 0..127 stage Q, the others dO
  const int64_t mine_ld = tid < 128 ? ld3 : (int64_t)H;
  const int t128 = tid & 127;
  uint4 pre[4];
  float pre_lse = 0.f, pre_delta = 0.f;
  auto fetch = [&](int q0) {
    fetch_tile(mine, mine_ld, q0, L - 1, t128, pre);
    if (tid < TK) {
      const int q = min(q0 + tid, L - 1);
      pre_lse = lse[(int64_t)bh * L + q];
      pre_delta = delta[(int64_t)bh * L + q];
    }
  };
  if (qstart < qend) fetch(qstart);
  for (int q0 = qstart; q0 < qend; q0 += TK) {
    __syncthreads();
    if (tid < 128) stash_tile<true, true>(pre, t128, Qs, Qt);
    else stash_tile<true, true>(pre, t128, Gs, Gt);
    if (tid < TK) { lse_s[tid] = -LOG2E * pre_lse; delta_s[tid] = pre_delta; }   // lse_s: ready for exp2
    __syncthreads();
    if (q0 + TK < qend) fetch(q0 + TK);
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      f32x16 s, dp;
      zero(s); zero(dp);
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) {
        s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(&Qs[32 * qb + kl][16 * kk + 8 * h]), kf[kk], s, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(&Gs[32 * qb + kl][16 * kk + 8 * h]), vf[kk], dp, 0, 0, 0);
      }
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int qq = 32 * qb + 8 * g + 4 * h;
        const float4 nl = *(const float4*)&lse_s[qq], dl = *(const float4*)&delta_s[qq];
        const float nls[4] = {nl.x, nl.y, nl.z, nl.w}, dls[4] = {dl.x, dl.y, dl.z, dl.w};
        // Dropout: this lane holds one key and four queries; a generator block covers four keys
        // of one query.  The four lanes of a quad (four neighbouring keys) each make the block of
        // one of the four queries and pass its words round: in turn t a lane receives, from the
        // lane t places on, the word of its own key for that lane's query.
        bool keep[4] = {true, true, true, true};
        if (DROP) {
          const int c = lane & 3;
          const int qmine = min(q0 + qq + c, L - 1);
          const uint4 w = attn_drop_words(drop, (int64_t)bh * L + qmine, (L + 3) >> 2, ki & ~3);
#pragma unroll
          for (int t = 0; t < 4; ++t) {
            const uint32_t got = __shfl(pick_word(w, (c - t) & 3), (lane & ~3) | ((c + t) & 3), 64);
            const bool k = got >= drop.thr;
            const int e = (c + t) & 3;
            keep[0] = e == 0 ? k : keep[0]; keep[1] = e == 1 ? k : keep[1];
            keep[2] = e == 2 ? k : keep[2]; keep[3] = e == 3 ? k : keep[3];
          }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g + e;
          const float p = fast_exp2(fmaf(s[r], c2, nls[e]));
          if (DROP) {
            s[r] = keep[e] ? p * drop.scale : 0.f;                         // what multiplied V in the forward
            dp[r] = p * ((keep[e] ? dp[r] * drop.scale : 0.f) - dls[e]);
          } else {
            s[r] = p;
            dp[r] = p * (dp[r] - dls[e]);
          }
        }
      }
      if (CAUSAL || q0 + TK > L) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int q = q0 + 32 * qb + 8 * (r >> 2) + 4 * h + (r & 3);
          if (q >= L || (CAUSAL && ki > q)) { s[r] = 0.f; dp[r] = 0.f; }
        }
      }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        const bf16x8 pf = regs_to_frag(s, c), dsf = regs_to_frag(dp, c);
#pragma unroll
        for (int db = 0; db < 2; ++db) {
          dv[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_t(Gt, 32 * db + kl, 32 * qb + 16 * c, h), pf, dv[db], 0, 0, 0);
          dk[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_t(Qt, 32 * db + kl, 32 * qb + 16 * c, h), dsf, dk[db], 0, 0, 0);
        }
      }
    }
  }
  if (ki < L) {
    if (ki >= Lk) { zero(dk[0]); zero(dk[1]); zero(dv[0]); zero(dv[1]); }   // whatever the lane's column held
    bf16_t* out = dqkv + ((int64_t)b * L + ki) * ld3 + hh * D;
    store_rows(out + H, dk, h, scale);
    store_rows(out + 2 * H, dv, h, 1.f);
  }
}

void attention_fwd_mfma(const void* qkv, void* ctx, float* lse, const int32_t* lens, int B, int L, int nh, int causal,
                        const DropDesc& drop, hipStream_t st) {
  dim3 grid((L + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, B * nh);
#define FWD_(C, D) hipLaunchKernelGGL((fa_fwd_kernel<C, D>), grid, dim3(256), 0, st, (const bf16_t*)qkv, (bf16_t*)ctx, lse, lens, L, nh, drop)
  if (drop.thr) { if (causal) FWD_(true, true); else FWD_(false, true); }
  else { if (causal) FWD_(true, false); else FWD_(false, false); }
#undef FWD_
}

void attention_bwd_mfma(const void* qkv, const void* ctx, const void* dctx, const float* lse, float* delta, void* dqkv,
                        const int32_t* lens, int B, int L, int nh, int causal, const DropDesc& drop, hipStream_t st) {
  dim3 grid((L + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK, B * nh);
#define BWD_(C, D)                                                                                               \
  hipLaunchKernelGGL((fa_bwd_dq_kernel<C, D>), grid, dim3(256), 0, st, (const bf16_t*)qkv, (const bf16_t*)ctx,  \
                     (const bf16_t*)dctx, lse, delta, (bf16_t*)dqkv, lens, L, nh, drop);                          \
  hipLaunchKernelGGL((fa_bwd_dkv_kernel<C, D>), grid, dim3(256), 0, st, (const bf16_t*)qkv, (const bf16_t*)dctx, lse, \
                     delta, (bf16_t*)dqkv, lens, L, nh, drop)
  if (drop.thr) { if (causal) { BWD_(true, true); } else { BWD_(false, true); } }
  else { if (causal) { BWD_(true, false); } else { BWD_(false, false); } }
#undef BWD_
}

}  // namespace mk
