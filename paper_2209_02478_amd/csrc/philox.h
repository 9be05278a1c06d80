// Counter-based random numbers for dropout: Philox4x32 with ten rounds (Salmon, Moraes, Dror,
// Shaw, SC'11).  A mask is a pure function of (seed, iteration, site, element number), so the
// forward of a checkpointed layer that is run again before its backward meets the masks of its
// first run without anything being stored.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace mk {

__device__ __forceinline__ uint4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                               uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c0), lo0 = M0 * c0;
    const uint32_t hi1 = __umulhi(M1, c2), lo1 = M1 * c2;
    c0 = hi1 ^ c1 ^ k0;
    c1 = lo1;
    c2 = hi0 ^ c3 ^ k1;
    c3 = lo0;
    k0 += W0;
    k1 += W1;
  }
  return make_uint4(c0, c1, c2, c3);
}

// the four words of block `block` (elements 4*block .. 4*block+3) at this site and iteration
__device__ __forceinline__ uint4 drop_words(const DropDesc& d, uint64_t block) {
  return philox4x32_10((uint32_t)block, (uint32_t)(block >> 32), d.site, d.step, d.k0, d.k1);
}

// Attention probabilities [B, nh, L, L]: every row of L keys is padded to a multiple of four, so
// four neighbouring keys of one query share a block whatever L is:
//   block = row * ceil(L / 4) + key / 4,  row = (b * nh + h) * L + query,  word = key % 4.
__device__ __forceinline__ uint4 attn_drop_words(const DropDesc& d, int64_t row, int L4q, int key) {
  return drop_words(d, (uint64_t)row * (uint64_t)L4q + (uint64_t)(key >> 2));
}
__device__ __forceinline__ uint32_t pick_word(const uint4& w, int i) {
  return i == 0 ? w.x : i == 1 ? w.y : i == 2 ? w.z : w.w;
}
__device__ __forceinline__ bool attn_keep(const DropDesc& d, int64_t row, int L4q, int key) {
  return pick_word(attn_drop_words(d, row, L4q, key), key & 3) >= d.thr;
}

}  // namespace mk
