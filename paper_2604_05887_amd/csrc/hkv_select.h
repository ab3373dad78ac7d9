// Block-wide radix selection of the m-th largest 32-bit key with exact tie accounting.
// Used for the Top-M visual tokens of static heads and the top-k chunks of dynamic heads
// (Appendix A of the paper); ties are later broken towards the lower index by the caller.
#pragma once

#include "hkv_device.h"

namespace hkv {

// Order-preserving map from float to uint32 (larger float -> larger key); -0.0 counts as +0.0.
__device__ __forceinline__ uint32_t float_order_key(float f) {
  uint32_t u = float_to_bits(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Finds T = key of the m_sel-th largest candidate among j in [0, n) and r_adm = how many
// candidates equal to T belong to the top m_sel (>= 1).  Requires 0 < m_sel <= #candidates.
// keyfn(j, key) returns whether j is a candidate and, if so, its key.
// `hist` is 256 words of shared memory, `bc` 2 words.  All NT threads of the block must call.
// EARLY: the search may stop at a prefix all of whose candidates are wanted; T is then the smallest key
// with that prefix -- no candidate's key, in general -- and still splits the candidates as above (key > T:
// in; key == T: in for the first r_adm of them; else out).  For callers that use T only in that way.
template <int NT, bool EARLY = false, class KeyFn>
__device__ __forceinline__ void radix_select(int n, int m_sel, KeyFn keyfn, uint32_t* hist, uint32_t* bc,
                                             uint32_t& T, int& r_adm) {
  const int tid = thread_index();
  uint32_t prefix = 0, mask = 0;
  int remaining = m_sel;
#pragma unroll 1
  for (int shift = 24; shift >= 0; shift -= 8) {
    for (int i = tid; i < 256; i += NT) hist[i] = 0;
    __syncthreads();
    for (int j = tid; j < n; j += NT) {
      uint32_t key;
      if (keyfn(j, key) && (key & mask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1u);
    }
    __syncthreads();
    if (tid < 64) {   // one wave scans the 256 bins from the top: lane l owns bins 4l..4l+3
      const int h0 = (int)hist[4 * tid + 0], h1 = (int)hist[4 * tid + 1];
      const int h2 = (int)hist[4 * tid + 2], h3 = (int)hist[4 * tid + 3];
      const int s = h0 + h1 + h2 + h3;
      const int incl = wave_inclusive_scan(s);
      const int total = __builtin_amdgcn_readlane(incl, 63);
      const int above = total - incl;          // candidates in bins owned by higher lanes
      if (above < remaining && remaining <= above + s) {   // exactly one lane
        int cum = above, d;
        if (cum + h3 >= remaining) d = 3;
        else { cum += h3;
          if (cum + h2 >= remaining) d = 2;
          else { cum += h2;
            if (cum + h1 >= remaining) d = 1;
            else { cum += h1; d = 0; } } }
        const int in_bin = d == 3 ? h3 : d == 2 ? h2 : d == 1 ? h1 : h0;
        bc[0] = (uint32_t)(4 * tid + d);
        // top bit: every candidate of the bin is wanted, so the bin's smallest possible key already separates
        // the top m_sel from the rest and the remaining digits need not be resolved
        bc[1] = (uint32_t)(remaining - cum) | (remaining - cum == in_bin ? 0x80000000u : 0u);
      }
    }
    __syncthreads();
    prefix |= bc[0] << shift;
    mask |= 0xFFu << shift;
    const uint32_t word = bc[1];
    remaining = (int)(word & 0x7fffffffu);
    __syncthreads();
    if (EARLY && (word >> 31)) break;          // block-uniform
  }
  T = prefix;
  r_adm = remaining;
}

}  // namespace hkv
