// Radix selection of the m-th largest 32-bit key with exact tie accounting, block-wide over keys in memory
// (radix_select) and wave-wide over keys in registers (wave_radix_kth).
// Used for the Top-M visual tokens of static heads, the top-k chunks of dynamic heads (Appendix A of the
// paper) and the per-row top-k of the head classification; ties are later broken towards the lower index
// by the caller.
#pragma once

#include "hkv_device.h"

namespace hkv {

// Order-preserving map from float to uint32 (larger float -> larger key); -0.0 counts as +0.0.
__device__ __forceinline__ uint32_t float_order_key(float f) {
  uint32_t u = float_to_bits(f + 0.0f);
  return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ void wave_lds_sync() {     // orders the wave's own shared-memory writes before its later reads
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The kth largest of the keys one wave holds (N per lane, the first n_used registers of every lane in use; an
// absent entry holds 0; keys below lo are left out, none lies above hi, lo >= 1, and at least kth keys lie in
// [lo, hi]), exactly: radix
// selection on key - lo, eight bits per round, through a 256-bin histogram in `hist` (the wave's own 256
// words of shared memory).  A round costs a handful of instructions per register where the bitwise search
// above costs three per register and BIT.
// max_rounds < 4: the search stops early and returns the smallest key that shares the decided bits with the
// kth largest -- a lower bound for it.
template <int N>
__device__ __forceinline__ uint32_t wave_radix_kth(const uint32_t (&key)[N], int n_used, int kth, uint32_t lo, uint32_t hi,
                                                   uint32_t* hist, int max_rounds = 4) {
  const int lane = thread_index() & 63;
  const uint32_t span = hi - lo;
  int shift = 32 - __builtin_clz(span | 1u);                 // bits of key - lo not yet decided (wave-uniform)
  uint32_t d[N];                                             // key - lo; an absent entry gets 2^32 - 1: above the span
                                                             // (lo >= 1), so it never shares a prefix with a real key
#pragma unroll
  for (int e = 0; e < N; ++e) d[e] = key[e] >= lo ? key[e] - lo : 0xFFFFFFFFu;
  uint32_t prefix = 0;                                       // the decided bits
  int need = kth;                                            // rank among the keys that share the prefix
  for (int round = 0; shift > 0 && round < max_rounds; ++round) {
    const int w = min(8, shift);
    const int hi_shift = shift;                              // keys in play: (key - lo) >> hi_shift == prefix
    shift -= w;
    *reinterpret_cast<uint4*>(hist + 4 * lane) = make_uint4(0, 0, 0, 0);
    wave_lds_sync();
    if (hi_shift >= 32) {                                    // first round of a full-width span: every real key is in play
#pragma unroll
      for (int e = 0; e < N; ++e)
        if (e < n_used && key[e] >= lo) atomicAdd(hist + (d[e] >> shift), 1u);
    } else {
#pragma unroll
      for (int e = 0; e < N; ++e)
        if (e < n_used && (d[e] >> hi_shift) == prefix) atomicAdd(hist + ((d[e] >> shift) & ((1u << w) - 1u)), 1u);
    }
    wave_lds_sync();
    const uint4 c = *reinterpret_cast<const uint4*>(hist + 4 * lane);          // bins 4 * lane .. 4 * lane + 3
    const int s = (int)(c.x + c.y + c.z + c.w);
    const int incl = wave_inclusive_scan_dpp(s);
    const int total = __builtin_amdgcn_readlane(incl, 63);
    const int a3 = total - incl;                             // keys in bins above this lane's
    // the largest bin b with (keys in bins >= b) >= need
    const int c3 = a3 + (int)c.w, c2 = c3 + (int)c.z, c1 = c2 + (int)c.y, c0 = c1 + (int)c.x;
    int cand = -1, above = 0;
    if (c0 >= need) { cand = 4 * lane; above = c1; }
    if (c1 >= need) { cand = 4 * lane + 1; above = c2; }
    if (c2 >= need) { cand = 4 * lane + 2; above = c3; }
    if (c3 >= need) { cand = 4 * lane + 3; above = a3; }
    const uint64_t has = __builtin_amdgcn_ballot_w64(cand >= 0);
    const int src = 63 - __builtin_clzll(has | 1ull);        // highest lane with a candidate holds the largest bin
    const int bin = __builtin_amdgcn_readlane(cand, src);
    need -= __builtin_amdgcn_readlane(above, src);
    prefix = (prefix << w) | (uint32_t)bin;
  }
  return lo + (prefix << shift);
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
