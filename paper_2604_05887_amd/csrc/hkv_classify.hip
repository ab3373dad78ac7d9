// Text-centric head classification (paper, Section 3.1) and the host side of the top-down budget
// allocation (Section 3.2): the two steps upstream of hkv_compress.
//
// Sparsity score of a KV head: every text token of the prompt attends over the whole prompt,
// S_text = softmax(Q_text K^T / sqrt(d)); a row contributes the sum of its k largest probabilities,
// k = ceil(focus * C); the score is the mean over the text rows (and over the G query heads that
// share the KV head).  Heads at or above a threshold are static, the others dynamic.
//
// Device plan, one (layer, sequence) pass at a time, all KV heads of the pass together.
// bf16 inputs with a focus fraction of at most 1/18 (the paper's 0.05 is) and rows of at most 65536 keys:
//   scan_rows_kernel  S = Q_text K^T on the matrix cores, formed once and never written out: per text row the
//                     running maximum and normaliser, per group of 16 keys of a row its four largest logits
//   row_final_kernel  per text row: a lower bound for the k-th largest logit from the groups' largest, the
//                     candidates at or above it (a group that may hold more than four is recomputed), the
//                     exact k-th largest of the candidates, the sum of the probabilities above it plus the
//                     admitted ties
//   reduce_kernel     mean of the row values of each head, in a fixed order
// Other inputs (fp32, larger focus fractions, longer rows): the logits of a pass are materialised
//   logits_kernel     S = Q_text K^T on the matrix cores, logits (log2 domain) written to the workspace
//   row top-k         per text row: row maximum, normaliser, exact k-th largest logit, sum of the
//                     probabilities above it plus the admitted ties -- one wave per row with the row in
//                     registers (row_topk_wave_kernel, up to 8192 keys), one workgroup per row
//                     (row_topk_reg_kernel, up to 32768 keys), or radix selection over the row in memory
//                     (row_topk_kernel)
//   reduce_kernel     as above
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <vector>

#include "hkv_internal.h"
#include "hkv_mma.h"
#include "hkv_select.h"

namespace hkv {

constexpr int kRowsPerBlock = 256;     // text rows staged per workgroup of logits_kernel
constexpr int kKeysPerLogitBlock = 512;

// grid = (key splits, row chunks, heads of the pass); block = 256 threads.
// Row r of a head is (g = r / T, t = r % T): query head head*G + g at the t-th text token
// (text_pos == nullptr: at token t itself).
template <typename T>
__global__ __launch_bounds__(256) void logits_kernel(const T* __restrict__ q_layer, const T* __restrict__ k_layer,
                                                     const int32_t* __restrict__ text_pos, int64_t seq_start, int C,
                                                     int n_text, int G, int n_q_heads, int n_kv_heads, int head0,
                                                     float scale_log2e, float* __restrict__ logits,
                                                     int64_t head_stride, int pitch) {
  constexpr int ROWB = kD * sizeof(T);
  constexpr int PITCH = ROWB + 16;
  constexpr int NPIECE = ROWB / 32;
  constexpr int PPR = ROWB / 16;
  extern __shared__ char qs[];                  // [kRowsPerBlock][PITCH]
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int head = head0 + blockIdx.z;
  const int rows = G * n_text;
  const int row0 = blockIdx.y * kRowsPerBlock;
  const int rows_here = min(kRowsPerBlock, rows - row0);
  const int n_rb = (rows_here + 31) / 32;
  const int key0 = blockIdx.x * kKeysPerLogitBlock;

  // stage the query rows of this chunk (zero rows past the end), eight independent loads per round
  for (int base = 0; base < n_rb * 32 * PPR; base += 256 * 8) {
    uint4 val[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = base + u * 256 + tid;
      const int rl = idx / PPR, piece = idx % PPR;
      val[u] = make_uint4(0, 0, 0, 0);
      if (idx < n_rb * 32 * PPR && rl < rows_here) {
        const int r = row0 + rl, g = r / n_text, t = r % n_text;
        const size_t src = ((size_t)(seq_start + (text_pos ? text_pos[t] : t)) * n_q_heads + (size_t)head * G + g) * ROWB;
        val[u] = ld16(reinterpret_cast<const char*>(q_layer) + src + piece * 16);
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int idx = base + u * 256 + tid;
      if (idx < n_rb * 32 * PPR) st16(qs + (size_t)(idx / PPR) * PITCH + (idx % PPR) * 16, val[u]);
    }
  }
  __syncthreads();

  const char* kbase = reinterpret_cast<const char*>(k_layer) + ((size_t)seq_start * n_kv_heads + head) * ROWB;
  const size_t kstride = (size_t)n_kv_heads * ROWB;
  float* out = logits + (size_t)blockIdx.z * head_stride;
  for (int kt = 0; kt < kKeysPerLogitBlock / 128; ++kt) {
    const int j0 = key0 + (kt * 4 + wv) * 32;
    if (j0 >= C) break;                          // wave-uniform
    const int key = j0 + l32;
    uint4 a[NPIECE];
#pragma unroll
    for (int j = 0; j < NPIECE; ++j) {
      a[j] = make_uint4(0, 0, 0, 0);
      if (key < C) a[j] = ld16(kbase + (size_t)key * kstride + j * 32 + half * 16);
    }
    for (int rb = 0; rb < n_rb; ++rb) {
      floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
      const char* qrow = qs + (size_t)(rb * 32 + l32) * PITCH + half * 16;
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) acc = mma_piece(a[j], ld16(qrow + j * 32), acc, T{});
      // acc[r] = q_row(rb*32 + l32) . k(j0 + 8*(r/4) + 4*half + r%4): four runs of four consecutive keys.
      // The row pitch is a multiple of 32 keys, so a run past C stays inside the row and is never read.
      const int rl = rb * 32 + l32;
      if (rl < rows_here) {
        float* dst = out + (size_t)(row0 + rl) * pitch + j0 + 4 * half;
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4)
          *reinterpret_cast<float4*>(dst + 8 * g4) =
              make_float4(acc[4 * g4] * scale_log2e, acc[4 * g4 + 1] * scale_log2e, acc[4 * g4 + 2] * scale_log2e,
                          acc[4 * g4 + 3] * scale_log2e);
      }
    }
  }
}

__device__ __forceinline__ float key_to_float(uint32_t key) {      // inverse of float_order_key
  return bits_to_float((key & 0x80000000u) ? (key & 0x7FFFFFFFu) : ~key);
}

// Block-wide reductions in thread order (deterministic); `red` holds 4 floats.  Two barriers each.
__device__ __forceinline__ float block_max(float v, float* red) {
  v = fmaxf(v, lane_xor(v, 1)); v = fmaxf(v, lane_xor(v, 2)); v = fmaxf(v, lane_xor(v, 4));
  v = fmaxf(v, lane_xor(v, 8)); v = fmaxf(v, lane_xor(v, 16)); v = fmaxf(v, lane_xor(v, 32));
  if ((thread_index() & 63) == 0) red[thread_index() >> 6] = v;
  __syncthreads();
  const float r = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  __syncthreads();
  return r;
}
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = sum64(v);
  if ((thread_index() & 63) == 0) red[thread_index() >> 6] = v;
  __syncthreads();
  const float r = (red[0] + red[1]) + (red[2] + red[3]);
  __syncthreads();
  return r;
}

// grid = rows of the pass (heads x G x T), block = 256 threads: one text row per workgroup.
// row value = (sum of the k_top largest probabilities of the row), ties at the k-th place counted as
// often as they are admitted.
__global__ __launch_bounds__(256) void row_topk_kernel(const float* __restrict__ logits, int64_t head_stride, int pitch,
                                                       const int32_t* __restrict__ text_pos, int C, int n_text,
                                                       int rows_per_head, int k_top, int causal,
                                                       float* __restrict__ row_value) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t bc[2];
  __shared__ float red[4];
  const int tid = thread_index();
  const int hp = blockIdx.x / rows_per_head, r = blockIdx.x % rows_per_head;
  const float* row = logits + (size_t)hp * head_stride + (size_t)r * pitch;
  const int n = causal ? min(C, text_pos[r % n_text] + 1) : C;       // keys this text token sees
  const int kt = min(k_top, n);

  float m = kNeg;
  for (int j = tid; j < n; j += 256) m = fmaxf(m, row[j]);
  m = block_max(m, red);
  float z = 0.f;
  for (int j = tid; j < n; j += 256) z += fast_exp2(row[j] - m);
  z = block_sum(z, red);

  uint32_t t_key = 0;
  int r_adm = 0;
  radix_select<256>(n, kt, [&](int j, uint32_t& key) { key = float_order_key(row[j]); return true; }, hist, bc, t_key,
                    r_adm);
  float above = 0.f;
  for (int j = tid; j < n; j += 256) {
    const float l = row[j];
    above += float_order_key(l) > t_key ? fast_exp2(l - m) : 0.f;
  }
  above = block_sum(above, red);
  if (tid == 0) row_value[blockIdx.x] = (above + (float)r_adm * fast_exp2(key_to_float(t_key) - m)) / z;
}

__device__ __forceinline__ uint32_t block_min_u32(uint32_t v, uint32_t* red) {
#pragma unroll
  for (int mask = 1; mask < 64; mask <<= 1) v = min(v, (uint32_t)lane_xor_i((int)v, mask));
  if ((thread_index() & 63) == 0) red[thread_index() >> 6] = v;
  __syncthreads();
  const uint32_t r = min(min(red[0], red[1]), min(red[2], red[3]));
  __syncthreads();
  return r;
}

// The kth largest of the keys the workgroup holds (N per thread; an absent entry holds 0, which is below
// every real key), given that at least kth of them lie in [lo, hi] and none above hi: bitwise search on
// key - lo over workgroup-wide vote counts, one barrier per bit of hi - lo.  cnt: [2][4] ints.
template <int N>
__device__ __forceinline__ uint32_t block_kth_largest(const uint32_t (&key)[N], int kth, uint32_t lo, uint32_t hi,
                                                      int (*cnt)[4]) {
  const int tid = thread_index(), wv = tid >> 6;
  const uint32_t span = hi - lo;
  const int nbits = 32 - __builtin_clz(span | 1u);          // block-uniform
  __syncthreads();                                          // cnt may still be read from an earlier search
  uint32_t thr = 0;
  int buf = 0;
  for (int bit = nbits - 1; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    if (cand > span) continue;                              // no key lies above hi (block-uniform; keeps lo + cand <= hi)
    int c = 0;
#pragma unroll
    for (int e = 0; e < N; ++e) c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= lo + cand));
    if ((tid & 63) == 0) cnt[buf][wv] = c;
    __syncthreads();                       // the other buffer is rewritten only after the next barrier
    const int total = cnt[buf][0] + cnt[buf][1] + cnt[buf][2] + cnt[buf][3];
    if (total >= kth) thr = cand;
    if (total == kth) break;               // block-uniform; the candidate separates the kth largest from the rest
    buf ^= 1;
  }
  return lo + thr;
}

// Same result as row_topk_kernel for rows of at most 256 * EPT keys, with the row read once and held in
// registers (EPT logits per thread).  The k-th largest key is found in two rounds of a bitwise search on
// workgroup-wide vote counts: first among the two largest keys of every group of 32 (a subset of the row,
// so its k-th largest is a lower bound L of the row's), then among the keys at or above L, which are few
// and are gathered in shared memory first.  Rows where that does not narrow the field (k above the
// subset's size, or more than kMaxCand keys at or above L) search all their keys.
constexpr int kMaxCand = 2048;
template <int EPT>
__global__ __launch_bounds__(256) void row_topk_reg_kernel(const float* __restrict__ logits, int64_t head_stride, int pitch,
                                                           const int32_t* __restrict__ text_pos, int C, int n_text,
                                                           int rows_per_head, int k_top, int causal,
                                                           float* __restrict__ row_value) {
  constexpr int NG = EPT / 32, SUB = 2 * NG, CE = kMaxCand / 256;
  __shared__ float red[4];
  __shared__ uint32_t redu[4];
  __shared__ int cnt[2][4];
  __shared__ int wcnt[4];
  __shared__ uint32_t cand_key[kMaxCand];
  __shared__ float cand_w[kMaxCand];
  const int tid = thread_index(), wv = tid >> 6;
  const int hp = blockIdx.x / rows_per_head, r = blockIdx.x % rows_per_head;
  const float* row = logits + (size_t)hp * head_stride + (size_t)r * pitch;
  const int n = causal ? min(C, text_pos[r % n_text] + 1) : C;
  const int kt = min(k_top, n);

  float v[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const int j = tid + 256 * e;
    v[e] = j < n ? row[j] : kNeg;
  }
  float m = v[0];
#pragma unroll
  for (int e = 1; e < EPT; ++e) m = fmaxf(m, v[e]);
  m = block_max(m, red);
  const uint32_t key_max = float_order_key(m);
  float z = 0.f;
  uint32_t key[EPT];
#pragma unroll
  for (int e = 0; e < EPT; ++e) {
    const bool in = tid + 256 * e < n;
    key[e] = in ? float_order_key(v[e]) : 0u;                      // 0 is below the key of every finite logit
    v[e] = in ? fast_exp2(v[e] - m) : 0.f;                         // from here on v holds the unnormalised weight
    z += v[e];
  }
  z = block_sum(z, red);

  // lower bound: the kt-th largest among the two largest keys of every group of 32 keys
  uint32_t L = 0;
  if (kt <= 256 * SUB) {                                           // block-uniform
    uint32_t sub[SUB];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      uint32_t a = 0, b = 0;
#pragma unroll
      for (int e = 0; e < 32; ++e) {
        const uint32_t k = key[g * 32 + e];
        b = max(b, min(a, k));
        a = max(a, k);
      }
      sub[2 * g] = a;
      sub[2 * g + 1] = b;
    }
    uint32_t lo = sub[0];
#pragma unroll
    for (int i = 1; i < SUB; ++i) lo = min(lo, sub[i]);
    lo = block_min_u32(lo, redu);                                  // 0 if some group has fewer than two keys
    L = block_kth_largest<SUB>(sub, kt, lo, key_max, cnt);         // 0 (no bound) if the subset has fewer than kt keys
  }

  // keys at or above L, gathered in shared memory (any order: only their count and their weights matter)
  int mine = 0;
#pragma unroll
  for (int e = 0; e < EPT; ++e)
    mine += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] != 0u && key[e] >= L));
  if ((tid & 63) == 0) wcnt[wv] = mine;
  __syncthreads();
  const int n_cand = wcnt[0] + wcnt[1] + wcnt[2] + wcnt[3];
  uint32_t thr;
  float above = 0.f, n_gt = 0.f;
  if (n_cand <= kMaxCand) {                                        // block-uniform
    int run = 0;
    for (int w = 0; w < wv; ++w) run += wcnt[w];
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      const bool take = key[e] != 0u && key[e] >= L;
      const unsigned long long bal = __builtin_amdgcn_ballot_w64(take);
      if (take) {
        const int pos = run + (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0u));
        cand_key[pos] = key[e];
        cand_w[pos] = v[e];
      }
      run += __builtin_popcountll(bal);
    }
    __syncthreads();
    uint32_t ck[CE];
    float cw[CE];
#pragma unroll
    for (int c = 0; c < CE; ++c) {
      const int idx = tid + 256 * c;
      ck[c] = idx < n_cand ? cand_key[idx] : 0u;
      cw[c] = idx < n_cand ? cand_w[idx] : 0.f;
    }
    thr = block_kth_largest<CE>(ck, kt, L, key_max, cnt);
#pragma unroll
    for (int c = 0; c < CE; ++c) {
      above += ck[c] > thr ? cw[c] : 0.f;
      n_gt += ck[c] > thr ? 1.f : 0.f;
    }
  } else {
    thr = block_kth_largest<EPT>(key, kt, 0u, key_max, cnt);
#pragma unroll
    for (int e = 0; e < EPT; ++e) {
      above += key[e] > thr ? v[e] : 0.f;
      n_gt += key[e] > thr ? 1.f : 0.f;
    }
  }
  above = block_sum(above, red);
  n_gt = block_sum(n_gt, red);             // exact: at most 2^24 keys
  // keys equal to the threshold fill the places left; a threshold that is no key of the row (the search stops
  // early at a value that separates the kt largest) leaves none, and its bit pattern need not be a number
  const float ties = (float)kt - n_gt;
  if (tid == 0) row_value[blockIdx.x] = (above + (ties > 0.f ? ties * fast_exp2(key_to_float(thr) - m) : 0.f)) / z;
}

__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
#pragma unroll
  for (int mask = 1; mask < 64; mask <<= 1) v = min(v, (uint32_t)lane_xor_i((int)v, mask));
  return v;
}
__device__ __forceinline__ float wave_max_f32(float v) {
#pragma unroll
  for (int mask = 1; mask < 64; mask <<= 1) v = fmaxf(v, lane_xor(v, mask));
  return v;
}
// Sum of a per-lane count over the wave, as a wave-uniform value (counts stay far below 2^24, so the float
// lane reduction is exact).
__device__ __forceinline__ int wave_total(int c) {
  return __builtin_amdgcn_readfirstlane((int)sum64((float)c));
}

// The kth largest of the keys one wave holds (N per lane, the first n_used registers of every lane in use;
// an absent entry holds 0), given that at least kth of them lie in [lo, hi] and none above hi: bitwise search
// on key - lo over the wave's counts.  No barrier, no memory traffic.  VOTE: the counts are taken with
// wave votes on the scalar unit (few registers per lane), else per lane with one lane reduction per step.
// STOP_EARLY = false: the search runs through all bits and returns the kth largest key itself.
template <int N, bool VOTE, bool STOP_EARLY = true>
__device__ __forceinline__ uint32_t wave_kth_largest(const uint32_t (&key)[N], int n_used, int kth, uint32_t lo,
                                                     uint32_t hi) {
  const uint32_t span = hi - lo;
  const int nbits = 32 - __builtin_clz(span | 1u);          // wave-uniform
  uint32_t thr = 0;
  for (int bit = nbits - 1; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    if (cand > span) continue;                              // no key lies above hi; keeps lo + cand <= hi
    const uint32_t x = lo + cand;
    int c = 0;
    if constexpr (VOTE) {
#pragma unroll
      for (int e = 0; e < N; ++e)
        if (e < n_used) c += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[e] >= x));   // uniform branch
    } else {
#pragma unroll
      for (int e = 0; e < N; ++e) c += key[e] >= x ? 1 : 0;
      c = wave_total(c);
    }
    if (c >= kth) thr = cand;
    // exactly kth keys at or above the candidate: it separates them from the rest, which is all the callers
    // need (a bound from below, or the sum of the weights at or above it), so the remaining bits are skipped
    if (STOP_EARLY && c == kth) break;
  }
  return lo + thr;
}

// Same result as row_topk_reg_kernel for rows of at most 64 * KPL keys, one text row per WAVE (four rows per
// workgroup): the row stays in the wave's registers (KPL values per lane), every reduction is a wave
// reduction, so a row needs no barrier at all.
// A logit v is held as key = ~bits(m - v), m the row maximum: m - v >= 0, and the bit pattern of a
// non-negative float grows with its value, so a larger logit has a larger key, the maximum has key
// 0xFFFFFFFF, and the weight comes back as exp2(-(m - v)) without any further conversion.  (Two logits whose
// distances to m round to the same float share a key; they also share the computed weight, so the sum of
// the k largest weights does not depend on which of them is taken.)
// Same two rounds as the workgroup version: lower bound from the two largest keys of every group of 32
// registers, then a search among the keys at or above it (gathered in the wave's own slice of shared
// memory; at most kWaveCand, else the wave searches all its keys).
constexpr int kWaveCand = 1024;
__device__ __forceinline__ float weight_of_key(uint32_t key) { return fast_exp2(-bits_to_float(~key)); }

template <int KPL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(KPL == 128 ? 2 : KPL == 64 ? 3 : 4)))
void row_topk_wave_kernel(const float* __restrict__ logits, int64_t head_stride, int pitch,
                          const int32_t* __restrict__ text_pos, int C, int n_text, int rows_per_head, int n_rows_total,
                          int k_top, int causal, float* __restrict__ row_value) {
  constexpr int NG = KPL / 32, SUB = 2 * NG, CW = kWaveCand / 64;
  __shared__ uint32_t cand_s[4][kWaveCand];
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int gr = blockIdx.x * 4 + wv;                               // global row of this wave
  if (gr >= n_rows_total) return;                                   // wave-uniform; no barrier below
  const int hp = gr / rows_per_head, r = gr % rows_per_head;
  const float* row = logits + (size_t)hp * head_stride + (size_t)r * pitch;
  const int n = causal ? min(C, text_pos[r % n_text] + 1) : C;
  const int kt = min(k_top, n);

  uint32_t key[KPL];                                                // first the logits' bits, then the keys, in place
  float z = 0.f;
  {
    float m = kNeg;
    if (n == 64 * KPL) {                                            // wave-uniform: a full row needs no bounds checks
#pragma unroll
      for (int e = 0; e < KPL; ++e) { key[e] = float_to_bits(row[lane + 64 * e]); m = fmaxf(m, bits_to_float(key[e])); }
    } else {
#pragma unroll
      for (int e = 0; e < KPL; ++e) {
        const int j = lane + 64 * e;
        key[e] = float_to_bits(j < n ? row[j] : kNeg);
        m = fmaxf(m, bits_to_float(key[e]));
      }
    }
    m = wave_max_f32(m);
#pragma unroll
    for (int e = 0; e < KPL; ++e) {
      const float d = m - bits_to_float(key[e]);                    // absent entries: about 1e30
      z += fast_exp2(-d);                                           // ... which adds exactly 0
      key[e] = ~float_to_bits(d);
    }
    if (n != 64 * KPL) {
#pragma unroll
      for (int e = 0; e < KPL; ++e) key[e] = lane + 64 * e < n ? key[e] : 0u;   // 0 is below every real key
    }
  }
  z = sum64(z);
  constexpr uint32_t key_max = 0xFFFFFFFFu;                         // the row maximum itself

  uint32_t L = 0;
  if (kt <= 64 * SUB) {                                             // wave-uniform
    uint32_t sub[SUB];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      uint32_t a = 0, b = 0;
#pragma unroll
      for (int e = 0; e < 32; ++e) {
        const uint32_t k = key[g * 32 + e];
        b = max(b, min(a, k));
        a = max(a, k);
      }
      sub[2 * g] = a;
      sub[2 * g + 1] = b;
    }
    uint32_t lo = sub[0];
#pragma unroll
    for (int i = 1; i < SUB; ++i) lo = min(lo, sub[i]);
    lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)wave_min_u32(lo));   // 0 if some group has fewer than two keys
    L = wave_kth_largest<SUB, true>(sub, SUB, kt, lo, key_max);     // 0 (no bound) if the subset has fewer than kt keys
  }

  const uint32_t Lc = max(L, 1u);                                   // absent entries (0) are never candidates
  int my_cand = 0;
#pragma unroll
  for (int e = 0; e < KPL; ++e) my_cand += key[e] >= Lc ? 1 : 0;
  const int n_cand = wave_total(my_cand);
  uint32_t thr;
  float above = 0.f;
  int n_gt = 0;
  if (n_cand <= kWaveCand) {                                        // wave-uniform
    // every lane writes its own candidates behind those of the lanes before it (any order will do)
    uint32_t* mine = cand_s[wv];
    int pos = wave_inclusive_scan(my_cand) - my_cand;
    uint32_t Lw = Lc;
    asm volatile("" : "+v"(Lw));            // a value of its own: the compares are redone here, one at a time,
                                            // instead of keeping KPL lane masks alive from the counting loop
#pragma unroll
    for (int e = 0; e < KPL; ++e)
      if (key[e] >= Lw) mine[pos++] = key[e];
    // the wave's shared-memory operations execute in issue order; the fences only keep the compiler from
    // moving the reads below above the writes
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    uint32_t ck[CW];
    const int n_used = (n_cand + 63) >> 6;
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      const int idx = lane + 64 * c;
      ck[c] = idx < n_cand ? mine[idx] : 0u;
    }
    thr = wave_kth_largest<CW, true>(ck, n_used, kt, L, key_max);
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      if (c < n_used) {                                             // wave-uniform
        const bool gt = ck[c] > thr;
        above += gt ? weight_of_key(ck[c]) : 0.f;
        n_gt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(gt));
      }
    }
  } else {
    thr = wave_kth_largest<KPL, false>(key, KPL, kt, 0u, key_max);
    int my_gt = 0;
#pragma unroll
    for (int e = 0; e < KPL; ++e) {
      const bool gt = key[e] > thr;
      above += gt ? weight_of_key(key[e]) : 0.f;
      my_gt += gt ? 1 : 0;
    }
    n_gt = wave_total(my_gt);
  }
  above = sum64(above);
  // keys equal to the threshold fill the places left; a threshold that is no key of the row (the search stops
  // early at a value that separates the kt largest) leaves none, and its bit pattern need not be a number
  if (lane == 0) row_value[gr] = (above + (kt > n_gt ? (float)(kt - n_gt) * weight_of_key(thr) : 0.f)) / z;
}

// ---- rows scanned on the fly (bf16, focus fraction up to 1/18) -----------------------------------------
// The two kernels below give the same row values as logits_kernel + row_topk_*_kernel without writing the
// logits out: the contraction runs once, and of every group of 16 logits of a row (the 16 that one lane
// holds for a 32-key tile) only the four largest are kept -- a quarter of the logits' bytes.
//   scan_rows_kernel   per text row: running maximum and normaliser; per (row, group): the four largest
//                      logits, in descending order.
//   row_final_kernel   one wave per row.  (1) A lower bound for the row's kt-th largest logit: the kt-th
//                      largest of the groups' two largest (of the groups' maxima on long rows).  These are
//                      different logits of the row, so the row's kt-th largest is at or above it, and every
//                      logit below the bound is out of the top kt.  With kt = 5 % of the keys about 5.4 % of
//                      the logits lie at or above the bound (9.6 % with the maxima alone).  (2) The
//                      candidates: the kept logits at or above the bound; a group whose FOURTH largest is
//                      still at or above the bound may hold more of them than were kept (about one group in
//                      a thousand), and the wave recomputes that group's 16 logits from the query row and
//                      the keys.  (3) The exact kt-th largest of the candidates (ties included) and the sum
//                      of the probabilities above it plus the admitted ties.
// Text rows run along the lanes of the 32x32 tiles (a lane owns one row of each of its wave's two row
// blocks); the rows stay in registers and the key tiles pass through shared memory once per workgroup,
// as in the window scoring of the compression pass.
// grid = (key splits, chunks of 256 rows, heads of the pass); block = 256 threads.
// Global row index R = blockIdx.z * rows + r.  part_stats [R][n_splits]; top4 [R][2][n_tiles] (group
// (half, tile) of row R holds the logits of keys 32 * tile + 8 * (i / 4) + 4 * half + i % 4, i = 0..15).
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void scan_rows_kernel(const bf16_t* __restrict__ q_layer, const bf16_t* __restrict__ k_layer,
                      const int32_t* __restrict__ text_pos, int64_t seq_start, int C, int n_text, int G,
                      int n_q_heads, int n_kv_heads, int head0, float s2, int causal, int tiles_per_block,
                      int n_splits, float2* __restrict__ part_stats, float4* __restrict__ top4) {
  constexpr int ROWB = kD * 2, NPIECE = ROWB / 32, PITCH = ROWB + 16;
  constexpr int PLANE = 64 * 16 + 16;                  // one tile's records of a wave's row block, padded
  __shared__ __attribute__((aligned(16))) char ktile[2][32 * PITCH];
  __shared__ __attribute__((aligned(16))) char rec[4][2][4 * PLANE];   // [wave][row block][tile % 4][lane] float4
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int head = head0 + blockIdx.z;
  const int rows = G * n_text;
  const int row0 = blockIdx.y * kRowsPerBlock;
  const int n_tiles_all = (C + 31) / 32;
  const int tile0 = blockIdx.x * tiles_per_block;
  const int n_tiles = min(tiles_per_block, n_tiles_all - tile0);
  const int key0 = tile0 * 32;
  const int n_my = min(2, max(0, (min(kRowsPerBlock, rows - row0) + 31) / 32 - 2 * wv));   // wave-uniform

  uint4 qreg[2][NPIECE];
  int pos_row[2];                       // prompt position of the row's text token (causal option)
  bool valid[2];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int r = row0 + (2 * wv + x) * 32 + l32;
    valid[x] = r < rows;
    pos_row[x] = 0x7fffffff;
#pragma unroll
    for (int j = 0; j < NPIECE; ++j) qreg[x][j] = make_uint4(0, 0, 0, 0);
    if (valid[x]) {
      const int g = r / n_text, t = r % n_text;
      const int p = text_pos ? text_pos[t] : t;
      if (causal) pos_row[x] = p;
      const char* src = reinterpret_cast<const char*>(q_layer) +
                        ((size_t)(seq_start + p) * n_q_heads + (size_t)head * G + g) * ROWB + half * 16;
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) qreg[x][j] = ld16(src + j * 32);
    }
  }
  float m_run[2] = {kNeg, kNeg}, z_run[2] = {0.f, 0.f};
  float4* top4_wg = top4 + ((size_t)blockIdx.z * rows + row0) * 2 * n_tiles_all;   // records of this workgroup's first row

  const char* kbase = reinterpret_cast<const char*>(k_layer) + ((size_t)seq_start * n_kv_heads + head) * ROWB;
  const uint32_t kstride = (uint32_t)n_kv_heads * ROWB;
  uint4 stage[2];
  auto fetch = [&](int kt) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p = tid + 256 * h, row = p >> 4, key = key0 + kt * 32 + row;
      stage[h] = make_uint4(0, 0, 0, 0);
      // (a row of keys is at most 16 KB long and a sequence at most 65536 tokens: the offset fits 32 bits)
      if (kt < n_tiles && key < C) stage[h] = ld16(kbase + ((uint32_t)key * kstride + (uint32_t)(p & 15) * 16u));
    }
  };
  auto park = [&](int buf) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p = tid + 256 * h;
      st16(ktile[buf] + (p >> 4) * PITCH + (p & 15) * 16, stage[h]);
    }
  };
  fetch(0);
  park(0);
  fetch(1);
  lds_barrier();
  for (int kt = 0; kt < n_tiles; ++kt) {
    const int j0 = key0 + kt * 32;
    const bool clean = !causal && j0 + 32 <= C;                 // wave-uniform: no logit of the tile is masked
    if (n_my > 0) {
      uint4 a[NPIECE];
      const char* krow = ktile[kt & 1] + l32 * PITCH + half * 16;
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) a[j] = ld16(krow + j * 32);
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        if (x >= n_my) continue;
        // acc[r] = q_row . k(j0 + 8*(r/4) + 4*half + r%4); the logit is acc[r] * s2, rounded once
        floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
        for (int j = 0; j < NPIECE; ++j) acc = mma_piece(a[j], qreg[x][j], acc, bf16_t{});
        // the selection works on the raw sums (the scale is positive); a masked logit becomes a value whose
        // scaled form still lies below every real logit and below kNeg's test in row_final_kernel
        constexpr float kRawNeg = -3.0e38f;
        if (!clean) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
            if (kk >= C || kk > pos_row[x]) acc[r] = kRawNeg;
          }
        }
        // the four largest, sorted: inserting v into t0 >= t1 >= t2 >= t3 leaves max(t0, v) first and the
        // median of each neighbouring pair with v behind it
        float t0 = kRawNeg, t1 = kRawNeg, t2 = kRawNeg, t3 = kRawNeg;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float n3 = __builtin_amdgcn_fmed3f(t2, t3, acc[r]);
          const float n2 = __builtin_amdgcn_fmed3f(t1, t2, acc[r]);
          const float n1 = __builtin_amdgcn_fmed3f(t0, t1, acc[r]);
          t0 = fmaxf(t0, acc[r]); t1 = n1; t2 = n2; t3 = n3;
        }
        t0 *= s2; t1 *= s2; t2 *= s2; t3 *= s2;                         // the logits themselves: sum * s2, rounded once
        const float mn = fmaxf(m_run[x], t0);
        float z = z_run[x] * fast_exp2(m_run[x] - mn);
#pragma unroll
        for (int r = 0; r < 16; ++r) z += fast_exp2(fmaf(acc[r], s2, -mn));   // masked: exp2 of a huge negative = 0
        z_run[x] = z; m_run[x] = mn;
        *reinterpret_cast<float4*>(rec[wv][x] + (kt & 3) * PLANE + lane * 16) = make_float4(t0, t1, t2, t3);
      }
      // every fourth tile (and after the last) the wave writes the records out: four lanes carry the four
      // tiles' records of one (row, half) list, 64 consecutive bytes in memory, 16 lists per instruction
      if ((kt & 3) == 3 || kt == n_tiles - 1) {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        const int kt4 = kt & ~3, piece = lane & 3;
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          if (x >= n_my) continue;
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int li = (lane >> 2) + 16 * i;                    // list = lane li of this wave: row li % 32, half li / 32
            const int rr = row0 + (2 * wv + x) * 32 + (li & 31);
            if (rr < rows && kt4 + piece <= kt) {
              const float4 val = *reinterpret_cast<const float4*>(rec[wv][x] + piece * PLANE + li * 16);
              // offset inside the workgroup's 256 rows: below 2^20 records
              const uint32_t off = (uint32_t)((((2 * wv + x) * 32 + (li & 31)) * 2 + (li >> 5)) * n_tiles_all + tile0 + kt4 + piece);
              top4_wg[off] = val;
            }
          }
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
      }
    }
    park((kt + 1) & 1);
    fetch(kt + 2);
    lds_barrier();
  }
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const float mo = lane_xor(m_run[x], 32), zo = lane_xor(z_run[x], 32);
    const float mn = fmaxf(m_run[x], mo);
    const float z = z_run[x] * fast_exp2(m_run[x] - mn) + zo * fast_exp2(mo - mn);
    const size_t R = (size_t)blockIdx.z * rows + row0 + (2 * wv + x) * 32 + l32;
    if (half == 0 && valid[x]) part_stats[R * n_splits + blockIdx.x] = make_float2(mn, z);
  }
}

// One text row per wave (four per workgroup); NGL = groups per lane (64 * NGL >= groups of the row).
// Candidates are held as keys ~bits(m - v) (see row_topk_wave_kernel); up to 64 * 2 * NGL of them are
// gathered in the wave's slice of shared memory and searched in registers, more (long runs of equal logits)
// go to the row's list in `spill` ([row][spill_pitch] keys) and are searched there, one pass per bit.
typedef __attribute__((ext_vector_type(2))) __bf16 bf16_pair;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {       // c + a.lo * b.lo + a.hi * b.hi
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16_pair, a), __builtin_bit_cast(bf16_pair, b), c, false);
}

constexpr int kExcList = 256;
template <int NGL>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(NGL == 8 ? 5 : NGL == 16 ? 3 : 1)))
void row_final_kernel(const float2* __restrict__ part_stats, int n_splits, const float4* __restrict__ top4, int n_tiles_all,
                      const bf16_t* __restrict__ q_layer, const bf16_t* __restrict__ k_layer,
                      const int32_t* __restrict__ text_pos, int64_t seq_start, int C, int n_text, int G, int n_q_heads,
                      int n_kv_heads, int head0, float s2, int rows_per_head, int n_rows_total, int k_top, int causal,
                      uint32_t* __restrict__ spill, int spill_pitch, float* __restrict__ row_value) {
  constexpr int CW = 2 * NGL, ROWB = kD * 2;
  constexpr bool TWO = NGL <= 16;                                   // bound from the two largest of every group
  constexpr int NK = TWO ? 2 * NGL : NGL;
  extern __shared__ uint32_t flat_s[];                              // [4][64 * CW + 64]
  __shared__ uint16_t exc_s[4 * kExcList];
  __shared__ __attribute__((aligned(16))) uint32_t hist_s[4 * 256];
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int gr = blockIdx.x * 4 + wv;
  if (gr >= n_rows_total) return;                                   // wave-uniform; no barrier below
  uint32_t* hist = hist_s + wv * 256;
  const int hp = gr / rows_per_head, r = gr % rows_per_head;
  const int g = r / n_text, tt = r % n_text;
  const int pos = text_pos ? text_pos[tt] : tt;
  const int n = causal ? min(C, pos + 1) : C;
  const int kt = min(k_top, n);
  const int n_groups = 2 * n_tiles_all;

  float m = kNeg;
  for (int s = lane; s < n_splits; s += 64) m = fmaxf(m, part_stats[(size_t)gr * n_splits + s].x);
  m = wave_max_f_dpp(m);
  float z = 0.f;
  for (int s = lane; s < n_splits; s += 64) {
    const float2 p = part_stats[(size_t)gr * n_splits + s];
    z += p.y * fast_exp2(p.x - m);
  }
  z = wave_sum_f_dpp(z);

  // the row's kept logits: lane holds groups lane, lane + 64, ...
  const float4* trow = top4 + (size_t)gr * n_groups;
  float4 T[NGL];
#pragma unroll
  for (int e = 0; e < NGL; ++e) {
    const int gi = lane + 64 * e;
    T[e] = gi < n_groups ? trow[gi] : make_float4(kNeg, kNeg, kNeg, kNeg);
  }
  // (1) the bound
  float t_lo = kNeg;
  {
    uint32_t key[NK];
    uint32_t lo = 0xFFFFFFFFu, hi = 0u;
#pragma unroll
    for (int e = 0; e < NGL; ++e) {
      const bool in = lane + 64 * e < n_groups;
      if constexpr (TWO) {
        key[2 * e] = in ? float_order_key(T[e].x) : 0u;
        key[2 * e + 1] = in ? float_order_key(T[e].y) : 0u;
        if (in) { lo = min(lo, key[2 * e + 1]); hi = max(hi, key[2 * e]); }
      } else {
        key[e] = in ? float_order_key(T[e].x) : 0u;
        if (in) { lo = min(lo, key[e]); hi = max(hi, key[e]); }
      }
    }
    lo = wave_min_u32_dpp(lo);
    hi = ~wave_min_u32_dpp(~hi);
    const int n_keys = TWO ? 2 * n_groups : n_groups;
    if (kt <= n_keys) {                                             // wave-uniform
      const int n_used = (TWO ? 2 : 1) * ((n_groups + 63) >> 6);
      // three rounds decide the top 24 bits of the span: the bound is low by a 2^-16th of its size at most
      t_lo = key_to_float(wave_radix_kth<NK>(key, n_used, kt, max(lo, 1u), hi, hist, 3));
    }
  }
  // (2) candidates.  A group whose fourth largest is a real logit at or above the bound is recomputed.
  const float tl = fmaxf(t_lo, -9.0e29f);                           // at or above the bound AND a real logit (> kNeg)
  int my_c = 0, my_x = 0;
#pragma unroll
  for (int e = 0; e < NGL; ++e) {
    const bool exc = T[e].w >= tl;
    my_x += exc ? 1 : 0;
    my_c += exc ? 0 : (T[e].x >= tl ? 1 : 0) + (T[e].y >= tl ? 1 : 0) + (T[e].z >= tl ? 1 : 0);
  }
  const int n_kept = wave_sum_i_dpp(my_c), n_exc = wave_sum_i_dpp(my_x);
  const bool in_lds = n_kept + 16 * n_exc <= 64 * CW;               // wave-uniform
  uint32_t* lds_list = flat_s + wv * (64 * CW + 64);                // 64 * CW candidates + one waste word per lane
  uint32_t* mem_list = spill + (size_t)gr * spill_pitch;
  auto key_of = [&](float v) { return ~float_to_bits(fmaxf(m - v, 0.f)); };
  auto put = [&](int at, uint32_t key) {                            // recomputed logits (few) and the spill path
    if (in_lds) lds_list[at] = key;
    else mem_list[at] = key;
  };
  {
    int at = wave_inclusive_scan_dpp(my_c) - my_c;
    if (in_lds) {
      // branch-free: a logit that is no candidate goes to the lane's waste word
      const int waste = 64 * CW + lane;
#pragma unroll
      for (int e = 0; e < NGL; ++e) {
        const bool exc = T[e].w >= tl;
        const bool c0 = !exc && T[e].x >= tl, c1 = !exc && T[e].y >= tl, c2 = !exc && T[e].z >= tl;
        lds_list[c0 ? at : waste] = key_of(T[e].x); at += c0 ? 1 : 0;
        lds_list[c1 ? at : waste] = key_of(T[e].y); at += c1 ? 1 : 0;
        lds_list[c2 ? at : waste] = key_of(T[e].z); at += c2 ? 1 : 0;
      }
    } else {
#pragma unroll
      for (int e = 0; e < NGL; ++e) {
        if (T[e].w >= tl) continue;
        if (T[e].x >= tl) mem_list[at++] = key_of(T[e].x);
        if (T[e].y >= tl) mem_list[at++] = key_of(T[e].y);
        if (T[e].z >= tl) mem_list[at++] = key_of(T[e].z);
      }
    }
  }
  int n_cand = n_kept;
  if (n_exc > 0) {                                                  // wave-uniform
    // The groups to recompute, listed in shared memory (at most kExcList; a row with more -- long runs of
    // equal logits -- takes the rest one at a time).  Lane (i = lane / 4, quarter = lane % 4) forms a
    // quarter of the dot product with the group's key i; two groups' keys are in flight at once.  A
    // recomputed logit may differ from the matrix cores' in the last bits, so the bound is taken a little
    // lower for them (more candidates never change the result).
    uint16_t* xl = exc_s + wv * kExcList;
    {
      int at = wave_inclusive_scan_dpp(my_x) - my_x;
#pragma unroll
      for (int e = 0; e < NGL; ++e) {
        const bool exc = T[e].w >= tl;
        if (exc) {
          if (at < kExcList) xl[at] = (uint16_t)(lane + 64 * e);
          ++at;
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    const float t_acc = t_lo - 1.0e-4f * fmaxf(1.f, fabsf(t_lo));
    const int ki = lane >> 2, qu = lane & 3;
    const char* qsrc = reinterpret_cast<const char*>(q_layer) +
                       ((size_t)(seq_start + pos) * n_q_heads + (size_t)(head0 + hp) * G + g) * ROWB + qu * 64;
    uint4 qp[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) qp[j] = ld16(qsrc + 16 * j);
    const char* kbase = reinterpret_cast<const char*>(k_layer) + ((size_t)seq_start * n_kv_heads + head0 + hp) * ROWB + qu * 64;
    const size_t kstride = (size_t)n_kv_heads * ROWB;
    auto key_index = [&](int gi) {
      const int hf = gi / n_tiles_all, tile = gi % n_tiles_all;
      return 32 * tile + 8 * (ki >> 2) + 4 * hf + (ki & 3);
    };
    auto finish = [&](const uint4 (&kv)[4], bool visible) {
      float acc = 0.f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        acc = dot2_bf16(kv[j].x, qp[j].x, acc);
        acc = dot2_bf16(kv[j].y, qp[j].y, acc);
        acc = dot2_bf16(kv[j].z, qp[j].z, acc);
        acc = dot2_bf16(kv[j].w, qp[j].w, acc);
      }
      acc += lane_xor(acc, 1);
      acc += lane_xor(acc, 2);
      const float v = acc * s2;
      const bool take = visible && qu == 0 && v >= t_acc;
      const uint64_t tm = __builtin_amdgcn_ballot_w64(take);
      if (take) put(n_cand + __builtin_popcountll(tm & ((1ull << lane) - 1ull)), key_of(v));
      n_cand += __builtin_popcountll(tm);
    };
    const int n_list = min(n_exc, kExcList);
    for (int i0 = 0; i0 < n_list; i0 += 2) {                        // wave-uniform
      uint4 kv[2][4];
      bool vis[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int kk = i0 + u < n_list ? key_index(xl[i0 + u]) : 0x7fffffff;
        vis[u] = kk < n;                                            // n <= C; with the causal option keys up to pos
#pragma unroll
        for (int j = 0; j < 4; ++j) kv[u][j] = vis[u] ? ld16(kbase + (size_t)kk * kstride + 16 * j) : make_uint4(0, 0, 0, 0);
      }
#pragma unroll
      for (int u = 0; u < 2; ++u)
        if (i0 + u < n_list) finish(kv[u], vis[u]);                 // wave-uniform
    }
    if (n_exc > kExcList) {
      // the list took the first kExcList groups in (lane, register) order; walk the same order over the
      // row's records in memory and skip those
      int seen = 0;
      for (int src = 0; src < 64; ++src) {
        for (int e = 0; e < NGL; ++e) {
          const int gi = src + 64 * e;
          if (gi >= n_groups) break;
          if (!(trow[gi].w >= tl)) continue;                        // wave-uniform (every lane reads the same record)
          if (seen++ < kExcList) continue;
          const int kk = key_index(gi);
          const bool visible = kk < n;
          uint4 kv[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) kv[j] = visible ? ld16(kbase + (size_t)kk * kstride + 16 * j) : make_uint4(0, 0, 0, 0);
          finish(kv, visible);
        }
      }
    }
  }
  // the wave's own writes, read back by other lanes of the wave
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");

  // (3) exact kt-th largest of the candidates
  constexpr uint32_t key_max = 0xFFFFFFFFu;                         // the row maximum itself
  uint32_t thr = 0u;
  float above = 0.f;
  int n_gt = 0;
  if (in_lds) {
    uint32_t ck[CW];
    uint32_t lo = key_max;
    const int n_used = (n_cand + 63) >> 6;
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      const int idx = lane + 64 * c;
      ck[c] = idx < n_cand ? lds_list[idx] : 0u;
      if (idx < n_cand) lo = min(lo, ck[c]);
    }
    if (n_cand > kt) {
      lo = wave_min_u32_dpp(lo);
      thr = wave_radix_kth<CW>(ck, n_used, kt, max(lo, 1u), key_max, hist);
    }                                                               // else every candidate counts: thr = 0 is below all
#pragma unroll
    for (int c = 0; c < CW; ++c) {
      if (c < n_used) {                                             // wave-uniform
        const bool gt = ck[c] > thr;
        above += gt ? weight_of_key(ck[c]) : 0.f;
        n_gt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(gt));
      }
    }
  } else {
    auto count_at_least = [&](uint32_t x, bool strictly, float* sum) {
      int c = 0;
      float s = 0.f;
      for (int j = lane; j < n_cand; j += 64) {
        const uint32_t key = mem_list[j];
        const bool in = strictly ? key > x : key >= x;
        c += in ? 1 : 0;
        s += in ? weight_of_key(key) : 0.f;
      }
      if (sum) *sum = s;
      return wave_sum_i_dpp(c);
    };
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t x = thr | (1u << bit);
      if (count_at_least(x, false, nullptr) >= kt) thr = x;
    }
    n_gt = count_at_least(thr, true, &above);
  }
  above = wave_sum_f_dpp(above);
  const int ties = min(kt, n_cand) - n_gt;      // candidates equal to the threshold fill the places left
  if (lane == 0) row_value[gr] = (above + (ties > 0 ? (float)ties * weight_of_key(thr) : 0.f)) / z;
}

// Cumulative focus count (Section 2.1, Eq. 1).  grid = rows of the pass (KV heads x G x steps), block = 256
// threads: one step's logit row of one query head per workgroup.  The k_top largest logits of the row
// (softmax is increasing, so these are the k_top most attended tokens; equal values go to the lower
// position) each add one to their token's counter.  counts: [n_q_heads][C] int32, head0 = first KV head of
// the pass.
__global__ __launch_bounds__(256) void row_focus_kernel(const float* __restrict__ logits, int64_t head_stride, int pitch,
                                                        int C, int n_steps, int rows_per_head, int k_top, int G,
                                                        int head0, int32_t* __restrict__ counts) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t bc[2];
  __shared__ int scan[6];
  const int tid = thread_index();
  const int hp = blockIdx.x / rows_per_head, r = blockIdx.x % rows_per_head;
  const float* row = logits + (size_t)hp * head_stride + (size_t)r * pitch;
  int32_t* out = counts + ((size_t)(head0 + hp) * G + r / n_steps) * C;
  const int kt = min(k_top, C);
  uint32_t t_key = 0;
  int r_adm = C;
  if (kt < C)
    radix_select<256, true>(C, kt, [&](int j, uint32_t& key) { key = float_order_key(row[j]); return true; }, hist, bc,
                            t_key, r_adm);
  int base_eq = 0;
  for (int j0 = 0; j0 < C; j0 += 256) {              // uniform trip count
    const int j = j0 + tid;
    const bool in = j < C;
    const uint32_t key = in ? float_order_key(row[j]) : 0u;
    const bool gt = in && key > t_key;
    const int eq = (in && key == t_key) ? 1 : 0;
    int tot_eq;
    const int eq_rank = base_eq + block_exclusive_scan<256>(eq, scan, &tot_eq);
    if (gt || (eq && eq_rank < r_adm)) atomicAdd(out + j, 1);
    base_eq += tot_eq;
  }
}

// grid = heads of the pass, block = 256 threads: mean of the head's row values, fixed summation order.
__global__ __launch_bounds__(256) void reduce_kernel(const float* __restrict__ row_value, int rows_per_head,
                                                     float* __restrict__ scores) {
  __shared__ float red[4];
  const int tid = thread_index();
  const float* v = row_value + (size_t)blockIdx.x * rows_per_head;
  float s = 0.f;
  for (int j = tid; j < rows_per_head; j += 256) s += v[j];
  s = block_sum(s, red);
  if (tid == 0) scores[blockIdx.x] = s / (float)rows_per_head;
}

}  // namespace hkv

using namespace hkv;

namespace {

constexpr size_t kAlignC = 256;
inline size_t align_up_c(size_t x) { return (x + kAlignC - 1) / kAlignC * kAlignC; }

// Floats per logit row: a multiple of 32 that covers n_keys, and never a multiple of 1024: rows that start
// a power-of-two number of bytes apart would all begin in the same memory channel, and the row kernels,
// which walk their rows in step, would queue up on one channel after another.
inline size_t logit_pitch(size_t n_keys) {
  size_t pitch = (n_keys + 31) / 32 * 32;
  if (pitch % 1024 == 0) pitch += 64;
  return pitch;
}

// Rows scanned on the fly (scan_rows_kernel and its companions): usable for bf16 inputs when the k-th largest
// of the groups' maxima is a useful bound, i.e. the row has clearly more groups of 16 keys than k.
constexpr int kScanTilesPerBlock = 32;
struct ScanShape {
  bool usable = false;
  int n_tiles = 0, n_splits = 0, n_groups = 0, spill_pitch = 0;
  size_t row_bytes = 0;                 // workspace bytes per text row, all arrays together
};
constexpr size_t kScanSlack = 4 * 256;  // alignment of the three arrays
ScanShape scan_shape(const hkv_config* cfg, int64_t C, int64_t k_top) {
  ScanShape sc;
  sc.n_tiles = (int)((C + 31) / 32);
  sc.n_splits = (sc.n_tiles + kScanTilesPerBlock - 1) / kScanTilesPerBlock;
  sc.n_groups = 2 * sc.n_tiles;
  sc.spill_pitch = 32 * sc.n_tiles;
  sc.usable = cfg->dtype == HKV_BF16 && k_top * 18 <= C && sc.n_groups <= 64 * 64;
  sc.row_bytes = (size_t)sc.n_splits * 8 + (size_t)sc.n_groups * 16 + (size_t)sc.spill_pitch * 4;
  return sc;
}
inline int k_top_of(double focus_fraction, int64_t C) {
  return (int)std::max<int64_t>(1, std::min<int64_t>(C, (int64_t)std::ceil(focus_fraction * (double)C - 1e-9)));
}

struct ClassifyShape {
  std::vector<int32_t> text_pos;        // all sequences, packed
  std::vector<int64_t> text_begin;      // [batch + 1]
  size_t off_pos = 0, off_rows = 0, off_logits = 0;
  size_t max_rows = 0;                  // G * T of the sequence with the most text
  size_t head_bytes_max = 0;            // logits of one head of the largest sequence
};

int classify_shape(const hkv_config* cfg, int32_t batch, const int32_t* cu, const uint8_t* is_visual, ClassifyShape& sh) {
  int rc = validate_config(cfg);
  if (rc != HKV_OK) return rc;
  if (!cu || !is_visual) return HKV_EINVAL;
  if (batch < 1 || batch > 4096 || cu[0] != 0) return HKV_ESHAPE;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  sh.text_begin.assign(batch + 1, 0);
  for (int b = 0; b < batch; ++b) {
    const int64_t C = (int64_t)cu[b + 1] - cu[b];
    if (C < 1 || C >= (1 << 24)) return HKV_ESHAPE;
    for (int64_t j = cu[b]; j < cu[b + 1]; ++j) {
      if (is_visual[j] > 1) return HKV_EINVAL;
      if (!is_visual[j]) sh.text_pos.push_back((int32_t)(j - cu[b]));
    }
    sh.text_begin[b + 1] = (int64_t)sh.text_pos.size();
    const size_t T = (size_t)(sh.text_begin[b + 1] - sh.text_begin[b]);
    const size_t pitch = logit_pitch((size_t)C);
    sh.max_rows = std::max(sh.max_rows, (size_t)G * T);
    sh.head_bytes_max = std::max(sh.head_bytes_max, (size_t)G * T * pitch * sizeof(float));
    // the scanning form's arrays for one head (whatever the focus fraction of the later call: the bound
    // holds for every k)
    sh.head_bytes_max = std::max(sh.head_bytes_max, (size_t)G * T * scan_shape(cfg, C, 1).row_bytes + kScanSlack);
  }
  sh.off_pos = 0;
  sh.off_rows = align_up_c(std::max<size_t>(1, sh.text_pos.size()) * 4);
  sh.off_logits = sh.off_rows + align_up_c(std::max<size_t>(1, (size_t)cfg->n_kv_heads * sh.max_rows) * 4);
  return HKV_OK;
}

}  // namespace

int hkv_head_scores_workspace_size(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens,
                                   const uint8_t* is_visual, size_t* min_bytes, size_t* best_bytes) {
  if (!min_bytes && !best_bytes) return HKV_EINVAL;
  ClassifyShape sh;
  int rc = classify_shape(cfg, batch, cu_seqlens, is_visual, sh);
  if (rc != HKV_OK) return rc;
  if (min_bytes) *min_bytes = sh.off_logits + align_up_c(sh.head_bytes_max);
  if (best_bytes) *best_bytes = sh.off_logits + align_up_c(sh.head_bytes_max * (size_t)cfg->n_kv_heads);
  return HKV_OK;
}

int hkv_head_scores(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens, const uint8_t* is_visual,
                    int n_layers_call, const void* q_prompt, const void* k, double focus_fraction, float* scores,
                    void* workspace, size_t workspace_bytes, void* stream) {
  ClassifyShape sh;
  int rc = classify_shape(cfg, batch, cu_seqlens, is_visual, sh);
  if (rc != HKV_OK) return rc;
  if (!q_prompt || !k || !scores || !workspace || n_layers_call < 1) return HKV_EINVAL;
  if (!(focus_fraction > 0.0) || !(focus_fraction <= 1.0)) return HKV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(q_prompt) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(workspace)) & 15u)
    return HKV_EALIGN;
  if (workspace_bytes < sh.off_logits + align_up_c(sh.head_bytes_max)) return HKV_ENOSPACE;
  const int Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, G = Hq / Hkv;
  const size_t es = cfg->dtype == HKV_BF16 ? 2 : 4;
  const int64_t total = cu_seqlens[batch];
  hipStream_t st = static_cast<hipStream_t>(stream);
  char* ws = static_cast<char*>(workspace);
  int32_t* d_pos = reinterpret_cast<int32_t*>(ws + sh.off_pos);
  float* d_rows = reinterpret_cast<float*>(ws + sh.off_rows);
  float* d_logits = reinterpret_cast<float*>(ws + sh.off_logits);
  // the text positions are the only host data the kernels need; the copy must be over before this
  // function's vectors go away, hence the one synchronisation
  if (!sh.text_pos.empty() &&
      (hipMemcpyAsync(d_pos, sh.text_pos.data(), sh.text_pos.size() * 4, hipMemcpyHostToDevice, st) != hipSuccess ||
       hipStreamSynchronize(st) != hipSuccess))
    return HKV_EHIP;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)kD);
  const float scale_log2e = scale * 1.4426950408889634f;
  const size_t logits_room = workspace_bytes - sh.off_logits;
  const size_t smem = (size_t)kRowsPerBlock * (kD * es + 16);
  static std::atomic<bool> attr_set[2] = {{false}, {false}};
  if (!attr_set[cfg->dtype == HKV_BF16].load(std::memory_order_acquire)) {
    const void* fn = cfg->dtype == HKV_BF16 ? reinterpret_cast<const void*>(&logits_kernel<bf16_t>)
                                            : reinterpret_cast<const void*>(&logits_kernel<float>);
    if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) return HKV_EHIP;
    attr_set[cfg->dtype == HKV_BF16].store(true, std::memory_order_release);
  }
  for (int l = 0; l < n_layers_call; ++l) {
    const char* q_layer = static_cast<const char*>(q_prompt) + (size_t)l * total * Hq * kD * es;
    const char* k_layer = static_cast<const char*>(k) + (size_t)l * total * Hkv * kD * es;
    for (int b = 0; b < batch; ++b) {
      const int C = cu_seqlens[b + 1] - cu_seqlens[b];
      const int T = (int)(sh.text_begin[b + 1] - sh.text_begin[b]);
      float* out = scores + ((size_t)l * batch + b) * Hkv;
      if (T == 0) {                              // no text token: the score is defined as 0
        if (hipMemsetAsync(out, 0, (size_t)Hkv * 4, st) != hipSuccess) return HKV_EHIP;
        continue;
      }
      const int rows = G * T;
      const int pitch = (int)logit_pitch((size_t)C);
      const int64_t head_stride = (int64_t)rows * pitch;
      const int heads_per_pass = (int)std::min<size_t>((size_t)Hkv, logits_room / ((size_t)head_stride * 4));
      const int k_top = k_top_of(focus_fraction, C);
      const int32_t* pos = d_pos + sh.text_begin[b];
      const ScanShape sc = scan_shape(cfg, C, k_top);
      if (sc.usable) {
        const size_t per_head = (size_t)rows * sc.row_bytes;
        const int hpp = (int)std::min<size_t>((size_t)Hkv, (logits_room - kScanSlack) / per_head);
        if (hpp < 1) return HKV_ENOSPACE;
        for (int h0 = 0; h0 < Hkv; h0 += hpp) {
          const int nh = std::min(hpp, Hkv - h0);
          const size_t nr = (size_t)nh * rows;
          char* base = reinterpret_cast<char*>(d_logits);
          size_t off = 0;
          auto take = [&](size_t bytes) { char* p = base + off; off = align_up_c(off + bytes); return p; };
          float2* d_part = reinterpret_cast<float2*>(take(nr * sc.n_splits * 8));
          float4* d_top4 = reinterpret_cast<float4*>(take(nr * sc.n_groups * 16));
          uint32_t* d_spill = reinterpret_cast<uint32_t*>(take(nr * sc.spill_pitch * 4));
          const dim3 grid(sc.n_splits, (rows + kRowsPerBlock - 1) / kRowsPerBlock, nh);
          const dim3 wgrid((unsigned)((nr + 3) / 4));
          const bf16_t* qb = reinterpret_cast<const bf16_t*>(q_layer);
          const bf16_t* kb = reinterpret_cast<const bf16_t*>(k_layer);
          hipLaunchKernelGGL(scan_rows_kernel, grid, dim3(256), 0, st, qb, kb, pos, (int64_t)cu_seqlens[b], C, T, G, Hq,
                             Hkv, h0, scale_log2e, cfg->score_causal, kScanTilesPerBlock, sc.n_splits, d_part, d_top4);
#define HKV_ROW_FINAL(NGL) \
  do { \
    constexpr size_t lds = (size_t)4 * (64 * 2 * NGL + 64) * 4; \
    static std::atomic<bool> big_lds{false}; \
    if (lds > 48 * 1024 && !big_lds.load(std::memory_order_acquire)) { \
      if (hipFuncSetAttribute(reinterpret_cast<const void*>(&row_final_kernel<NGL>), \
                              hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return HKV_EHIP; \
      big_lds.store(true, std::memory_order_release); \
    } \
    hipLaunchKernelGGL(row_final_kernel<NGL>, wgrid, dim3(256), lds, st, d_part, sc.n_splits, d_top4, sc.n_tiles, qb, kb, pos, \
                       (int64_t)cu_seqlens[b], C, T, G, Hq, Hkv, h0, scale_log2e, rows, (int)nr, k_top, cfg->score_causal, \
                       d_spill, sc.spill_pitch, d_rows); \
  } while (0)
          if (sc.n_groups <= 64 * 8) HKV_ROW_FINAL(8);
          else if (sc.n_groups <= 64 * 16) HKV_ROW_FINAL(16);
          else if (sc.n_groups <= 64 * 32) HKV_ROW_FINAL(32);
          else HKV_ROW_FINAL(64);
#undef HKV_ROW_FINAL
          hipLaunchKernelGGL(reduce_kernel, dim3(nh), dim3(256), 0, st, d_rows, rows, out + h0);
          if (hipGetLastError() != hipSuccess) return HKV_EHIP;
        }
        continue;
      }
      for (int h0 = 0; h0 < Hkv; h0 += heads_per_pass) {
        const int nh = std::min(heads_per_pass, Hkv - h0);
        const dim3 grid((C + kKeysPerLogitBlock - 1) / kKeysPerLogitBlock, (rows + kRowsPerBlock - 1) / kRowsPerBlock, nh);
        if (cfg->dtype == HKV_BF16)
          hipLaunchKernelGGL(logits_kernel<bf16_t>, grid, dim3(256), smem, st, reinterpret_cast<const bf16_t*>(q_layer),
                             reinterpret_cast<const bf16_t*>(k_layer), pos, (int64_t)cu_seqlens[b], C, T, G, Hq, Hkv, h0,
                             scale_log2e, d_logits, head_stride, pitch);
        else
          hipLaunchKernelGGL(logits_kernel<float>, grid, dim3(256), smem, st, reinterpret_cast<const float*>(q_layer),
                             reinterpret_cast<const float*>(k_layer), pos, (int64_t)cu_seqlens[b], C, T, G, Hq, Hkv, h0,
                             scale_log2e, d_logits, head_stride, pitch);
        const dim3 rgrid((unsigned)(nh * rows));
#define HKV_ROW_TOPK(KERNEL) \
  hipLaunchKernelGGL(KERNEL, rgrid, dim3(256), 0, st, d_logits, head_stride, pitch, pos, C, T, rows, k_top, \
                     cfg->score_causal, d_rows)
#define HKV_ROW_TOPK_WAVE(KERNEL) \
  hipLaunchKernelGGL(KERNEL, dim3((unsigned)((nh * rows + 3) / 4)), dim3(256), 0, st, d_logits, head_stride, pitch, pos, C, T, \
                     rows, nh * rows, k_top, cfg->score_causal, d_rows)
        if (C <= 64 * 32) HKV_ROW_TOPK_WAVE(row_topk_wave_kernel<32>);        // one row per wave, no barriers
        else if (C <= 64 * 64) HKV_ROW_TOPK_WAVE(row_topk_wave_kernel<64>);
        else if (C <= 64 * 128) HKV_ROW_TOPK_WAVE(row_topk_wave_kernel<128>);
        else if (C <= 256 * 64) HKV_ROW_TOPK(row_topk_reg_kernel<64>);
        else if (C <= 256 * 128) HKV_ROW_TOPK(row_topk_reg_kernel<128>);
        else HKV_ROW_TOPK(row_topk_kernel);      // longer rows are re-read from memory on every pass
#undef HKV_ROW_TOPK
#undef HKV_ROW_TOPK_WAVE
        hipLaunchKernelGGL(reduce_kernel, dim3(nh), dim3(256), 0, st, d_rows, rows, out + h0);
        if (hipGetLastError() != hipSuccess) return HKV_EHIP;
      }
    }
  }
  return HKV_OK;
}

// ---- budget allocation (host arithmetic, Section 3.2) ---------------------------------------------
namespace {
struct FocusShape { size_t off_logits = 0, head_bytes = 0; int pitch = 0; };
int focus_shape(const hkv_config* cfg, int32_t n_steps, int32_t context_len, FocusShape& fs) {
  int rc = validate_config(cfg);
  if (rc != HKV_OK) return rc;
  if (n_steps < 1 || n_steps > (1 << 20) || context_len < 1 || context_len >= (1 << 24)) return HKV_ESHAPE;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  fs.pitch = (int)logit_pitch((size_t)context_len);
  fs.head_bytes = (size_t)G * n_steps * fs.pitch * sizeof(float);
  fs.off_logits = 0;
  return HKV_OK;
}
}  // namespace

int hkv_focus_counts_workspace_size(const hkv_config* cfg, int32_t n_steps, int32_t context_len, size_t* min_bytes,
                                    size_t* best_bytes) {
  if (!min_bytes && !best_bytes) return HKV_EINVAL;
  FocusShape fs;
  int rc = focus_shape(cfg, n_steps, context_len, fs);
  if (rc != HKV_OK) return rc;
  if (min_bytes) *min_bytes = align_up_c(fs.head_bytes);
  if (best_bytes) *best_bytes = align_up_c(fs.head_bytes * (size_t)cfg->n_kv_heads);
  return HKV_OK;
}

int hkv_focus_counts(const hkv_config* cfg, int32_t n_steps, int32_t context_len, const void* q_steps, const void* k,
                     double focus_fraction, int32_t* counts, void* workspace, size_t workspace_bytes, void* stream) {
  FocusShape fs;
  int rc = focus_shape(cfg, n_steps, context_len, fs);
  if (rc != HKV_OK) return rc;
  if (!q_steps || !k || !counts || !workspace) return HKV_EINVAL;
  if (!(focus_fraction > 0.0) || !(focus_fraction <= 1.0)) return HKV_EINVAL;
  if ((reinterpret_cast<uintptr_t>(q_steps) | reinterpret_cast<uintptr_t>(k) | reinterpret_cast<uintptr_t>(workspace) |
       reinterpret_cast<uintptr_t>(counts)) & 15u)
    return HKV_EALIGN;
  if (workspace_bytes < align_up_c(fs.head_bytes)) return HKV_ENOSPACE;
  const int Hq = cfg->n_q_heads, Hkv = cfg->n_kv_heads, G = Hq / Hkv, C = context_len;
  const size_t es = cfg->dtype == HKV_BF16 ? 2 : 4;
  hipStream_t st = static_cast<hipStream_t>(stream);
  float* d_logits = static_cast<float*>(workspace);
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)kD);
  const float scale_log2e = scale * 1.4426950408889634f;
  const size_t smem = (size_t)kRowsPerBlock * (kD * es + 16);
  const void* fn = cfg->dtype == HKV_BF16 ? reinterpret_cast<const void*>(&logits_kernel<bf16_t>)
                                          : reinterpret_cast<const void*>(&logits_kernel<float>);
  if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem) != hipSuccess) return HKV_EHIP;
  if (hipMemsetAsync(counts, 0, (size_t)Hq * C * sizeof(int32_t), st) != hipSuccess) return HKV_EHIP;
  const int rows = G * n_steps;
  const int64_t head_stride = (int64_t)rows * fs.pitch;
  const int heads_per_pass = (int)std::min<size_t>((size_t)Hkv, workspace_bytes / fs.head_bytes);
  const int k_top = std::max(1, std::min(C, (int)std::ceil(focus_fraction * C - 1e-9)));
  for (int h0 = 0; h0 < Hkv; h0 += heads_per_pass) {
    const int nh = std::min(heads_per_pass, Hkv - h0);
    const dim3 grid((C + kKeysPerLogitBlock - 1) / kKeysPerLogitBlock, (rows + kRowsPerBlock - 1) / kRowsPerBlock, nh);
    if (cfg->dtype == HKV_BF16)
      hipLaunchKernelGGL(logits_kernel<bf16_t>, grid, dim3(256), smem, st, static_cast<const bf16_t*>(q_steps),
                         static_cast<const bf16_t*>(k), (const int32_t*)nullptr, (int64_t)0, C, n_steps, G, Hq, Hkv, h0,
                         scale_log2e, d_logits, head_stride, fs.pitch);
    else
      hipLaunchKernelGGL(logits_kernel<float>, grid, dim3(256), smem, st, static_cast<const float*>(q_steps),
                         static_cast<const float*>(k), (const int32_t*)nullptr, (int64_t)0, C, n_steps, G, Hq, Hkv, h0,
                         scale_log2e, d_logits, head_stride, fs.pitch);
    hipLaunchKernelGGL(row_focus_kernel, dim3((unsigned)(nh * rows)), dim3(256), 0, st, d_logits, head_stride, fs.pitch,
                       C, n_steps, rows, k_top, G, h0, counts);
    if (hipGetLastError() != hipSuccess) return HKV_EHIP;
  }
  return HKV_OK;
}

