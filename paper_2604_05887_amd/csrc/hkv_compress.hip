// Prefill-compression kernels of libhkv (gfx950), following the paper's Appendix A:
//   score_kernel<pass 1>  observation-window logits on the matrix cores + per-row max / sum
//   stats_finalize        combine the per-key-split row statistics in fixed order
//   score_kernel<pass 2>  same logits again, softmax with the final row statistics, mean over the
//                         G*w window rows -> relevance vector s_w over all prompt tokens
//   select_kernel         Top-M of s_w over the historical visual tokens (radix select, ties to the
//                         lower position) + window + historical text -> ascending kept positions
//   compact_kernel        fp32: copy the kept K/V rows into the head's ragged cache segment
//   adopt_kernel          fp32, dynamic heads: copy the whole K/V head-major into the cache and reduce
//                         every chunk's keys to their mean (the chunk-level index)
//   pack_rows_kernel      bf16, static heads: the compaction, into the blocked layout the matrix-core
//                         decode kernel reads (8-row blocks, V transposed inside a block)
//   adopt_blocks_kernel   bf16, dynamic heads: the whole prompt into that layout and the chunk means,
//                         from one read of K
#include "hkv_device.h"
#include "hkv_internal.h"
#include "hkv_mma.h"
#include "hkv_select.h"

namespace hkv {

// grid = (key splits, static units of the call); block = 256 threads (4 waves).
// Each block covers kKeysPerBlock keys of one static head; each wave 32 keys at a time against all
// G*w window rows (row blocks of 32).  The matrix-core tile has keys along its register/row axis and
// window rows along lanes, so row statistics reduce inside a lane and column sums across lanes.
template <typename T, int PASS>
__global__ __launch_bounds__(256) void score_kernel(CacheView cv, int layer_begin, int static_begin,
                                                    const T* __restrict__ q_window, const T* __restrict__ k,
                                                    int64_t total_tokens, float2* __restrict__ part_stats,
                                                    const float2* __restrict__ final_stats, int n_splits_max) {
  constexpr int ROWB = kD * sizeof(T);          // bytes per row
  constexpr int PITCH = ROWB + 16;              // padded shared-memory pitch (bank spread)
  constexpr int NPIECE = ROWB / 32;             // 32-byte piece pairs per row: 8 (bf16) / 16 (f32)
  constexpr int NRB = kMaxScoreRows / 32;
  extern __shared__ char qs[];                  // [rows_pad][PITCH]
  __shared__ float2 wstats[4][kMaxScoreRows];

  const int su = blockIdx.y;
  const UnitDesc d = cv.units[cv.static_units[static_begin + su]];
  const int key0 = blockIdx.x * kKeysPerBlock;
  if (key0 >= d.C) return;
  const int G = cv.G, w = cv.window;
  const int rows = G * w;
  const int n_rb = (rows + 31) / 32;
  const int lrel = d.layer - layer_begin;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;

  // stage the window queries: row r = g * w + i  <-  q_window[lrel][seq][i][head*G + g][:]
  // (eight independent loads per round: a load-then-store loop would pay one memory round trip per piece)
  {
    constexpr int PPR = ROWB / 16;              // 16-byte pieces per row
    const int n_pieces = n_rb * 32 * PPR;
    for (int base = 0; base < n_pieces; base += 256 * 8) {
      uint4 val[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int idx = base + u * 256 + tid;
        const int r = idx / PPR, piece = idx % PPR;
        val[u] = make_uint4(0, 0, 0, 0);
        if (idx < n_pieces && r < rows) {
          const int g = r / w, i = r % w;
          const size_t src = ((((size_t)lrel * cv.batch + d.seq) * w + i) * cv.n_q_heads + (size_t)d.head * G + g) * ROWB;
          val[u] = ld16(reinterpret_cast<const char*>(q_window) + src + piece * 16);
        }
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int idx = base + u * 256 + tid;
        if (idx < n_pieces) st16(qs + (size_t)(idx / PPR) * PITCH + (idx % PPR) * 16, val[u]);
      }
    }
  }
  __syncthreads();

  float m_run[NRB], z_run[NRB];
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) { m_run[rb] = kNeg; z_run[rb] = 0.f; }

  float2 fstat[NRB];                            // pass 2: this lane's rows' (maximum, 1/(Z*G*w))
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    fstat[rb] = make_float2(0.f, 0.f);
    if constexpr (PASS == 2) {
      if (rb < n_rb) fstat[rb] = final_stats[(size_t)su * kMaxScoreRows + rb * 32 + l32];
    }
  }

  const char* kbase = reinterpret_cast<const char*>(k) +
                      (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * ROWB;
  const size_t kstride = (size_t)cv.n_kv_heads * ROWB;
  const int hist_end = d.C - w;

  for (int kt = 0; kt < kKeysPerBlock / 128; ++kt) {
    const int j0 = key0 + (kt * 4 + wv) * 32;
    if (j0 >= d.C) break;                        // wave-uniform
    const int key = j0 + l32;
    uint4 a[NPIECE];
#pragma unroll
    for (int j = 0; j < NPIECE; ++j) {
      a[j] = make_uint4(0, 0, 0, 0);
      if (key < d.C) a[j] = ld16(kbase + (size_t)key * kstride + j * 32 + half * 16);
    }
    float col[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) col[r] = 0.f;
    // a tile is clean when none of its 32 keys is past the end or (with the causal option) inside the
    // window: then no logit is masked and the scale folds into the exponent's multiply-add
    const bool clean = (j0 + 32 <= d.C) && (!cv.causal || j0 + 31 <= hist_end);      // wave-uniform
    const float s2 = cv.scale_log2e;

#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      if (rb < n_rb) {
        floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        const char* qrow = qs + (size_t)(rb * 32 + l32) * PITCH + half * 16;
#pragma unroll
        for (int j = 0; j < NPIECE; ++j) acc = mma_piece(a[j], ld16(qrow + j * 32), acc, T{});
        // acc[r] = q_row(rb*32 + l32) . k(j0 + 8*(r/4) + 4*half + r%4); the logit is acc[r] * s2, and both
        // passes form "logit - row maximum" as one fused multiply-add, so they agree bit for bit
        const int qr = rb * 32 + l32;
        if (clean) {
          if constexpr (PASS == 1) {
            float mx = acc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
            const float mn = fmaxf(m_run[rb], mx * s2);
            float z = z_run[rb] * fast_exp2(m_run[rb] - mn);
#pragma unroll
            for (int r = 0; r < 16; ++r) z += fast_exp2(fmaf(acc[r], s2, -mn));
            z_run[rb] = z; m_run[rb] = mn;
          } else {
            const float2 st = fstat[rb];         // (row max, 1/(Z*G*w)); zero for pad rows
#pragma unroll
            for (int r = 0; r < 16; ++r) col[r] = fmaf(fast_exp2(fmaf(acc[r], s2, -st.x)), st.y, col[r]);
          }
        } else {
          const int qi = qr % w;                 // position of the row inside the window
          bool masked[16];
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int kk = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
            masked[r] = (kk >= d.C) || (cv.causal && kk > hist_end + qi);
          }
          if constexpr (PASS == 1) {
            float mx = kNeg;
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = masked[r] ? mx : fmaxf(mx, acc[r] * s2);
            const float mn = fmaxf(m_run[rb], mx);
            float z = z_run[rb] * fast_exp2(m_run[rb] - mn);
#pragma unroll
            for (int r = 0; r < 16; ++r) z += masked[r] ? 0.f : fast_exp2(fmaf(acc[r], s2, -mn));
            z_run[rb] = z; m_run[rb] = mn;
          } else {
            const float2 st = fstat[rb];
#pragma unroll
            for (int r = 0; r < 16; ++r)
              col[r] = masked[r] ? col[r] : fmaf(fast_exp2(fmaf(acc[r], s2, -st.x)), st.y, col[r]);
          }
        }
      }
    }
    if constexpr (PASS == 2) {
      float* sc = cv.scores + d.aux_off;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float tot = sum32(col[r]);         // over the 32 window rows held by this half-wave, then row blocks were already added
        const int kk = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
        if (l32 == 0 && kk < d.C) sc[kk] = tot;
      }
    }
  }

  if constexpr (PASS == 1) {
    // fold the two half-waves (same window row, different keys), then the four waves
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
      const float mo = lane_xor(m_run[rb], 32), zo = lane_xor(z_run[rb], 32);
      const float mn = fmaxf(m_run[rb], mo);
      z_run[rb] = z_run[rb] * fast_exp2(m_run[rb] - mn) + zo * fast_exp2(mo - mn);
      m_run[rb] = mn;
      if (half == 0) wstats[wv][rb * 32 + l32] = make_float2(m_run[rb], z_run[rb]);
    }
    __syncthreads();
    for (int r = tid; r < kMaxScoreRows; r += 256) {
      float mn = kNeg;
      for (int x = 0; x < 4; ++x) mn = fmaxf(mn, wstats[x][r].x);
      float z = 0.f;
      for (int x = 0; x < 4; ++x) z += wstats[x][r].y * fast_exp2(wstats[x][r].x - mn);
      part_stats[((size_t)su * n_splits_max + blockIdx.x) * kMaxScoreRows + r] = make_float2(mn, z);
    }
  }
}

// bf16 form of score_kernel with the window rows in registers and the keys staged through shared memory.
// The form above re-reads a query piece from LDS for every matrix instruction (1 KB per wave per
// instruction: the LDS port's whole bandwidth at full matrix rate), its 70 KB of staged rows leave two
// workgroups per compute unit, and every lane fetches its own key row from memory (32 cache lines per load
// instruction).  Here wave w keeps the two 32-row blocks 2w and 2w + 1 of the (at most 256) window rows in
// registers for the whole key range of the block; the workgroup brings every 32-key tile in once, each
// load instruction covering four whole 256-byte rows, a tile ahead of its use, and parks it in a
// double-buffered shared array from which the four waves read their operands (8 KB per wave and tile for 16
// matrix instructions).  One barrier per tile.
//   pass 1  keys along the tile's register axis, window rows along lanes: a lane owns its rows' running
//           maximum and sum outright; nothing crosses lanes until the block's end.
//   pass 2  the operands swap places -- window rows along the register axis, keys along lanes -- so the sum
//           over the rows of a column is a sum inside the lane (plus one exchange between the half-waves);
//           the weight of an element is exp2(logit - c_row) with c_row = row maximum + log2(Z * G * w), one
//           constant per row.  Per key tile a wave leaves the column sums of its rows in a shared array; the
//           four waves' sums are added in wave order when the block is done.
// grid = (key splits, static units of the call); block = 256 threads; a block covers keys_per_block keys (a
// multiple of 32, at most 32 * kScoreMaxTiles), chosen by the host so that the grid fills whole rounds of
// resident workgroups (three per compute unit).
constexpr int kScoreMaxTiles = 32;
template <int PASS>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void score_rows_kernel(CacheView cv, int layer_begin, int static_begin, const bf16_t* __restrict__ q_window,
                       const bf16_t* __restrict__ k, int64_t total_tokens, float2* __restrict__ part_stats,
                       const float2* __restrict__ final_stats, int n_splits_max, int keys_per_block) {
  constexpr int ROWB = kD * 2, NPIECE = ROWB / 32, NT = kScoreMaxTiles, PITCH = ROWB + 16;
  __shared__ __attribute__((aligned(16))) char ktile[2][32 * PITCH];   // the key tile in use and the next one
  __shared__ float colpart[PASS == 2 ? NT : 1][4][32];                  // pass 2: per key tile and wave, the column sums of the wave's rows
  __shared__ __attribute__((aligned(16))) float crow_lds[kMaxScoreRows];
  __shared__ __attribute__((aligned(16))) int qpos_lds[PASS == 2 ? kMaxScoreRows : 4];
  const int su = blockIdx.y;
  const UnitDesc d = cv.units[cv.static_units[static_begin + su]];
  const int key0 = blockIdx.x * keys_per_block;
  if (key0 >= d.C) return;
  const int G = cv.G, w = cv.window, rows = G * w;
  const int lrel = d.layer - layer_begin;
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int half = lane >> 5, l32 = lane & 31;
  const int n_my = min(2, max(0, (rows + 31) / 32 - 2 * wv));         // row blocks this wave really has (wave-uniform)

  // this lane's two window rows (row r = g * w + i), 16 bytes of every 32-byte piece pair
  uint4 qreg[2][NPIECE];
#pragma unroll
  for (int x = 0; x < 2; ++x) {
    const int r = (2 * wv + x) * 32 + l32;
#pragma unroll
    for (int j = 0; j < NPIECE; ++j) qreg[x][j] = make_uint4(0, 0, 0, 0);
    if (r < rows) {
      const int g = r / w, i = r % w;
      const char* src = reinterpret_cast<const char*>(q_window) +
                        ((((size_t)lrel * cv.batch + d.seq) * w + i) * cv.n_q_heads + (size_t)d.head * G + g) * ROWB + half * 16;
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) qreg[x][j] = ld16(src + j * 32);
    }
  }
  // pass 1: running statistics of this lane's rows.  pass 2: c_row of every window row in shared memory (a
  // lane meets 16 rows of a row block per tile and reads their constants as four broadcast 16-byte loads);
  // rows that do not exist get a constant that zeroes their weight
  float m_run[2] = {kNeg, kNeg}, z_run[2] = {0.f, 0.f};
  if constexpr (PASS == 2) {
    float c = 1.0e30f;
    if (tid < rows) {
      const float2 st = final_stats[(size_t)su * kMaxScoreRows + tid];           // (row maximum, 1 / (Z * G * w))
      c = st.x - __builtin_amdgcn_logf(st.y);                                      // log2
    }
    crow_lds[tid] = c;                          // blockDim.x == kMaxScoreRows; visible after the first barrier below
    qpos_lds[tid] = tid % w;                    // position of the row inside the window (causal masking)
  }

  const char* kbase = reinterpret_cast<const char*>(k) +
                      (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * ROWB;
  const size_t kstride = (size_t)cv.n_kv_heads * ROWB;
  const int hist_end = d.C - w;
  const float s2 = cv.scale_log2e;
  const int n_tiles = min(keys_per_block / 32, (d.C - key0 + 31) / 32);

  // staging: thread t carries the 16-byte pieces t and t + 256 of a tile (piece p = row p / 16, bytes 16 * (p % 16))
  uint4 stage[2];
  auto fetch = [&](int kt) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int p = tid + 256 * h, row = p >> 4, key = key0 + kt * 32 + row;
      stage[h] = make_uint4(0, 0, 0, 0);
      if (kt < n_tiles && key < d.C) stage[h] = ld16(kbase + (size_t)key * kstride + (p & 15) * 16);
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
    // a tile is clean when none of its 32 keys is past the end or (with the causal option) inside the
    // window: then no logit is masked
    const bool clean = (j0 + 32 <= d.C) && (!cv.causal || j0 + 31 <= hist_end);      // wave-uniform
    if (n_my > 0) {
      uint4 a[NPIECE];
      const char* krow = ktile[kt & 1] + l32 * PITCH + half * 16;
#pragma unroll
      for (int j = 0; j < NPIECE; ++j) a[j] = ld16(krow + j * 32);
      float colsum = 0.f;
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        if (x >= n_my) continue;
        floatx16 acc = {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
        if constexpr (PASS == 1) {
          // acc[r] = q_row((2*wv+x)*32 + l32) . k(j0 + 8*(r/4) + 4*half + r%4)
#pragma unroll
          for (int j = 0; j < NPIECE; ++j) acc = mma_piece(a[j], qreg[x][j], acc, bf16_t{});
          if (clean) {
            float mx = acc[0];
#pragma unroll
            for (int r = 1; r < 16; ++r) mx = fmaxf(mx, acc[r]);
            const float mn = fmaxf(m_run[x], mx * s2);
            float z = z_run[x] * fast_exp2(m_run[x] - mn);
#pragma unroll
            for (int r = 0; r < 16; ++r) z += fast_exp2(fmaf(acc[r], s2, -mn));
            z_run[x] = z; m_run[x] = mn;
          } else {
            const int qi = ((2 * wv + x) * 32 + l32) % w;       // position of the row inside the window
            bool masked[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int kk = j0 + 8 * (r >> 2) + 4 * half + (r & 3);
              masked[r] = (kk >= d.C) || (cv.causal && kk > hist_end + qi);
            }
            float mx = kNeg;
#pragma unroll
            for (int r = 0; r < 16; ++r) mx = masked[r] ? mx : fmaxf(mx, acc[r] * s2);
            const float mn = fmaxf(m_run[x], mx);
            float z = z_run[x] * fast_exp2(m_run[x] - mn);
#pragma unroll
            for (int r = 0; r < 16; ++r) z += masked[r] ? 0.f : fast_exp2(fmaf(acc[r], s2, -mn));
            z_run[x] = z; m_run[x] = mn;
          }
        } else {
          // operands swapped: acc[r] = q_row((2*wv+x)*32 + 8*(r/4) + 4*half + r%4) . k(j0 + l32)
#pragma unroll
          for (int j = 0; j < NPIECE; ++j) acc = mma_piece(qreg[x][j], a[j], acc, bf16_t{});
          float crow[16];
#pragma unroll
          for (int qd = 0; qd < 4; ++qd) {
            const float4 c4 = *reinterpret_cast<const float4*>(crow_lds + (2 * wv + x) * 32 + 8 * qd + 4 * half);
            crow[4 * qd] = c4.x; crow[4 * qd + 1] = c4.y; crow[4 * qd + 2] = c4.z; crow[4 * qd + 3] = c4.w;
          }
          if (clean) {
#pragma unroll
            for (int r = 0; r < 16; ++r) colsum += fast_exp2(fmaf(acc[r], s2, -crow[r]));
          } else {
            // key j0 + l32 is masked for a row when it lies past the end, or (causal option) behind the row's
            // own position: position in the window < key - (C - w)
            const int kk = j0 + l32;
            const int lim = kk >= d.C ? 0x7fffffff : (cv.causal ? kk - hist_end : -1);
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
              const int4 p4 = *reinterpret_cast<const int4*>(qpos_lds + (2 * wv + x) * 32 + 8 * qd + 4 * half);
              colsum += p4.x < lim ? 0.f : fast_exp2(fmaf(acc[4 * qd], s2, -crow[4 * qd]));
              colsum += p4.y < lim ? 0.f : fast_exp2(fmaf(acc[4 * qd + 1], s2, -crow[4 * qd + 1]));
              colsum += p4.z < lim ? 0.f : fast_exp2(fmaf(acc[4 * qd + 2], s2, -crow[4 * qd + 2]));
              colsum += p4.w < lim ? 0.f : fast_exp2(fmaf(acc[4 * qd + 3], s2, -crow[4 * qd + 3]));
            }
          }
        }
      }
      if constexpr (PASS == 2) {
        colsum += lane_xor(colsum, 32);            // the other half-wave holds the other 16 rows of each block
        if (half == 0) colpart[kt][wv][l32] = colsum;
      }
    }
    park((kt + 1) & 1);                            // the buffer the workgroup left at the previous barrier
    fetch(kt + 2);
    lds_barrier();
  }

  if constexpr (PASS == 1) {
    // fold the two half-waves (same window row, different keys); the rows belong to this wave alone
#pragma unroll
    for (int x = 0; x < 2; ++x) {
      const float mo = lane_xor(m_run[x], 32), zo = lane_xor(z_run[x], 32);
      const float mn = fmaxf(m_run[x], mo);
      const float z = z_run[x] * fast_exp2(m_run[x] - mn) + zo * fast_exp2(mo - mn);
      const int r = (2 * wv + x) * 32 + l32;
      if (half == 0) part_stats[((size_t)su * n_splits_max + blockIdx.x) * kMaxScoreRows + r] = make_float2(mn, z);
    }
  } else {
    const int n_wv = (rows + 63) / 64;           // waves that have rows
    float* sc = cv.scores + d.aux_off;
    for (int idx = tid; idx < n_tiles * 32; idx += 256) {
      const int kt = idx >> 5, c = idx & 31;
      float tot = 0.f;
      for (int x = 0; x < n_wv; ++x) tot += colpart[kt][x][c];
      const int kk = key0 + idx;
      if (kk < d.C) sc[kk] = tot;
    }
  }
}

// grid = static units of the call, block = kMaxScoreRows threads (one per window row).
__global__ __launch_bounds__(kMaxScoreRows) void stats_finalize_kernel(CacheView cv, int static_begin,
                                                                       const float2* __restrict__ part_stats,
                                                                       float2* __restrict__ final_stats,
                                                                       int n_splits_max, int keys_per_block) {
  const int su = blockIdx.x, r = threadIdx.x;
  const UnitDesc d = cv.units[cv.static_units[static_begin + su]];
  const int n_splits = (d.C + keys_per_block - 1) / keys_per_block;
  const int rows = cv.G * cv.window;
  float2 res = make_float2(0.f, 0.f);
  if (r < rows) {
    const float2* p = part_stats + (size_t)su * n_splits_max * kMaxScoreRows + r;
    float mn = kNeg;
    for (int s = 0; s < n_splits; ++s) mn = fmaxf(mn, p[(size_t)s * kMaxScoreRows].x);
    float z = 0.f;
    for (int s = 0; s < n_splits; ++s) {
      const float2 v = p[(size_t)s * kMaxScoreRows];
      z += v.y * fast_exp2(v.x - mn);
    }
    res = make_float2(mn, 1.0f / (z * (float)rows));
  }
  final_stats[(size_t)su * kMaxScoreRows + r] = res;
}

// grid = static units of the call, block = 1024 threads.
__global__ __launch_bounds__(1024) void select_kernel(CacheView cv, int static_begin) {
  __shared__ uint32_t hist[256];
  __shared__ uint32_t bc[2];
  __shared__ int scan[18];
  const UnitDesc d = cv.units[cv.static_units[static_begin + blockIdx.x]];
  const float* sc = cv.scores + d.aux_off;
  const uint8_t* vis = cv.is_visual + d.seq_start;
  const int C = d.C, hist_end = d.C - cv.window, mode = d.sel_mode;
  const int tid = threadIdx.x;

  auto is_cand = [&](int j) -> bool {
    if (mode == kSelVisual) return j < hist_end && vis[j] != 0;
    if (mode == kSelText) return j < hist_end && vis[j] == 0;
    return false;
  };
  auto is_fixed = [&](int j) -> bool {
    if (mode == kSelVisual) return j >= hist_end || vis[j] == 0;
    if (mode == kSelText) return j >= hist_end;
    return j >= C - d.n_prompt_rows;
  };

  uint32_t T_key = 0xFFFFFFFFu;   // nothing is greater or equal: selects no candidate
  int r_adm = 0;
  if (d.m_sel >= d.n_cand) { T_key = 0; r_adm = d.n_cand; }       // everything (keys are >= 0)
  else if (d.m_sel > 0) {
    radix_select<1024, true>(C, d.m_sel,
                       [&](int j, uint32_t& key) { if (!is_cand(j)) return false; key = float_to_bits(sc[j]); return true; },
                       hist, bc, T_key, r_adm);
  }
  int base_eq = 0, base_keep = 0;
  int32_t* kept = cv.kept_idx + d.idx_off;
  for (int j0 = 0; j0 < C; j0 += 1024) {
    const int j = j0 + tid;
    const bool in = j < C;
    const bool cand = in && is_cand(j);
    const uint32_t key = cand ? float_to_bits(sc[j]) : 0u;
    const int eq = (cand && key == T_key) ? 1 : 0;
    const int gt = (cand && key > T_key) ? 1 : 0;
    int tot_eq, tot_keep;
    const int eq_rank = base_eq + block_exclusive_scan<1024>(eq, scan, &tot_eq);
    const int keep = ((in && is_fixed(j)) ? 1 : 0) | gt | (eq & (eq_rank < r_adm ? 1 : 0));
    const int pos = base_keep + block_exclusive_scan<1024>(keep, scan, &tot_keep);
    if (keep && pos < d.n_prompt_rows) kept[pos] = j;
    base_eq += tot_eq;
    base_keep += tot_keep;
  }
}

// grid = (row tiles of 64, static units of the call); block = 256 threads.
template <typename T>
__global__ __launch_bounds__(256) void compact_kernel(CacheView cv, int layer_begin, int static_begin,
                                                      const T* __restrict__ k, const T* __restrict__ v,
                                                      int64_t total_tokens) {
  constexpr int LPR = Elem<T>::kLanesPerRow, ROWB = kD * sizeof(T);
  const UnitDesc d = cv.units[cv.static_units[static_begin + blockIdx.y]];
  const int row_base = blockIdx.x * 64;
  if (row_base >= d.n_prompt_rows) return;
  const int lrel = d.layer - layer_begin;
  const int sub = threadIdx.x % LPR, slot = threadIdx.x / LPR;
  const int32_t* kept = cv.kept_idx + d.idx_off;
  const size_t src0 = (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * ROWB;
  const size_t sstride = (size_t)cv.n_kv_heads * ROWB;
  for (int i = row_base + slot; i < row_base + 64 && i < d.n_prompt_rows; i += 256 / LPR) {
    const int pos = min(max(kept[i], 0), d.C - 1);
    const size_t src = src0 + (size_t)pos * sstride + sub * 16;
    const size_t dst = (size_t)(d.kv_row_off + i) * ROWB + sub * 16;
    st16(reinterpret_cast<char*>(cv.k_rows) + dst, ld16(reinterpret_cast<const char*>(k) + src));
    st16(reinterpret_cast<char*>(cv.v_rows) + dst, ld16(reinterpret_cast<const char*>(v) + src));
  }
}

// grid = (chunk groups of 4, dynamic units of the call); block = 256 threads, one wave per chunk.
template <typename T>
__global__ __launch_bounds__(256) void adopt_kernel(CacheView cv, int layer_begin, int dynamic_begin,
                                                    const T* __restrict__ k, const T* __restrict__ v,
                                                    int64_t total_tokens) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RPW = 64 / LPR, ROWB = kD * sizeof(T);
  const UnitDesc d = cv.units[cv.dynamic_units[dynamic_begin + blockIdx.y]];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int ch = blockIdx.x * 4 + wv;
  if (ch >= d.n_chunks) return;               // wave-uniform
  const int c = 1 << d.c_log2;
  const int r_begin = ch * c, r_end = min(r_begin + c, d.C);
  const int lrel = d.layer - layer_begin;
  const int sub = lane % LPR, grp = lane / LPR;
  const size_t src0 = (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * ROWB;
  const size_t sstride = (size_t)cv.n_kv_heads * ROWB;
  // The mean is formed exactly: the keys are summed in double precision (a sum of c fp32 values of similar
  // size has no rounding error to speak of there), divided in double precision and rounded once to the
  // cache's type, which is the definition the summaries are checked against.
  double acc[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) acc[e] = 0.0;
  for (int r = r_begin + grp; r < r_begin + c; r += RPW) {     // uniform trip count (c is a multiple of RPW)
    if (r < r_end) {
      const size_t src = src0 + (size_t)r * sstride + sub * 16;
      const size_t dst = (size_t)(d.kv_row_off + r) * ROWB + sub * 16;
      const uint4 kraw = ld16(reinterpret_cast<const char*>(k) + src);
      st16(reinterpret_cast<char*>(cv.k_dyn) + dst, kraw);
      st16(reinterpret_cast<char*>(cv.v_dyn) + dst, ld16(reinterpret_cast<const char*>(v) + src));
      float kf[EPL];
      unpack16(kraw, kf, T{});
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[e] += (double)kf[e];
    }
  }
#pragma unroll
  for (int mask = LPR; mask < 64; mask <<= 1) {
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[e] += lane_xor_f64(acc[e], mask);
  }
  if (grp == 0) {
    const double n_rows = (double)(r_end - r_begin);
    float mf[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) mf[e] = (float)(acc[e] / n_rows);      // one rounding, to nearest even
    st16(reinterpret_cast<char*>(cv.mu) + (size_t)(d.aux_off + ch) * ROWB + sub * 16, pack16(mf, T{}));
  }
}

// bf16 caches, static heads: gather the kept rows, 8 at a time, into one K block and one V block of the
// blocked layout.  grid = (groups of 4 blocks, static units of the call); block = 256 threads, one wave
// per 8-row block.
__global__ __launch_bounds__(256) void pack_rows_kernel(CacheView cv, int layer_begin, int list_begin,
                                                        const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                        int64_t total_tokens) {
  __shared__ __attribute__((aligned(16))) uint16_t vt[4][kBlkRows][kD + 8];
  const UnitDesc d = cv.units[cv.static_units[list_begin + blockIdx.y]];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int n_src = d.n_prompt_rows;
  const int blk = blockIdx.x * 4 + wv;
  const int n_blk = (n_src + kBlkRows - 1) / kBlkRows;
  if (blockIdx.x * 4 * kBlkRows >= n_src) return;           // whole workgroup beyond the unit
  const bool active = blk < n_blk;                          // wave-uniform
  const int lrel = d.layer - layer_begin;
  const size_t src0 = (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * (kD * 2);
  const size_t sstride = (size_t)cv.n_kv_heads * kD * 2;
  const int32_t* kept = cv.kept_idx + d.idx_off;
  char* kdst = reinterpret_cast<char*>(cv.k_rows) + ((size_t)d.kv_row_off / kBlkRows + blk) * kBlkBytes;
  char* vdst = reinterpret_cast<char*>(cv.v_rows) + ((size_t)d.kv_row_off / kBlkRows + blk) * kBlkBytes;
  // each lane moves two 16-byte pieces of K and of V: piece p = lane, lane + 64 -> row e = p / 16, dims 8*(p % 16)
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int p = lane + 64 * h, e = p >> 4, d8 = p & 15;
    const int r = blk * kBlkRows + e;
    uint4 kk = make_uint4(0, 0, 0, 0), vv = make_uint4(0, 0, 0, 0);
    if (active && r < n_src) {
      const int pos = min(max(kept[r], 0), d.C - 1);
      kk = ld16(reinterpret_cast<const char*>(k) + src0 + (size_t)pos * sstride + d8 * 16);
      vv = ld16(reinterpret_cast<const char*>(v) + src0 + (size_t)pos * sstride + d8 * 16);
    }
    if (active) st16(kdst + k_piece_index(e, d8) * 16, kk);
    *reinterpret_cast<uint4*>(&vt[wv][e][d8 * 8]) = vv;
  }
  __syncthreads();
  if (!active) return;
  // transpose V: lane writes the pieces of dims 2*lane and 2*lane + 1 (8 rows each)
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int dd = 2 * lane + h;
    uint4 o;
    o.x = (uint32_t)vt[wv][0][dd] | ((uint32_t)vt[wv][1][dd] << 16);
    o.y = (uint32_t)vt[wv][2][dd] | ((uint32_t)vt[wv][3][dd] << 16);
    o.z = (uint32_t)vt[wv][4][dd] | ((uint32_t)vt[wv][5][dd] << 16);
    o.w = (uint32_t)vt[wv][6][dd] | ((uint32_t)vt[wv][7][dd] << 16);
    st16(vdst + dd * 16, o);
  }
}

// bf16 caches, dynamic heads: adopt the head's whole prompt into the blocked layout AND reduce every chunk's
// keys to their mean (the chunk-level index of the paper's Appendix A) from the same read of K.
// grid = (groups of 32 prompt rows, dynamic units of the call); block = 256 threads.  A workgroup takes
// W = max(chunk size, 32) consecutive rows -- whole chunks -- so units with larger chunks use fewer of the
// grid's workgroups; wave w packs the 8-row blocks w, w + 4, ... of those rows, as pack_rows_kernel does.
// The mean is formed exactly: bf16 keys summed in double precision (no rounding at all while the chunk's
// values span fewer than 35 binary orders of magnitude), divided in double precision, rounded once to
// bf16.  Partial sums are combined in a fixed order (lanes, then waves in wave order).
__global__ __launch_bounds__(256) void adopt_blocks_kernel(CacheView cv, int layer_begin, int dynamic_begin,
                                                           const bf16_t* __restrict__ k, const bf16_t* __restrict__ v,
                                                           int64_t total_tokens) {
  __shared__ __attribute__((aligned(16))) uint16_t vt[4][kBlkRows][kD + 8];
  __shared__ double wsum[4][kD];
  const UnitDesc d = cv.units[cv.dynamic_units[dynamic_begin + blockIdx.y]];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int c = 1 << d.c_log2;
  const int W = max(c, 4 * kBlkRows);                       // rows of this workgroup
  const int row0 = blockIdx.x * W;
  if (row0 >= d.C) return;                                  // whole workgroup beyond the unit
  const int n_blk = (d.C + kBlkRows - 1) / kBlkRows;
  const int lrel = d.layer - layer_begin;
  const size_t src0 = (((size_t)lrel * total_tokens + d.seq_start) * cv.n_kv_heads + d.head) * (kD * 2);
  const size_t sstride = (size_t)cv.n_kv_heads * kD * 2;
  char* kdst0 = reinterpret_cast<char*>(cv.k_dyn) + ((size_t)d.kv_row_off / kBlkRows) * kBlkBytes;
  char* vdst0 = reinterpret_cast<char*>(cv.v_dyn) + ((size_t)d.kv_row_off / kBlkRows) * kBlkBytes;
  const int e0 = lane >> 4, d8 = lane & 15;                 // this lane's pieces: rows e0 and e0 + 4, dims 8*d8..8*d8+7
  double acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.0;
  const int blocks_per_wave = W / (4 * kBlkRows);           // uniform over the workgroup
  for (int it = 0; it < blocks_per_wave; ++it) {
    const int blk = row0 / kBlkRows + it * 4 + wv;
    const bool active = blk < n_blk;                        // wave-uniform
    uint4 kk[2], vv[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int r = blk * kBlkRows + e0 + 4 * h;
      kk[h] = make_uint4(0, 0, 0, 0); vv[h] = make_uint4(0, 0, 0, 0);
      if (active && r < d.C) {
        kk[h] = ld16(reinterpret_cast<const char*>(k) + src0 + (size_t)r * sstride + d8 * 16);
        vv[h] = ld16(reinterpret_cast<const char*>(v) + src0 + (size_t)r * sstride + d8 * 16);
      }
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (active) st16(kdst0 + (size_t)blk * kBlkBytes + k_piece_index(e0 + 4 * h, d8) * 16, kk[h]);
      *reinterpret_cast<uint4*>(&vt[wv][e0 + 4 * h][d8 * 8]) = vv[h];
      float kf[8];
      unpack16(kk[h], kf, bf16_t{});
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += (double)kf[e];  // rows past the end contribute zeros
    }
    // the wave's own staging area: written and read by this wave only
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (active) {
      // transpose V: lane writes the pieces of dims 2*lane and 2*lane + 1 (8 rows each)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int dd = 2 * lane + h;
        uint4 o;
        o.x = (uint32_t)vt[wv][0][dd] | ((uint32_t)vt[wv][1][dd] << 16);
        o.y = (uint32_t)vt[wv][2][dd] | ((uint32_t)vt[wv][3][dd] << 16);
        o.z = (uint32_t)vt[wv][4][dd] | ((uint32_t)vt[wv][5][dd] << 16);
        o.w = (uint32_t)vt[wv][6][dd] | ((uint32_t)vt[wv][7][dd] << 16);
        st16(vdst0 + (size_t)blk * kBlkBytes + dd * 16, o);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                        // the next block overwrites the staging area
  }
  // rows of the wave's blocks -> one sum per dim: fold the four row groups of the wave
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    acc[e] += lane_xor_f64(acc[e], 16);
    acc[e] += lane_xor_f64(acc[e], 32);
  }
  if (lane < 16) {
#pragma unroll
    for (int e = 0; e < 8; ++e) wsum[wv][d8 * 8 + e] = acc[e];
  }
  __syncthreads();
  // chunks of this workgroup: W / c of them (1, 2 or 4), each summed over its 4 * c / W waves in wave order
  const int n_ch = W / c, wpc = 4 / n_ch;
  for (int idx = threadIdx.x; idx < n_ch * kD; idx += 256) {
    const int j = idx / kD, dd = idx % kD;
    const int ch = row0 / c + j;
    if (ch >= d.n_chunks) continue;
    double sum = 0.0;
    for (int x = 0; x < wpc; ++x) sum += wsum[j * wpc + x][dd];
    const int n_rows = min(c, d.C - ch * c);
    reinterpret_cast<uint16_t*>(cv.mu)[(size_t)(d.aux_off + ch) * kD + dd] = f64_to_bf16_rne(sum / (double)n_rows);
  }
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
template <typename T>
static hipError_t launch_score_t(const CacheView& cv, int layer_begin, int static_begin, int n_static, int max_C,
                                 const void* q_window, const void* k, int64_t total_tokens, float2* part_stats,
                                 float2* final_stats, int keys_per_block, hipStream_t st) {
  if constexpr (sizeof(T) == 2) {
    if (keys_per_block < 32 || keys_per_block % 32 != 0 || keys_per_block > 32 * kScoreMaxTiles) return hipErrorInvalidValue;
    const int n_splits = (max_C + keys_per_block - 1) / keys_per_block;
    const dim3 grid(n_splits, n_static);
    hipLaunchKernelGGL(score_rows_kernel<1>, grid, dim3(256), 0, st, cv, layer_begin, static_begin, (const bf16_t*)q_window,
                       (const bf16_t*)k, total_tokens, part_stats, (const float2*)final_stats, n_splits, keys_per_block);
    hipLaunchKernelGGL(stats_finalize_kernel, dim3(n_static), dim3(kMaxScoreRows), 0, st, cv, static_begin,
                       (const float2*)part_stats, final_stats, n_splits, keys_per_block);
    hipLaunchKernelGGL(score_rows_kernel<2>, grid, dim3(256), 0, st, cv, layer_begin, static_begin, (const bf16_t*)q_window,
                       (const bf16_t*)k, total_tokens, part_stats, (const float2*)final_stats, n_splits, keys_per_block);
    return hipGetLastError();
  }
  const int n_splits = (max_C + kKeysPerBlock - 1) / kKeysPerBlock;
  const dim3 grid(n_splits, n_static);
  const int rows_pad = ((cv.G * cv.window + 31) / 32) * 32;
  const size_t smem = (size_t)rows_pad * (kD * sizeof(T) + 16);
  hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_kernel<T, 1>),
                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(&score_kernel<T, 2>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((score_kernel<T, 1>), grid, dim3(256), smem, st, cv, layer_begin, static_begin,
                     (const T*)q_window, (const T*)k, total_tokens, part_stats, (const float2*)final_stats, n_splits);
  hipLaunchKernelGGL(stats_finalize_kernel, dim3(n_static), dim3(kMaxScoreRows), 0, st, cv, static_begin,
                     (const float2*)part_stats, final_stats, n_splits, kKeysPerBlock);
  hipLaunchKernelGGL((score_kernel<T, 2>), grid, dim3(256), smem, st, cv, layer_begin, static_begin,
                     (const T*)q_window, (const T*)k, total_tokens, part_stats, (const float2*)final_stats, n_splits);
  return hipGetLastError();
}

hipError_t launch_score(const CacheView& cv, int dtype, int layer_begin, int static_begin, int n_static, int max_C,
                        const void* q_window, const void* k, int64_t total_tokens, float2* part_stats,
                        float2* final_stats, int keys_per_block, hipStream_t st) {
  if (n_static <= 0) return hipSuccess;
  if (dtype == HKV_F32)
    return launch_score_t<float>(cv, layer_begin, static_begin, n_static, max_C, q_window, k, total_tokens,
                                 part_stats, final_stats, keys_per_block, st);
  return launch_score_t<bf16_t>(cv, layer_begin, static_begin, n_static, max_C, q_window, k, total_tokens,
                                part_stats, final_stats, keys_per_block, st);
}

hipError_t launch_select(const CacheView& cv, int static_begin, int n_static, hipStream_t st) {
  if (n_static <= 0) return hipSuccess;
  hipLaunchKernelGGL(select_kernel, dim3(n_static), dim3(1024), 0, st, cv, static_begin);
  return hipGetLastError();
}

hipError_t launch_compact(const CacheView& cv, int dtype, int layer_begin, int static_begin, int n_static,
                          int max_rows, const void* k, const void* v, int64_t total_tokens, hipStream_t st) {
  if (n_static <= 0 || max_rows <= 0) return hipSuccess;
  if (dtype == HKV_F32)
    hipLaunchKernelGGL(compact_kernel<float>, dim3((max_rows + 63) / 64, n_static), dim3(256), 0, st, cv, layer_begin,
                       static_begin, (const float*)k, (const float*)v, total_tokens);
  else
    hipLaunchKernelGGL(pack_rows_kernel, dim3((max_rows + 4 * kBlkRows - 1) / (4 * kBlkRows), n_static),
                       dim3(256), 0, st, cv, layer_begin, static_begin, (const bf16_t*)k, (const bf16_t*)v,
                       total_tokens);
  return hipGetLastError();
}

hipError_t launch_adopt(const CacheView& cv, int dtype, int layer_begin, int dynamic_begin, int n_dynamic,
                        int max_chunks, int max_C, const void* k, const void* v, int64_t total_tokens,
                        hipStream_t st) {
  if (n_dynamic <= 0 || max_chunks <= 0) return hipSuccess;
  const dim3 grid((max_chunks + 3) / 4, n_dynamic);
  if (dtype == HKV_F32) {
    hipLaunchKernelGGL(adopt_kernel<float>, grid, dim3(256), 0, st, cv, layer_begin, dynamic_begin, (const float*)k,
                       (const float*)v, total_tokens);
  } else {
    hipLaunchKernelGGL(adopt_blocks_kernel, dim3((max_C + 4 * kBlkRows - 1) / (4 * kBlkRows), n_dynamic),
                       dim3(256), 0, st, cv, layer_begin, dynamic_begin, (const bf16_t*)k, (const bf16_t*)v,
                       total_tokens);
  }
  return hipGetLastError();
}

}  // namespace hkv
