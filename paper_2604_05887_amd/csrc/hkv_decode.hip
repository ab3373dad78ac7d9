// Decode-step kernels of libhkv (gfx950):
//   decode_kernel         a block either owns a dynamic head: it scores all chunk summaries with the
//                         group-summed query, picks the top-k chunks (paper, Appendix A, "KV Cache
//                         Retrieval for Dynamic Heads"), attends the gathered rows and combines its own
//                         tiles into the output rows (or stops after the selection); or it owns one
//                         split-K tile of a static head's compacted rows and leaves a record in the
//                         workspace
//   dynamic_tiles_kernel  split-K tiles of the dynamic heads (each repeating its head's selection when
//                         asked to), with the static heads' tiles in the same grid: the whole step in
//                         one launch
//   unit_kernel           one wide workgroup per head, selection to output rows, no records (short heads)
//   stream_kernel         every workgroup walks an equal share of the rows of all heads of the call
//   chunk_score_sum_kernel / chunk_score_max_kernel
//                         the chunk scores in a launch of their own, ahead of kernels that then only pick
//   attn_merge_kernel     log-sum-exp combination of the tiles in fixed order, cast to the output dtype
//   full_attn_kernel      the same attention over caller-held, uncompressed K/V (comparison kernel)
// The step's new K/V row is appended by the attention block whose tile contains it.
//
// All of them are short kernels on small inputs, so their structure is driven by memory latency as
// much as by bandwidth: descriptors come in through scalar loads, every thread issues its global
// loads in independent batches, and nothing walks a dependent chain longer than it must.
#include "hkv_device.h"
#include <hip/hip_ext.h>

#include <type_traits>

#include "hkv_internal.h"
#include "hkv_select.h"

#include <algorithm>
#include <atomic>

// A launch that carries start/stop events when a profiled call asks for them and is a plain launch
// otherwise (plain launches are what stream capture records).
#define HKV_LAUNCH(kernel, grid, block, smem, stream, ev0, ev1, ...)                                   \
  do {                                                                                                 \
    if ((ev0) != nullptr) hipExtLaunchKernelGGL(kernel, grid, block, smem, stream, ev0, ev1, 0u, __VA_ARGS__); \
    else hipLaunchKernelGGL(kernel, grid, block, smem, stream, __VA_ARGS__);                           \
  } while (0)

namespace hkv {

// Where the logical rows of one head live.
struct RowMap {
  const char* kbase;
  const char* vbase;
  int64_t ktail;         // blocked caches: bytes from kbase / vbase to the base of the unit's decode tail
  int64_t vtail;         //   (the tail may live in another memory than the gathered prompt rows)
  uint32_t stride;       // bytes between consecutive physical rows
  const int32_t* sel;    // dynamic: selected chunk ids (ascending)
  int32_t dynamic;
  int32_t n_sel_rows;    // dynamic: k_sel << c_log2
  int32_t c_log2;
  int32_t C;             // dynamic: prompt rows
  int32_t tail_row;      // physical row of the first appended token (row-major caches: static = retained rows, dynamic = C)
  int32_t n_chunks_prompt;   // dynamic, generated tokens indexed: picks at or above this id are chunks of the tail
  int32_t gen0;              // ... and the tail's first row that no complete chunk covers
  int32_t n_rows;        // logical rows to attend (prompt part + tail)
};

__device__ __forceinline__ bool resolve_row(const RowMap& rm, int r, int64_t& phys) {
  if (!rm.dynamic) { phys = r; return true; }
  if (r < rm.n_sel_rows) {
    const int ch = rm.sel[r >> rm.c_log2];
    phys = ((int64_t)ch << rm.c_log2) + (r & ((1 << rm.c_log2) - 1));
    return phys >= 0 && phys < rm.C;    // the last chunk of the prompt may be short
  }
  phys = (int64_t)rm.tail_row + (r - rm.n_sel_rows);
  return true;
}


// Where a tile's split-K record goes: o = [G][128] unnormalised outputs (512-byte rows), ml = [8][2]
// (running max in the log2 domain, sum) -- one fully written 64-byte line per tile.  Records are
// whole, aligned lines on purpose: partially written lines made the memory side read-modify-write
// and cost the attention kernel 8 % of its time.
struct PartOut {
  float* o;
  float* ml;
  uint16_t* out_bf16;    // not null: the tile is its unit's only one -- write the G normalised output rows (bf16)
                         // here instead of a record
  void* out_all;         // not null (bf16 caches): the call's output tensor; a split-K tile that turns out to be
                         // its unit's only tile at this step writes the unit's rows there, and the combination
                         // kernel leaves such units alone
};
constexpr int kMlStride = kMlFloats;

// Combine NS online-softmax streams staged in shared memory ([stream][G][kPartStride]: max, sum, pad,
// pad, o[128]) in stream order and store the tile's record.  All NT threads; smem must be ready.
template <int G, int NS, int NT = 256>
__device__ __forceinline__ void combine_streams_and_store(const float* smem, const PartOut& po) {
  const int tid = thread_index();
  if (po.out_bf16 != nullptr) {                 // block-uniform
    for (int idx = tid; idx < G * kD; idx += NT) {
      const int g = idx >> 7, dd = idx & (kD - 1);
      float mm = kNeg;
#pragma unroll
      for (int st = 0; st < NS; ++st) mm = fmaxf(mm, smem[(st * G + g) * kPartStride]);
      float oo = 0.f, ll = 0.f;
#pragma unroll
      for (int st = 0; st < NS; ++st) {
        const float c = fast_exp2(smem[(st * G + g) * kPartStride] - mm);
        oo = fmaf(smem[(st * G + g) * kPartStride + 4 + dd], c, oo);
        ll = fmaf(smem[(st * G + g) * kPartStride + 1], c, ll);
      }
      po.out_bf16[idx] = f32_to_bf16_rne(ll > 0.f ? oo / ll : 0.f);
    }
    return;
  }
  for (int idx = tid; idx < G * kD; idx += NT) {
    const int g = idx >> 7, dd = idx & (kD - 1);
    float mm = kNeg;
#pragma unroll
    for (int st = 0; st < NS; ++st) mm = fmaxf(mm, smem[(st * G + g) * kPartStride]);
    float oo = 0.f;
#pragma unroll
    for (int st = 0; st < NS; ++st)
      oo = fmaf(smem[(st * G + g) * kPartStride + 4 + dd], fast_exp2(smem[(st * G + g) * kPartStride] - mm), oo);
    __builtin_nontemporal_store(oo, po.o + idx);
  }
  if (tid < 8) {
    float mm = 0.f, ll = 0.f;
    if (tid < G) {
      mm = kNeg;
#pragma unroll
      for (int st = 0; st < NS; ++st) mm = fmaxf(mm, smem[(st * G + tid) * kPartStride]);
#pragma unroll
      for (int st = 0; st < NS; ++st)
        ll = fmaf(smem[(st * G + tid) * kPartStride + 1], fast_exp2(smem[(st * G + tid) * kPartStride] - mm), ll);
    }
    __builtin_nontemporal_store(mm, po.ml + 2 * tid);
    __builtin_nontemporal_store(ll, po.ml + 2 * tid + 1);
  }
}

// ---------------------------------------------------------------------------------------------
// generic tile (any dtype; used for fp32): 16 or 32 lanes per row, fp32 FMAs, wave reductions
// ---------------------------------------------------------------------------------------------
// One tile (kTileF32 logical rows starting at row0) of one KV head for its G query heads.
// Writes G records of kPartStride floats: [0]=running max (log2 domain), [1]=sum, [4..131]=unnormalised o.
template <typename T, int G>
__device__ __forceinline__ void attn_tile(const RowMap& rm, const T* __restrict__ q, float scale_log2e, int row0,
                                          const PartOut& part, float* smem) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RPW = 64 / LPR;
  constexpr int WROWS = kTileF32 / 4;
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int sub = lane % LPR, grp = lane / LPR;

  float qf[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    unpack16(ld16(reinterpret_cast<const char*>(q) + ((size_t)g * kD) * sizeof(T) + sub * 16), qf[g], T{});
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[g][e] *= scale_log2e;
  }
  float m[G], l[G], acc[G][EPL];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNeg; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < EPL; ++e) acc[g][e] = 0.f;
  }

  const int wrow0 = row0 + wv * WROWS;
  if (wrow0 < rm.n_rows) {
#pragma unroll 2
    for (int it = 0; it < WROWS / RPW; ++it) {
      const int r = wrow0 + it * RPW + grp;
      bool valid = r < rm.n_rows;
      int64_t phys = 0;
      if (valid) valid = resolve_row(rm, r, phys);
      uint4 kraw = make_uint4(0, 0, 0, 0), vraw = make_uint4(0, 0, 0, 0);
      if (valid) {
        kraw = ld16_stream(rm.kbase + phys * rm.stride + sub * 16);
        vraw = ld16_stream(rm.vbase + phys * rm.stride + sub * 16);
      }
      float kf[EPL], vf[EPL];
      unpack16(kraw, kf, T{});
      unpack16(vraw, vf, T{});
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(qf[g][e], kf[e], s);
        s = sum_lanes<LPR>(s);
        const float mn = valid ? fmaxf(m[g], s) : m[g];
        const float corr = fast_exp2(m[g] - mn);
        const float p = valid ? fast_exp2(s - mn) : 0.f;
        l[g] = fmaf(l[g], corr, p);
#pragma unroll
        for (int e = 0; e < EPL; ++e) acc[g][e] = fmaf(acc[g][e], corr, p * vf[e]);
        m[g] = mn;
      }
    }
  }
  // fold the RPW row groups of the wave together (every group ends with the wave's result)
#pragma unroll
  for (int mask = LPR; mask < 64; mask <<= 1) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float mo = lane_xor(m[g], mask), lo = lane_xor(l[g], mask);
      const float mn = fmaxf(m[g], mo);
      const float c0 = fast_exp2(m[g] - mn), c1 = fast_exp2(mo - mn);
      l[g] = l[g] * c0 + lo * c1;
#pragma unroll
      for (int e = 0; e < EPL; ++e) acc[g][e] = acc[g][e] * c0 + lane_xor(acc[g][e], mask) * c1;
      m[g] = mn;
    }
  }
  // waves -> shared memory -> one record per query head
  float* mine = smem + (size_t)wv * G * kPartStride;
  if (grp == 0) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      if (sub == 0) { mine[g * kPartStride + 0] = m[g]; mine[g * kPartStride + 1] = l[g]; }
#pragma unroll
      for (int e = 0; e < EPL; ++e) mine[g * kPartStride + 4 + sub * EPL + e] = acc[g][e];
    }
  }
  __syncthreads();
  combine_streams_and_store<G, 4>(smem, part);
}

// ---------------------------------------------------------------------------------------------
// bf16 tile: packed dot products, transpose-reduce across the 16 lanes of a row
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2bf(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2_t v = {(__bf16)lo, (__bf16)hi};        // round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}
template <int CTRL> __device__ __forceinline__ float dpp_max(float x) {
  const int xi = __builtin_bit_cast(int, x);
  return fmaxf(x, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(xi, xi, CTRL, 0xf, 0xf, false)));
}
__device__ __forceinline__ float max16(float x) {
  x = dpp_max<0xB1>(x); x = dpp_max<0x4E>(x); x = dpp_max<0x141>(x); return dpp_max<0x140>(x);
}

constexpr int kStreams = 16;          // 4 waves x 4 row groups, each an independent online-softmax stream
constexpr int kPGroupStride = 40;     // dwords per (wave, group) in the weight exchange buffer (32 + pad)
constexpr float kRescaleSlack = 8.f;  // a stream's reference maximum may lag the true one by 2^8
template <int G> constexpr size_t attn_bf16_smem_bytes() {
  return (size_t)kStreams * G * kPartStride * sizeof(float) + (size_t)kStreams * kPGroupStride * 4;
}

// One tile of 128 * NHB logical rows.  Lane (grp = lane / 16, sub = lane % 16) loads 16 bytes (8 dims)
// of row 4*i + grp for i = 0..7 of each 32-row half batch; per query head the 8 partial dot products
// are summed across the 16 lanes by a butterfly that leaves lane `sub` with the full score of row
// i = sub % 8.  Softmax weights go through shared memory as bf16 pairs of two rows so that the
// weighted sum of V uses packed dot products as well.  The softmax reference maximum of a stream is
// only raised when a score exceeds it by more than kRescaleSlack, which keeps every weight below 2^8
// and removes the rescaling of the accumulators from almost every half batch.
template <int G, int NHB, bool DYN>
__device__ __forceinline__ void attn_tile_bf16(const RowMap& rm, const bf16_t* __restrict__ q, float scale_log2e,
                                               int row0, const PartOut& part, float* smem) {
  const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  uint32_t* pbuf = reinterpret_cast<uint32_t*>(smem + (size_t)kStreams * G * kPartStride) +
                   (size_t)(wv * 4 + grp) * kPGroupStride;

  uint32_t qp[G][4];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const uint4 t = ld16(reinterpret_cast<const char*>(q) + (size_t)g * kD * 2 + sub * 16);
    qp[g][0] = t.x; qp[g][1] = t.y; qp[g][2] = t.z; qp[g][3] = t.w;
  }
  float m[G], l[G], acc[G][8];
#pragma unroll
  for (int g = 0; g < G; ++g) {
    m[g] = kNeg; l[g] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
  }
  const bool b4 = (sub & 4) != 0, b2 = (sub & 2) != 0, b1 = (sub & 1) != 0;
  const int wrow0 = __builtin_amdgcn_readfirstlane(row0 + wv * 32 * NHB);
  const uint32_t lane_off = (uint32_t)sub * 16u;
  const uint32_t cmask = (1u << rm.c_log2) - 1u;

#pragma unroll 1
  for (int hb = 0; hb < NHB; ++hb) {
    const int rbase = wrow0 + hb * 32;
    if (rbase >= rm.n_rows) break;                       // wave-uniform
    // ---- addresses: invalid rows are redirected to a row that exists and masked out below ----
    uint32_t off[8];
    uint32_t vmask = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + 4 * i + grp;
      uint32_t phys;
      bool valid;
      if constexpr (!DYN) {
        valid = r < rm.n_rows;
        phys = (uint32_t)min(r, rm.n_rows - 1);
      } else {
        if (rbase + 4 * i < rm.n_sel_rows) {              // wave-uniform: chunks are multiples of 4 rows
          const int ch = rm.sel[(rbase + 4 * i) >> rm.c_log2];
          phys = ((uint32_t)ch << rm.c_log2) + ((uint32_t)r & cmask);
          valid = phys < (uint32_t)rm.C;                  // the last chunk of the prompt may be short
        } else {
          phys = (uint32_t)rm.tail_row + (uint32_t)(r - rm.n_sel_rows);
          valid = r < rm.n_rows;
        }
        phys = valid ? phys : 0u;
      }
      off[i] = __umul24(phys, rm.stride) + lane_off;   // < 2^32 (checked on the host)
      vmask |= valid ? (1u << i) : 0u;
    }
    uint4 kraw[8], vraw[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) kraw[i] = ld16_stream(rm.kbase + off[i]);
#pragma unroll
    for (int i = 0; i < 8; ++i) vraw[i] = ld16_stream(rm.vbase + off[i]);

    // ---- scores: partial dot products, all-reduce over the mirror pair, then reduce-scatter ----
    float v[8][G];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        float s = dot2bf(kraw[i].x, qp[g][0], 0.f);
        s = dot2bf(kraw[i].y, qp[g][1], s);
        s = dot2bf(kraw[i].z, qp[g][2], s);
        s = dot2bf(kraw[i].w, qp[g][3], s);
        v[i][g] = s + dpp_mov<0x140>(s);                 // row_mirror: lanes sub and 15 - sub
      }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float keep = b4 ? v[i + 4][g] : v[i][g], send = b4 ? v[i][g] : v[i + 4][g];
        v[i][g] = keep + dpp_mov<0x141>(send);           // row_half_mirror: partner sub ^ 7
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float keep = b2 ? v[i + 2][g] : v[i][g], send = b2 ? v[i][g] : v[i + 2][g];
        v[i][g] = keep + dpp_mov<0x4E>(send);            // quad_perm [2,3,0,1]: partner sub ^ 2
      }
    }
    const bool my_valid = (vmask >> (sub & 7)) & 1u;     // lane sub now owns row i = sub & 7 of its group
    float s[G];
    bool raise = false;
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float keep = b1 ? v[1][g] : v[0][g], send = b1 ? v[0][g] : v[1][g];
      const float x = (keep + dpp_mov<0xB1>(send)) * scale_log2e;   // quad_perm [1,0,3,2]: partner sub ^ 1
      s[g] = my_valid ? x : kNeg;
      raise |= s[g] > m[g] + kRescaleSlack;
    }
    if (__builtin_amdgcn_ballot_w64(raise) != 0) {       // wave-uniform and rare after the first half batch
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float mn = fmaxf(m[g], max16(s[g]));       // maximum over the row group's rows
        const float corr = fast_exp2(m[g] - mn);
        l[g] *= corr;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] *= corr;
        m[g] = mn;
      }
    }
    // ---- weights -> shared memory as bf16 pairs of rows (2t, 2t+1): dword [t][g] ----
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float p = my_valid ? fast_exp2(s[g] - m[g]) : 0.f;
      l[g] += p;                                         // lanes sub >= 8 hold duplicates; dropped at the end
      const float pn = dpp_mov<0xB1>(p);                 // weight of the next row (lane sub ^ 1)
      if ((sub & 9) == 0) pbuf[(sub >> 1) * 8 + g] = pack_bf16(p, pn);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // ---- weighted sum of V: two rows per packed dot product ----
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      uint32_t pp[8];
      const uint4 p0 = *reinterpret_cast<const uint4*>(pbuf + t * 8);
      pp[0] = p0.x; pp[1] = p0.y; pp[2] = p0.z; pp[3] = p0.w;
      if constexpr (G > 4) {
        const uint4 p1 = *reinterpret_cast<const uint4*>(pbuf + t * 8 + 4);
        pp[4] = p1.x; pp[5] = p1.y; pp[6] = p1.z; pp[7] = p1.w;
      }
      const uint32_t va[4] = {vraw[2 * t].x, vraw[2 * t].y, vraw[2 * t].z, vraw[2 * t].w};
      const uint32_t vb[4] = {vraw[2 * t + 1].x, vraw[2 * t + 1].y, vraw[2 * t + 1].z, vraw[2 * t + 1].w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t lo = __builtin_amdgcn_perm(vb[j], va[j], 0x05040100u);   // (va.lo16, vb.lo16)
        const uint32_t hi = __builtin_amdgcn_perm(vb[j], va[j], 0x07060302u);   // (va.hi16, vb.hi16)
#pragma unroll
        for (int g = 0; g < G; ++g) {
          acc[g][2 * j] = dot2bf(lo, pp[g], acc[g][2 * j]);
          acc[g][2 * j + 1] = dot2bf(hi, pp[g], acc[g][2 * j + 1]);
        }
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();                     // the next half batch overwrites pbuf
  }

  // every (wave, row group) is one stream: (m, l, acc) -> shared memory -> fixed-order combination
  float* mine = smem + (size_t)(wv * 4 + grp) * G * kPartStride;
#pragma unroll
  for (int g = 0; g < G; ++g) {
    const float lt = sum16(sub < 8 ? l[g] : 0.f);
    if (sub == 0) { mine[g * kPartStride + 0] = m[g]; mine[g * kPartStride + 1] = lt; }
    float4* dst = reinterpret_cast<float4*>(mine + g * kPartStride + 4 + sub * 8);
    dst[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
    dst[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
  }
  __syncthreads();
  combine_streams_and_store<G, kStreams>(smem, part);
}

// ---------------------------------------------------------------------------------------------
// bf16 tile on the matrix cores, for caches in the blocked layout (hkv_internal.h)
// ---------------------------------------------------------------------------------------------
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;

// Physical 8-row block that holds logical rows Lr .. Lr+7 (Lr a multiple of 8) and how many of them
// are real (0..8).  A block with no real row is redirected to block 0, which always exists.
template <int DYN>
__device__ __forceinline__ void resolve_block(const RowMap& rm, int Lr, uint32_t& blk, int& nv, bool& tail) {
  int pb;
  tail = false;
  if constexpr (DYN == 0) {
    pb = Lr;
    nv = rm.n_rows - Lr;
  } else {
    if (Lr < rm.n_sel_rows) {
      const int ch = rm.sel[Lr >> rm.c_log2];
      const int off = Lr & ((1 << rm.c_log2) - 1);
      if (DYN == 2 && ch >= rm.n_chunks_prompt) {       // a complete chunk of generated tokens
        pb = ((ch - rm.n_chunks_prompt) << rm.c_log2) + off;
        nv = kBlkRows;
        tail = true;
      } else {
        pb = (ch << rm.c_log2) + off;
        nv = rm.C - pb;                                 // the last chunk of the prompt may be short
      }
    } else {
      pb = (DYN == 2 ? rm.gen0 : 0) + (Lr - rm.n_sel_rows);   // row of the tail, counted from the tail's base
      nv = rm.n_rows - Lr;
      tail = true;
    }
  }
  nv = min(max(nv, 0), kBlkRows);
  blk = nv > 0 ? (uint32_t)pb >> 3 : 0u;
  if (nv <= 0) tail = false;
}

// Operands of one 32-row step in flight: eight 16-byte K pieces and eight V pieces per lane, and how many
// of the 8 rows of this lane's V block exist.
struct StepBufs {
  uint4 ka[8], va[8];
  int nv;
};

// Issues the loads of step `st` of the tile at row0 for this lane (wave-uniform st).  Rows past the end of
// the unit resolve to its block 0 with no valid rows, so any step number is safe to ask for.
template <int DYN>
__device__ __forceinline__ void issue_step_loads(const RowMap& rm, int row0, int st, StepBufs& sb) {
  const int lane = thread_index() & 63;
  const int qi = lane & 15, jv = lane >> 4, ja = qi >> 2, e1 = lane & 3;
  uint32_t ba, bv;
  int unused;
  bool ta, tv;
  resolve_block<DYN>(rm, row0 + st * 32 + 8 * ja, ba, unused, ta);
  resolve_block<DYN>(rm, row0 + st * 32 + 8 * jv, bv, sb.nv, tv);
  const char* kp = rm.kbase + ((int64_t)ba * kBlkBytes + (ta ? rm.ktail : (int64_t)0)) + (uint32_t)(jv * 4 + e1) * 16u;
  const char* vp = rm.vbase + ((int64_t)bv * kBlkBytes + (tv ? rm.vtail : (int64_t)0)) + (uint32_t)qi * 16u;
#pragma unroll
  for (int i = 0; i < 8; ++i) sb.ka[i] = ld16_stream(kp + i * 256);     // i = 2 * kstep + half tile
#pragma unroll
  for (int i = 0; i < 8; ++i) sb.va[i] = ld16_stream(vp + i * 256);     // i = 16-dim block of the output
}

struct NoHook { __device__ __forceinline__ void operator()() const {} };

// One tile of `tile_rows` logical rows (a multiple of 32).  The tile is cut into steps of 32 keys;
// wave w of the NW waves of the workgroup takes steps w, w+NW, w+2NW, ... and keeps one step of loads in
// flight ahead of its arithmetic.
// Scores S^T = K Q^T: the A operand is a K block piece (key-major), the B operand the query rows
// (zero beyond G), so lane (q = lane % 16, j = lane / 16) ends with the scores of query head q for
// the 8 rows of block j of the step -- which is exactly the B operand the second contraction
// O^T += V^T P^T needs from that lane, so the weights never move between lanes.  The A operand of the
// second contraction is a 16-byte piece of the transposed V block.  No operand is staged through LDS.
// `sb` holds the operands in flight; with `preloaded` the caller has already issued this wave's first
// step into it.  `between` runs after the last step's arithmetic and before the combination of the
// waves, when `sb` is free again (a hook for callers that overlap something with the combination).
template <int G, int DYN, class Between = NoHook, int NW = 4>
__device__ __forceinline__ void attn_tile_mfma(const RowMap& rm, const bf16_t* __restrict__ q, float scale_log2e,
                                               int row0, int tile_rows, const PartOut& part, float* smem,
                                               StepBufs& sb, bool preloaded = false, Between between = Between()) {
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int qi = lane & 15, jv = lane >> 4, ja = qi >> 2, e1 = lane & 3;

  bf16x8 qb[4];
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    uint4 t = make_uint4(0, 0, 0, 0);
    if (qi < G) t = ld16(reinterpret_cast<const char*>(q) + (size_t)qi * kD * 2 + (32 * s + 8 * jv) * 2);
    qb[s] = __builtin_bit_cast(bf16x8, t);
  }
  const int rows_here = min(tile_rows, rm.n_rows - row0);
  const int n_steps = (rows_here + 31) >> 5;
  const uint32_t k_lane = (uint32_t)(jv * 4 + e1) * 16u, v_lane = (uint32_t)qi * 16u;

  floatx4 o[8];
#pragma unroll
  for (int db = 0; db < 8; ++db) o[db] = floatx4{0.f, 0.f, 0.f, 0.f};
  float m = kNeg, lsum = 0.f;

  uint4 (&ka)[8] = sb.ka;
  uint4 (&va)[8] = sb.va;
  int st = wv;                                           // wave-uniform
  if (st < n_steps && !preloaded) issue_step_loads<DYN>(rm, row0, st, sb);
  int nv = sb.nv;
#pragma unroll 1
  while (st < n_steps) {
    floatx4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[2 * s]), qb[s], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[2 * s + 1]), qb[s], s1, 0, 0, 0);
    }
    // next step's addresses and K loads go out while this step's softmax and second contraction run
    const int nst = st + NW;
    const bool more = nst < n_steps;                     // wave-uniform
    uint32_t bv_next = 0;
    int nv_next = 0;
    bool tv_next = false;
    if (more) {
      uint32_t ba;
      int unused;
      bool ta;
      resolve_block<DYN>(rm, row0 + nst * 32 + 8 * ja, ba, unused, ta);
      resolve_block<DYN>(rm, row0 + nst * 32 + 8 * jv, bv_next, nv_next, tv_next);
      const char* kp = rm.kbase + ((int64_t)ba * kBlkBytes + (ta ? rm.ktail : (int64_t)0)) + k_lane;
#pragma unroll
      for (int i = 0; i < 8; ++i) ka[i] = ld16_stream(kp + i * 256);
    }
    float sc[8];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sc[e] = e < nv ? s0[e] * scale_log2e : kNeg;        // rows 0..3 of block jv
      sc[e + 4] = e + 4 < nv ? s1[e] * scale_log2e : kNeg;  // rows 4..7
    }
    float mx = sc[0];
#pragma unroll
    for (int e = 1; e < 8; ++e) mx = fmaxf(mx, sc[e]);
    if (__builtin_amdgcn_ballot_w64(mx > m + kRescaleSlack) != 0) {   // wave-uniform, rare after the first step
      mx = fmaxf(mx, lane_xor(mx, 16));
      mx = fmaxf(mx, lane_xor(mx, 32));                  // over the four lanes that share a query head
      const float mn = fmaxf(m, mx);
      const float corr = fast_exp2(m - mn);
      lsum *= corr;
#pragma unroll
      for (int db = 0; db < 8; ++db) o[db] *= corr;
      m = mn;
    }
    float p[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      p[e] = e < nv ? fast_exp2(sc[e] - m) : 0.f;
      lsum += p[e];
    }
    uint4 pw;
    pw.x = pack_bf16(p[0], p[1]); pw.y = pack_bf16(p[2], p[3]);
    pw.z = pack_bf16(p[4], p[5]); pw.w = pack_bf16(p[6], p[7]);
    const bf16x8 pb = __builtin_bit_cast(bf16x8, pw);
#pragma unroll
    for (int db = 0; db < 8; ++db)
      o[db] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, va[db]), pb, o[db], 0, 0, 0);
    if (more) {
      const char* vp = rm.vbase + ((int64_t)bv_next * kBlkBytes + (tv_next ? rm.vtail : (int64_t)0)) + v_lane;
#pragma unroll
      for (int i = 0; i < 8; ++i) va[i] = ld16_stream(vp + i * 256);
    }
    nv = nv_next;
    st = nst;
  }

  between();
  lsum += lane_xor(lsum, 16);
  lsum += lane_xor(lsum, 32);
  float* mine = smem + (size_t)wv * G * kPartStride;
  if (qi < G) {
    if (jv == 0) { mine[qi * kPartStride] = m; mine[qi * kPartStride + 1] = lsum; }
#pragma unroll
    for (int db = 0; db < 8; ++db)      // o[db][r] is output dim 16*db + 4*jv + r of query head qi
      *reinterpret_cast<float4*>(mine + qi * kPartStride + 4 + 16 * db + 4 * jv) =
          make_float4(o[db][0], o[db][1], o[db][2], o[db][3]);
  }
  lds_barrier();                       // staging is LDS only; loads for the next tile may be in flight
  combine_streams_and_store<G, NW, NW * 64>(smem, part);
}

constexpr int kNhbBf16 = kTileBf16 / 128;
// BLOCKED: the K/V rows are in the blocked cache layout (bf16 caches) -> matrix-core tile.
template <typename T, int G, bool BLOCKED> constexpr size_t attn_smem_bytes() {
  if constexpr (sizeof(T) == 2 && !BLOCKED) return attn_bf16_smem_bytes<G>();
  else return (size_t)4 * G * kPartStride * sizeof(float);
}
template <typename T> __device__ __forceinline__ constexpr int tile_of() { return sizeof(T) == 2 ? kTileBf16 : kTileF32; }

template <typename T, int G, bool BLOCKED, int NW = 4, bool INDEXED = false>
__device__ __forceinline__ void run_tile(const RowMap& rm, const T* __restrict__ q, float scale_log2e, int row0,
                                         int tile_rows, const PartOut& part, float* smem) {
  if constexpr (sizeof(T) == 2 && BLOCKED) {
    StepBufs sb;
    sb.nv = 0;
    if constexpr (INDEXED) {               // kernels of caches that index their generated tokens
      if (rm.dynamic) attn_tile_mfma<G, 2, NoHook, NW>(rm, q, scale_log2e, row0, tile_rows, part, smem, sb);
      else attn_tile_mfma<G, 0, NoHook, NW>(rm, q, scale_log2e, row0, tile_rows, part, smem, sb);
      return;
    }
    if (rm.dynamic) attn_tile_mfma<G, 1, NoHook, NW>(rm, q, scale_log2e, row0, tile_rows, part, smem, sb);
    else attn_tile_mfma<G, 0, NoHook, NW>(rm, q, scale_log2e, row0, tile_rows, part, smem, sb);
  } else if constexpr (sizeof(T) == 2) {
    attn_tile_bf16<G, kNhbBf16, false>(rm, q, scale_log2e, row0, part, smem);   // row-major rows, never gathered
  } else {
    attn_tile<T, G>(rm, q, scale_log2e, row0, part, smem);
  }
}

// Combine the n_tiles records of one (unit, query head) in tile order -- eight records per round
// of independent loads -- and write the output row.  blockDim.x == 128, one thread per element.
// o0 / ml0 point at the first tile's entries for this query head; consecutive tiles are rec_o floats
// (resp. kMlStride floats) apart.
template <typename T>
__device__ __forceinline__ void merge_head(const float* __restrict__ o0, const float* __restrict__ ml0, int n_tiles,
                                           int rec_o, T* __restrict__ out_row) {
  const int dd = threadIdx.x;
  float M = kNeg, L = 0.f, O = 0.f;
  for (int t0 = 0; t0 < n_tiles; t0 += 8) {
    float mv[8], lv[8], ov[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool in = t0 + j < n_tiles;
      const int t = in ? t0 + j : t0;
      const float2 ml = *reinterpret_cast<const float2*>(ml0 + (size_t)t * kMlStride);
      mv[j] = in ? ml.x : kNeg; lv[j] = in ? ml.y : 0.f; ov[j] = in ? o0[(size_t)t * rec_o + dd] : 0.f;
    }
    float bm = mv[0];
#pragma unroll
    for (int j = 1; j < 8; ++j) bm = fmaxf(bm, mv[j]);
    const float Mn = fmaxf(M, bm);
    const float c = fast_exp2(M - Mn);
    L *= c; O *= c;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float cj = fast_exp2(mv[j] - Mn);
      L = fmaf(lv[j], cj, L);
      O = fmaf(ov[j], cj, O);
    }
    M = Mn;
  }
  const float o = L > 0.f ? O / L : 0.f;
  if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(out_row)[dd] = o;
  else reinterpret_cast<uint16_t*>(out_row)[dd] = f32_to_bf16_rne(o);
}

// ------------------------------------------------------------------------------------------
// hybrid cache kernels
// ------------------------------------------------------------------------------------------
// A decode step runs in one of two shapes, fixed when the cache is laid out.
// Fused (dynamic heads of moderate length):
//   1  decode_kernel: blocks [0, n_dyn) each own one dynamic unit of the call -- chunk selection, then
//      attention over all gathered rows, then the unit's output rows; the remaining blocks run the
//      split-K tiles of the static units.  The two kinds of work do not depend on each other, and the
//      dynamic blocks -- the longest dependent chains -- are dispatched first, so their latency hides
//      behind the static heads' streaming.
//   2  attn_merge_kernel over the static units only.
// Split (large steps, bound by memory throughput):
//   1  decode_kernel with the dynamic blocks stopping after the chunk selection,
//   2  dynamic_tiles_kernel: split-K tiles of the dynamic units (they need the picks),
//   3  attn_merge_kernel over all units.
// Repeated selection (small steps, bound by the chain of dependent launches): one launch of
// dynamic_tiles_kernel over all tiles, every dynamic tile repeating its head's chunk selection (the
// summaries are a small fraction of the step and mostly come from the L2), then attn_merge_kernel
// over all units.
// The step's new K/V row is written by the one block whose tile contains it, before that block reads;
// the block that owns the first tile of (sequence 0, head 0) moves the layer's tail counter on.
// Tail length: t_arg >= 0 is the length before this step, known to the host, and the counter is
// updated in place since nobody reads it; t_arg < 0 reads the device counter cnt_a[layer], the new
// length goes to cnt_b, and a follow-up kernel publishes it once every reader is done.

// Top-k of up to 64 * R chunk scores held in shared memory (sig), without block-wide passes: every wave
// keeps all keys in registers (R per lane; chunk 64 * m + lane in register m) and wave 0 searches.
// k <= 32: the k-th largest of the 64 lanes' largest keys, to its upper 20 bits, is a lower bound for the
// k-th largest key (k of the lanes' maxima reach it) that usually leaves little more than k keys at or above it
// (for k = 32 it is the median of the lanes' maxima: about 45 of 1000 keys reach it).  32 < k <= kBoundPicks: the
// same with every lane's two largest keys, 128 values.
// If at most 64 keys reach the bound (128 in the second case), they go to one lane each (two a lane), in chunk
// order; a bitwise search on wave votes over that register (those two) finds the k-th largest exactly, and the
// picks -- keys above it, those equal to it in chunk order up to the k-th place -- leave from there, ascending
// by chunk id.  (Scores of one head share their sign and
// size: over the whole key range a radix round's histogram adds all hit the same few words.)
// Otherwise: wave 0 finds the k-th largest key by radix selection on its own histogram; after the one barrier
// that hands it over, every wave counts with wave votes, and wave m % 4 emits the picks of register m.
// All NT threads call (the barrier); waves beyond the fourth only take part in it.
constexpr int kBoundPicks = 64;
// The search from the lanes' largest keys (TWO: largest and second largest, for 32 < k <= 64) described above, by one
// wave; false if more keys reach the bound than there are candidate places (64, TWO: 128), nothing written then.
// lane_max = this lane's largest key, hi = the largest key of all; cand_lds: 128 (key, chunk id) pairs.
template <int R, bool TWO>
__device__ __forceinline__ bool topk_from_lane_maxima(const uint32_t (&key)[R], int k, uint32_t lane_max, uint32_t hi,
                                                      uint2* cand_lds, bool to_memory, int32_t* sel_mem, int32_t* sel_lds) {
  const int lane = thread_index() & 63;
  constexpr int kPlaces = TWO ? 128 : 64;
  uint32_t second = 0u;                                      // this lane's second largest key (an equal one counts)
  if constexpr (TWO) {
    uint32_t first = 0u;
#pragma unroll
    for (int m = 0; m < R; ++m) { second = max(second, min(first, key[m])); first = max(first, key[m]); }
  }
  auto reach = [&](uint32_t t) {                             // how many of the lanes' keys in play reach t (wave-uniform)
    int n = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane_max >= t));
    if constexpr (TWO) n += __builtin_popcountll(__builtin_amdgcn_ballot_w64(second >= t));
    return n;
  };
  // the searches skip the bits that cannot differ: no key exceeds hi, so a threshold that keeps hi's sign and
  // exponent bits and is reached often enough is the start for the remaining bits
  uint32_t bound = 0;
  int bit0 = 31;
  const uint32_t top = hi & 0xFF800000u;
  if (reach(top) >= k) { bound = top; bit0 = 22; }
#pragma unroll 4
  for (int bit = bit0; bit >= 12; --bit) {
    const uint32_t cand = bound | (1u << bit);
    if (reach(cand) >= k) bound = cand;
  }
  int n_cand = 0;
#pragma unroll
  for (int m = 0; m < R; ++m) {                              // (registers without a chunk hold 0: never at the bound)
    const bool in = key[m] != 0u && key[m] >= bound;
    const unsigned long long inb = __builtin_amdgcn_ballot_w64(in);
    const int pos = n_cand + lanes_below(inb);
    if (in && pos < kPlaces) cand_lds[pos] = make_uint2(key[m], (uint32_t)(lane + 64 * m));
    n_cand += __builtin_popcountll(inb);
  }
  if (n_cand > kPlaces) return false;                        // the lanes' maxima are low, or many keys tie at the bound
  wave_lds_sync();
  const uint2 c0 = lane < n_cand ? cand_lds[lane] : make_uint2(0u, 0u);
  uint2 c1 = make_uint2(0u, 0u);
  if constexpr (TWO) {
    if (lane + 64 < n_cand) c1 = cand_lds[lane + 64];
  }
  // every candidate lies in [bound, hi]: the bits above the first one in which the two differ are decided
  const int free_bits = 32 - __builtin_clz((hi ^ bound) | 1u);
  uint32_t thr = free_bits >= 32 ? 0u : (hi >> free_bits) << free_bits;
#pragma unroll 4
  for (int bit = free_bits - 1; bit >= 0; --bit) {
    const uint32_t cand = thr | (1u << bit);
    int cnt = __builtin_popcountll(__builtin_amdgcn_ballot_w64(c0.x >= cand));
    if constexpr (TWO) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(c1.x >= cand));
    if (cnt >= k) thr = cand;                                // wave-uniform
    if (cnt == k) break;                                     // exactly k keys reach it: they are the picks
  }
  // candidate places are in chunk order: place `lane`, then (TWO) place 64 + lane
  const unsigned long long gt0 = __builtin_amdgcn_ballot_w64(c0.x > thr);
  const unsigned long long eq0 = __builtin_amdgcn_ballot_w64(c0.x == thr && lane < n_cand);
  unsigned long long gt1 = 0ull, eq1 = 0ull;
  if constexpr (TWO) {
    gt1 = __builtin_amdgcn_ballot_w64(c1.x > thr);
    eq1 = __builtin_amdgcn_ballot_w64(c1.x == thr && lane + 64 < n_cand);
  }
  const int r_adm = k - __builtin_popcountll(gt0) - __builtin_popcountll(gt1);   // places left for keys equal to the threshold
  {
    const int eq_before = lanes_below(eq0);
    if (((gt0 >> lane) & 1ull) || (((eq0 >> lane) & 1ull) && eq_before < r_adm)) {
      const int pos = lanes_below(gt0) + min(eq_before, r_adm);
      if (to_memory) sel_mem[pos] = (int32_t)c0.y;
      if (sel_lds) sel_lds[pos] = (int32_t)c0.y;
    }
  }
  if constexpr (TWO) {
    const int eq_before = __builtin_popcountll(eq0) + lanes_below(eq1);
    if (((gt1 >> lane) & 1ull) || (((eq1 >> lane) & 1ull) && eq_before < r_adm)) {
      const int pos = __builtin_popcountll(gt0) + lanes_below(gt1) + min(eq_before, r_adm);
      if (to_memory) sel_mem[pos] = (int32_t)c1.y;
      if (sel_lds) sel_lds[pos] = (int32_t)c1.y;
    }
  }
  return true;
}

template <int R, int NT>
__device__ __forceinline__ void topk_chunks_in_registers(const float* sig, int n_c, int k, uint32_t* hist, uint32_t* bc,
                                                         bool to_memory, int32_t* sel_mem, int32_t* sel_lds) {
  const int tid = thread_index(), lane = tid & 63, wv = tid >> 6;
  const int n_used = (n_c + 63) >> 6;
  uint32_t key[R];
#pragma unroll
  for (int m = 0; m < R; ++m) {
    const int ch = lane + 64 * m;
    key[m] = (m < n_used && ch < n_c) ? float_order_key(sig[ch]) : 0u;      // 0: no chunk (below every real key)
  }
  if (wv == 0) {
    uint32_t lane_max = 0u;                                  // absent entries are 0
#pragma unroll
    for (int m = 0; m < R; ++m) lane_max = max(lane_max, key[m]);
    const uint32_t hi = ~wave_min_u32_dpp(~lane_max);        // the largest key
    uint2* cand_lds = reinterpret_cast<uint2*>(hist);        // the histogram's 256 words, not in use on this path
    bool picked = false;                                     // wave-uniform
    if (k <= 32) picked = topk_from_lane_maxima<R, false>(key, k, lane_max, hi, cand_lds, to_memory, sel_mem, sel_lds);
    else if (k <= kBoundPicks) picked = topk_from_lane_maxima<R, true>(key, k, lane_max, hi, cand_lds, to_memory, sel_mem, sel_lds);
    if (!picked) {
      uint32_t lo = 0xFFFFFFFFu;
#pragma unroll
      for (int m = 0; m < R; ++m)
        if (key[m] != 0u) lo = min(lo, key[m]);
      lo = wave_min_u32_dpp(lo);
      const uint32_t t = wave_radix_kth<R>(key, n_used, k, max(lo, 1u), hi, hist);
      if (lane == 0) bc[0] = t;
    }
    if (lane == 0) bc[1] = picked ? 1u : 0u;
  }
  __syncthreads();
  if (bc[1]) return;                                         // wave 0 has left the picks
  const uint32_t thr = bc[0];
  if (wv >= 4) return;
  int n_gt = 0;
#pragma unroll
  for (int m = 0; m < R; ++m)
    if (m < n_used) n_gt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[m] > thr));   // wave-uniform branch
  const int r_adm = k - n_gt;                            // >= 1 places left for keys equal to the threshold
  const unsigned long long below = (1ull << lane) - 1ull;
  int gt_run = 0, eq_run = 0;
#pragma unroll
  for (int m = 0; m < R; ++m) {
    if (m >= n_used) break;                              // wave-uniform
    const unsigned long long gtb = __builtin_amdgcn_ballot_w64(key[m] > thr);
    const unsigned long long eqb = __builtin_amdgcn_ballot_w64(key[m] == thr);   // absent entries are 0 < thr
    if ((m & 3) == wv) {
      const bool is_gt = (gtb >> lane) & 1ull, is_eq = (eqb >> lane) & 1ull;
      const int eq_before = eq_run + __builtin_popcountll(eqb & below);
      if (is_gt || (is_eq && eq_before < r_adm)) {
        const int pos = gt_run + __builtin_popcountll(gtb & below) + min(eq_before, r_adm);
        if (to_memory) sel_mem[pos] = lane + 64 * m;
        if (sel_lds) sel_lds[pos] = lane + 64 * m;
      }
    }
    gt_run += __builtin_popcountll(gtb);
    eq_run += __builtin_popcountll(eqb);
  }
}

// Scores of the chunks [ch_begin, ch_end) of one dynamic unit that has n_c chunks: the inner product of the
// group-summed query (summed in head order) with every chunk summary; whole block (NT threads).  sig (shared
// memory, indexed by chunk; may be null) and, with to_memory, the unit's score array take the results.  One
// routine for the step's kernels and for the launch that scores ahead of them, so that both give the same bits.
template <typename T, int NT>
__device__ __forceinline__ void score_chunk_range(const CacheView& cv, const UnitDesc& d, int lrel, const T* __restrict__ q,
                                                  int ch_begin, int ch_end, int n_c, float* sig, bool to_memory) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RP = NT / LPR;
  const int tid = thread_index();
  const int sub = tid % LPR, slot = tid / LPR;
  float qf[EPL];
#pragma unroll
  for (int e = 0; e < EPL; ++e) qf[e] = 0.f;
  const char* qb = reinterpret_cast<const char*>(q) +
                   (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * cv.G) * kD * sizeof(T) + sub * 16;
  const char* mu = reinterpret_cast<const char*>(cv.mu) + (size_t)d.aux_off * kD * sizeof(T) + sub * 16;
  uint4 qraw[kMaxG];
#pragma unroll
  for (int g = 0; g < kMaxG; ++g) qraw[g] = g < cv.G ? ld16(qb + (size_t)g * kD * sizeof(T)) : make_uint4(0, 0, 0, 0);
  for (int ch0 = ch_begin; ch0 < ch_end; ch0 += RP * 16) {      // uniform trip count; sixteen independent loads per round
    uint4 raw[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int ch = ch0 + j * RP + slot;
      raw[j] = ld16(mu + (size_t)min(ch, n_c - 1) * kD * sizeof(T));
    }
    if (ch0 == ch_begin) {
#pragma unroll
      for (int g = 0; g < kMaxG; ++g) {
        float t[EPL];
        unpack16(qraw[g], t, T{});
#pragma unroll
        for (int e = 0; e < EPL; ++e) qf[e] += t[e];
      }
    }
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int ch = ch0 + j * RP + slot;
      float mf[EPL];
      unpack16(raw[j], mf, T{});
      float dot = 0.f;
#pragma unroll
      for (int e = 0; e < EPL; ++e) dot = fmaf(qf[e], mf[e], dot);
      dot = sum_lanes<LPR>(dot);
      if (ch < ch_end && sub == 0) {
        if (sig) sig[ch] = dot;
        if (to_memory) cv.sigma[d.aux_off + ch] = dot;
      }
    }
  }
}

// Chunk scoring and chunk top-k of one dynamic unit; whole block (NT threads).
constexpr int kSelHeader = 256 + 16;       // words before the chunk scores: histogram, 2 broadcast words, scan area
template <typename T, int NT = 256>
__device__ __forceinline__ void select_chunks_of_unit(const CacheView& cv, const UnitDesc& d, int lrel,
                                                      const T* __restrict__ q, int use_stored_sigma, float* dsm,
                                                      int32_t* sel_lds = nullptr, bool to_memory = true,
                                                      int n_c_now = -1, int k_now = -1,
                                                      unsigned long long* t_scores = nullptr) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RP = NT / LPR;
  const int tid = thread_index();
  uint32_t* hist = reinterpret_cast<uint32_t*>(dsm);         // [256]
  uint32_t* bc = hist + 256;                                 // [2]
  int* scan = reinterpret_cast<int*>(bc + 2);                // [NT / 64 + 1 <= 14]
  float* sig = dsm + kSelHeader;                             // [n_chunks rounded up to 4]
  // caches that index generated tokens pass the chunks there are at this step and how many to pick
  const int n_c = n_c_now >= 0 ? n_c_now : d.n_chunks;
  const int k_sel = k_now >= 0 ? k_now : d.k_sel;
  const int n_c4 = (n_c + 3) & ~3;
  unsigned long long* key64 = reinterpret_cast<unsigned long long*>(sig + n_c4);   // [n_c4], 8-byte aligned

  if (!use_stored_sigma) {
    score_chunk_range<T, NT>(cv, d, lrel, q, 0, n_c, n_c, sig, to_memory);
  } else {
    for (int ch = tid; ch < n_c; ch += NT) sig[ch] = cv.sigma[d.aux_off + ch];
  }
  __syncthreads();
  if (t_scores && tid == 0) *t_scores = wall_clock64();       // diagnostic: the scores are in shared memory

  // top-k chunks, ties to the lower chunk id, emitted ascending by chunk id
  if (n_c <= 256) {
    // Every wave holds all keys (four per lane) and finds the k-th largest key value by a bitwise search
    // on wave-wide vote counts -- no barrier, no memory traffic; the four waves do the same arithmetic.
    // Chunks with a key above it are picked, those equal to it in chunk order up to the k-th place.
    const int lane = tid & 63, wv = tid >> 6;
    if (NT > 256 && wv >= 4) return;                       // the first four waves cover all 256 chunks
    const int k = k_sel;
    uint32_t key[4];
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const int ch = lane + 64 * m;
      key[m] = ch < n_c ? float_order_key(sig[ch]) : 0u;   // 0 is below every candidate threshold
    }
    // (a candidate that exactly k keys reach already separates the picks from the rest: the search stops
    // there, usually a dozen bits in, and the code below picks the keys at or above it)
    uint32_t thr = 0;
#pragma unroll 4
    for (int bit = 31; bit >= 0; --bit) {
      const uint32_t cand = thr | (1u << bit);
      int cnt = 0;
#pragma unroll
      for (int m = 0; m < 4; ++m) cnt += __builtin_popcountll(__builtin_amdgcn_ballot_w64(key[m] >= cand));
      if (cnt >= k) thr = cand;                             // wave-uniform
      if (cnt == k) break;
    }
    const unsigned long long below = (1ull << lane) - 1ull;
    int n_gt = 0, gt_before = 0, eq_before = 0;
    bool is_gt = false, is_eq = false;
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const unsigned long long gtb = __builtin_amdgcn_ballot_w64(key[m] > thr);
      const unsigned long long eqb = __builtin_amdgcn_ballot_w64(key[m] == thr && lane + 64 * m < n_c);
      n_gt += __builtin_popcountll(gtb);
      if (m < wv) { gt_before += __builtin_popcountll(gtb); eq_before += __builtin_popcountll(eqb); }
      if (m == wv) {                                       // this thread's own chunk is 64 * wv + lane
        gt_before += __builtin_popcountll(gtb & below);
        eq_before += __builtin_popcountll(eqb & below);
        is_gt = (gtb >> lane) & 1ull;
        is_eq = (eqb >> lane) & 1ull;
      }
    }
    const int r_adm = k - n_gt;                            // >= 1 places left for keys equal to the threshold
    if (is_gt || (is_eq && eq_before < r_adm)) {
      const int pos = gt_before + min(eq_before, r_adm);   // picks with a lower chunk id
      if (to_memory) cv.sel[d.idx_off + pos] = tid;
      if (sel_lds) sel_lds[pos] = tid;
    }
    return;
  }
  // up to 2048 chunks: the keys fit a wave's registers and the selection needs one barrier instead of the
  // block-wide radix passes and scans below (about sixty barriers at 1600 chunks)
  if (n_c <= 64 * 32) {
    int32_t* sel_mem = cv.sel + d.idx_off;
    if (n_c <= 64 * 8) topk_chunks_in_registers<8, NT>(sig, n_c, k_sel, hist, bc, to_memory, sel_mem, sel_lds);
    else if (n_c <= 64 * 16) topk_chunks_in_registers<16, NT>(sig, n_c, k_sel, hist, bc, to_memory, sel_mem, sel_lds);
    else topk_chunks_in_registers<32, NT>(sig, n_c, k_sel, hist, bc, to_memory, sel_mem, sel_lds);
    return;
  }
  uint32_t T_key = 0;
  int r_adm = n_c;
  if (k_sel < n_c) {
    radix_select<NT, true>(n_c, k_sel,
                     [&](int j, uint32_t& key) { key = float_order_key(sig[j]); return true; },
                     hist, bc, T_key, r_adm);
  }
  int base_eq = 0, base_keep = 0;
  for (int ch0 = 0; ch0 < n_c; ch0 += NT) {
    const int ch = ch0 + tid;
    uint32_t key = 0;
    const bool in = ch < n_c;
    if (in) key = float_order_key(sig[ch]);
    const int eq = (in && key == T_key) ? 1 : 0;
    const int gt = (in && key > T_key) ? 1 : 0;
    int tot_eq, tot_keep;
    const int eq_rank = base_eq + block_exclusive_scan<NT>(eq, scan, &tot_eq);
    const int keep = gt | (eq & (eq_rank < r_adm ? 1 : 0));
    const int pos = base_keep + block_exclusive_scan<NT>(keep, scan, &tot_keep);
    if (keep && pos < k_sel) {
      if (to_memory) cv.sel[d.idx_off + pos] = ch;
      if (sel_lds) sel_lds[pos] = ch;
    }
    base_eq += tot_eq;
    base_keep += tot_keep;
  }
}

// Writes the step's new K/V row of one unit into its tail (all threads of the block; ends with a barrier,
// so the row is in memory before any lane of this block reads it).
template <typename T>
__device__ __forceinline__ void append_row(const CacheView& cv, int seq, int head, int64_t tail_off, int lrel, int t_before,
                                           const T* __restrict__ k_new, const T* __restrict__ v_new) {
  constexpr int LPR = Elem<T>::kLanesPerRow;
  const int tid = thread_index();
  const size_t src_row = (((size_t)lrel * cv.batch + seq) * cv.n_kv_heads + head) * kD * sizeof(T);
  const int64_t prow = tail_off + t_before;                    // row in the device arrays
  if constexpr (sizeof(T) == 2) {
    // blocked cache: 16 key pieces go to their slots of the row's block, V is scattered one element per dim
    const size_t blk_off = (size_t)(prow >> 3) * kBlkBytes;
    const int e = (int)(prow & 7);
    if (tid < 16)
      st16(reinterpret_cast<char*>(cv.k_rows) + blk_off + k_piece_index(e, tid) * 16,
           ld16(reinterpret_cast<const char*>(k_new) + src_row + tid * 16));
    if (tid >= 64 && tid < 64 + kD) {
      const int dd = tid - 64;
      *reinterpret_cast<uint16_t*>(reinterpret_cast<char*>(cv.v_rows) + blk_off + dd * 16 + e * 2) =
          *reinterpret_cast<const uint16_t*>(reinterpret_cast<const char*>(v_new) + src_row + dd * 2);
    }
  } else if (tid < 2 * LPR) {
    const int which = tid / LPR, sub = tid % LPR;
    const size_t dst = (size_t)prow * kD * sizeof(T) + sub * 16;
    if (which == 0) st16(reinterpret_cast<char*>(cv.k_rows) + dst, ld16(reinterpret_cast<const char*>(k_new) + src_row + sub * 16));
    else st16(reinterpret_cast<char*>(cv.v_rows) + dst, ld16(reinterpret_cast<const char*>(v_new) + src_row + sub * 16));
  }
  __threadfence_block();
  __syncthreads();                        // the row is in memory before any lane of this block reads it
}

// Caches that index their generated tokens (bf16): the chunk of generated tokens g of a dynamic unit has
// just been completed by this block's append; its metadata -- the exact mean of its keys, rounded once to
// bf16 like the prompt's -- goes behind the prompt's chunk summaries, where the next step's selection
// finds it.  Threads 0..127 take one dimension each; the chunk's rows are read back from the blocked tail.
__device__ __forceinline__ void index_generated_chunk(const CacheView& cv, const AttnItem& it, int g) {
  const int dd = thread_index();
  if (dd >= kD) return;
  const int c = 1 << it.c_log2;
  const char* tail = reinterpret_cast<const char*>(cv.k_rows) + (size_t)it.tail_off * kD * 2;
  double acc = 0.0;                    // exact, as for the prompt's chunks: double sum, double divide, one rounding
  for (int r = 0; r < c; ++r) {
    const int row = g * c + r;
    const uint16_t bits = *reinterpret_cast<const uint16_t*>(tail + (size_t)(row >> 3) * kBlkBytes +
                                                             k_piece_index(row & 7, dd >> 3) * 16 + (dd & 7) * 2);
    acc += (double)bits_to_float((uint32_t)bits << 16);
  }
  reinterpret_cast<uint16_t*>(cv.mu)[(size_t)(it.aux_off + it.n_chunks + g) * kD + dd] = f64_to_bf16_rne(acc / (double)c);
}

// One split-K tile of the hybrid cache: optional tail append, then attention, record -> workspace.
// NW: waves of the workgroup (bf16 matrix-core tile only).  out_rows (bf16 caches, a tile that covers its
// whole unit): the unit's G output rows are written there and no record is made.
template <typename T, int G, int NW = 4, bool INDEXED = false>
__device__ __forceinline__ void attention_item(const CacheView& cv, const AttnItem& it, int layer_begin, int slot_base,
                                               const T* __restrict__ q, const T* __restrict__ k_new,
                                               const T* __restrict__ v_new, const PartOut& partials, int t_arg,
                                               int TILE, float* smem, const int32_t* sel_override = nullptr,
                                               uint16_t* out_rows = nullptr) {
  constexpr int LPR = Elem<T>::kLanesPerRow;
  const int tid = threadIdx.x;
  const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[it.layer];
  const bool append = (k_new != nullptr) && (t_before < cv.max_new);
  // INDEXED, dynamic unit: it.n_prompt_rows counts the rows of the chunks picked this step (prompt or
  // generated); of the tail only the rows behind its last complete chunk are attended unconditionally
  const int gen0 = (INDEXED && it.dynamic) ? (t_before >> it.c_log2) << it.c_log2 : 0;
  const int t_rest = t_before - gen0;
  RowMap rm;
  rm.n_rows = it.n_prompt_rows + t_rest + (append ? 1 : 0);
  if (it.row0 == 0 && it.seq == 0 && it.head == 0 && tid == 0)     // one block per layer moves the tail counter on
    (t_arg >= 0 ? cv.cnt_a : cv.cnt_b)[it.layer] = t_before + (append ? 1 : 0);
  if (it.row0 >= rm.n_rows) return;          // tile reserved for tail growth, not reached yet
  const int lrel = it.layer - layer_begin;
  const int new_row = it.n_prompt_rows + t_rest;            // logical index of the appended row
  if (append && new_row >= it.row0 && new_row < it.row0 + TILE) {  // block-uniform
    append_row<T>(cv, it.seq, it.head, it.tail_off, lrel, t_before, k_new, v_new);
    if constexpr (INDEXED && sizeof(T) == 2) {
      if (it.dynamic && ((t_before + 1) & ((1 << it.c_log2) - 1)) == 0)    // the new token completes a chunk
        index_generated_chunk(cv, it, t_before >> it.c_log2);
    }
  }
  rm.kbase = reinterpret_cast<const char*>(it.dynamic ? cv.k_dyn : cv.k_rows) + (size_t)it.kv_row_off * kD * sizeof(T);
  rm.vbase = reinterpret_cast<const char*>(it.dynamic ? cv.v_dyn : cv.v_rows) + (size_t)it.kv_row_off * kD * sizeof(T);
  rm.ktail = (int64_t)(reinterpret_cast<intptr_t>(cv.k_rows) + it.tail_off * (int64_t)(kD * sizeof(T)) -
                       reinterpret_cast<intptr_t>(rm.kbase));
  rm.vtail = (int64_t)(reinterpret_cast<intptr_t>(cv.v_rows) + it.tail_off * (int64_t)(kD * sizeof(T)) -
                       reinterpret_cast<intptr_t>(rm.vbase));
  rm.stride = kD * sizeof(T);
  rm.dynamic = it.dynamic;
  rm.sel = sel_override ? sel_override : cv.sel + it.sel_off;
  rm.n_sel_rows = it.n_prompt_rows;
  rm.c_log2 = it.c_log2;
  rm.C = it.C;
  rm.tail_row = it.tail_row;
  rm.n_chunks_prompt = it.n_chunks;
  rm.gen0 = gen0;
  const size_t qoff = (((size_t)lrel * cv.batch + it.seq) * cv.n_q_heads + (size_t)it.head * G) * kD;
  if constexpr (sizeof(T) == 2) {
    // the unit's rows all fall into this tile: no record, no combination (same arithmetic, one pass)
    if (!out_rows && partials.out_all && it.row0 == 0 && rm.n_rows <= TILE)
      out_rows = reinterpret_cast<uint16_t*>(partials.out_all) + qoff;
  }
  const PartOut part = {out_rows ? nullptr : partials.o + (size_t)(it.slot - slot_base) * G * kD,
                        out_rows ? nullptr : partials.ml + (size_t)(it.slot - slot_base) * kMlStride, out_rows, nullptr};
  run_tile<T, G, true, NW, INDEXED>(rm, q + qoff, cv.scale_log2e, it.row0, TILE, part, smem);
}

// Combine the tiles [0, n_tiles) of one unit, whose records this block wrote itself, and write the G
// output rows.  All 256 threads.
template <typename T>
__device__ __forceinline__ void merge_own_tiles(const PartOut& first, int n_tiles, int G, T* __restrict__ out_rows) {
  for (int idx = threadIdx.x; idx < G * kD; idx += 256) {
    const int g = idx >> 7;
    float M = kNeg, L = 0.f, O = 0.f;
    for (int t = 0; t < n_tiles; ++t) {
      const float2 ml = *reinterpret_cast<const float2*>(first.ml + (size_t)t * kMlStride + 2 * g);
      const float ov = first.o[(size_t)t * G * kD + idx];
      const float Mn = fmaxf(M, ml.x);
      const float c0 = fast_exp2(M - Mn), c1 = fast_exp2(ml.x - Mn);
      L = L * c0 + ml.y * c1;
      O = O * c0 + ov * c1;
      M = Mn;
    }
    const float o = L > 0.f ? O / L : 0.f;
    if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(out_rows)[idx] = o;
    else reinterpret_cast<uint16_t*>(out_rows)[idx] = f32_to_bf16_rne(o);
  }
}

constexpr int kWholeUnit = 1 << 28;   // tile size that covers any unit (row counts stay below 2^24)

// Chunk scores under the other reading for grouped query heads (hkv_config.chunk_score_group = 1): every
// query head of the group scores every chunk and a chunk takes the largest of its G scores.  A launch of
// its own, ahead of the step's kernels, which then pick from the stored scores; the default reading stays
// inside those kernels.  grid = dynamic units of the call, block = 256 threads.
template <typename T>
__global__ __launch_bounds__(256) void chunk_score_max_kernel(CacheView cv, int layer_begin, int dyn_begin,
                                                              const T* __restrict__ q, int t_arg) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RP = 256 / LPR;
  const UnitDesc d = cv.dyn_descs[dyn_begin + blockIdx.x];
  const int lrel = d.layer - layer_begin;
  int n_c = d.n_chunks;
  if (cv.index_gen) n_c += (t_arg >= 0 ? t_arg : cv.cnt_a[d.layer]) >> d.c_log2;    // complete chunks of generated tokens
  const int tid = thread_index(), sub = tid % LPR, slot = tid / LPR;
  const char* qb = reinterpret_cast<const char*>(q) +
                   (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * cv.G) * kD * sizeof(T) + sub * 16;
  const char* mu = reinterpret_cast<const char*>(cv.mu) + (size_t)d.aux_off * kD * sizeof(T) + sub * 16;
  uint4 qraw[kMaxG];
#pragma unroll
  for (int g = 0; g < kMaxG; ++g) qraw[g] = g < cv.G ? ld16(qb + (size_t)g * kD * sizeof(T)) : make_uint4(0, 0, 0, 0);
  for (int ch0 = 0; ch0 < n_c; ch0 += RP * 4) {       // uniform trip count; four independent loads per round
    uint4 raw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ch = ch0 + j * RP + slot;
      raw[j] = ld16(mu + (size_t)min(ch, n_c - 1) * kD * sizeof(T));
    }
    float best[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) best[j] = -INFINITY;
#pragma unroll
    for (int g = 0; g < kMaxG; ++g) {
      if (g < cv.G) {                                  // uniform
        float t[EPL];
        unpack16(qraw[g], t, T{});
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          float mf[EPL];
          unpack16(raw[j], mf, T{});
          float dot = 0.f;
#pragma unroll
          for (int e = 0; e < EPL; ++e) dot = fmaf(t[e], mf[e], dot);
          best[j] = fmaxf(best[j], sum_lanes<LPR>(dot));
        }
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int ch = ch0 + j * RP + slot;
      if (ch < n_c && sub == 0) cv.sigma[d.aux_off + ch] = best[j];
    }
  }
}

// Chunk scores under the default reading in a launch of their own, ahead of the step's kernels, which then
// pick from the stored scores: for calls in which a dynamic tile's chunk selection is the longest chain of
// the launch -- one workgroup bringing in all summaries of its head -- the summaries go through many compute
// units instead.  grid = (dynamic units of the call, blocks of 256 chunks), block = 256 threads; same
// arithmetic as inside the step's kernels (score_chunk_range), so the scores and the picks are the same bits.
template <typename T>
__global__ __launch_bounds__(256) void chunk_score_sum_kernel(CacheView cv, int layer_begin, int dyn_begin,
                                                              const T* __restrict__ q) {
  const UnitDesc d = cv.dyn_descs[dyn_begin + blockIdx.x];
  const int ch_begin = (int)blockIdx.y * 256;
  if (ch_begin >= d.n_chunks) return;
  score_chunk_range<T, 256>(cv, d, d.layer - layer_begin, q, ch_begin, min(d.n_chunks, ch_begin + 256), d.n_chunks,
                            nullptr, true);
}

// INDEXED: the cache indexes its generated tokens (bf16 caches; see attention_item).
template <typename T, int G, bool INDEXED = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void decode_kernel(CacheView cv, int layer_begin, int dyn_begin, int n_dyn, int sitem_begin, int slot_base,
                   const T* __restrict__ q, const T* __restrict__ k_new, const T* __restrict__ v_new,
                   PartOut partials, T* __restrict__ out, int t_arg, int use_stored_sigma, int select_only) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  if ((int)blockIdx.x >= n_dyn) {
    const AttnItem it = cv.static_items[sitem_begin + ((int)blockIdx.x - n_dyn)];
    attention_item<T, G, 4, INDEXED>(cv, it, layer_begin, slot_base, q, k_new, v_new, partials, t_arg, cv.tile_rows, smem);
    return;
  }
  const UnitDesc d = cv.dyn_descs[dyn_begin + blockIdx.x];
  const int lrel = d.layer - layer_begin;
  const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[d.layer];
  // chunks there are at this step and how many of them are picked
  int n_c_now = d.n_chunks, k_now = d.k_sel;
  if constexpr (INDEXED) {
    n_c_now += t_before >> d.c_log2;                    // complete chunks of generated tokens
    k_now = min(d.k_sel, n_c_now);
  }
  select_chunks_of_unit<T>(cv, d, lrel, q, use_stored_sigma | cv.sigma_max, smem, nullptr, true, n_c_now, k_now);
  if (select_only) return;
  // ---- the rest of the dynamic unit, in this block ----
  __threadfence_block();
  __syncthreads();                          // the picks are in memory before the tile code reads them
  const int rows_sel = INDEXED ? (k_now << d.c_log2) : d.n_prompt_rows;
  const int t_rest = INDEXED ? t_before - ((t_before >> d.c_log2) << d.c_log2) : t_before;
  const int t_after = t_rest + ((k_new != nullptr && t_before < cv.max_new) ? 1 : 0);
  // the matrix-core tile takes any number of rows, so the whole unit is one tile and one record;
  // the fp32 tile has a fixed size
  const int TILE = sizeof(T) == 2 ? kWholeUnit : cv.tile_rows;
  const int n_tiles = sizeof(T) == 2 ? 1 : (rows_sel + t_after + TILE - 1) / TILE;
  AttnItem it;
  it.kv_row_off = d.kv_row_off; it.sel_off = (int32_t)d.idx_off; it.n_prompt_rows = rows_sel;
  it.C = d.C; it.c_log2 = d.c_log2; it.dynamic = 1; it.layer = d.layer; it.seq = d.seq; it.head = d.head;
  it.tail_row = d.tail_row; it.tail_off = d.tail_off; it.n_chunks = d.n_chunks; it.aux_off = d.aux_off;
  for (int t = 0; t < n_tiles; ++t) {
    if (t > 0) __syncthreads();             // the previous tile's staging area is free again
    it.row0 = t * TILE;
    it.slot = d.item_begin + t;
    attention_item<T, G, 4, INDEXED>(cv, it, layer_begin, slot_base, q, k_new, v_new, partials, t_arg, TILE, smem);
  }
  if (sizeof(T) == 2 && partials.out_all) return;   // the unit's single tile has written the output rows itself
  __threadfence_block();
  __syncthreads();                          // this block's own records are visible to all its threads
  const PartOut first = {partials.o + (size_t)(d.item_begin - slot_base) * G * kD,
                         partials.ml + (size_t)(d.item_begin - slot_base) * kMlStride};
  T* orow = out + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G) * kD;
  merge_own_tiles<T>(first, n_tiles, G, orow);
}

// Split-K tiles of the dynamic units.  reselect = 0: the picks are already in memory (an earlier launch
// made them).  reselect = 1: every block first repeats its unit's chunk selection, so that no launch
// boundary is needed; all blocks of a unit compute and store identical picks.  In that shape the grid
// also carries the static tiles: blocks [n_ditems, n_ditems + n_sitems), which wait static_hold x 512
// clocks before their first loads.
// NW: waves per workgroup.
// STAMPS: thread 0 of workgroup b < n_stamps leaves a record of HKV_STAMP_WORDS 64-bit words in stamps (values
// of the constant 100 MHz counter): [0] start, [1] tile descriptor read, [2] chunk selection done (0 for a
// static tile), [3] the tile's rows read and its record or output rows written (0: tile not reached at this
// tail length), [4] first logical row of the tile, [5] 1 for a dynamic tile, [6] chunk scores in shared memory
// (dynamic tiles).  A diagnostic instantiation.
template <typename T, int G, bool INDEXED = false, int NW = 4, bool STAMPS = false>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(3, 3)))
void dynamic_tiles_kernel(CacheView cv, int layer_begin, int ditem_begin, int n_ditems, int sitem_begin,
                          int slot_base, const T* __restrict__ q, const T* __restrict__ k_new,
                          const T* __restrict__ v_new, PartOut partials, int t_arg, int reselect, int lds_sel_off,
                          int static_hold, unsigned long long* __restrict__ stamps, int n_stamps) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  unsigned long long* rec = nullptr;
  if constexpr (STAMPS) {
    if (threadIdx.x == 0 && (int)blockIdx.x < n_stamps) {
      rec = stamps + (size_t)blockIdx.x * HKV_STAMP_WORDS;
      rec[0] = wall_clock64();
      for (int i = 1; i < HKV_STAMP_WORDS; ++i) rec[i] = 0;
    }
  }
  if ((int)blockIdx.x >= n_ditems) {
    const AttnItem it = cv.static_items[sitem_begin + ((int)blockIdx.x - n_ditems)];
    if constexpr (STAMPS) {
      if (rec) { asm volatile("" ::"v"(it.row0), "v"(it.slot) : "memory"); rec[1] = wall_clock64(); rec[4] = (unsigned long long)it.row0; }
    }
    // When the whole grid is resident at once, every block asks for its first rows at the same moment and
    // the dynamic heads' summary reads -- the head of the longest dependent chain of the launch -- queue
    // behind all of them.  The static tiles therefore start a little later: static_hold x 512 clocks,
    // the time the summaries need on the memory system (0 for grids of several rounds).
    for (int i = 0; i < static_hold; ++i) __builtin_amdgcn_s_sleep(8);
    attention_item<T, G, NW, INDEXED>(cv, it, layer_begin, slot_base, q, k_new, v_new, partials, t_arg, cv.tile_rows, smem);
    if constexpr (STAMPS) {
      if (rec) rec[3] = wall_clock64();
    }
    return;
  }
  // Workgroups go to the eight dies in rotation (workgroup b runs on die b % 8) and each die has its own L2.
  // The tiles of a unit all read the unit's chunk summaries, so the dynamic tiles are dealt out in eight
  // contiguous runs, one per die: die x takes tiles [x * xq + min(x, xr), ...) in order.
  const int xq = n_ditems >> 3, xr = n_ditems & 7, xx = blockIdx.x & 7;
  AttnItem it = cv.dynamic_items[ditem_begin + xx * xq + min(xx, xr) + ((int)blockIdx.x >> 3)];
  if constexpr (STAMPS) {
    if (rec) { asm volatile("" ::"v"(it.row0), "v"(it.slot) : "memory"); rec[1] = wall_clock64(); rec[4] = (unsigned long long)it.row0; rec[5] = 1; }
  }
  const int32_t* picks = nullptr;
  if (reselect) {
    const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[it.layer];
    int n_c_now = it.n_chunks, k_now = it.k_sel, t_rest = t_before;
    if constexpr (INDEXED) {                                    // chunks there are at this step, picks, rows they give
      n_c_now += t_before >> it.c_log2;
      k_now = min(it.k_sel, n_c_now);
      it.n_prompt_rows = k_now << it.c_log2;
      t_rest = t_before & ((1 << it.c_log2) - 1);
    }
    if (it.row0 >= it.n_prompt_rows + t_rest + 1) return;       // tile not reached yet, with or without an append
    UnitDesc d;                                                 // the fields the selection reads
    d.aux_off = it.aux_off; d.idx_off = it.sel_off; d.n_chunks = it.n_chunks; d.k_sel = it.k_sel;
    d.seq = it.seq; d.head = it.head;
    int32_t* sel_lds = reinterpret_cast<int32_t*>(smem + lds_sel_off);
    // the picks stay in LDS for this block's own tile; the first tile also leaves them (and the chunk
    // scores) in memory for export
    select_chunks_of_unit<T, NW * 64>(cv, d, it.layer - layer_begin, q, cv.sigma_max, smem, sel_lds, it.row0 == 0, n_c_now, k_now,
                                      STAMPS && rec ? rec + 6 : nullptr);
    __syncthreads();
    picks = sel_lds;
    if constexpr (STAMPS) {
      if (rec) rec[2] = wall_clock64();
    }
  }
  attention_item<T, G, NW, INDEXED>(cv, it, layer_begin, slot_base, q, k_new, v_new, partials, t_arg, cv.tile_rows, smem, picks);
  if constexpr (STAMPS) {
    if (rec) rec[3] = wall_clock64();
  }
}

// One workgroup of kUnitWaves waves per unit (bf16 caches): chunk selection for a dynamic unit, then attention
// over all rows of the unit as a single tile -- the waves share the 32-row steps and combine in shared
// memory -- and the unit's output rows.  No records, no second launch: the shape for steps whose units
// are few enough to give every unit a compute unit of its own.  grid = dynamic units of the call, then
// static units.
constexpr int kUnitWaves = 12;
template <int G, bool INDEXED = false>
__global__ __launch_bounds__(kUnitWaves * 64) __attribute__((amdgpu_waves_per_eu(3, 3)))
void unit_kernel(CacheView cv, int layer_begin, int dyn_begin, int n_dyn, int static_begin,
                 const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
                 bf16_t* __restrict__ out, int t_arg, int lds_sel_off) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const bool dyn = (int)blockIdx.x < n_dyn;                  // block-uniform
  const UnitDesc d = dyn ? cv.dyn_descs[dyn_begin + blockIdx.x] : cv.static_descs[static_begin + ((int)blockIdx.x - n_dyn)];
  const int lrel = d.layer - layer_begin;
  const int32_t* picks = nullptr;
  int rows_sel = d.n_prompt_rows;
  if (dyn) {
    int n_c_now = d.n_chunks, k_now = d.k_sel;
    if constexpr (INDEXED) {
      const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[d.layer];
      n_c_now += t_before >> d.c_log2;                       // complete chunks of generated tokens
      k_now = min(d.k_sel, n_c_now);
      rows_sel = k_now << d.c_log2;
    }
    int32_t* sel_lds = reinterpret_cast<int32_t*>(smem + lds_sel_off);
    select_chunks_of_unit<bf16_t, kUnitWaves * 64>(cv, d, lrel, q, cv.sigma_max, smem, sel_lds, true, n_c_now, k_now);
    __syncthreads();                                         // the picks are in shared memory; the scratch is free
    picks = sel_lds;
  }
  AttnItem it;
  it.kv_row_off = d.kv_row_off; it.sel_off = (int32_t)d.idx_off; it.n_prompt_rows = rows_sel;
  it.C = d.C; it.c_log2 = d.c_log2; it.dynamic = dyn ? 1 : 0; it.layer = d.layer; it.seq = d.seq; it.head = d.head;
  it.tail_row = d.tail_row; it.tail_off = d.tail_off; it.row0 = 0; it.slot = 0; it.n_chunks = d.n_chunks;
  it.aux_off = d.aux_off;
  uint16_t* orow = reinterpret_cast<uint16_t*>(out) +
                   (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G) * kD;
  const PartOut none = {nullptr, nullptr, nullptr};
  attention_item<bf16_t, G, kUnitWaves, INDEXED>(cv, it, layer_begin, 0, q, k_new, v_new, none, t_arg, kWholeUnit, smem,
                                                 picks, orow);
}

// ------------------------------------------------------------------------------------------
// streamed shape: every workgroup takes an equal share of the step's rows
// ------------------------------------------------------------------------------------------
// The rows a step attends (every unit of the call, in unit order, each unit's rows in steps of 32) form one
// line of work; the host cuts it into as many equal shares as the launch has workgroups (a table made when
// the cache was laid out, one per call shape and reference tail length) and workgroup i walks its share:
// it may end one unit, cross several whole units and begin another.  Per unit it touches it leaves one
// record at slot i + (unit's position in the call) -- those sums grow along the line of work, so slots
// are unique -- or, when the unit lies wholly inside its share, the unit's output rows themselves.  All
// workgroups read the same number of bytes and end together; what a fresh workgroup per tile pays at
// every tile (dispatch, descriptor, first loads' latency, record) is paid once per unit crossed.
// A boundary (unit, row) has 0 <= row < rows of the unit at the table's reference tail length, row a
// multiple of 32; the end of a unit is written as the start of the next.  A segment that reaches its
// unit's end in the table takes every row the unit has now (the tail may be longer than the table
// assumed); one that begins beyond the rows the unit has now is empty and leaves a neutral record.
// Dynamic units: a workgroup selects the chunks of every dynamic unit it touches (like the tiles that repeat
// the selection); the workgroup holding row 0 leaves scores and picks in memory for export.
// Where the logical rows of a unit live, for a step in which the unit has n_rows of them.
__device__ __forceinline__ RowMap row_map_of_unit(const CacheView& cv, const UnitDesc& d, int n_rows, const int32_t* picks) {
  const bool dyn = d.kind == HKV_DYNAMIC;
  RowMap rm;
  rm.n_rows = n_rows;
  rm.kbase = reinterpret_cast<const char*>(dyn ? cv.k_dyn : cv.k_rows) + (size_t)d.kv_row_off * kD * 2;
  rm.vbase = reinterpret_cast<const char*>(dyn ? cv.v_dyn : cv.v_rows) + (size_t)d.kv_row_off * kD * 2;
  rm.ktail = (int64_t)(reinterpret_cast<intptr_t>(cv.k_rows) + d.tail_off * (int64_t)(kD * 2) - reinterpret_cast<intptr_t>(rm.kbase));
  rm.vtail = (int64_t)(reinterpret_cast<intptr_t>(cv.v_rows) + d.tail_off * (int64_t)(kD * 2) - reinterpret_cast<intptr_t>(rm.vbase));
  rm.stride = kD * 2;
  rm.dynamic = dyn ? 1 : 0;
  rm.sel = picks;
  rm.n_sel_rows = d.n_prompt_rows;
  rm.c_log2 = d.c_log2;
  rm.C = d.C;
  rm.tail_row = d.tail_row;
  rm.n_chunks_prompt = d.n_chunks;
  rm.gen0 = 0;
  return rm;
}

template <int G>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(3, 3)))
void stream_kernel(CacheView cv, const StreamBound* __restrict__ bounds, int unit_base, int layer_begin,
                   const bf16_t* __restrict__ q, const bf16_t* __restrict__ k_new, const bf16_t* __restrict__ v_new,
                   PartOut partials, bf16_t* __restrict__ out, int t_arg, int lds_sel_off) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  const StreamBound b0 = bounds[blockIdx.x], b1 = bounds[blockIdx.x + 1];
  int u = __builtin_amdgcn_readfirstlane(b0.unit), ra = __builtin_amdgcn_readfirstlane(b0.row);
  const int u_last = __builtin_amdgcn_readfirstlane(b1.unit), r_last = __builtin_amdgcn_readfirstlane(b1.row);
  StepBufs sb;                   // the operands in flight
  sb.nv = 0;
  bool here = u < u_last || (u == u_last && ra < r_last);        // workgroup-uniform
  while (here) {
    const UnitDesc d = cv.units[unit_base + u];
    const bool more = u + 1 < u_last || (u + 1 == u_last && 0 < r_last);     // another unit of the share follows
    const int lrel = d.layer - layer_begin;
    const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[d.layer];
    const bool append = (k_new != nullptr) && (t_before < cv.max_new);
    const int n_rows = d.n_prompt_rows + t_before + (append ? 1 : 0);      // logical rows the unit has in this step
    const bool to_end = u < u_last;                                       // else the share ends inside this unit
    const int rb = to_end ? n_rows : min(r_last, n_rows);
    if (ra == 0 && d.seq == 0 && d.head == 0 && thread_index() == 0)       // one workgroup per layer moves the tail counter on
      (t_arg >= 0 ? cv.cnt_a : cv.cnt_b)[d.layer] = t_before + (append ? 1 : 0);
    const int new_row = n_rows - 1;                                        // logical index of the appended row, if any
    const bool appends_here = append && ra <= new_row && new_row < rb;
    const size_t qoff = (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G) * kD;
    const bool whole = ra == 0 && to_end;                                  // the unit lies inside this share: write its output rows
    const size_t slot = (size_t)blockIdx.x + (size_t)u;
    const PartOut part = {whole ? nullptr : partials.o + slot * G * kD, whole ? nullptr : partials.ml + slot * kMlStride,
                          whole ? reinterpret_cast<uint16_t*>(out) + qoff : nullptr};
    if (d.kind == HKV_DYNAMIC) {
      const int32_t* picks = nullptr;
      if (ra < rb) {
        int32_t* sel_lds = reinterpret_cast<int32_t*>(smem + lds_sel_off);
        select_chunks_of_unit<bf16_t>(cv, d, lrel, q, cv.sigma_max, smem, sel_lds, ra == 0);
        __syncthreads();                                                   // the picks are in shared memory; the scratch is free
        picks = sel_lds;
      }
      if (appends_here) append_row<bf16_t>(cv, d.seq, d.head, d.tail_off, lrel, t_before, k_new, v_new);
      attn_tile_mfma<G, 1>(row_map_of_unit(cv, d, n_rows, picks), q + qoff, cv.scale_log2e, ra, rb - ra, part, smem, sb,
                           false);
    } else {
      if (appends_here) append_row<bf16_t>(cv, d.seq, d.head, d.tail_off, lrel, t_before, k_new, v_new);
      attn_tile_mfma<G, 0>(row_map_of_unit(cv, d, n_rows, nullptr), q + qoff, cv.scale_log2e, ra, rb - ra, part, smem, sb,
                           false);
    }
    lds_barrier();                                                         // the staging area is free for the next unit
    u += 1;
    ra = 0;
    here = more;
  }
}

// Combination of the records of the units that more than one workgroup of stream_kernel touched.
// grid = listed units x G, block = 128 threads.
template <typename T>
__global__ __launch_bounds__(128) void stream_merge_kernel(CacheView cv, const StreamMulti* __restrict__ multi, int unit_base,
                                                           int layer_begin, PartOut partials, T* __restrict__ out) {
  const int G = cv.G;
  const int g = blockIdx.x % G;
  const StreamMulti m = multi[blockIdx.x / G];
  const UnitDesc d = cv.units[unit_base + m.unit];
  const int lrel = d.layer - layer_begin;
  const float* o0 = partials.o + ((size_t)m.slot0 * G + g) * kD;
  const float* ml0 = partials.ml + (size_t)m.slot0 * kMlStride + 2 * g;
  T* orow = out + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G + g) * kD;
  merge_head<T>(o0, ml0, m.n_rec, G * kD, orow);
}

// grid = n_units x G, block = 128 threads; descs points at the first unit's descriptor.
template <typename T>
__global__ __launch_bounds__(128) void attn_merge_kernel(CacheView cv, const UnitDesc* __restrict__ descs,
                                                         int layer_begin, int slot_base, PartOut partials,
                                                         T* __restrict__ out, int t_arg, int appending) {
  const int G = cv.G;
  const int g = blockIdx.x % G;
  const UnitDesc d = descs[blockIdx.x / G];
  const int t_before = t_arg >= 0 ? t_arg : cv.cnt_a[d.layer];
  const int t = t_before + ((appending && t_before < cv.max_new) ? 1 : 0);
  const int TILE = cv.tile_rows;
  int rows = d.n_prompt_rows + t;
  if (cv.index_gen && d.kind == HKV_DYNAMIC) {     // picked chunks (prompt or generated) + the tail behind its last complete chunk
    const int k_now = min(d.k_sel, d.n_chunks + (t_before >> d.c_log2));
    rows = (k_now << d.c_log2) + (t_before & ((1 << d.c_log2) - 1)) + (t - t_before);
  }
  const int n_tiles = (rows + TILE - 1) / TILE;
  if (sizeof(T) == 2 && partials.out_all && n_tiles == 1) return;    // its only tile has written the rows
  const int lrel = d.layer - layer_begin;
  const float* o0 = partials.o + ((size_t)(d.item_begin - slot_base) * G + g) * kD;
  const float* ml0 = partials.ml + (size_t)(d.item_begin - slot_base) * kMlStride + 2 * g;
  T* orow = out + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G + g) * kD;
  merge_head<T>(o0, ml0, n_tiles, G * kD, orow);
}

__global__ void publish_tail_kernel(CacheView cv, int layer_begin, int layer_end) {
  const int i = layer_begin + blockIdx.x * blockDim.x + threadIdx.x;
  if (i < layer_end) cv.cnt_a[i] = cv.cnt_b[i];
}

__global__ void rewind_kernel(CacheView cv, int layer_begin, int layer_end) {
  const int i = layer_begin + blockIdx.x * blockDim.x + threadIdx.x;
  if (i < layer_end) { cv.cnt_a[i] = 0; cv.cnt_b[i] = 0; }
}

// ------------------------------------------------------------------------------------------
// full-KV comparison kernels: same tile and combination code, rows read in place
// ------------------------------------------------------------------------------------------
template <typename T, int G>
__global__ __launch_bounds__(256) void full_attn_kernel(FullView fv, const T* __restrict__ q,
                                                        const T* __restrict__ k, const T* __restrict__ v,
                                                        PartOut partials) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  constexpr int TILE = tile_of<T>();
  const int unit = blockIdx.y;                       // (lrel * batch + b) * Hkv + h
  const int h = unit % fv.n_kv_heads;
  const int b = (unit / fv.n_kv_heads) % fv.batch;
  const int lrel = unit / (fv.n_kv_heads * fv.batch);
  RowMap rm;
  rm.n_rows = fv.cu[b + 1] - fv.cu[b];
  const int row0 = blockIdx.x * TILE;
  if (row0 >= rm.n_rows) return;
  const size_t off = (((size_t)lrel * fv.total_tokens + fv.cu[b]) * fv.n_kv_heads + h) * kD * sizeof(T);
  rm.kbase = reinterpret_cast<const char*>(k) + off;
  rm.vbase = reinterpret_cast<const char*>(v) + off;
  rm.stride = (uint32_t)fv.n_kv_heads * kD * sizeof(T);
  rm.dynamic = 0; rm.sel = nullptr; rm.n_sel_rows = 0; rm.c_log2 = 0; rm.C = rm.n_rows; rm.tail_row = rm.n_rows;
  rm.ktail = 0; rm.vtail = 0;
  const size_t qoff = (((size_t)lrel * fv.batch + b) * fv.n_q_heads + (size_t)h * G) * kD;
  const size_t slot = (size_t)unit * fv.n_tiles_max + blockIdx.x;
  const PartOut part = {partials.o + slot * G * kD, partials.ml + slot * kMlStride};
  run_tile<T, G, false>(rm, q + qoff, fv.scale_log2e, row0, TILE, part, smem);
}

template <typename T>
__global__ __launch_bounds__(128) void full_merge_kernel(FullView fv, PartOut partials, T* __restrict__ out) {
  const int G = fv.G;
  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int h = unit % fv.n_kv_heads;
  const int b = (unit / fv.n_kv_heads) % fv.batch;
  const int lrel = unit / (fv.n_kv_heads * fv.batch);
  const int n_rows = fv.cu[b + 1] - fv.cu[b];
  constexpr int TILE = tile_of<T>();
  const int n_tiles = (n_rows + TILE - 1) / TILE;
  const float* o0 = partials.o + (((size_t)unit * fv.n_tiles_max) * G + g) * kD;
  const float* ml0 = partials.ml + (size_t)unit * fv.n_tiles_max * kMlStride + 2 * g;
  T* orow = out + (((size_t)lrel * fv.batch + b) * fv.n_q_heads + (size_t)h * G + g) * kD;
  merge_head<T>(o0, ml0, n_tiles, G * kD, orow);
}

// ------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------
#define HKV_DISPATCH_G(G_, ...)                 \
  switch (G_) {                                 \
    case 1: { constexpr int GG = 1; __VA_ARGS__; break; } \
    case 2: { constexpr int GG = 2; __VA_ARGS__; break; } \
    case 3: { constexpr int GG = 3; __VA_ARGS__; break; } \
    case 4: { constexpr int GG = 4; __VA_ARGS__; break; } \
    case 5: { constexpr int GG = 5; __VA_ARGS__; break; } \
    case 6: { constexpr int GG = 6; __VA_ARGS__; break; } \
    case 7: { constexpr int GG = 7; __VA_ARGS__; break; } \
    case 8: { constexpr int GG = 8; __VA_ARGS__; break; } \
    default: return hipErrorInvalidValue;       \
  }

static size_t select_smem_bytes(int max_chunks) {
  const size_t n4 = ((size_t)max_chunks + 3) & ~(size_t)3;
  return (kSelHeader + n4) * sizeof(float) + n4 * sizeof(unsigned long long);
}

template <typename T, int G, bool INDEXED = false>
static hipError_t launch_decode_t(const CacheView& cv, int layer_begin, int dyn_begin, int n_dyn, int sitem_begin,
                                  int n_sitems, int slot_base, const void* q, const void* k_new, const void* v_new,
                                  float* parts_o, float* parts_ml, void* out, int t_arg, int use_stored_sigma,
                                  int select_only, int max_chunks, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const PartOut partials = {parts_o, parts_ml, nullptr, sizeof(T) == 2 ? out : nullptr};
  const size_t smem = std::max(attn_smem_bytes<T, G, true>(), select_smem_bytes(max_chunks));
  static std::atomic<size_t> attr{0};      // per instantiation; the attribute is sticky for the process
  if (smem > attr.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_kernel<T, G, INDEXED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr.store(smem, std::memory_order_release);
  }
  if (n_dyn + n_sitems > 0)
    HKV_LAUNCH((decode_kernel<T, G, INDEXED>), dim3(n_dyn + n_sitems), dim3(256), (uint32_t)smem, st, ev0, ev1, cv,
                          layer_begin, dyn_begin, n_dyn, sitem_begin, slot_base, (const T*)q, (const T*)k_new,
                          (const T*)v_new, partials, (T*)out, t_arg, use_stored_sigma, select_only);
  return hipGetLastError();
}

hipError_t launch_chunk_score_sum(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int max_chunks,
                                  const void* q, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (n_dyn <= 0) return hipSuccess;
  const dim3 grid(n_dyn, (max_chunks + 255) / 256);
  if (dtype == HKV_F32)
    HKV_LAUNCH(chunk_score_sum_kernel<float>, grid, dim3(256), 0u, st, ev0, ev1, cv, layer_begin, dyn_begin,
               static_cast<const float*>(q));
  else
    HKV_LAUNCH(chunk_score_sum_kernel<bf16_t>, grid, dim3(256), 0u, st, ev0, ev1, cv, layer_begin, dyn_begin,
               static_cast<const bf16_t*>(q));
  return hipGetLastError();
}

hipError_t launch_chunk_score_max(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, const void* q,
                                  int t_arg, hipStream_t st) {
  if (n_dyn <= 0) return hipSuccess;
  if (dtype == HKV_F32)
    hipLaunchKernelGGL(chunk_score_max_kernel<float>, dim3(n_dyn), dim3(256), 0, st, cv, layer_begin, dyn_begin,
                       (const float*)q, t_arg);
  else
    hipLaunchKernelGGL(chunk_score_max_kernel<bf16_t>, dim3(n_dyn), dim3(256), 0, st, cv, layer_begin, dyn_begin,
                       (const bf16_t*)q, t_arg);
  return hipGetLastError();
}

hipError_t launch_decode(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int sitem_begin,
                         int n_sitems, int slot_base, const void* q, const void* k_new, const void* v_new,
                         float* parts_o, float* parts_ml, void* out, int t_arg, int use_stored_sigma, int select_only,
                         int max_chunks, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (cv.index_gen) {        // bf16 caches only (checked when the cache is laid out)
    if (dtype != HKV_BF16) return hipErrorInvalidValue;
    HKV_DISPATCH_G(cv.G, return (launch_decode_t<bf16_t, GG, true>(cv, layer_begin, dyn_begin, n_dyn, sitem_begin,
                                                                   n_sitems, slot_base, q, k_new, v_new, parts_o, parts_ml,
                                                                   out, t_arg, use_stored_sigma, select_only, max_chunks,
                                                                   st, ev0, ev1)));
  }
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(cv.G, return (launch_decode_t<float, GG>(cv, layer_begin, dyn_begin, n_dyn, sitem_begin, n_sitems,
                                                            slot_base, q, k_new, v_new, parts_o, parts_ml, out, t_arg,
                                                            use_stored_sigma, select_only, max_chunks, st, ev0, ev1)));
  } else {
    HKV_DISPATCH_G(cv.G, return (launch_decode_t<bf16_t, GG>(cv, layer_begin, dyn_begin, n_dyn, sitem_begin, n_sitems,
                                                             slot_base, q, k_new, v_new, parts_o, parts_ml, out, t_arg,
                                                             use_stored_sigma, select_only, max_chunks, st, ev0, ev1)));
  }
  return hipErrorInvalidValue;
}

template <typename T, int G, bool INDEXED = false, int NW = 4, bool STAMPS = false>
static hipError_t launch_dynamic_tiles_t(const CacheView& cv, int layer_begin, int ditem_begin, int n_ditems,
                                         int sitem_begin, int n_sitems, int slot_base, const void* q,
                                         const void* k_new, const void* v_new, float* parts_o, float* parts_ml,
                                         void* out, int t_arg, int reselect, int static_hold, int max_chunks, hipStream_t st,
                                         hipEvent_t ev0, hipEvent_t ev1, unsigned long long* stamps = nullptr,
                                         int n_stamps = 0) {
  const PartOut partials = {parts_o, parts_ml, nullptr, sizeof(T) == 2 ? out : nullptr};
  // reselect: selection scratch and the tile's staging area share the front; the picks sit behind both
  const size_t staging = NW == 4 ? attn_smem_bytes<T, G, true>() : (size_t)NW * G * kPartStride * sizeof(float);
  const size_t front = std::max(staging, reselect ? select_smem_bytes(max_chunks) : (size_t)0);
  const size_t smem = front + (reselect ? (((size_t)max_chunks + 3) & ~(size_t)3) * sizeof(int32_t) : 0);
  static std::atomic<size_t> attr{0};
  if (smem > attr.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dynamic_tiles_kernel<T, G, INDEXED, NW, STAMPS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr.store(smem, std::memory_order_release);
  }
  HKV_LAUNCH((dynamic_tiles_kernel<T, G, INDEXED, NW, STAMPS>), dim3(n_ditems + n_sitems), dim3(NW * 64), (uint32_t)smem, st, ev0, ev1,
                        cv, layer_begin, ditem_begin, n_ditems, sitem_begin, slot_base, (const T*)q, (const T*)k_new,
                        (const T*)v_new, partials, t_arg, reselect, (int)(front / sizeof(float)), static_hold, stamps, n_stamps);
  return hipGetLastError();
}

hipError_t launch_dynamic_tiles(const CacheView& cv, int dtype, int layer_begin, int ditem_begin, int n_ditems,
                                int sitem_begin, int n_sitems, int slot_base, const void* q, const void* k_new,
                                const void* v_new, float* parts_o, float* parts_ml, void* out, int t_arg, int reselect,
                                int static_hold, int max_chunks, void* stamps, int n_stamps, hipStream_t st,
                                hipEvent_t ev0, hipEvent_t ev1) {
  if (n_ditems + n_sitems <= 0) return hipSuccess;
  if (stamps && dtype == HKV_BF16 && !cv.index_gen) {      // diagnostic instantiation with time stamps
    HKV_DISPATCH_G(cv.G, return (launch_dynamic_tiles_t<bf16_t, GG, false, 4, true>(
                             cv, layer_begin, ditem_begin, n_ditems, sitem_begin, n_sitems, slot_base, q, k_new, v_new,
                             parts_o, parts_ml, out, t_arg, reselect, static_hold, max_chunks, st, ev0, ev1,
                             static_cast<unsigned long long*>(stamps), n_stamps)));
    return hipErrorInvalidValue;
  }
  if (cv.index_gen) {        // bf16 caches, tiles that repeat the selection
    if (dtype != HKV_BF16 || !reselect) return hipErrorInvalidValue;
    HKV_DISPATCH_G(cv.G, return (launch_dynamic_tiles_t<bf16_t, GG, true>(cv, layer_begin, ditem_begin, n_ditems, sitem_begin,
                                                                          n_sitems, slot_base, q, k_new, v_new, parts_o,
                                                                          parts_ml, out, t_arg, reselect, static_hold, max_chunks,
                                                                          st, ev0, ev1)));
  }
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(cv.G, return (launch_dynamic_tiles_t<float, GG>(cv, layer_begin, ditem_begin, n_ditems, sitem_begin,
                                                                   n_sitems, slot_base, q, k_new, v_new, parts_o,
                                                                   parts_ml, out, t_arg, reselect, static_hold, max_chunks, st, ev0, ev1)));
  } else {
    HKV_DISPATCH_G(cv.G, return (launch_dynamic_tiles_t<bf16_t, GG>(cv, layer_begin, ditem_begin, n_ditems, sitem_begin,
                                                                    n_sitems, slot_base, q, k_new, v_new, parts_o,
                                                                    parts_ml, out, t_arg, reselect, static_hold, max_chunks, st, ev0, ev1)));
  }
  return hipErrorInvalidValue;
}

template <int G, bool INDEXED = false>
static hipError_t launch_units_t(const CacheView& cv, int layer_begin, int dyn_begin, int n_dyn, int static_begin,
                                 int n_static, const void* q, const void* k_new, const void* v_new, void* out, int t_arg,
                                 int max_chunks, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  // selection scratch and the waves' staging area share the front; the picks sit behind both
  const size_t front = std::max((size_t)kUnitWaves * G * kPartStride * sizeof(float), select_smem_bytes(max_chunks));
  const size_t smem = front + (((size_t)max_chunks + 3) & ~(size_t)3) * sizeof(int32_t);
  static std::atomic<size_t> attr{0};
  if (smem > attr.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&unit_kernel<G, INDEXED>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr.store(smem, std::memory_order_release);
  }
  HKV_LAUNCH((unit_kernel<G, INDEXED>), dim3(n_dyn + n_static), dim3(kUnitWaves * 64), (uint32_t)smem, st, ev0, ev1, cv, layer_begin,
             dyn_begin, n_dyn, static_begin, (const bf16_t*)q, (const bf16_t*)k_new, (const bf16_t*)v_new, (bf16_t*)out,
             t_arg, (int)(front / sizeof(float)));
  return hipGetLastError();
}

hipError_t launch_units(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int static_begin,
                        int n_static, const void* q, const void* k_new, const void* v_new, void* out, int t_arg,
                        int max_chunks, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (dtype != HKV_BF16) return hipErrorInvalidValue;
  if (n_dyn + n_static <= 0) return hipSuccess;
  if (cv.index_gen) {
    HKV_DISPATCH_G(cv.G, return (launch_units_t<GG, true>(cv, layer_begin, dyn_begin, n_dyn, static_begin, n_static, q,
                                                          k_new, v_new, out, t_arg, max_chunks, st, ev0, ev1)));
  }
  HKV_DISPATCH_G(cv.G, return (launch_units_t<GG>(cv, layer_begin, dyn_begin, n_dyn, static_begin, n_static, q, k_new,
                                                  v_new, out, t_arg, max_chunks, st, ev0, ev1)));
  return hipErrorInvalidValue;
}

hipError_t launch_attn_merge(const CacheView& cv, int dtype, const UnitDesc* descs, int n_units, int layer_begin,
                             int layer_end, int slot_base, float* parts_o, float* parts_ml, void* out, int t_arg,
                             int appending, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  const PartOut partials = {parts_o, parts_ml, nullptr, dtype == HKV_BF16 ? out : nullptr};
  const int n_blocks = n_units * cv.G;
  if (n_blocks > 0) {
    if (dtype == HKV_F32)
      HKV_LAUNCH(attn_merge_kernel<float>, dim3(n_blocks), dim3(128), 0u, st, ev0, ev1, cv, descs,
                            layer_begin, slot_base, partials, (float*)out, t_arg, appending);
    else
      HKV_LAUNCH(attn_merge_kernel<bf16_t>, dim3(n_blocks), dim3(128), 0u, st, ev0, ev1, cv, descs,
                            layer_begin, slot_base, partials, (bf16_t*)out, t_arg, appending);
  }
  if (t_arg < 0 && layer_end > layer_begin)
    hipLaunchKernelGGL(publish_tail_kernel, dim3((layer_end - layer_begin + 63) / 64), dim3(64), 0, st, cv, layer_begin,
                       layer_end);
  return hipGetLastError();
}

template <int G>
static hipError_t launch_stream_t(const CacheView& cv, const StreamBound* bounds, int n_wg, int unit_base, int layer_begin,
                                  const void* q, const void* k_new, const void* v_new, float* parts_o,
                                  float* parts_ml, void* out, int t_arg, int max_chunks, hipStream_t st, hipEvent_t ev0,
                                  hipEvent_t ev1) {
  const PartOut partials = {parts_o, parts_ml, nullptr};
  // selection scratch and the waves' staging area share the front; the picks sit behind both
  const size_t front = std::max(attn_smem_bytes<bf16_t, G, true>(), select_smem_bytes(max_chunks));
  const size_t smem = front + (((size_t)max_chunks + 3) & ~(size_t)3) * sizeof(int32_t);
  static std::atomic<size_t> attr{0};          // per instantiation; the attribute is sticky for the process
  if (smem > attr.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&stream_kernel<G>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr.store(smem, std::memory_order_release);
  }
  HKV_LAUNCH((stream_kernel<G>), dim3(n_wg), dim3(256), (uint32_t)smem, st, ev0, ev1, cv, bounds, unit_base, layer_begin,
             (const bf16_t*)q, (const bf16_t*)k_new, (const bf16_t*)v_new, partials, (bf16_t*)out, t_arg,
             (int)(front / sizeof(float)));
  return hipGetLastError();
}

hipError_t launch_stream(const CacheView& cv, int dtype, const StreamBound* bounds, int n_wg, int unit_base, int layer_begin,
                         const void* q, const void* k_new, const void* v_new, float* parts_o, float* parts_ml,
                         void* out, int t_arg, int max_chunks, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (dtype != HKV_BF16 || cv.index_gen) return hipErrorInvalidValue;
  if (n_wg <= 0) return hipSuccess;
  HKV_DISPATCH_G(cv.G, return (launch_stream_t<GG>(cv, bounds, n_wg, unit_base, layer_begin, q, k_new, v_new, parts_o,
                                                   parts_ml, out, t_arg, max_chunks, st, ev0, ev1)));
  return hipErrorInvalidValue;
}

hipError_t launch_stream_merge(const CacheView& cv, int dtype, const StreamMulti* multi, int n_multi, int unit_base,
                               int layer_begin, int layer_end, float* parts_o, float* parts_ml, void* out, int t_arg,
                               hipStream_t st, hipEvent_t ev0, hipEvent_t ev1) {
  if (dtype != HKV_BF16) return hipErrorInvalidValue;
  const PartOut partials = {parts_o, parts_ml, nullptr};
  if (n_multi > 0)
    HKV_LAUNCH(stream_merge_kernel<bf16_t>, dim3(n_multi * cv.G), dim3(128), 0u, st, ev0, ev1, cv, multi, unit_base,
               layer_begin, partials, (bf16_t*)out);
  if (t_arg < 0 && layer_end > layer_begin)
    hipLaunchKernelGGL(publish_tail_kernel, dim3((layer_end - layer_begin + 63) / 64), dim3(64), 0, st, cv, layer_begin,
                       layer_end);
  return hipGetLastError();
}

hipError_t launch_rewind(const CacheView& cv, int layer_begin, int layer_end, hipStream_t st) {
  if (layer_end <= layer_begin) return hipSuccess;
  hipLaunchKernelGGL(rewind_kernel, dim3((layer_end - layer_begin + 63) / 64), dim3(64), 0, st, cv, layer_begin,
                     layer_end);
  return hipGetLastError();
}

template <typename T, int G>
static hipError_t launch_full_t(const FullView& fv, const void* q, const void* k, const void* v, float* parts_o,
                                float* parts_ml, void* out, hipStream_t st) {
  const PartOut partials = {parts_o, parts_ml};
  constexpr size_t smem = attn_smem_bytes<T, G, false>();
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&full_attn_kernel<T, G>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set.store(true, std::memory_order_release);
  }
  const int n_units = fv.n_layers_call * fv.batch * fv.n_kv_heads;
  hipLaunchKernelGGL((full_attn_kernel<T, G>), dim3(fv.n_tiles_max, n_units), dim3(256), smem, st, fv, (const T*)q,
                     (const T*)k, (const T*)v, partials);
  hipLaunchKernelGGL(full_merge_kernel<T>, dim3(n_units * G), dim3(128), 0, st, fv, partials, (T*)out);
  return hipGetLastError();
}

hipError_t launch_full_attn(const FullView& fv, int dtype, const void* q, const void* k, const void* v,
                            float* parts_o, float* parts_ml, void* out, hipStream_t st) {
  const int n_units = fv.n_layers_call * fv.batch * fv.n_kv_heads;
  if (n_units <= 0 || fv.n_tiles_max <= 0) return hipSuccess;
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(fv.G, return (launch_full_t<float, GG>(fv, q, k, v, parts_o, parts_ml, out, st)));
  } else {
    HKV_DISPATCH_G(fv.G, return (launch_full_t<bf16_t, GG>(fv, q, k, v, parts_o, parts_ml, out, st)));
  }
  return hipErrorInvalidValue;
}

}  // namespace hkv
