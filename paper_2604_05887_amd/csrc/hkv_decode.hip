// Decode-step kernels of libhkv (gfx950):
//   prepare_kernel   append the step's K/V rows to every head's tail; for dynamic heads score all
//                    chunk summaries with the group-summed query and pick the top-k chunks
//                    (paper, Appendix A, "KV Cache Retrieval for Dynamic Heads")
//   attn_partial     split-K softmax attention over a tile of a head's retained rows: compacted
//                    rows (static heads), gathered chunk rows (dynamic heads) or all rows (full KV)
//   attn_merge       log-sum-exp combination of the tiles in fixed order, cast to the output dtype
#include "hkv_device.h"
#include "hkv_internal.h"
#include "hkv_select.h"

namespace hkv {

// Where the logical rows of one head live.
struct RowMap {
  const char* kbase;
  const char* vbase;
  int64_t stride;        // bytes between consecutive physical rows
  const int32_t* sel;    // dynamic: selected chunk ids (ascending)
  int32_t dynamic;
  int32_t n_sel_rows;    // dynamic: k_sel << c_log2
  int32_t c_log2;
  int32_t C;             // dynamic: prompt rows (tail starts at physical row C)
  int32_t n_rows;        // logical rows to attend (prompt part + tail)
};

__device__ __forceinline__ bool resolve_row(const RowMap& rm, int r, int64_t& phys) {
  if (!rm.dynamic) { phys = r; return true; }
  if (r < rm.n_sel_rows) {
    const int ch = rm.sel[r >> rm.c_log2];
    phys = ((int64_t)ch << rm.c_log2) + (r & ((1 << rm.c_log2) - 1));
    return phys >= 0 && phys < rm.C;    // the last chunk of the prompt may be short
  }
  phys = (int64_t)rm.C + (r - rm.n_sel_rows);
  return true;
}

// One tile (kTileF32 logical rows starting at row0) of one KV head for its G query heads; any dtype.
// Writes G records of kPartStride floats: [0]=running max (log2 domain), [1]=sum, [4..131]=unnormalised o.
template <typename T, int G>
__device__ __forceinline__ void attn_tile(const RowMap& rm, const T* __restrict__ q, float scale_log2e, int row0,
                                          float* __restrict__ part, float* smem) {
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
        kraw = ld16(rm.kbase + phys * rm.stride + sub * 16);
        vraw = ld16(rm.vbase + phys * rm.stride + sub * 16);
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
  if (tid < kD) {
#pragma unroll
    for (int g = 0; g < G; ++g) {
      float mm = kNeg;
#pragma unroll
      for (int w = 0; w < 4; ++w) mm = fmaxf(mm, smem[(w * G + g) * kPartStride]);
      float ll = 0.f, oo = 0.f;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const float c = fast_exp2(smem[(w * G + g) * kPartStride] - mm);
        ll = fmaf(smem[(w * G + g) * kPartStride + 1], c, ll);
        oo = fmaf(smem[(w * G + g) * kPartStride + 4 + tid], c, oo);
      }
      part[g * kPartStride + 4 + tid] = oo;
      if (tid == 0) { part[g * kPartStride] = mm; part[g * kPartStride + 1] = ll; }
    }
  }
}

// ---- bf16 tile: packed dot products, transpose-reduce across the 16 lanes of a row ----------------
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ float dot2bf(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}
template <int CTRL> __device__ __forceinline__ float dpp_max(float x) { return fmaxf(x, dpp_mov<CTRL>(x)); }

constexpr int kStreams = 16;          // 4 waves x 4 row groups, each an independent online-softmax stream
constexpr int kPGroupStride = 40;     // dwords per (wave, group) in the weight exchange buffer (32 + pad)
template <int G> constexpr size_t attn_bf16_smem_bytes() {
  return (size_t)kStreams * G * kPartStride * sizeof(float) + (size_t)kStreams * kPGroupStride * 4;
}

// One tile of kTileBf16 logical rows.  Lane (grp = lane / 16, sub = lane % 16) loads 16 bytes (8 dims) of
// row 4*i + grp for i = 0..7 of each 32-row half batch; per query head the 8 partial dot products are
// summed across the 16 lanes by a butterfly that leaves lane `sub` with the full score of row i = sub % 8.
// Softmax weights go through shared memory as bf16 pairs of two rows so that the weighted sum of V uses
// packed dot products as well.
template <int G>
__device__ __forceinline__ void attn_tile_bf16(const RowMap& rm, const bf16_t* __restrict__ q, float scale_log2e,
                                               int row0, float* __restrict__ part, float* smem) {
  constexpr int HB = 32, NHB = kTileBf16 / 4 / HB;
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

#pragma unroll 1
  for (int hb = 0; hb < NHB; ++hb) {
    const int rbase = row0 + (wv * NHB + hb) * HB;
    if (rbase >= rm.n_rows) break;                       // wave-uniform
    uint4 kraw[8], vraw[8];
    uint32_t vmask = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int r = rbase + 4 * i + grp;
      bool valid = r < rm.n_rows;
      int64_t phys = 0;
      if (valid) valid = resolve_row(rm, r, phys);
      kraw[i] = make_uint4(0, 0, 0, 0); vraw[i] = make_uint4(0, 0, 0, 0);
      if (valid) {
        kraw[i] = ld16(rm.kbase + phys * rm.stride + sub * 16);
        vraw[i] = ld16(rm.vbase + phys * rm.stride + sub * 16);
        vmask |= 1u << i;
      }
    }
    // partial scores, then all-reduce over the mirror pair (stage 1 of the butterfly)
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
    // reduce-scatter: after the three stages lane sub holds row i = sub & 7, summed over all 16 lanes
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
    const bool my_valid = (vmask >> (sub & 7)) & 1u;
    float p[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float keep = b1 ? v[1][g] : v[0][g], send = b1 ? v[0][g] : v[1][g];
      float s = (keep + dpp_mov<0xB1>(send)) * scale_log2e;   // quad_perm [1,0,3,2]: partner sub ^ 1
      s = my_valid ? s : kNeg;
      float gm = dpp_max<0xB1>(s);
      gm = dpp_max<0x4E>(gm);
      gm = dpp_max<0x141>(gm);
      gm = dpp_max<0x140>(gm);                           // maximum over the row group's 8 rows
      const float mn = fmaxf(m[g], gm);
      const float corr = fast_exp2(m[g] - mn);
      p[g] = my_valid ? fast_exp2(s - mn) : 0.f;
      l[g] = fmaf(l[g], corr, sub < 8 ? p[g] : 0.f);     // lanes sub >= 8 hold duplicates of rows 0..7
      m[g] = mn;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[g][e] *= corr;
    }
    // weights -> shared memory as bf16, paired by rows (2t, 2t+1): dword [t][g] = (p_2t, p_2t+1)
    if (sub < 8) {
      uint16_t* ph = reinterpret_cast<uint16_t*>(pbuf) + (size_t)((sub >> 1) * 8) * 2 + (sub & 1);
#pragma unroll
      for (int g = 0; g < G; ++g) ph[g * 2] = f32_to_bf16_rne(p[g]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
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
    const float lt = sum16(l[g]);
    if (sub == 0) { mine[g * kPartStride + 0] = m[g]; mine[g * kPartStride + 1] = lt; }
    float4* dst = reinterpret_cast<float4*>(mine + g * kPartStride + 4 + sub * 8);
    dst[0] = make_float4(acc[g][0], acc[g][1], acc[g][2], acc[g][3]);
    dst[1] = make_float4(acc[g][4], acc[g][5], acc[g][6], acc[g][7]);
  }
  __syncthreads();
  for (int idx = tid; idx < G * kD; idx += 256) {
    const int g = idx >> 7, dd = idx & (kD - 1);
    float mm = kNeg;
#pragma unroll
    for (int s = 0; s < kStreams; ++s) mm = fmaxf(mm, smem[(s * G + g) * kPartStride]);
    float ll = 0.f, oo = 0.f;
#pragma unroll
    for (int s = 0; s < kStreams; ++s) {
      const float c = fast_exp2(smem[(s * G + g) * kPartStride] - mm);
      ll = fmaf(smem[(s * G + g) * kPartStride + 1], c, ll);
      oo = fmaf(smem[(s * G + g) * kPartStride + 4 + dd], c, oo);
    }
    part[g * kPartStride + 4 + dd] = oo;
    if (dd == 0) { part[g * kPartStride] = mm; part[g * kPartStride + 1] = ll; }
  }
}

template <typename T, int G> constexpr size_t attn_smem_bytes() {
  if constexpr (sizeof(T) == 2) return attn_bf16_smem_bytes<G>() + 16;
  else return (size_t)4 * G * kPartStride * sizeof(float) + 16;
}
template <typename T> __device__ __forceinline__ constexpr int tile_of() { return sizeof(T) == 2 ? kTileBf16 : kTileF32; }

template <typename T, int G>
__device__ __forceinline__ void run_tile(const RowMap& rm, const T* __restrict__ q, float scale_log2e, int row0,
                                         float* __restrict__ part, float* smem) {
  if constexpr (sizeof(T) == 2) attn_tile_bf16<G>(rm, q, scale_log2e, row0, part, smem);
  else attn_tile<T, G>(rm, q, scale_log2e, row0, part, smem);
}

// After a block has written its record: count it; the block that completes the unit combines all
// n_tiles records in tile order (so the result does not depend on which block that is), writes the
// G output rows and re-arms the counter.  Returns true in the combining block.
template <typename T>
__device__ __forceinline__ bool finish_unit(const float* __restrict__ unit_parts, int n_tiles, int G, int32_t* counter,
                                            T* __restrict__ out_rows, int* flag) {
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    const int old = n_tiles > 1 ? atomicAdd(counter, 1) : 0;
    *flag = (old == n_tiles - 1) ? 1 : 0;
  }
  __syncthreads();
  if (!*flag) return false;
  __threadfence();
  const int rec = G * kPartStride;
  for (int idx = threadIdx.x; idx < G * kD; idx += blockDim.x) {
    const int g = idx >> 7, dd = idx & (kD - 1);
    const float* p0 = unit_parts + g * kPartStride;
    float mm = kNeg;
    for (int t = 0; t < n_tiles; ++t) mm = fmaxf(mm, __builtin_nontemporal_load(p0 + (size_t)t * rec));
    float ll = 0.f, oo = 0.f;
    for (int t = 0; t < n_tiles; ++t) {
      const float* p = p0 + (size_t)t * rec;
      const float c = fast_exp2(__builtin_nontemporal_load(p) - mm);
      ll = fmaf(__builtin_nontemporal_load(p + 1), c, ll);
      oo = fmaf(__builtin_nontemporal_load(p + 4 + dd), c, oo);
    }
    const float o = ll > 0.f ? oo / ll : 0.f;
    if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(out_rows)[idx] = o;
    else reinterpret_cast<uint16_t*>(out_rows)[idx] = f32_to_bf16_rne(o);
  }
  if (threadIdx.x == 0 && n_tiles > 1) *counter = 0;
  return true;
}

// ------------------------------------------------------------------------------------------
// hybrid cache kernels
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void prepare_kernel(CacheView cv, int layer_begin, int unit_begin,
                                                      const T* __restrict__ q, const T* __restrict__ k_new,
                                                      const T* __restrict__ v_new, int use_stored_sigma,
                                                      int do_step) {
  extern __shared__ float dsm[];
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow;
  const int tid = threadIdx.x;
  const UnitDesc d = cv.units[unit_begin + blockIdx.x];
  const int lrel = d.layer - layer_begin;

  if (do_step) {
    const int t = cv.cnt_a[d.layer];
    const bool append = (k_new != nullptr) && (t < cv.max_new);
    if (append && tid < 2 * LPR) {
      const int which = tid / LPR, sub = tid % LPR;
      const int64_t base_rows = d.kind == HKV_STATIC ? d.n_prompt_rows : d.C;
      const size_t src = (((size_t)lrel * cv.batch + d.seq) * cv.n_kv_heads + d.head) * kD * sizeof(T) + sub * 16;
      const size_t dst = (size_t)(d.kv_row_off + base_rows + t) * kD * sizeof(T) + sub * 16;
      if (which == 0) st16(reinterpret_cast<char*>(cv.k_rows) + dst, ld16(reinterpret_cast<const char*>(k_new) + src));
      else st16(reinterpret_cast<char*>(cv.v_rows) + dst, ld16(reinterpret_cast<const char*>(v_new) + src));
    }
    if (d.seq == 0 && d.head == 0 && tid == 0) cv.cnt_b[d.layer] = t + (append ? 1 : 0);
  }
  if (d.kind != HKV_DYNAMIC) return;

  float* qsum = dsm;                                         // [128]
  uint32_t* hist = reinterpret_cast<uint32_t*>(dsm + kD);    // [256]
  uint32_t* bc = hist + 256;                                 // [2]
  int* scan = reinterpret_cast<int*>(bc + 2);                // [6]
  float* sig = dsm + kD + 256 + 8;                           // [n_chunks]
  const int n_c = d.n_chunks;

  if (!use_stored_sigma) {
    if (tid < kD) {
      const T* qp = q + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * cv.G) * kD + tid;
      float s = 0.f;
      for (int g = 0; g < cv.G; ++g) {
        float x;
        if constexpr (sizeof(T) == 4) x = reinterpret_cast<const float*>(qp)[(size_t)g * kD];
        else x = bits_to_float((uint32_t)reinterpret_cast<const uint16_t*>(qp)[(size_t)g * kD] << 16);
        s += x;
      }
      qsum[tid] = s;
    }
    __syncthreads();
    const int sub = tid % LPR, slot = tid / LPR;
    constexpr int RP = 256 / LPR;
    float qf[EPL];
#pragma unroll
    for (int e = 0; e < EPL; ++e) qf[e] = qsum[sub * EPL + e];
    const char* mu = reinterpret_cast<const char*>(cv.mu) + (size_t)d.aux_off * kD * sizeof(T);
    for (int ch0 = 0; ch0 < n_c; ch0 += RP) {       // uniform trip count
      const int ch = ch0 + slot;
      float dot = 0.f;
      if (ch < n_c) {
        float mf[EPL];
        unpack16(ld16(mu + (size_t)ch * kD * sizeof(T) + sub * 16), mf, T{});
#pragma unroll
        for (int e = 0; e < EPL; ++e) dot = fmaf(qf[e], mf[e], dot);
      }
      dot = sum_lanes<LPR>(dot);
      if (ch < n_c && sub == 0) { sig[ch] = dot; cv.sigma[d.aux_off + ch] = dot; }
    }
  } else {
    for (int ch = tid; ch < n_c; ch += 256) sig[ch] = cv.sigma[d.aux_off + ch];
  }
  __syncthreads();

  // top-k chunks, ties to the lower chunk id, emitted ascending
  uint32_t T_key = 0;
  int r_adm = n_c;
  if (d.k_sel < n_c) {
    radix_select<256>(n_c, d.k_sel,
                      [&](int j, uint32_t& key) { key = float_order_key(sig[j]); return true; },
                      hist, bc, T_key, r_adm);
  }
  int base_eq = 0, base_keep = 0;
  for (int ch0 = 0; ch0 < n_c; ch0 += 256) {
    const int ch = ch0 + tid;
    uint32_t key = 0;
    const bool in = ch < n_c;
    if (in) key = float_order_key(sig[ch]);
    const int eq = (in && key == T_key) ? 1 : 0;
    const int gt = (in && key > T_key) ? 1 : 0;
    int tot_eq, tot_keep;
    const int eq_rank = base_eq + block_exclusive_scan<256>(eq, scan, &tot_eq);
    const int keep = gt | (eq & (eq_rank < r_adm ? 1 : 0));
    const int pos = base_keep + block_exclusive_scan<256>(keep, scan, &tot_keep);
    if (keep && pos < d.k_sel) cv.sel[d.idx_off + pos] = ch;
    base_eq += tot_eq;
    base_keep += tot_keep;
  }
}

template <typename T, int G>
__global__ __launch_bounds__(256) void attn_kernel(CacheView cv, int layer_begin, int item_begin,
                                                   const T* __restrict__ q, float* __restrict__ partials,
                                                   T* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) float smem[];
  constexpr int TILE = tile_of<T>();
  const int2 item = cv.items[item_begin + blockIdx.x];
  const UnitDesc d = cv.units[item.x];
  const int t = cv.cnt_b[d.layer];
  RowMap rm;
  rm.n_rows = d.n_prompt_rows + t;
  const int row0 = item.y * TILE;
  if (row0 >= rm.n_rows) return;          // tile reserved for tail growth, not reached yet
  rm.kbase = reinterpret_cast<const char*>(cv.k_rows) + (size_t)d.kv_row_off * kD * sizeof(T);
  rm.vbase = reinterpret_cast<const char*>(cv.v_rows) + (size_t)d.kv_row_off * kD * sizeof(T);
  rm.stride = kD * sizeof(T);
  rm.dynamic = d.kind == HKV_DYNAMIC;
  rm.sel = cv.sel + d.idx_off;
  rm.n_sel_rows = d.n_prompt_rows;
  rm.c_log2 = d.c_log2;
  rm.C = d.C;
  const int lrel = d.layer - layer_begin;
  const size_t qoff = (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G) * kD;
  float* part = partials + (size_t)blockIdx.x * G * kPartStride;
  run_tile<T, G>(rm, q + qoff, cv.scale_log2e, row0, part, smem);

  const int n_tiles = (rm.n_rows + TILE - 1) / TILE;
  int* flag = reinterpret_cast<int*>(smem + attn_smem_bytes<T, G>() / sizeof(float) - 4);
  const float* unit_parts = partials + (size_t)(d.item_begin - item_begin) * G * kPartStride;
  if (finish_unit<T>(unit_parts, n_tiles, G, cv.done + item.x, out + qoff, flag)) {
    // the step is complete for this unit; one unit per layer moves the tail counter on
    if (d.seq == 0 && d.head == 0 && threadIdx.x == 0) cv.cnt_a[d.layer] = t;
  }
}

__global__ void rewind_kernel(CacheView cv, int layer_begin, int layer_end) {
  const int i = layer_begin + blockIdx.x * blockDim.x + threadIdx.x;
  if (i < layer_end) { cv.cnt_a[i] = 0; cv.cnt_b[i] = 0; }
}

// ------------------------------------------------------------------------------------------
// full-KV comparison kernel: same tile code and the same fused combination, rows read in place
// ------------------------------------------------------------------------------------------
__global__ void zero_kernel(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <typename T, int G>
__global__ __launch_bounds__(256) void full_attn_kernel(FullView fv, const T* __restrict__ q,
                                                        const T* __restrict__ k, const T* __restrict__ v,
                                                        float* __restrict__ partials, T* __restrict__ out) {
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
  rm.stride = (int64_t)fv.n_kv_heads * kD * sizeof(T);
  rm.dynamic = 0; rm.sel = nullptr; rm.n_sel_rows = 0; rm.c_log2 = 0; rm.C = rm.n_rows;
  const size_t qoff = (((size_t)lrel * fv.batch + b) * fv.n_q_heads + (size_t)h * G) * kD;
  float* unit_parts = partials + (size_t)unit * fv.n_tiles_max * G * kPartStride;
  run_tile<T, G>(rm, q + qoff, fv.scale_log2e, row0, unit_parts + (size_t)blockIdx.x * G * kPartStride, smem);
  const int n_tiles = (rm.n_rows + TILE - 1) / TILE;
  int* flag = reinterpret_cast<int*>(smem + attn_smem_bytes<T, G>() / sizeof(float) - 4);
  finish_unit<T>(unit_parts, n_tiles, G, fv.done + unit, out + qoff, flag);
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

hipError_t launch_prepare(const CacheView& cv, int dtype, int layer_begin, int layer_end, const void* q,
                          const void* k_new, const void* v_new, int use_stored_sigma, int do_step,
                          int max_chunks, hipStream_t st) {
  const int upl = cv.batch * cv.n_kv_heads;
  const int n_units = (layer_end - layer_begin) * upl;
  if (n_units <= 0) return hipSuccess;
  const size_t smem = (size_t)(kD + 256 + 8 + max_chunks) * sizeof(float);
  if (dtype == HKV_F32)
    hipLaunchKernelGGL(prepare_kernel<float>, dim3(n_units), dim3(256), smem, st, cv, layer_begin, layer_begin * upl,
                       (const float*)q, (const float*)k_new, (const float*)v_new, use_stored_sigma, do_step);
  else
    hipLaunchKernelGGL(prepare_kernel<bf16_t>, dim3(n_units), dim3(256), smem, st, cv, layer_begin, layer_begin * upl,
                       (const bf16_t*)q, (const bf16_t*)k_new, (const bf16_t*)v_new, use_stored_sigma, do_step);
  return hipGetLastError();
}

template <typename T, int G>
static hipError_t launch_attn_t(const CacheView& cv, int layer_begin, int item_begin, int n_items, const void* q,
                                float* partials, void* out, hipStream_t st) {
  constexpr size_t smem = attn_smem_bytes<T, G>();
  static bool attr_set = false;     // per instantiation; the attribute is sticky for the process
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<T, G>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL((attn_kernel<T, G>), dim3(n_items), dim3(256), smem, st, cv, layer_begin, item_begin,
                     (const T*)q, partials, (T*)out);
  return hipGetLastError();
}

hipError_t launch_attn(const CacheView& cv, int dtype, int layer_begin, int item_begin, int n_items, const void* q,
                       float* partials, void* out, hipStream_t st) {
  if (n_items <= 0) return hipSuccess;
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(cv.G, return (launch_attn_t<float, GG>(cv, layer_begin, item_begin, n_items, q, partials, out, st)));
  } else {
    HKV_DISPATCH_G(cv.G, return (launch_attn_t<bf16_t, GG>(cv, layer_begin, item_begin, n_items, q, partials, out, st)));
  }
  return hipErrorInvalidValue;
}

hipError_t launch_rewind(const CacheView& cv, int layer_begin, int layer_end, hipStream_t st) {
  if (layer_end <= layer_begin) return hipSuccess;
  hipLaunchKernelGGL(rewind_kernel, dim3((layer_end - layer_begin + 63) / 64), dim3(64), 0, st, cv, layer_begin,
                     layer_end);
  return hipGetLastError();
}

template <typename T, int G>
static hipError_t launch_full_t(const FullView& fv, const void* q, const void* k, const void* v, float* partials,
                                void* out, hipStream_t st) {
  constexpr size_t smem = attn_smem_bytes<T, G>();
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&full_attn_kernel<T, G>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int n_units = fv.n_layers_call * fv.batch * fv.n_kv_heads;
  hipLaunchKernelGGL(zero_kernel, dim3((n_units + 255) / 256), dim3(256), 0, st, fv.done, n_units);
  hipLaunchKernelGGL((full_attn_kernel<T, G>), dim3(fv.n_tiles_max, n_units), dim3(256), smem, st, fv, (const T*)q,
                     (const T*)k, (const T*)v, partials, (T*)out);
  return hipGetLastError();
}

hipError_t launch_full_attn(const FullView& fv, int dtype, const void* q, const void* k, const void* v,
                            float* partials, void* out, hipStream_t st) {
  const int n_units = fv.n_layers_call * fv.batch * fv.n_kv_heads;
  if (n_units <= 0 || fv.n_tiles_max <= 0) return hipSuccess;
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(fv.G, return (launch_full_t<float, GG>(fv, q, k, v, partials, out, st)));
  } else {
    HKV_DISPATCH_G(fv.G, return (launch_full_t<bf16_t, GG>(fv, q, k, v, partials, out, st)));
  }
  return hipErrorInvalidValue;
}

}  // namespace hkv
