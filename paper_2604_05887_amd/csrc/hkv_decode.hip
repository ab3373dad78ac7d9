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

// One tile (kTile logical rows starting at row0) of one KV head for its G query heads.
// Writes G records of kPartStride floats: [0]=running max (log2 domain), [1]=sum, [4..131]=unnormalised o.
template <typename T, int G>
__device__ __forceinline__ void attn_tile(const RowMap& rm, const T* __restrict__ q, float scale_log2e, int row0,
                                          float* __restrict__ part, float* smem) {
  constexpr int EPL = Elem<T>::kPer16, LPR = Elem<T>::kLanesPerRow, RPW = 64 / LPR;
  constexpr int WROWS = kTile / 4;
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

// Combine n_tiles records of one (unit, query head) in tile order and write the output row.
template <typename T>
__device__ __forceinline__ void merge_tiles(const float* __restrict__ part0, int n_tiles, int tile_stride,
                                            T* __restrict__ out_row) {
  const int tid = threadIdx.x;   // 128 threads, one per output element
  float mm = kNeg;
  for (int t = 0; t < n_tiles; ++t) mm = fmaxf(mm, part0[(size_t)t * tile_stride]);
  float ll = 0.f, oo = 0.f;
  for (int t = 0; t < n_tiles; ++t) {
    const float* p = part0 + (size_t)t * tile_stride;
    const float c = fast_exp2(p[0] - mm);
    ll = fmaf(p[1], c, ll);
    oo = fmaf(p[4 + tid], c, oo);
  }
  const float o = ll > 0.f ? oo / ll : 0.f;
  if constexpr (sizeof(T) == 4) reinterpret_cast<float*>(out_row)[tid] = o;
  else reinterpret_cast<uint16_t*>(out_row)[tid] = f32_to_bf16_rne(o);
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
__global__ __launch_bounds__(256) void attn_partial_kernel(CacheView cv, int layer_begin, int item_begin,
                                                           const T* __restrict__ q, float* __restrict__ partials) {
  __shared__ float smem[4 * G * kPartStride];
  const int2 item = cv.items[item_begin + blockIdx.x];
  const UnitDesc d = cv.units[item.x];
  const int t = cv.cnt_b[d.layer];
  RowMap rm;
  rm.n_rows = d.n_prompt_rows + t;
  const int row0 = item.y * kTile;
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
  const T* qh = q + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G) * kD;
  float* part = partials + (size_t)blockIdx.x * G * kPartStride;
  attn_tile<T, G>(rm, qh, cv.scale_log2e, row0, part, smem);
}

template <typename T>
__global__ __launch_bounds__(128) void attn_merge_kernel(CacheView cv, int layer_begin, int unit_begin,
                                                         int item_base, const float* __restrict__ partials,
                                                         T* __restrict__ out, int advance_tail) {
  const int G = cv.G;
  const int u = unit_begin + blockIdx.x / G, g = blockIdx.x % G;
  const UnitDesc d = cv.units[u];
  const int t = cv.cnt_b[d.layer];
  const int n_rows = d.n_prompt_rows + t;
  const int n_tiles = (n_rows + kTile - 1) / kTile;
  const int lrel = d.layer - layer_begin;
  const float* p0 = partials + ((size_t)(d.item_begin - item_base) * G + g) * kPartStride;
  T* orow = out + (((size_t)lrel * cv.batch + d.seq) * cv.n_q_heads + (size_t)d.head * G + g) * kD;
  merge_tiles<T>(p0, n_tiles, G * kPartStride, orow);
  if (advance_tail && d.seq == 0 && d.head == 0 && g == 0 && threadIdx.x == 0) cv.cnt_a[d.layer] = t;
}

__global__ void rewind_kernel(CacheView cv, int layer_begin, int layer_end) {
  const int i = layer_begin + blockIdx.x * blockDim.x + threadIdx.x;
  if (i < layer_end) { cv.cnt_a[i] = 0; cv.cnt_b[i] = 0; }
}

// ------------------------------------------------------------------------------------------
// full-KV comparison kernels
// ------------------------------------------------------------------------------------------
template <typename T, int G>
__global__ __launch_bounds__(256) void full_partial_kernel(FullView fv, const T* __restrict__ q,
                                                           const T* __restrict__ k, const T* __restrict__ v,
                                                           float* __restrict__ partials) {
  __shared__ float smem[4 * G * kPartStride];
  const int unit = blockIdx.y;                       // (lrel * batch + b) * Hkv + h
  const int h = unit % fv.n_kv_heads;
  const int b = (unit / fv.n_kv_heads) % fv.batch;
  const int lrel = unit / (fv.n_kv_heads * fv.batch);
  RowMap rm;
  rm.n_rows = fv.cu[b + 1] - fv.cu[b];
  const int row0 = blockIdx.x * kTile;
  if (row0 >= rm.n_rows) return;
  const size_t off = (((size_t)lrel * fv.total_tokens + fv.cu[b]) * fv.n_kv_heads + h) * kD * sizeof(T);
  rm.kbase = reinterpret_cast<const char*>(k) + off;
  rm.vbase = reinterpret_cast<const char*>(v) + off;
  rm.stride = (int64_t)fv.n_kv_heads * kD * sizeof(T);
  rm.dynamic = 0; rm.sel = nullptr; rm.n_sel_rows = 0; rm.c_log2 = 0; rm.C = rm.n_rows;
  const T* qh = q + (((size_t)lrel * fv.batch + b) * fv.n_q_heads + (size_t)h * G) * kD;
  float* part = partials + ((size_t)unit * fv.n_tiles_max + blockIdx.x) * G * kPartStride;
  attn_tile<T, G>(rm, qh, fv.scale_log2e, row0, part, smem);
}

template <typename T>
__global__ __launch_bounds__(128) void full_merge_kernel(FullView fv, const float* __restrict__ partials,
                                                         T* __restrict__ out) {
  const int G = fv.G;
  const int unit = blockIdx.x / G, g = blockIdx.x % G;
  const int h = unit % fv.n_kv_heads;
  const int b = (unit / fv.n_kv_heads) % fv.batch;
  const int lrel = unit / (fv.n_kv_heads * fv.batch);
  const int n_rows = fv.cu[b + 1] - fv.cu[b];
  const int n_tiles = (n_rows + kTile - 1) / kTile;
  const float* p0 = partials + (((size_t)unit * fv.n_tiles_max) * G + g) * kPartStride;
  T* orow = out + (((size_t)lrel * fv.batch + b) * fv.n_q_heads + (size_t)h * G + g) * kD;
  merge_tiles<T>(p0, n_tiles, G * kPartStride, orow);
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

hipError_t launch_attn_partial(const CacheView& cv, int dtype, int layer_begin, int item_begin, int n_items,
                               const void* q, float* partials, hipStream_t st) {
  if (n_items <= 0) return hipSuccess;
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(cv.G, hipLaunchKernelGGL((attn_partial_kernel<float, GG>), dim3(n_items), dim3(256), 0, st, cv,
                                            layer_begin, item_begin, (const float*)q, partials));
  } else {
    HKV_DISPATCH_G(cv.G, hipLaunchKernelGGL((attn_partial_kernel<bf16_t, GG>), dim3(n_items), dim3(256), 0, st, cv,
                                            layer_begin, item_begin, (const bf16_t*)q, partials));
  }
  return hipGetLastError();
}

hipError_t launch_attn_merge(const CacheView& cv, int dtype, int layer_begin, int layer_end, int item_base,
                             const float* partials, void* out, int advance_tail, hipStream_t st) {
  const int upl = cv.batch * cv.n_kv_heads;
  const int n_blocks = (layer_end - layer_begin) * upl * cv.G;
  if (n_blocks <= 0) return hipSuccess;
  if (dtype == HKV_F32)
    hipLaunchKernelGGL(attn_merge_kernel<float>, dim3(n_blocks), dim3(128), 0, st, cv, layer_begin, layer_begin * upl,
                       item_base, partials, (float*)out, advance_tail);
  else
    hipLaunchKernelGGL(attn_merge_kernel<bf16_t>, dim3(n_blocks), dim3(128), 0, st, cv, layer_begin,
                       layer_begin * upl, item_base, partials, (bf16_t*)out, advance_tail);
  return hipGetLastError();
}

hipError_t launch_rewind(const CacheView& cv, int layer_begin, int layer_end, hipStream_t st) {
  if (layer_end <= layer_begin) return hipSuccess;
  hipLaunchKernelGGL(rewind_kernel, dim3((layer_end - layer_begin + 63) / 64), dim3(64), 0, st, cv, layer_begin,
                     layer_end);
  return hipGetLastError();
}

hipError_t launch_full_attn(const FullView& fv, int dtype, const void* q, const void* k, const void* v,
                            float* partials, void* out, hipStream_t st) {
  const int n_units = fv.n_layers_call * fv.batch * fv.n_kv_heads;
  if (n_units <= 0 || fv.n_tiles_max <= 0) return hipSuccess;
  const dim3 grid(fv.n_tiles_max, n_units);
  if (dtype == HKV_F32) {
    HKV_DISPATCH_G(fv.G, hipLaunchKernelGGL((full_partial_kernel<float, GG>), grid, dim3(256), 0, st, fv,
                                            (const float*)q, (const float*)k, (const float*)v, partials));
    hipLaunchKernelGGL(full_merge_kernel<float>, dim3(n_units * fv.G), dim3(128), 0, st, fv, partials, (float*)out);
  } else {
    HKV_DISPATCH_G(fv.G, hipLaunchKernelGGL((full_partial_kernel<bf16_t, GG>), grid, dim3(256), 0, st, fv,
                                            (const bf16_t*)q, (const bf16_t*)k, (const bf16_t*)v, partials));
    hipLaunchKernelGGL(full_merge_kernel<bf16_t>, dim3(n_units * fv.G), dim3(128), 0, st, fv, partials, (bf16_t*)out);
  }
  return hipGetLastError();
}

}  // namespace hkv
