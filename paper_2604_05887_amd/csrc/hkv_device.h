// Device-side helpers for the libhkv kernels (gfx950, wave64).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hkv {

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global load and
// store the wave has in flight; a wave that has already asked for its next tile's rows, or has just
// stored a record nobody in the workgroup reads, must not stall on those at a barrier that only guards
// shared memory.
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// threadIdx.x behind an optimisation barrier.  In a kernel whose workgroups loop over many tiles the
// compiler otherwise hoists every per-thread address term of every inner loop out of the tile loop and
// then spills them; an opaque copy per use keeps those terms local to the tile (a handful of ALU ops).
__device__ __forceinline__ int thread_index() {
  int t = (int)threadIdx.x;
  asm volatile("" : "+v"(t));
  return t;
}


struct bf16_t { uint16_t bits; };   // storage type of bfloat16 tensors

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int kPer16 = 4;              // elements per 16-byte piece
  static constexpr int kLanesPerRow = 32;       // lanes that cover one 128-element row
};
template <> struct Elem<bf16_t> {
  static constexpr int kPer16 = 8;
  static constexpr int kLanesPerRow = 16;
};

__device__ __forceinline__ float bits_to_float(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t float_to_bits(float f) { return __builtin_bit_cast(uint32_t, f); }

// float -> bfloat16 bits, round to nearest even (NaN stays NaN).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  uint32_t u = float_to_bits(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// double -> bfloat16 bits in ONE rounding to nearest even (going through float first could round twice):
// the double's significand is cut to bfloat16's 8 bits in place, after which the conversion to float and
// the cut to its upper half are exact.  For finite values of normal bfloat16 magnitude, and zero.
__device__ __forceinline__ uint16_t f64_to_bf16_rne(double x) {
  uint64_t u = __builtin_bit_cast(uint64_t, x);
  u = (u + ((1ull << 44) - 1ull) + ((u >> 45) & 1ull)) & ~((1ull << 45) - 1ull);
  return (uint16_t)(float_to_bits((float)__builtin_bit_cast(double, u)) >> 16);
}

// Unpack one 16-byte piece into floats.
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[4], float) {
  f[0] = bits_to_float(v.x); f[1] = bits_to_float(v.y); f[2] = bits_to_float(v.z); f[3] = bits_to_float(v.w);
}
__device__ __forceinline__ void unpack16(const uint4& v, float (&f)[8], bf16_t) {
  f[0] = bits_to_float(v.x << 16); f[1] = bits_to_float(v.x & 0xffff0000u);
  f[2] = bits_to_float(v.y << 16); f[3] = bits_to_float(v.y & 0xffff0000u);
  f[4] = bits_to_float(v.z << 16); f[5] = bits_to_float(v.z & 0xffff0000u);
  f[6] = bits_to_float(v.w << 16); f[7] = bits_to_float(v.w & 0xffff0000u);
}

__device__ __forceinline__ uint4 pack16(const float (&f)[4], float) {
  return make_uint4(float_to_bits(f[0]), float_to_bits(f[1]), float_to_bits(f[2]), float_to_bits(f[3]));
}
__device__ __forceinline__ uint4 pack16(const float (&f)[8], bf16_t) {
  uint4 v;
  v.x = (uint32_t)f32_to_bf16_rne(f[0]) | ((uint32_t)f32_to_bf16_rne(f[1]) << 16);
  v.y = (uint32_t)f32_to_bf16_rne(f[2]) | ((uint32_t)f32_to_bf16_rne(f[3]) << 16);
  v.z = (uint32_t)f32_to_bf16_rne(f[4]) | ((uint32_t)f32_to_bf16_rne(f[5]) << 16);
  v.w = (uint32_t)f32_to_bf16_rne(f[6]) | ((uint32_t)f32_to_bf16_rne(f[7]) << 16);
  return v;
}

__device__ __forceinline__ uint4 ld16(const void* p) { return *reinterpret_cast<const uint4*>(p); }
// 16-byte load of data that is read once per launch (cache rows): marked non-temporal, so that the rows
// streaming through do not push the small reused arrays (chunk summaries, descriptors, queries) out of the L2.
typedef unsigned int u32x4_stream __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld16_stream(const void* p) {
  const u32x4_stream v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_stream*>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16(void* p, const uint4& v) { *reinterpret_cast<uint4*>(p) = v; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// ---- cross-lane primitives -------------------------------------------------------------
template <int CTRL> __device__ __forceinline__ float dpp_mov(float x) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float lane_xor(float x, int mask) {
  const int lane = (int)__lane_id();
  return __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, __builtin_bit_cast(int, x)));
}
__device__ __forceinline__ double lane_xor_f64(double x, int mask) {
  const int lane = (int)__lane_id();
  const uint64_t u = __builtin_bit_cast(uint64_t, x);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)(uint32_t)u);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, (int)(uint32_t)(u >> 32));
  return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ int lane_xor_i(int x, int mask) {
  const int lane = (int)__lane_id();
  return __builtin_amdgcn_ds_bpermute((lane ^ mask) << 2, x);
}

// Sum over each aligned group of 16 lanes; every lane of the group gets the total.
__device__ __forceinline__ float sum16(float x) {
  x += dpp_mov<0xB1>(x);    // quad_perm [1,0,3,2]
  x += dpp_mov<0x4E>(x);    // quad_perm [2,3,0,1]
  x += dpp_mov<0x141>(x);   // row_half_mirror
  x += dpp_mov<0x140>(x);   // row_mirror
  return x;
}
__device__ __forceinline__ float sum32(float x) { x = sum16(x); return x + lane_xor(x, 16); }
__device__ __forceinline__ float sum64(float x) { x = sum32(x); return x + lane_xor(x, 32); }
template <int LANES> __device__ __forceinline__ float sum_lanes(float x) {
  if constexpr (LANES == 16) return sum16(x);
  else if constexpr (LANES == 32) return sum32(x);
  else return sum64(x);
}

// Number of set bits of a wave vote below this lane.
__device__ __forceinline__ int lanes_below(unsigned long long votes) {
  return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(votes >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)votes, 0u));
}

// Wave-wide inclusive prefix sum of ints (wave64).
__device__ __forceinline__ int wave_inclusive_scan(int v) {
  const int lane = (int)__lane_id();
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    int n = __builtin_amdgcn_ds_bpermute(((lane - off) & 63) << 2, v);
    if (lane >= off) v += n;
  }
  return v;
}

// The same prefix sum without shared-memory traffic: shifts inside each row of 16 lanes, then the last lane
// of a row added to the rows behind it (row broadcasts).  A lane without a source adds 0.
__device__ __forceinline__ int wave_inclusive_scan_dpp(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return v;
}

// Wave-wide reductions on the same pattern: after the six steps lane 63 holds the result, which is handed
// back as a wave-uniform value.  `IDENT` is what a lane without a source contributes.
#define HKV_DPP_REDUCE(TYPE, OP, IDENT, BITS_IN, BITS_OUT)                                                          \
  do {                                                                                                               \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x111, 0xf, 0xf, false)));          \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x112, 0xf, 0xf, false)));          \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x114, 0xf, 0xf, false)));          \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x118, 0xf, 0xf, false)));          \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x142, 0xa, 0xf, false)));          \
    v = OP(v, BITS_OUT(__builtin_amdgcn_update_dpp(BITS_IN(IDENT), BITS_IN(v), 0x143, 0xc, 0xf, false)));          \
  } while (0)
__device__ __forceinline__ int hkv_as_int(float f) { return __builtin_bit_cast(int, f); }
__device__ __forceinline__ float hkv_as_float(int i) { return __builtin_bit_cast(float, i); }
__device__ __forceinline__ int hkv_keep_int(int i) { return i; }
__device__ __forceinline__ int hkv_add_i(int a, int b) { return a + b; }
__device__ __forceinline__ float hkv_add_f(float a, float b) { return a + b; }
__device__ __forceinline__ int hkv_min_u(int a, int b) { return (int)min((uint32_t)a, (uint32_t)b); }
__device__ __forceinline__ int wave_sum_i_dpp(int v) {
  HKV_DPP_REDUCE(int, hkv_add_i, 0, hkv_keep_int, hkv_keep_int);
  return __builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ uint32_t wave_min_u32_dpp(uint32_t x) {
  int v = (int)x;
  HKV_DPP_REDUCE(int, hkv_min_u, -1, hkv_keep_int, hkv_keep_int);
  return (uint32_t)__builtin_amdgcn_readlane(v, 63);
}
__device__ __forceinline__ float wave_sum_f_dpp(float v) {           // lanes added in a fixed order
  HKV_DPP_REDUCE(float, hkv_add_f, 0.f, hkv_as_int, hkv_as_float);
  return hkv_as_float(__builtin_amdgcn_readlane(hkv_as_int(v), 63));
}
__device__ __forceinline__ float wave_max_f_dpp(float v) {
  HKV_DPP_REDUCE(float, fmaxf, -3.0e38f, hkv_as_int, hkv_as_float);
  return hkv_as_float(__builtin_amdgcn_readlane(hkv_as_int(v), 63));
}
#undef HKV_DPP_REDUCE

// Block-wide exclusive prefix sum for blockDim.x == NT (multiple of 64).  `smem` holds NT/64 + 1 ints.
// Returns the exclusive prefix of `v`; *total gets the block sum.  Contains two barriers.
template <int NT> __device__ __forceinline__ int block_exclusive_scan(int v, int* smem, int* total) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int inc = wave_inclusive_scan(v);
  if (lane == 63) smem[wv] = inc;
  __syncthreads();
  if (threadIdx.x == 0) {
    int run = 0;
    for (int i = 0; i < NW; ++i) { int t = smem[i]; smem[i] = run; run += t; }
    smem[NW] = run;
  }
  __syncthreads();
  const int res = smem[wv] + inc - v;
  *total = smem[NW];
  __syncthreads();   // smem may be reused by the caller's next scan
  return res;
}

// Block-wide exclusive count of set flags for blockDim.x == NT (multiple of 64): the number of threads
// with a lower index whose flag is set; *total gets the block count.  `smem` holds NT/64 ints.  One
// barrier; the caller separates two uses of the same `smem` by a barrier of its own.
template <int NT> __device__ __forceinline__ int block_exclusive_count(bool flag, int* smem, int* total) {
  constexpr int NW = NT / 64;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const unsigned long long b = __builtin_amdgcn_ballot_w64(flag);
  const int pre = __builtin_popcountll(b & ((1ull << lane) - 1ull));
  if (lane == 0) smem[wv] = __builtin_popcountll(b);
  __syncthreads();
  int base = 0, tot = 0;
#pragma unroll
  for (int i = 0; i < NW; ++i) {
    const int t = smem[i];
    base += i < wv ? t : 0;
    tot += t;
  }
  *total = tot;
  return base + pre;
}

}  // namespace hkv
