// Internal declarations shared by the host API and the HIP kernels of libhkv.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hkv.h"

namespace hkv {

constexpr int kD = 128;          // head_dim
constexpr int kMaxG = 8;         // query heads per KV head
constexpr int kTileF32 = 128;    // logical rows per split-K work item of decode attention, fp32 path
constexpr int kTileBf16 = 256;   // same, bf16 rows read in place (full-KV kernel); smallest tile of a bf16 cache
constexpr int kTileBf16Max = 1024;   // bf16 caches pick 256, 512 or 1024 rows per tile from the amount of work
constexpr int kPartStride = 132; // floats per (stream, query head) in the shared-memory staging: m, l, 2 pad, o[128]
constexpr int kMlFloats = 16;    // floats per split-K tile in the workspace's (max, sum) array: 8 query heads x 2
constexpr int kKeysPerBlock = 512;   // keys one scoring block covers
constexpr int kMaxScoreRows = 256;   // G * window upper bound
constexpr int kFullMaxBatch = 256;
constexpr float kNeg = -1.0e30f;     // "minus infinity" that stays finite under subtraction

// bf16 caches store K and V in blocks of 8 rows (2048 bytes per block each) laid out so that the
// matrix-core operands of decode attention are plain 16-byte loads:
//   K block: 128 pieces of 16 bytes; the piece holding dims 8*d8 .. 8*d8+7 of row e sits at index
//            (((d8 / 4) * 2 + e / 4) * 4 + d8 % 4) * 4 + e % 4
//   V block: piece d (0..127) holds the 8 rows' values of dim d (row e at byte 2 * e)
// fp32 caches keep plain row-major rows.
constexpr int kBlkRows = 8;
constexpr int kBlkBytes = kBlkRows * kD * 2;
__host__ __device__ inline int k_piece_index(int e, int d8) { return ((((d8 >> 2) * 2 + (e >> 2)) * 4 + (d8 & 3)) * 4) + (e & 3); }

enum SelMode : int32_t { kSelVisual = 0, kSelText = 1, kSelSuffix = 2 };

// One (sequence, layer, KV head) unit.  Units are numbered layer-major:
// u = (layer * batch + seq) * n_kv_heads + head, so a layer range is a contiguous unit range.
struct UnitDesc {
  int64_t kv_row_off;   // first prompt row of the unit in the K / V row arrays (dynamic units: the k_dyn / v_dyn arrays)
  int64_t aux_off;      // static: element offset into scores[]; dynamic: chunk offset into mu[] rows and sigma[]
  int64_t idx_off;      // static: offset into kept_idx[]; dynamic: offset into sel[]
  int32_t seq_start;    // first token of the sequence in the packed prompt tensors
  int32_t C;            // prompt length of the sequence
  int32_t kind;         // hkv_head_type
  int32_t n_prompt_rows;// static: retained prompt rows; dynamic: k_sel * chunk (logical gathered rows)
  int32_t c_log2;       // dynamic: log2(chunk size)
  int32_t n_chunks;     // dynamic
  int32_t k_sel;        // dynamic: chunks gathered per step
  int32_t sel_mode;     // static: SelMode
  int32_t m_sel;        // static: candidates to pick
  int32_t n_cand;       // static: candidates available
  int32_t item_begin;   // first split-K work item of the unit (global numbering)
  int32_t n_tiles_max;  // work items reserved for the unit (tail at full capacity)
  int32_t seq, layer, head;
  int32_t type_ord;     // ordinal among the static (or dynamic) units, layer-major
  int32_t tail_row;     // physical row (within the unit) of the first appended decode token
  int32_t pad_;
  int64_t tail_off;     // first row of the unit's decode tail in the device K / V row arrays
};

// One split-K tile of decode attention: everything the attention block needs, in one record.
struct AttnItem {
  int64_t kv_row_off;   // first row of the unit in the cache K / V row arrays
  int32_t sel_off;      // dynamic: offset into sel[]
  int32_t n_prompt_rows;
  int32_t row0;         // first logical row of the tile
  int32_t C;
  int32_t c_log2;
  int32_t dynamic;
  int32_t layer, seq, head;
  int32_t tail_row;     // physical row of the first appended decode token
  int32_t slot;         // global index of the tile's record in the split-K workspace
  int32_t n_chunks;     // dynamic: chunks of the prompt
  int32_t k_sel;        // dynamic: chunks attended per step
  int32_t pad_;
  int64_t aux_off;      // dynamic: first chunk's offset into sigma[] / mu[]
  int64_t tail_off;     // first row of the unit's decode tail in the device K / V row arrays
};

// Streamed decode shape: boundary of a workgroup's share of the step's rows (unit counted from the first
// unit of the call, row a multiple of 32 inside that unit), and a unit whose rows more than one workgroup
// reads (its records sit in consecutive slots).
struct StreamBound { int32_t unit; int32_t row; };
struct StreamMulti { int32_t unit; int32_t slot0; int32_t n_rec; int32_t pad_; };

struct CacheView {
  const UnitDesc* units;
  const AttnItem* static_items;   // tiles of static units, layer-major
  const AttnItem* dynamic_items;  // tiles of dynamic units, layer-major
  const int32_t* static_units;
  const int32_t* dynamic_units;
  const UnitDesc* dyn_descs;      // descriptors of the dynamic units in dynamic_units order
  const UnitDesc* static_descs;   // descriptors of the static units in static_units order
  const uint8_t* is_visual;
  int32_t* cnt_a;             // [n_layers] tail length before the step in flight
  int32_t* cnt_b;             // [n_layers] tail length the step in flight attends
  int32_t* kept_idx;
  int32_t* sel;
  float* scores;
  float* sigma;
  void* mu;
  void* k_rows;               // static units' rows and every unit's decode tail (device memory)
  void* v_rows;
  void* k_dyn;                // dynamic units' prompt rows: k_rows / v_rows, or the host tier's arrays
  void* v_dyn;
  int32_t n_layers, batch, n_q_heads, n_kv_heads, G, window, max_new, causal;
  int32_t tile_rows;          // logical rows per split-K tile of this cache
  int32_t sigma_max;          // chunk score of a group: 0 = summed query, 1 = largest of the heads' inner products
  int32_t index_gen;          // dynamic heads: complete chunks of generated tokens are indexed and retrieved like the prompt's
  float scale_log2e;          // softmax scale * log2(e)
};

// ---- launchers implemented in the kernel translation units (all asynchronous on `st`) ----
// decode
// Field-by-field check of a configuration (HKV_OK or the status the entry points return for it).
int validate_config(const hkv_config* cfg);

// The launches of a decode step over a layer range.  t_arg: tail length before the step if the host
// knows it, else -1 (device counters).  select_only: the dynamic blocks stop after the chunk selection.
// launch_attn_merge also publishes the new tail counters when t_arg < 0, so it runs last.
// ev0 / ev1 (both or neither) receive the kernel's own start and stop time stamps.
// Scores of the chunks under hkv_config.chunk_score_group = 1, stored for the step's kernels to pick from.
hipError_t launch_chunk_score_sum(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int max_chunks,
                                  const void* q, hipStream_t st, hipEvent_t ev0, hipEvent_t ev1);
hipError_t launch_chunk_score_max(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, const void* q,
                                  int t_arg, hipStream_t st);
hipError_t launch_decode(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int sitem_begin,
                         int n_sitems, int slot_base, const void* q, const void* k_new, const void* v_new,
                         float* parts_o, float* parts_ml, void* out, int t_arg, int use_stored_sigma, int select_only,
                         int max_chunks, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
hipError_t launch_dynamic_tiles(const CacheView& cv, int dtype, int layer_begin, int ditem_begin, int n_ditems,
                                int sitem_begin, int n_sitems, int slot_base, const void* q, const void* k_new,
                                const void* v_new, float* parts_o, float* parts_ml, void* out, int t_arg, int reselect,
                                int static_hold, int max_chunks, void* stamps, int n_stamps, hipStream_t st,
                                hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// One wide workgroup per unit, outputs written directly (bf16 caches only; no workspace, no merge).
hipError_t launch_units(const CacheView& cv, int dtype, int layer_begin, int dyn_begin, int n_dyn, int static_begin,
                        int n_static, const void* q, const void* k_new, const void* v_new, void* out, int t_arg,
                        int max_chunks, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
hipError_t launch_attn_merge(const CacheView& cv, int dtype, const UnitDesc* descs, int n_units, int layer_begin,
                             int layer_end, int slot_base, float* parts_o, float* parts_ml, void* out, int t_arg,
                             int appending, hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
// Streamed shape (bf16 caches that do not index generated tokens): n_wg workgroups walk equal shares of the
// call's rows, then the units several workgroups touched are combined (also publishes device-side tail
// counters when t_arg < 0).
hipError_t launch_stream(const CacheView& cv, int dtype, const StreamBound* bounds, int n_wg, int unit_base, int layer_begin,
                         const void* q, const void* k_new, const void* v_new, float* parts_o, float* parts_ml,
                         void* out, int t_arg, int max_chunks, hipStream_t st, hipEvent_t ev0 = nullptr,
                         hipEvent_t ev1 = nullptr);
hipError_t launch_stream_merge(const CacheView& cv, int dtype, const StreamMulti* multi, int n_multi, int unit_base,
                               int layer_begin, int layer_end, float* parts_o, float* parts_ml, void* out, int t_arg,
                               hipStream_t st, hipEvent_t ev0 = nullptr, hipEvent_t ev1 = nullptr);
hipError_t launch_rewind(const CacheView& cv, int layer_begin, int layer_end, hipStream_t st);

struct FullView {
  int32_t cu[kFullMaxBatch + 1];
  int32_t batch, n_layers_call, n_q_heads, n_kv_heads, G, n_tiles_max;
  int64_t total_tokens;
  float scale_log2e;
};
hipError_t launch_full_attn(const FullView& fv, int dtype, const void* q, const void* k, const void* v,
                            float* parts_o, float* parts_ml, void* out, hipStream_t st);

// compress
// keys_per_block: keys one scoring block covers on the bf16 path (a multiple of 32 from kKeysPerBlock to
// 2 * kKeysPerBlock, so that the row-statistics workspace sized for kKeysPerBlock always suffices); the fp32
// path uses kKeysPerBlock.
hipError_t launch_score(const CacheView& cv, int dtype, int layer_begin, int static_begin, int n_static,
                        int max_C, const void* q_window, const void* k, int64_t total_tokens,
                        float2* part_stats, float2* final_stats, int keys_per_block, hipStream_t st);
hipError_t launch_select(const CacheView& cv, int static_begin, int n_static, hipStream_t st);
hipError_t launch_compact(const CacheView& cv, int dtype, int layer_begin, int static_begin, int n_static,
                          int max_rows, const void* k, const void* v, int64_t total_tokens, hipStream_t st);
hipError_t launch_adopt(const CacheView& cv, int dtype, int layer_begin, int dynamic_begin, int n_dynamic,
                        int max_chunks, int max_C, const void* k, const void* v, int64_t total_tokens,
                        hipStream_t st);

}  // namespace hkv
