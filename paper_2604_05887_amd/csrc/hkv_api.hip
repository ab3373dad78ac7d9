// Host side of libhkv: argument validation, cache layout planning, descriptor upload and kernel
// sequencing behind the C ABI declared in hkv.h.  No device memory is allocated here.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <memory>
#include <mutex>
#include <vector>

#include "hkv_internal.h"

namespace hkv {

int validate_config(const hkv_config* cfg) {
  if (!cfg) return HKV_EINVAL;
  if (cfg->struct_size != sizeof(hkv_config) || cfg->abi_version != HKV_ABI_VERSION) return HKV_EINVAL;
  if (cfg->dtype != HKV_F32 && cfg->dtype != HKV_BF16) return HKV_EINVAL;
  if (cfg->score_causal != 0 && cfg->score_causal != 1) return HKV_EINVAL;
  if (cfg->head_dim != kD) return HKV_ESHAPE;
  if (cfg->n_layers < 1 || cfg->n_q_heads < 1 || cfg->n_kv_heads < 1) return HKV_ESHAPE;
  if (cfg->n_q_heads % cfg->n_kv_heads != 0) return HKV_ESHAPE;
  const int G = cfg->n_q_heads / cfg->n_kv_heads;
  if (G < 1 || G > kMaxG) return HKV_ESHAPE;
  if (cfg->window < 1 || G * cfg->window > kMaxScoreRows) return HKV_ESHAPE;
  if (cfg->max_new_tokens < 0) return HKV_ESHAPE;
  if (cfg->decode_tile_rows != 0) {
    const int t = cfg->decode_tile_rows;
    if (cfg->dtype != HKV_BF16 || t < 128 || t > 4096 || t % 32 != 0) return HKV_ESHAPE;
  }
  if (cfg->decode_dynamic < 0 || cfg->decode_dynamic > 5) return HKV_EINVAL;
  if (cfg->decode_dynamic >= 4 && cfg->dtype != HKV_BF16) return HKV_ESHAPE;   // the per-unit and streamed shapes are bf16 only
  if (cfg->chunk_score_group != 0 && cfg->chunk_score_group != 1) return HKV_EINVAL;
  if (cfg->index_generated != 0 && cfg->index_generated != 1) return HKV_EINVAL;
  if (cfg->index_generated) {               // bf16 caches; not the shape that selects in one launch and gathers in the next
    if (cfg->dtype != HKV_BF16) return HKV_ESHAPE;
    if (cfg->decode_dynamic == 2 || cfg->decode_dynamic == 5) return HKV_ESHAPE;
  }
  if (!(cfg->softmax_scale >= 0.f) || !std::isfinite(cfg->softmax_scale)) return HKV_EINVAL;
  return HKV_OK;
}

}  // namespace hkv

using namespace hkv;

// Split-K records of hkv_decode_attn_noalloc: one array per GPU inside the library's code object, so that
// the call needs neither an allocation nor a caller workspace.  In host code the array's name is only a
// handle for the runtime, not a device address: scratch_of_current_device() asks the runtime for the
// array's address on the current device (every GPU holds its own copy) and keeps it, and everything
// that touches the array's memory -- kernel arguments included -- uses that address.
static __device__ __align__(256) unsigned char scratch[HKV_NOALLOC_SCRATCH_BYTES];

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on the current device (looked up once per device); *device gets the device id.
hipError_t scratch_of_current_device(void** ptr, int* device) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p || reinterpret_cast<uintptr_t>(p) % kAlign != 0) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  *device = dev;
  return hipSuccess;
}
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t elem_size(int dtype) { return dtype == HKV_BF16 ? 2 : 4; }

// Streamed decode shape: the equal shares of one call shape (all layers, or one layer) at one reference
// tail length.  Offsets are relative to the start of the cache's stream-table section.
struct StreamTable {
  int32_t t_ref = 0, n_wg = 0, n_multi = 0, share_rows = 0;
  size_t off_bounds = 0, off_multi = 0;
};
struct StreamShape {
  int32_t unit_begin = 0, n_units = 0;
  std::vector<StreamTable> tables;        // ascending t_ref
};

struct Layout {
  // streamed shape (bf16 caches that do not index generated tokens): [0] = all layers, [1 + l] = layer l alone
  std::vector<StreamShape> stream_shapes;
  std::vector<char> stream_blob;          // every table's boundaries and multi-workgroup unit lists, as uploaded
  size_t off_stream = 0, rows_end = 0;     // arena offset of the tables; end of the K / V row arrays
  int64_t stream_slots_max = 0;           // most record slots a streamed call can use
  // host tables
  std::vector<UnitDesc> units;
  std::vector<AttnItem> sitems, ditems;
  int64_t n_items = 0;
  std::vector<int32_t> static_units, dynamic_units;
  std::vector<int32_t> static_begin, dynamic_begin, item_begin, sitem_begin, ditem_begin;   // [n_layers + 1]
  std::vector<int64_t> dmu_begin;  // [n_layers + 1] summary bytes read by the dynamic tiles of the layers before
  std::vector<int32_t> cu;
  int64_t total_tokens = 0;
  int32_t max_C = 0, max_rows_static = 0, max_rows_dynamic = 0, max_chunks = 0;
  int64_t step_bytes0 = 0, reselect_extra_bytes = 0;   // per step at an empty tail; extra summary reads of mode 3
  int mode = 2;                    // how decode steps run the dynamic heads (hkv_config.decode_dynamic, resolved)
  bool mode_by_rule = true;        // the automatic rule chose it (a caller's explicit choice is followed to the letter)
  // element counts
  int64_t n_kept = 0, n_sel = 0, n_scores = 0, n_sigma = 0, n_rows = 0;
  // host tier (bf16 caches only): the dynamic units' prompt rows live in mapped host memory
  bool tiered = false;
  int64_t n_rows_host = 0;
  size_t host_off_k = 0, host_off_v = 0, host_bytes = 0;
  // arena offsets (bytes)
  size_t off_units = 0, off_sitems = 0, off_ditems = 0, off_static_descs = 0, off_static = 0, off_dynamic = 0, off_dyn_descs = 0, off_vis = 0, off_cnt = 0, off_kept = 0,
         off_sel = 0, off_scores = 0, off_sigma = 0, off_mu = 0, off_k = 0, off_v = 0, arena_bytes = 0;
  size_t ws_bytes = 0, ws_o_bytes = 0;
  int tile = 0;
  // A second tiling of the same cache with larger tiles (bf16 caches under the automatic tile rule): only its
  // unit and tile tables differ; they sit behind the first tiling's arena.  A call picks one of the two.
  std::shared_ptr<Layout> second;
  size_t s2off_units = 0, s2off_sitems = 0, s2off_ditems = 0, s2off_static_descs = 0, s2off_dyn_descs = 0;
};

inline bool pow2_ge4(int c) { return c >= 4 && (c & (c - 1)) == 0; }

int plan_layout_tile(const hkv_config* cfg, const hkv_plan* plan, Layout& lo, int tile, bool tiered) {
  int rc = validate_config(cfg);
  if (rc != HKV_OK) return rc;
  if (tiered && cfg->dtype != HKV_BF16) return HKV_ESHAPE;   // the host tier exists for bf16 caches only
  lo.tiered = tiered;
  if (!plan || !plan->cu_seqlens || !plan->is_visual || !plan->head_type || !plan->budget) return HKV_EINVAL;
  if (plan->batch < 1 || plan->batch > 4096) return HKV_ESHAPE;
  const int B = plan->batch, L = cfg->n_layers, H = cfg->n_kv_heads, w = cfg->window;
  const int G = cfg->n_q_heads / H;
  const bool blocked = cfg->dtype == HKV_BF16;
  lo.tile = tile;
  if (plan->cu_seqlens[0] != 0) return HKV_EINVAL;
  lo.cu.assign(plan->cu_seqlens, plan->cu_seqlens + B + 1);
  std::vector<int32_t> n_txt(B), n_vis(B), csz(B);
  for (int b = 0; b < B; ++b) {
    const int64_t C = (int64_t)lo.cu[b + 1] - lo.cu[b];
    if (C < w || C < 1) return HKV_ESHAPE;               // the window must fit in the prompt
    csz[b] = plan->chunk_size ? plan->chunk_size[b] : cfg->chunk_size;
    if (!pow2_ge4(csz[b])) return HKV_ESHAPE;
    int t = 0, v = 0;
    for (int64_t j = lo.cu[b]; j < lo.cu[b + 1] - w; ++j) {
      if (plan->is_visual[j] > 1) return HKV_EINVAL;
      (plan->is_visual[j] ? v : t)++;
    }
    n_txt[b] = t; n_vis[b] = v;
    lo.max_C = std::max<int32_t>(lo.max_C, (int32_t)C);
  }
  lo.total_tokens = lo.cu[B];

  lo.units.resize((size_t)L * B * H);
  lo.static_begin.assign(L + 1, 0); lo.dynamic_begin.assign(L + 1, 0); lo.item_begin.assign(L + 1, 0);
  lo.sitem_begin.assign(L + 1, 0); lo.ditem_begin.assign(L + 1, 0); lo.dmu_begin.assign(L + 1, 0);
  for (int l = 0; l < L; ++l) {
    lo.static_begin[l] = (int32_t)lo.static_units.size();
    lo.dynamic_begin[l] = (int32_t)lo.dynamic_units.size();
    lo.item_begin[l] = (int32_t)lo.n_items;
    lo.sitem_begin[l] = (int32_t)lo.sitems.size();
    lo.ditem_begin[l] = (int32_t)lo.ditems.size();
    lo.dmu_begin[l + 1] = lo.dmu_begin[l];
    for (int b = 0; b < B; ++b) {
      const int32_t C = lo.cu[b + 1] - lo.cu[b];
      for (int h = 0; h < H; ++h) {
        const size_t pi = ((size_t)b * L + l) * H + h;       // plan arrays are [batch][layer][head]
        const int32_t u = (int32_t)(((size_t)l * B + b) * H + h);
        const int ht = plan->head_type[pi];
        const int64_t budget = plan->budget[pi];
        if (ht != HKV_STATIC && ht != HKV_DYNAMIC) return HKV_EINVAL;
        if (budget < 1) return HKV_EBUDGET;
        UnitDesc d;
        std::memset(&d, 0, sizeof(d));
        d.seq_start = lo.cu[b]; d.C = C; d.kind = ht; d.seq = b; d.layer = l; d.head = h;
        d.kv_row_off = lo.n_rows;
        int64_t phys_rows;
        bool rows_on_host = false;
        if (ht == HKV_STATIC) {
          // Keep set = window + historical text + Top-M historical visual, M = budget - w - #text
          // (Appendix A); text outranks visual when the budget is short (Section 3.3).
          if (budget < w) { d.sel_mode = kSelSuffix; d.m_sel = 0; d.n_cand = 0; d.n_prompt_rows = (int32_t)budget; }
          else {
            const int64_t M = budget - w - n_txt[b];
            if (M < 0) { d.sel_mode = kSelText; d.m_sel = (int32_t)(budget - w); d.n_cand = n_txt[b]; d.n_prompt_rows = (int32_t)budget; }
            else { d.sel_mode = kSelVisual; d.m_sel = (int32_t)std::min<int64_t>(M, n_vis[b]); d.n_cand = n_vis[b];
                   d.n_prompt_rows = w + n_txt[b] + d.m_sel; }
          }
          d.aux_off = lo.n_scores; lo.n_scores += C;
          d.idx_off = lo.n_kept; lo.n_kept += d.n_prompt_rows;
          d.type_ord = (int32_t)lo.static_units.size();
          lo.static_units.push_back(u);
          lo.max_rows_static = std::max(lo.max_rows_static, d.n_prompt_rows);
          phys_rows = d.n_prompt_rows;
          d.tail_row = d.n_prompt_rows;
        } else {
          const int c = csz[b];
          int lg = 0; while ((1 << lg) < c) ++lg;
          d.c_log2 = lg;
          d.n_chunks = (C + c - 1) / c;
          // caches that index their generated tokens keep room for the chunks generation can complete
          const int max_gen = cfg->index_generated ? cfg->max_new_tokens / c : 0;
          d.k_sel = (int32_t)std::min<int64_t>(std::max<int64_t>(1, budget / c), d.n_chunks + max_gen);
          d.n_prompt_rows = d.k_sel * c;
          d.aux_off = lo.n_sigma; lo.n_sigma += d.n_chunks + max_gen;
          d.idx_off = lo.n_sel; lo.n_sel += d.k_sel;
          d.type_ord = (int32_t)lo.dynamic_units.size();
          lo.dynamic_units.push_back(u);
          lo.max_chunks = std::max(lo.max_chunks, d.n_chunks + max_gen);
          lo.max_rows_dynamic = std::max(lo.max_rows_dynamic, d.n_prompt_rows + cfg->max_new_tokens);
          if (blocked && c < kBlkRows) return HKV_ESHAPE;     // bf16 caches gather whole 8-row blocks
          phys_rows = blocked ? (C + kBlkRows - 1) / kBlkRows * kBlkRows : C;
          d.tail_row = (int32_t)phys_rows;
          rows_on_host = tiered;
        }
        if (rows_on_host) {
          // prompt rows in the host arrays, the decode tail (whole blocks) in the device arrays
          d.kv_row_off = lo.n_rows_host;
          lo.n_rows_host += phys_rows;
          d.tail_off = lo.n_rows;
          lo.n_rows += ((int64_t)cfg->max_new_tokens + kBlkRows - 1) / kBlkRows * kBlkRows;
        } else {
          d.tail_off = d.kv_row_off + d.tail_row;
          const int64_t cap = phys_rows + cfg->max_new_tokens;
          lo.n_rows += blocked ? (cap + kBlkRows - 1) / kBlkRows * kBlkRows : cap;
        }
        {
          const int64_t R = (int64_t)kD * (blocked ? 2 : 4);
          lo.step_bytes0 += 2 * R * d.n_prompt_rows + (ht == HKV_DYNAMIC ? R * d.n_chunks : 0);
          if (ht == HKV_DYNAMIC) lo.reselect_extra_bytes += R * d.n_chunks * ((d.n_prompt_rows + tile - 1) / tile - 1);
        }
        d.item_begin = (int32_t)lo.n_items;
        // rows a unit can attend: its prompt rows and its whole tail -- or, for a dynamic unit of a cache that
        // indexes generated tokens, the picked chunks and at most one chunk's worth of tail
        const int tail_rows_max = (ht == HKV_DYNAMIC && cfg->index_generated)
                                      ? std::min(cfg->max_new_tokens, 1 << d.c_log2) : cfg->max_new_tokens;
        d.n_tiles_max = std::max(1, (d.n_prompt_rows + tail_rows_max + tile - 1) / tile);
        if ((int64_t)C + cfg->max_new_tokens >= (1 << 24)) return HKV_ESHAPE;   // 24-bit row arithmetic in the kernels
        for (int t = 0; t < d.n_tiles_max; ++t) {
          AttnItem it;
          std::memset(&it, 0, sizeof(it));
          it.kv_row_off = d.kv_row_off;
          it.sel_off = ht == HKV_DYNAMIC ? (int32_t)d.idx_off : 0;
          it.n_prompt_rows = d.n_prompt_rows;
          it.row0 = t * tile;
          it.C = C;
          it.c_log2 = d.c_log2;
          it.dynamic = ht == HKV_DYNAMIC;
          it.layer = l; it.seq = b; it.head = h;
          it.tail_row = d.tail_row;
          it.tail_off = d.tail_off;
          it.slot = (int32_t)lo.n_items++;
          if (ht == HKV_DYNAMIC) {
            it.n_chunks = d.n_chunks; it.k_sel = d.k_sel; it.aux_off = d.aux_off;
            lo.dmu_begin[l + 1] += (int64_t)d.n_chunks * kD * (blocked ? 2 : 4);
          }
          (ht == HKV_DYNAMIC ? lo.ditems : lo.sitems).push_back(it);
        }
        if (lo.n_items > (int64_t)0x7fffff00) return HKV_ESHAPE;
        lo.units[u] = d;
      }
    }
  }
  lo.static_begin[L] = (int32_t)lo.static_units.size();
  lo.dynamic_begin[L] = (int32_t)lo.dynamic_units.size();
  lo.item_begin[L] = (int32_t)lo.n_items;
  lo.sitem_begin[L] = (int32_t)lo.sitems.size();
  lo.ditem_begin[L] = (int32_t)lo.ditems.size();
  // LDS of the chunk selection: histogram, scores, 64-bit keys and the picks of every chunk
  if ((size_t)(256 + 16 + lo.max_chunks + 4) * 4 + (size_t)(lo.max_chunks + 4) * 12 > 150 * 1024) return HKV_ESHAPE;

  const size_t es = elem_size(cfg->dtype);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
  lo.off_units = take(lo.units.size() * sizeof(UnitDesc));
  lo.off_sitems = take(std::max<size_t>(1, lo.sitems.size()) * sizeof(AttnItem));
  lo.off_ditems = take(std::max<size_t>(1, lo.ditems.size()) * sizeof(AttnItem));
  lo.off_static_descs = take(std::max<size_t>(1, lo.static_units.size()) * sizeof(UnitDesc));
  lo.off_static = take(std::max<size_t>(1, lo.static_units.size()) * 4);
  lo.off_dynamic = take(std::max<size_t>(1, lo.dynamic_units.size()) * 4);
  lo.off_dyn_descs = take(std::max<size_t>(1, lo.dynamic_units.size()) * sizeof(UnitDesc));
  lo.off_vis = take((size_t)lo.total_tokens);
  lo.off_cnt = take((size_t)2 * L * 4);
  lo.off_kept = take((size_t)std::max<int64_t>(1, lo.n_kept) * 4);
  lo.off_sel = take((size_t)std::max<int64_t>(1, lo.n_sel) * 4);
  lo.off_scores = take((size_t)std::max<int64_t>(1, lo.n_scores) * 4);
  lo.off_sigma = take((size_t)std::max<int64_t>(1, lo.n_sigma) * 4);
  lo.off_mu = take((size_t)std::max<int64_t>(1, lo.n_sigma) * kD * es);
  lo.off_k = take((size_t)lo.n_rows * kD * es);
  lo.off_v = take((size_t)lo.n_rows * kD * es);
  lo.arena_bytes = off;
  lo.host_off_k = 0;
  lo.host_off_v = align_up((size_t)lo.n_rows_host * kD * es);
  lo.host_bytes = tiered ? std::max<size_t>(kAlign, lo.host_off_v + align_up((size_t)lo.n_rows_host * kD * es)) : 0;

  const int n_splits = (lo.max_C + kKeysPerBlock - 1) / kKeysPerBlock;
  const size_t ws_compress = align_up(lo.static_units.size() * (size_t)n_splits * kMaxScoreRows * sizeof(float2)) +
                             align_up(lo.static_units.size() * (size_t)kMaxScoreRows * sizeof(float2));
  lo.ws_o_bytes = align_up((size_t)lo.n_items * G * kD * sizeof(float));
  const size_t ws_decode = lo.ws_o_bytes + align_up((size_t)lo.n_items * kMlFloats * sizeof(float));
  lo.ws_bytes = std::max<size_t>(kAlign, std::max(ws_compress, ws_decode));
  return HKV_OK;
}

// Streamed decode shape: cut the rows of a call's units (unit order, every unit's rows in steps of 32, tail at
// the reference length t_ref) into n_wg shares of equal size; see stream_kernel.  n_wg = as many as the
// device keeps resident (three workgroups on each compute unit), fewer when a share would drop below
// kStreamMinSteps steps.
constexpr int kDeviceCus = 256;          // compute units of the device this library is written for (MI355X)
constexpr int kStreamMinSteps = 8;
constexpr int kStreamMaxWg = 3 * 256;
constexpr int kPreScoreChunks = 512;      // chunks per head from which a one-round call scores them in a launch of its own
constexpr int kStreamAutoRows = 2048;     // the automatic rule streams when every workgroup's share is at least this long
// A dynamic unit costs more than its rows: whoever touches it reads its chunk summaries (one 32-row step
// of K and V is 16 KB) and waits for the selection's dependent chain (about the time of kSelLatencySteps
// steps of a streaming workgroup).  That cost sits at the front of the unit on the line of work; a
// boundary that falls inside it becomes the unit's row 0.
constexpr int kSelLatencySteps = 3;
void build_stream_table(const Layout& lo, int unit_begin, int n_units, int t_ref, StreamTable& tb, std::vector<char>& blob) {
  std::vector<int64_t> start(n_units + 1, 0), lead(n_units, 0);     // first step of every unit; its selection cost
  std::vector<int32_t> ref_rows(n_units, 0);
  for (int i = 0; i < n_units; ++i) {
    const UnitDesc& d = lo.units[unit_begin + i];
    ref_rows[i] = d.n_prompt_rows + t_ref;
    if (d.kind == HKV_DYNAMIC) lead[i] = ((int64_t)d.n_chunks * kD * 2 + 16383) / 16384 + kSelLatencySteps;
    start[i + 1] = start[i] + lead[i] + ((int64_t)ref_rows[i] + 31) / 32;
  }
  const int64_t S = start[n_units];
  const int n_wg = (int)std::max<int64_t>(1, std::min<int64_t>(kStreamMaxWg, S / kStreamMinSteps));
  std::vector<StreamBound> bounds(n_wg + 1);
  int u = 0;
  for (int j = 0; j <= n_wg; ++j) {
    const int64_t pos = j == n_wg ? S : S * j / n_wg;
    while (u < n_units && start[u + 1] <= pos) ++u;           // unit that holds step `pos` (n_units at the very end)
    bounds[j].unit = u;
    bounds[j].row = u < n_units ? (int32_t)(std::max<int64_t>(0, pos - start[u] - lead[u]) * 32) : 0;
  }
  // who touches which unit: walk every workgroup's share as the kernel does
  std::vector<int32_t> first(n_units, -1), last(n_units, -1);
  for (int j = 0; j < n_wg; ++j) {
    int uu = bounds[j].unit, ra = bounds[j].row;
    while (uu < bounds[j + 1].unit || (uu == bounds[j + 1].unit && ra < bounds[j + 1].row)) {
      if (first[uu] < 0) first[uu] = j;
      last[uu] = j;
      ++uu; ra = 0;
    }
  }
  std::vector<StreamMulti> multi;
  for (int i = 0; i < n_units; ++i)
    if (last[i] > first[i]) multi.push_back(StreamMulti{i, first[i] + i, last[i] - first[i] + 1, 0});
  tb.t_ref = t_ref; tb.n_wg = n_wg; tb.n_multi = (int32_t)multi.size();
  tb.share_rows = (int32_t)std::min<int64_t>(S * 32 / n_wg, 0x7fffffff);
  auto put = [&](const void* src, size_t bytes) {
    const size_t off = (blob.size() + 255) / 256 * 256;
    blob.resize(off + std::max<size_t>(bytes, 16));
    if (bytes) std::memcpy(blob.data() + off, src, bytes);      // an empty list has no data pointer to copy from
    return off;
  };
  tb.off_bounds = put(bounds.data(), bounds.size() * sizeof(StreamBound));
  tb.off_multi = put(multi.data(), multi.size() * sizeof(StreamMulti));
}

void build_stream_shapes(const hkv_config* cfg, int batch, Layout& lo) {
  lo.stream_shapes.clear(); lo.stream_blob.clear(); lo.stream_slots_max = 0;
  if (cfg->dtype != HKV_BF16 || cfg->index_generated) return;
  // reference tail lengths: every 32 tokens up to 256, every 128 up to 1024, then doubling
  std::vector<int> rungs;
  for (int t = 0; t <= cfg->max_new_tokens; t += t < 256 ? 32 : (t < 1024 ? 128 : t)) rungs.push_back(t);
  const int L = cfg->n_layers, upl = batch * cfg->n_kv_heads;
  const int n_shapes = L > 1 ? 1 + L : 1;
  lo.stream_shapes.resize(n_shapes);
  for (int s = 0; s < n_shapes; ++s) {
    StreamShape& sh = lo.stream_shapes[s];
    sh.unit_begin = s == 0 ? 0 : (s - 1) * upl;
    sh.n_units = s == 0 ? L * upl : upl;
    sh.tables.resize(rungs.size());
    for (size_t r = 0; r < rungs.size(); ++r) {
      build_stream_table(lo, sh.unit_begin, sh.n_units, rungs[r], sh.tables[r], lo.stream_blob);
      lo.stream_slots_max = std::max<int64_t>(lo.stream_slots_max, (int64_t)sh.tables[r].n_wg + sh.n_units);
    }
  }
}

// Tile size: fp32 caches use 128 rows; bf16 caches start at 256 rows and double (up to 1024) while the
// whole cache still yields three tiles per compute unit (one full round of resident workgroups), so that
// small steps keep every compute unit busy and large ones amortise the per-tile cost.
// Dynamic heads: every dynamic tile repeats its head's chunk selection, so that the step is one launch
// plus the combination, as long as the repeated reads of the chunk summaries stay below a quarter of
// the step's bytes (they mostly hit the L2); with many small chunks the selection runs once per head
// and the tiles follow in a second launch.  Heads of at most kUnitShapeMaxRows rows (tail at full
// capacity included; bf16 caches) are not split at all: measured on the 7B shape, one wide workgroup per
// head is ahead of the split-K shapes up to about that length and behind them beyond.
constexpr int kUnitShapeMaxRows = 768;
int plan_layout(const hkv_config* cfg, const hkv_plan* plan, Layout& lo, bool tiered = false) {
  int rc;
  if (cfg && cfg->dtype != HKV_BF16) rc = plan_layout_tile(cfg, plan, lo, kTileF32, tiered);
  else if (cfg && cfg->decode_tile_rows != 0) rc = plan_layout_tile(cfg, plan, lo, cfg->decode_tile_rows, tiered);
  else {
    int tile = kTileBf16;
    rc = plan_layout_tile(cfg, plan, lo, tile, tiered);
    while (rc == HKV_OK && tile < kTileBf16Max) {
      Layout next;
      if (plan_layout_tile(cfg, plan, next, tile * 2, tiered) != HKV_OK || next.n_items < 3 * kDeviceCus) break;
      tile *= 2;
      lo = std::move(next);
    }
  }
  if (rc != HKV_OK) return rc;
  // A bf16 cache under the automatic rule carries a second tiling, and every call takes the one that suits its
  // tile count (call_uses_second_tiling).  First tiling below kTileBf16Max rows: the second has kTileBf16Max --
  // small steps, a whole-model call of a short-context cache, run faster when every tile has a compute unit to
  // itself.  First tiling grown to kTileBf16Max (a large cache): the second has kTileBf16 rows, for calls over
  // few layers, which would leave most compute units without a tile otherwise.
  if (cfg->dtype == HKV_BF16 && cfg->decode_tile_rows == 0) {
    const int tile2 = lo.tile < kTileBf16Max ? kTileBf16Max : kTileBf16;
    auto co = std::make_shared<Layout>();
    if (plan_layout_tile(cfg, plan, *co, tile2, tiered) == HKV_OK && co->n_items != lo.n_items) {
      size_t off = lo.arena_bytes;
      auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
      lo.s2off_units = take(co->units.size() * sizeof(UnitDesc));
      lo.s2off_sitems = take(std::max<size_t>(1, co->sitems.size()) * sizeof(AttnItem));
      lo.s2off_ditems = take(std::max<size_t>(1, co->ditems.size()) * sizeof(AttnItem));
      lo.s2off_static_descs = take(std::max<size_t>(1, co->static_units.size()) * sizeof(UnitDesc));
      lo.s2off_dyn_descs = take(std::max<size_t>(1, co->dynamic_units.size()) * sizeof(UnitDesc));
      lo.arena_bytes = off;
      lo.ws_bytes = std::max(lo.ws_bytes, co->ws_bytes);       // the finer tiling has more records
      lo.second = std::move(co);
    }
  }
  lo.rows_end = lo.second ? lo.s2off_units : lo.arena_bytes;
  build_stream_shapes(cfg, plan->batch, lo);
  if (!lo.stream_blob.empty()) {
    lo.off_stream = align_up(lo.arena_bytes);
    lo.arena_bytes = lo.off_stream + align_up(lo.stream_blob.size());
    const size_t G = (size_t)(cfg->n_q_heads / cfg->n_kv_heads);
    const size_t ws_stream = align_up((size_t)lo.stream_slots_max * G * kD * sizeof(float)) +
                             align_up((size_t)lo.stream_slots_max * kMlFloats * sizeof(float));
    lo.ws_bytes = std::max(lo.ws_bytes, ws_stream);
  }
  lo.mode_by_rule = cfg->decode_dynamic == 0;
  if (cfg->decode_dynamic != 0) lo.mode = cfg->decode_dynamic;
  else if (cfg->dtype == HKV_BF16 &&
           std::max(lo.max_rows_static + cfg->max_new_tokens, lo.max_rows_dynamic) <= kUnitShapeMaxRows)
    lo.mode = 4;         // short heads: one wide workgroup each beats split-K plus the combination launch
  else if (!lo.stream_shapes.empty() && lo.stream_shapes[0].tables[0].n_wg == kStreamMaxWg &&
           lo.stream_shapes[0].tables[0].share_rows >= kStreamAutoRows)
    lo.mode = 5;         // large steps: equal shares of the rows beat tiles (measured from about 1 GB per step on)
  else lo.mode = 4 * lo.reselect_extra_bytes <= lo.step_bytes0 ? 3 : (cfg->index_generated ? 1 : 2);
  return HKV_OK;
}

}  // namespace

struct hkv_cache {
  hkv_config cfg;
  int32_t batch;
  Layout lo;
  CacheView cv;
  char* arena;
  char* host_tier = nullptr;          // host address of the host tier (null: every row is in device memory)
  std::vector<int32_t> host_tail;     // [n_layers] appended tokens (host mirror of the device counter)
  bool device_tail = false;           // decode calls take the tail length from the device counters only
  std::vector<uint8_t> compressed;    // [n_layers]
  std::vector<hipEvent_t> events;     // 6 per profiled decode call: start and stop of up to three kernels
  int prof_calls = 0, prof_max = 0;
  void* stamps = nullptr;             // device buffer for per-workgroup time stamps of the tile launch (diagnosis)
  int n_stamps = 0;
  int n_cus = 256;                    // compute units of the device the cache lives on
  int clock_khz = 2400000;            // that device's shader clock
  int device = -1;                    // device that was current when the cache was created
  void* scratch_dev = nullptr;        // that device's copy of the library's split-K record array
  CacheView cv_second;                // cv with the tables of the coarse tiling (if lo.second)
  hipStream_t prof_stream = nullptr;  // stream of the profiled calls
  std::vector<uint8_t> prof_mask;     // per profiled call: bit j set if kernel j was launched
};

extern "C" {

uint32_t hkv_abi_version(void) { return HKV_ABI_VERSION; }

const char* hkv_strerror(int status) {
  switch (status) {
    case HKV_OK: return "ok";
    case HKV_EINVAL: return "invalid argument";
    case HKV_ESHAPE: return "unsupported shape";
    case HKV_EBUDGET: return "budget must be at least 1 token";
    case HKV_EALIGN: return "device pointer not 16-byte aligned";
    case HKV_ENOSPACE: return "buffer too small or decode tail full";
    case HKV_ESTATE: return "call out of order";
    case HKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int hkv_query_sizes(const hkv_config* cfg, const hkv_plan* plan, size_t* cache_bytes, size_t* workspace_bytes) {
  if (!cache_bytes || !workspace_bytes) return HKV_EINVAL;
  Layout lo;
  const int rc = plan_layout(cfg, plan, lo);
  if (rc != HKV_OK) return rc;
  *cache_bytes = lo.arena_bytes;
  *workspace_bytes = lo.ws_bytes;
  return HKV_OK;
}

int hkv_query_tier_sizes(const hkv_config* cfg, const hkv_plan* plan, size_t* cache_bytes, size_t* host_bytes,
                         size_t* workspace_bytes) {
  if (!cache_bytes || !host_bytes || !workspace_bytes) return HKV_EINVAL;
  Layout lo;
  const int rc = plan_layout(cfg, plan, lo, true);
  if (rc != HKV_OK) return rc;
  *cache_bytes = lo.arena_bytes;
  *host_bytes = lo.host_bytes;
  *workspace_bytes = lo.ws_bytes;
  return HKV_OK;
}

static int create_cache(const hkv_config* cfg, const hkv_plan* plan, void* cache_dev, size_t cache_bytes,
                        void* host_tier, size_t host_bytes, bool tiered, hkv_cache** out) {
  if (!out || !cache_dev || (tiered && !host_tier)) return HKV_EINVAL;
  if (reinterpret_cast<uintptr_t>(cache_dev) % kAlign != 0) return HKV_EALIGN;
  if (tiered && reinterpret_cast<uintptr_t>(host_tier) % kAlign != 0) return HKV_EALIGN;
  hkv_cache* c = new (std::nothrow) hkv_cache();
  if (!c) return HKV_EINVAL;
  int rc = plan_layout(cfg, plan, c->lo, tiered);
  if (rc != HKV_OK) { delete c; return rc; }
  if (cache_bytes < c->lo.arena_bytes || (tiered && host_bytes < c->lo.host_bytes)) { delete c; return HKV_ENOSPACE; }
  char* host_dev = nullptr;            // the host tier as the kernels address it
  if (tiered) {
    // The tier must be page-locked host memory that the current device can address; anything else
    // (pageable memory, a device allocation) is turned away here, before a kernel could touch it.
    hipPointerAttribute_t at;
    std::memset(&at, 0, sizeof(at));
    if (hipPointerGetAttributes(&at, host_tier) != hipSuccess) { (void)hipGetLastError(); delete c; return HKV_EINVAL; }
    if (at.type != hipMemoryTypeHost || !at.devicePointer || !at.hostPointer) { delete c; return HKV_EINVAL; }
    host_dev = static_cast<char*>(at.devicePointer);
    if (reinterpret_cast<uintptr_t>(host_dev) % kAlign != 0) { delete c; return HKV_EALIGN; }
    // unwritten rows of a short last chunk still enter the weighted sums with weight zero: keep them finite
    std::memset(host_tier, 0, c->lo.host_bytes);
  }
  c->host_tier = static_cast<char*>(host_tier);
  c->cfg = *cfg;
  c->batch = plan->batch;
  {
    int dev = 0, cus = 0, khz = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0)
      c->n_cus = cus;
    if (hipDeviceGetAttribute(&khz, hipDeviceAttributeClockRate, dev) == hipSuccess && khz > 0) c->clock_khz = khz;
  }
  // set-up is where the library's own record array is located on this device (hkv_decode_attn_noalloc
  // itself then makes no runtime call besides its launches)
  if (scratch_of_current_device(&c->scratch_dev, &c->device) != hipSuccess) { (void)hipGetLastError(); delete c; return HKV_EHIP; }
  c->arena = static_cast<char*>(cache_dev);
  c->host_tail.assign(cfg->n_layers, 0);
  c->compressed.assign(cfg->n_layers, 0);
  const Layout& lo = c->lo;
  char* a = c->arena;
  CacheView& cv = c->cv;
  cv.units = reinterpret_cast<const UnitDesc*>(a + lo.off_units);
  cv.static_items = reinterpret_cast<const AttnItem*>(a + lo.off_sitems);
  cv.dynamic_items = reinterpret_cast<const AttnItem*>(a + lo.off_ditems);
  cv.static_descs = reinterpret_cast<const UnitDesc*>(a + lo.off_static_descs);
  cv.static_units = reinterpret_cast<const int32_t*>(a + lo.off_static);
  cv.dynamic_units = reinterpret_cast<const int32_t*>(a + lo.off_dynamic);
  cv.dyn_descs = reinterpret_cast<const UnitDesc*>(a + lo.off_dyn_descs);
  cv.is_visual = reinterpret_cast<const uint8_t*>(a + lo.off_vis);
  cv.cnt_a = reinterpret_cast<int32_t*>(a + lo.off_cnt);
  cv.cnt_b = cv.cnt_a + cfg->n_layers;
  cv.kept_idx = reinterpret_cast<int32_t*>(a + lo.off_kept);
  cv.sel = reinterpret_cast<int32_t*>(a + lo.off_sel);
  cv.scores = reinterpret_cast<float*>(a + lo.off_scores);
  cv.sigma = reinterpret_cast<float*>(a + lo.off_sigma);
  cv.mu = a + lo.off_mu;
  cv.k_rows = a + lo.off_k;
  cv.v_rows = a + lo.off_v;
  cv.k_dyn = tiered ? host_dev + lo.host_off_k : cv.k_rows;
  cv.v_dyn = tiered ? host_dev + lo.host_off_v : cv.v_rows;
  cv.n_layers = cfg->n_layers; cv.batch = plan->batch; cv.n_q_heads = cfg->n_q_heads; cv.n_kv_heads = cfg->n_kv_heads;
  cv.G = cfg->n_q_heads / cfg->n_kv_heads; cv.window = cfg->window; cv.max_new = cfg->max_new_tokens;
  cv.causal = cfg->score_causal;
  cv.tile_rows = lo.tile;
  cv.sigma_max = cfg->chunk_score_group;
  cv.index_gen = cfg->index_generated;
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  cv.scale_log2e = scale * 1.4426950408889634f;

  hipError_t e = hipSuccess;
  auto up = [&](size_t off, const void* src, size_t bytes) {
    if (e == hipSuccess && bytes) e = hipMemcpy(a + off, src, bytes, hipMemcpyHostToDevice);
  };
  up(lo.off_units, lo.units.data(), lo.units.size() * sizeof(UnitDesc));
  up(lo.off_sitems, lo.sitems.data(), lo.sitems.size() * sizeof(AttnItem));
  up(lo.off_ditems, lo.ditems.data(), lo.ditems.size() * sizeof(AttnItem));
  {
    std::vector<UnitDesc> sd;
    for (int32_t u : lo.static_units) sd.push_back(lo.units[u]);
    up(lo.off_static_descs, sd.data(), sd.size() * sizeof(UnitDesc));
  }
  up(lo.off_static, lo.static_units.data(), lo.static_units.size() * 4);
  up(lo.off_dynamic, lo.dynamic_units.data(), lo.dynamic_units.size() * 4);
  {
    std::vector<UnitDesc> dd;
    for (int32_t u : lo.dynamic_units) dd.push_back(lo.units[u]);
    up(lo.off_dyn_descs, dd.data(), dd.size() * sizeof(UnitDesc));
  }
  c->cv_second = cv;
  if (lo.second) {
    const Layout& co = *lo.second;
    CacheView& cc = c->cv_second;
    cc.units = reinterpret_cast<const UnitDesc*>(a + lo.s2off_units);
    cc.static_items = reinterpret_cast<const AttnItem*>(a + lo.s2off_sitems);
    cc.dynamic_items = reinterpret_cast<const AttnItem*>(a + lo.s2off_ditems);
    cc.static_descs = reinterpret_cast<const UnitDesc*>(a + lo.s2off_static_descs);
    cc.dyn_descs = reinterpret_cast<const UnitDesc*>(a + lo.s2off_dyn_descs);
    cc.tile_rows = co.tile;
    up(lo.s2off_units, co.units.data(), co.units.size() * sizeof(UnitDesc));
    up(lo.s2off_sitems, co.sitems.data(), co.sitems.size() * sizeof(AttnItem));
    up(lo.s2off_ditems, co.ditems.data(), co.ditems.size() * sizeof(AttnItem));
    std::vector<UnitDesc> sd, dd;
    for (int32_t u : co.static_units) sd.push_back(co.units[u]);
    for (int32_t u : co.dynamic_units) dd.push_back(co.units[u]);
    up(lo.s2off_static_descs, sd.data(), sd.size() * sizeof(UnitDesc));
    up(lo.s2off_dyn_descs, dd.data(), dd.size() * sizeof(UnitDesc));
  }
  up(lo.off_vis, plan->is_visual, (size_t)lo.total_tokens);
  if (e == hipSuccess) e = hipMemset(a + lo.off_cnt, 0, (size_t)2 * cfg->n_layers * 4);
  // rows that are allocated but not (yet) written must hold finite values: masked rows still enter the
  // weighted sum with weight zero
  if (e == hipSuccess) e = hipMemset(a + lo.off_k, 0, lo.rows_end - lo.off_k);
  up(lo.off_stream, lo.stream_blob.data(), lo.stream_blob.size());
  if (e != hipSuccess) { delete c; return HKV_EHIP; }
  *out = c;
  return HKV_OK;
}

int hkv_cache_create(const hkv_config* cfg, const hkv_plan* plan, void* cache_dev, size_t cache_bytes,
                     hkv_cache** out) {
  return create_cache(cfg, plan, cache_dev, cache_bytes, nullptr, 0, false, out);
}

int hkv_cache_create_tiered(const hkv_config* cfg, const hkv_plan* plan, void* cache_dev, size_t cache_bytes,
                            void* host_tier, size_t host_bytes, hkv_cache** out) {
  return create_cache(cfg, plan, cache_dev, cache_bytes, host_tier, host_bytes, true, out);
}

int hkv_profile_disable(hkv_cache* c) {
  if (!c) return HKV_EINVAL;
  for (hipEvent_t e : c->events) (void)hipEventDestroy(e);
  c->events.clear();
  c->prof_calls = c->prof_max = 0;
  return HKV_OK;
}

int hkv_profile_enable(hkv_cache* c, int max_calls) {
  if (!c || max_calls < 1 || max_calls > (1 << 20)) return HKV_EINVAL;
  hkv_profile_disable(c);
  c->events.resize((size_t)6 * max_calls);
  for (size_t i = 0; i < c->events.size(); ++i) {
    if (hipEventCreate(&c->events[i]) != hipSuccess) {
      c->events.resize(i);
      hkv_profile_disable(c);
      return HKV_EHIP;
    }
  }
  c->prof_max = max_calls;
  c->prof_mask.assign(max_calls, 0);
  return HKV_OK;
}

int hkv_profile_read(hkv_cache* c, double* ms, int* n_calls) {
  if (!c || !ms || !n_calls) return HKV_EINVAL;
  ms[0] = ms[1] = ms[2] = 0.0;
  if (c->prof_calls > 0 && hipStreamSynchronize(c->prof_stream) != hipSuccess) return HKV_EHIP;
  for (int i = 0; i < c->prof_calls; ++i) {
    hipEvent_t* e = &c->events[(size_t)6 * i];
    for (int j = 0; j < 3; ++j) {
      if (!(c->prof_mask[i] >> j & 1)) continue;        // that kernel was not part of the call
      float t = 0.f;
      if (hipEventElapsedTime(&t, e[2 * j], e[2 * j + 1]) != hipSuccess) return HKV_EHIP;
      ms[j] += t;
    }
  }
  *n_calls = c->prof_calls;
  c->prof_calls = 0;
  return HKV_OK;
}

void hkv_cache_destroy(hkv_cache* cache) {
  if (cache) hkv_profile_disable(cache);
  delete cache;
}

static int check_range(const hkv_cache* c, int lb, int le) {
  if (!c) return HKV_EINVAL;
  if (lb < 0 || le > c->cfg.n_layers || lb >= le) return HKV_EINVAL;
  return HKV_OK;
}

static int compress_impl(hkv_cache* c, int lb, int le, const void* q_window, const void* k, const void* v,
                         void* workspace, size_t workspace_bytes, void* stream, bool do_scoring) {
  int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  if (!k || !v || (do_scoring && (!q_window || !workspace))) return HKV_EINVAL;
  if (!aligned16(k) || !aligned16(v) || (do_scoring && (!aligned16(q_window) || !aligned16(workspace)))) return HKV_EALIGN;
  if (do_scoring && workspace_bytes < c->lo.ws_bytes) return HKV_ENOSPACE;
  const Layout& lo = c->lo;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int sb = lo.static_begin[lb], ns = lo.static_begin[le] - sb;
  const int db = lo.dynamic_begin[lb], nd = lo.dynamic_begin[le] - db;
  hipError_t e = hipSuccess;
  if (do_scoring && ns > 0) {
    const int n_splits = (lo.max_C + kKeysPerBlock - 1) / kKeysPerBlock;
    float2* part = static_cast<float2*>(workspace);
    float2* fin = reinterpret_cast<float2*>(static_cast<char*>(workspace) +
                                            align_up((size_t)ns * n_splits * kMaxScoreRows * sizeof(float2)));
    // Keys per scoring block: the one from kKeysPerBlock to twice that (whole 32-key tiles) whose grid takes the
    // fewest tile-times -- rounds of resident workgroups (three per compute unit) times tiles per block.  A grid
    // that overflows its last round by a few blocks costs a whole round.
    int keys_per_block = kKeysPerBlock;
    {
      const int64_t resident = 3 * (int64_t)c->n_cus;
      int64_t best = -1;
      for (int tiles = kKeysPerBlock / 32; tiles <= 2 * kKeysPerBlock / 32; ++tiles) {
        int64_t blocks = 0;
        for (int i = 0; i < ns; ++i) blocks += (lo.units[lo.static_units[sb + i]].C + 32 * tiles - 1) / (32 * tiles);
        const int64_t cost = (blocks + resident - 1) / resident * tiles;
        if (best < 0 || cost < best) { best = cost; keys_per_block = 32 * tiles; }
      }
    }
    e = launch_score(c->cv, c->cfg.dtype, lb, sb, ns, lo.max_C, q_window, k, lo.total_tokens, part, fin, keys_per_block, st);
  }
  if (e == hipSuccess) e = launch_select(c->cv, sb, ns, st);
  if (e == hipSuccess) e = launch_compact(c->cv, c->cfg.dtype, lb, sb, ns, lo.max_rows_static, k, v, lo.total_tokens, st);
  if (e == hipSuccess) e = launch_adopt(c->cv, c->cfg.dtype, lb, db, nd, lo.max_chunks, lo.max_C, k, v, lo.total_tokens, st);
  if (e == hipSuccess) e = launch_rewind(c->cv, lb, le, st);
  if (e != hipSuccess) return HKV_EHIP;
  for (int l = lb; l < le; ++l) { c->compressed[l] = 1; c->host_tail[l] = 0; }
  return HKV_OK;
}

int hkv_compress(hkv_cache* cache, int layer_begin, int layer_end, const void* q_window, const void* k,
                 const void* v, void* workspace, size_t workspace_bytes, void* stream) {
  return compress_impl(cache, layer_begin, layer_end, q_window, k, v, workspace, workspace_bytes, stream, true);
}

int hkv_compress_from_scores(hkv_cache* cache, int layer_begin, int layer_end, const void* k, const void* v,
                             void* stream) {
  return compress_impl(cache, layer_begin, layer_end, nullptr, k, v, nullptr, 0, stream, false);
}

// Which tiling a decode call over [lb, le) takes.  With a coarser second tiling: the first, unless the call has
// more of its tiles than the device has compute units and the second gives every tile a compute unit of its
// own (measured on the 7B shape at 8K context, all layers in one call: 228 tiles of 1024 rows take 21.8 us
// per step, 678 tiles of 256 rows 24.8 us; a call per layer is 23 % slower with the large tiles).
static bool call_uses_second_tiling(const hkv_cache* c, int lb, int le) {
  if (!c->lo.second || c->lo.mode == 4) return false;
  const Layout& s2 = *c->lo.second;
  const int first_tiles = c->lo.item_begin[le] - c->lo.item_begin[lb];
  const int second_tiles = s2.item_begin[le] - s2.item_begin[lb];
  if (s2.tile > c->lo.tile) return first_tiles > c->n_cus && second_tiles <= c->n_cus;
  // finer second tiling (large caches): for calls whose large tiles would not even give every compute unit one
  // (a call per layer of the 72B video shape: 28 tiles of 1024 rows 32.3 us, 96 of 256 rows 26.3 us)
  return first_tiles <= c->n_cus;
}

// The table a streamed call over [lb, le) walks, or null when the call does not run streamed: the cache is
// not in that shape, or the range is neither all layers nor a single one (such calls take the tiles).
// The table is the one made for the largest reference tail length not above the tail the host knows of.
static const StreamTable* stream_table_of_call(const hkv_cache* c, int lb, int le, const StreamShape** shape) {
  if (c->lo.mode != 5 || c->lo.stream_shapes.empty()) return nullptr;
  const int L = c->cfg.n_layers;
  int s = -1;
  if (lb == 0 && le == L) s = 0;
  else if (le == lb + 1) s = 1 + lb;
  if (s < 0 || s >= (int)c->lo.stream_shapes.size()) return nullptr;
  const StreamShape& sh = c->lo.stream_shapes[s];
  const int t = c->host_tail[lb];
  const StreamTable* tb = &sh.tables[0];
  for (const StreamTable& x : sh.tables) if (x.t_ref <= t) tb = &x;
  // under the automatic rule a call per layer streams only when its shares are long enough as well; shorter
  // ones pay the unit crossings (descriptor, repeated selection) too often and run as tiles (measured on the
  // serving mix: 56 vs 59 us per call)
  if (c->lo.mode_by_rule && s > 0 && tb->share_rows < kStreamAutoRows) return nullptr;
  if (shape) *shape = &sh;
  return tb;
}

// Record slots a decode call over [lb, le) may write (tail at full capacity for the tile shapes).
static size_t call_record_slots(const hkv_cache* c, int lb, int le) {
  const StreamShape* sh = nullptr;
  if (const StreamTable* tb = stream_table_of_call(c, lb, le, &sh)) return (size_t)tb->n_wg + (size_t)sh->n_units;
  const Layout& lo = call_uses_second_tiling(c, lb, le) ? *c->lo.second : c->lo;
  return (size_t)(lo.item_begin[le] - lo.item_begin[lb]);
}

int hkv_cache_call_tiling(const hkv_cache* c, int lb, int le, int32_t* tile_rows, int32_t* n_tiles) {
  const int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  if (const StreamTable* tb = stream_table_of_call(c, lb, le, nullptr)) {
    if (tile_rows) *tile_rows = tb->share_rows;
    if (n_tiles) *n_tiles = tb->n_wg;
    return HKV_OK;
  }
  const Layout& lo = call_uses_second_tiling(c, lb, le) ? *c->lo.second : c->lo;
  if (tile_rows) *tile_rows = lo.tile;
  if (n_tiles) *n_tiles = lo.item_begin[le] - lo.item_begin[lb];
  return HKV_OK;
}

// Argument checks shared by the decode entry points (everything but the workspace).
static int check_decode_args(const hkv_cache* c, int lb, int le, const void* q, const void* k_new, const void* v_new,
                             const void* out) {
  int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  if (!q || !out) return HKV_EINVAL;
  if ((k_new == nullptr) != (v_new == nullptr)) return HKV_EINVAL;
  if (!aligned16(q) || !aligned16(out) || !aligned16(k_new) || !aligned16(v_new)) return HKV_EALIGN;
  for (int l = lb; l < le; ++l) {
    if (!c->compressed[l]) return HKV_ESTATE;
    if (k_new && !c->device_tail && c->host_tail[l] + 1 > c->cfg.max_new_tokens) return HKV_ENOSPACE;
  }
  return HKV_OK;
}

// The launches of one decode step over layers [lb, le), arguments already checked.  `records`: room for the
// call's split-K records, [slots][G][128] floats followed (256-byte aligned) by their (max, sum) lines,
// [slots][16] floats, slots = call_record_slots().
static int decode_launches(hkv_cache* c, int lb, int le, const void* q, const void* k_new, const void* v_new, void* out,
                           void* records, void* stream) {
  const size_t n_slots = call_record_slots(c, lb, le);
  float* parts = static_cast<float*>(records);
  float* parts_ml = reinterpret_cast<float*>(static_cast<char*>(records) +
                                             align_up(n_slots * (size_t)(c->cfg.n_q_heads / c->cfg.n_kv_heads) * kD * sizeof(float)));
  const bool use_second = call_uses_second_tiling(c, lb, le);
  const Layout& lo = use_second ? *c->lo.second : c->lo;
  const CacheView& cv = use_second ? c->cv_second : c->cv;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int slot_base = lo.item_begin[lb];
  const int db = lo.dynamic_begin[lb], nd = lo.dynamic_begin[le] - db;
  const int sb = lo.sitem_begin[lb], ns = lo.sitem_begin[le] - sb;
  const int dib = lo.ditem_begin[lb], ndi = lo.ditem_begin[le] - dib;
  const int sub = lo.static_begin[lb], nsu = lo.static_begin[le] - sub;
  const int ub = lb * c->batch * c->cfg.n_kv_heads, nu = (le - lb) * c->batch * c->cfg.n_kv_heads;
  // tail length: when every layer of the call has the same one (the normal case) it travels as a
  // kernel argument; otherwise the kernels read the per-layer device counters
  int t_before = c->device_tail ? -1 : c->host_tail[lb];
  for (int l = lb; l < le; ++l) if (c->host_tail[l] != t_before) t_before = -1;
  hipEvent_t none[6] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  const bool prof = c->prof_max > 0 && c->prof_calls < c->prof_max;
  hipEvent_t* ev = prof ? &c->events[(size_t)6 * c->prof_calls] : none;
  hipError_t e = hipSuccess;
  const int dt = c->cfg.dtype, app = k_new ? 1 : 0;
  const StreamShape* sshape = nullptr;
  const StreamTable* stable = stream_table_of_call(c, lb, le, &sshape);
  const int mode = c->lo.mode == 5 && !stable ? 3 : c->lo.mode;      // streamed caches run other layer ranges as tiles
  const int resident = 3 * c->n_cus;      // workgroups resident at once (three per compute unit)
  if (c->cfg.chunk_score_group == 1) {    // the other group reading scores the chunks in a launch of its own
    e = launch_chunk_score_max(cv, dt, lb, db, nd, q, t_before, st);
    if (e != hipSuccess) return HKV_EHIP;
  }
  if (mode == 5) {
    // equal shares of the call's rows, one per workgroup; units that several workgroups touched are combined after
    const char* tables = c->arena + c->lo.off_stream;
    e = launch_stream(c->cv, dt, reinterpret_cast<const StreamBound*>(tables + stable->off_bounds), stable->n_wg,
                      sshape->unit_begin, lb, q, k_new, v_new, parts, parts_ml, out, t_before,
                      c->lo.max_chunks, st, ev[0], ev[1]);
    if (e == hipSuccess)
      e = launch_stream_merge(c->cv, dt, reinterpret_cast<const StreamMulti*>(tables + stable->off_multi), stable->n_multi,
                              sshape->unit_begin, lb, le, parts, parts_ml, out, t_before, st, ev[4], ev[5]);
    if (e != hipSuccess) return HKV_EHIP;
    if (prof) {
      c->prof_mask[c->prof_calls] = (uint8_t)(1 | (stable->n_multi > 0 ? 4 : 0));
      c->prof_calls += 1;
      c->prof_stream = st;
    }
    if (k_new && !c->device_tail) for (int l = lb; l < le; ++l) c->host_tail[l] += 1;
    return HKV_OK;
  }
  if (mode == 4) {
    // one wide workgroup per unit writes the unit's output rows itself: no records, no combination
    e = launch_units(cv, dt, lb, db, nd, sub, nsu, q, k_new, v_new, out, t_before, lo.max_chunks, st, ev[0], ev[1]);
    if (e == hipSuccess) e = launch_attn_merge(cv, dt, nullptr, 0, lb, le, slot_base, parts, parts_ml, out, t_before,
                                               app, st);          // publishes device-side tail counters, if in use
    if (e != hipSuccess) return HKV_EHIP;
    if (prof) {
      c->prof_mask[c->prof_calls] = 1;
      c->prof_calls += 1;
      c->prof_stream = st;
    }
    if (k_new && !c->device_tail) for (int l = lb; l < le; ++l) c->host_tail[l] += 1;
    return HKV_OK;
  }
  bool pre_scored = false;
  if (mode == 3) {
    // a grid that is resident in one round: the static tiles wait for the time the dynamic tiles' summary
    // reads take at kSummaryRate (what a launch's first reads were measured to draw while every workgroup
    // asks at once), in units of 512 clocks of the device's shader clock, at most 16
    constexpr double kSummaryRate = 5.0e12;   // bytes per second
    int hold = 0;
    if (ndi > 0 && ndi + ns <= resident) {
      const double seconds = (double)(lo.dmu_begin[le] - lo.dmu_begin[lb]) / kSummaryRate;
      hold = (int)std::min<int64_t>(16, (int64_t)(seconds * c->clock_khz * 1e3 / 512.0));
    }
    // A grid of one round on a cache whose heads have many chunks would end with a dynamic tile whose four waves
    // bring in all summaries of its head before its rows (12-35 us of a 49 us launch for a call per layer of the
    // serving mix, up to 1218 chunks per head).  Under the automatic rule the scores then come from a launch of
    // their own, spread over the compute units, and the tiles only pick: a call per layer of the serving mix
    // 55.8 -> 45.6 us, of the 72B video shape 24.6 -> 23.9; at 512 chunks per head (32k shape) it costs
    // 21.5 -> 21.9, at 256 (8k shape) 14.4 -> 17.1, hence the threshold.
    const bool pre_score = c->lo.mode_by_rule && ndi > 0 && ndi + ns <= resident && lo.max_chunks > kPreScoreChunks &&
                           !c->cfg.chunk_score_group && !c->cfg.index_generated;
    CacheView cvs = cv;
    if (pre_score) {
      e = launch_chunk_score_sum(cv, dt, lb, db, nd, lo.max_chunks, q, st, ev[2], ev[3]);
      if (e != hipSuccess) return HKV_EHIP;
      cvs.sigma_max = 1;              // the tiles read the stored scores
      pre_scored = true;
    }
    e = launch_dynamic_tiles(cvs, dt, lb, dib, ndi, sb, ns, slot_base, q, k_new, v_new, parts, parts_ml, out, t_before, 1,
                             pre_score ? 0 : hold, lo.max_chunks, c->stamps, c->n_stamps, st, ev[0], ev[1]);
  } else {
    e = launch_decode(cv, dt, lb, db, nd, sb, ns, slot_base, q, k_new, v_new, parts, parts_ml, out, t_before, 0,
                      mode == 2 ? 1 : 0, lo.max_chunks, st, ev[0], ev[1]);
    if (e == hipSuccess && mode == 2)
      e = launch_dynamic_tiles(cv, dt, lb, dib, ndi, sb, 0, slot_base, q, k_new, v_new, parts, parts_ml, out, t_before, 0,
                               0, lo.max_chunks, nullptr, 0, st, ev[2], ev[3]);
  }
  if (e == hipSuccess)
    e = mode == 1 ? launch_attn_merge(cv, dt, cv.static_descs + sub, nsu, lb, le, slot_base, parts, parts_ml, out,
                                      t_before, app, st, ev[4], ev[5])
                  : launch_attn_merge(cv, dt, cv.units + ub, nu, lb, le, slot_base, parts, parts_ml, out, t_before,
                                      app, st, ev[4], ev[5]);
  if (e != hipSuccess) return HKV_EHIP;
  if (prof) {
    c->prof_mask[c->prof_calls] = (uint8_t)(1 | (((mode == 2 && ndi > 0) || pre_scored) ? 2 : 0) | ((mode == 1 ? nsu : nu) > 0 ? 4 : 0));
    c->prof_calls += 1;
    c->prof_stream = st;
  }
  if (k_new && !c->device_tail) for (int l = lb; l < le; ++l) c->host_tail[l] += 1;
  return HKV_OK;
}

int hkv_decode_attn(hkv_cache* c, int lb, int le, const void* q, const void* k_new, const void* v_new, void* out,
                    void* workspace, size_t workspace_bytes, void* stream) {
  const int rc = check_decode_args(c, lb, le, q, k_new, v_new, out);
  if (rc != HKV_OK) return rc;
  if (!workspace) return HKV_EINVAL;
  if (!aligned16(workspace)) return HKV_EALIGN;
  if (workspace_bytes < c->lo.ws_bytes) return HKV_ENOSPACE;
  return decode_launches(c, lb, le, q, k_new, v_new, out, workspace, stream);
}

int hkv_decode_attn_noalloc(hkv_cache* c, int lb, int le, const void* q, const void* k_new, const void* v_new,
                            void* out, void* stream) {
  int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  // the records of this call must fit the library's array (tile shapes: tail at full capacity, as the tables count them)
  const size_t n_slots = call_record_slots(c, lb, le);
  const size_t G = (size_t)(c->cfg.n_q_heads / c->cfg.n_kv_heads);
  const size_t need = align_up(n_slots * G * kD * sizeof(float)) + align_up(n_slots * kMlFloats * sizeof(float));
  if (need > (size_t)HKV_NOALLOC_SCRATCH_BYTES) return HKV_ENOSPACE;
  rc = check_decode_args(c, lb, le, q, k_new, v_new, out);
  if (rc != HKV_OK) return rc;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return HKV_EHIP;
  if (dev != c->device || !c->scratch_dev) return HKV_ESTATE;      // the array's address belongs to the cache's device
  return decode_launches(c, lb, le, q, k_new, v_new, out, c->scratch_dev, stream);
}

int hkv_reselect_chunks(hkv_cache* c, int lb, int le, void* stream) {
  int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  const Layout& lo = c->lo;
  const int db = lo.dynamic_begin[lb], nd = lo.dynamic_begin[le] - db;
  hipError_t e = launch_decode(c->cv, c->cfg.dtype, lb, db, nd, 0, 0, 0, nullptr, nullptr, nullptr, nullptr, nullptr,
                               nullptr, -1, 1, 1, lo.max_chunks, static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HKV_OK : HKV_EHIP;
}

int hkv_cache_set_device_tail(hkv_cache* c, int enable, void* stream) {
  if (!c || (enable != 0 && enable != 1)) return HKV_EINVAL;
  if (!enable && c->device_tail) {
    // back to host bookkeeping: fetch what the device counted meanwhile
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (hipMemcpyAsync(c->host_tail.data(), c->cv.cnt_a, (size_t)c->cfg.n_layers * 4, hipMemcpyDeviceToHost, st) != hipSuccess ||
        hipStreamSynchronize(st) != hipSuccess) return HKV_EHIP;
  }
  c->device_tail = enable != 0;
  return HKV_OK;
}

int hkv_cache_rewind(hkv_cache* c, void* stream) {
  if (!c) return HKV_EINVAL;
  hipError_t e = launch_rewind(c->cv, 0, c->cfg.n_layers, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return HKV_EHIP;
  std::fill(c->host_tail.begin(), c->host_tail.end(), 0);
  return HKV_OK;
}

static int full_view(const hkv_config* cfg, int32_t batch, const int32_t* cu, int n_layers_call, FullView& fv) {
  int rc = validate_config(cfg);
  if (rc != HKV_OK) return rc;
  if (!cu) return HKV_EINVAL;
  if (batch < 1 || batch > kFullMaxBatch || n_layers_call < 1) return HKV_ESHAPE;
  if (cu[0] != 0) return HKV_EINVAL;
  int32_t max_len = 0;
  for (int b = 0; b < batch; ++b) {
    if (cu[b + 1] <= cu[b]) return HKV_ESHAPE;
    // 24-bit row index times row stride must fit 32 bits inside the kernels
    if ((int64_t)(cu[b + 1] - cu[b]) >= (1 << 24) ||
        (int64_t)(cu[b + 1] - cu[b]) * cfg->n_kv_heads * kD * 4 >= ((int64_t)1 << 32)) return HKV_ESHAPE;
    max_len = std::max(max_len, cu[b + 1] - cu[b]);
  }
  std::memset(&fv, 0, sizeof(fv));
  std::memcpy(fv.cu, cu, (size_t)(batch + 1) * 4);
  fv.batch = batch; fv.n_layers_call = n_layers_call; fv.n_q_heads = cfg->n_q_heads; fv.n_kv_heads = cfg->n_kv_heads;
  fv.G = cfg->n_q_heads / cfg->n_kv_heads;
  const int tile = cfg->dtype == HKV_BF16 ? kTileBf16 : kTileF32;
  fv.n_tiles_max = (max_len + tile - 1) / tile;
  fv.total_tokens = cu[batch];
  const float scale = cfg->softmax_scale > 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  fv.scale_log2e = scale * 1.4426950408889634f;
  if ((int64_t)n_layers_call * batch * cfg->n_kv_heads > 65535) return HKV_ESHAPE;
  return HKV_OK;
}

int hkv_full_workspace_size(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens, int n_layers_call,
                            size_t* workspace_bytes) {
  if (!workspace_bytes) return HKV_EINVAL;
  FullView fv;
  int rc = full_view(cfg, batch, cu_seqlens, n_layers_call, fv);
  if (rc != HKV_OK) return rc;
  const size_t n_slots = (size_t)n_layers_call * batch * cfg->n_kv_heads * fv.n_tiles_max;
  *workspace_bytes = align_up(n_slots * fv.G * kD * sizeof(float)) + align_up(n_slots * kMlFloats * sizeof(float));
  return HKV_OK;
}

int hkv_full_decode_attn(const hkv_config* cfg, int32_t batch, const int32_t* cu_seqlens, int n_layers_call,
                         const void* q, const void* k, const void* v, void* out, void* workspace,
                         size_t workspace_bytes, void* stream) {
  FullView fv;
  int rc = full_view(cfg, batch, cu_seqlens, n_layers_call, fv);
  if (rc != HKV_OK) return rc;
  if (!q || !k || !v || !out || !workspace) return HKV_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out) || !aligned16(workspace)) return HKV_EALIGN;
  size_t need = 0;
  hkv_full_workspace_size(cfg, batch, cu_seqlens, n_layers_call, &need);
  if (workspace_bytes < need) return HKV_ENOSPACE;
  const size_t n_slots = (size_t)n_layers_call * batch * cfg->n_kv_heads * fv.n_tiles_max;
  float* parts_ml = reinterpret_cast<float*>(static_cast<char*>(workspace) + align_up(n_slots * fv.G * kD * sizeof(float)));
  hipError_t e = launch_full_attn(fv, cfg->dtype, q, k, v, static_cast<float*>(workspace), parts_ml, out,
                                  static_cast<hipStream_t>(stream));
  return e == hipSuccess ? HKV_OK : HKV_EHIP;
}

static const UnitDesc* find_unit(const hkv_cache* c, int seq, int layer, int head) {
  if (!c || seq < 0 || seq >= c->batch || layer < 0 || layer >= c->cfg.n_layers || head < 0 ||
      head >= c->cfg.n_kv_heads)
    return nullptr;
  return &c->lo.units[((size_t)layer * c->batch + seq) * c->cfg.n_kv_heads + head];
}

int hkv_cache_unit_info(const hkv_cache* c, int seq, int layer, int head, int32_t* prompt_rows, int32_t* n_chunks,
                        int32_t* k_chunks) {
  const UnitDesc* d = find_unit(c, seq, layer, head);
  if (!d) return HKV_EINVAL;
  if (prompt_rows) *prompt_rows = d->n_prompt_rows;
  if (n_chunks) *n_chunks = d->kind == HKV_DYNAMIC ? d->n_chunks : 0;
  if (k_chunks) *k_chunks = d->kind == HKV_DYNAMIC ? d->k_sel : 0;
  return HKV_OK;
}

int hkv_plan_unit_info(const hkv_config* cfg, const hkv_plan* plan, int seq, int layer, int head,
                       int32_t* prompt_rows, int32_t* n_chunks, int32_t* k_chunks) {
  Layout lo;
  const int rc = plan_layout(cfg, plan, lo);
  if (rc != HKV_OK) return rc;
  if (seq < 0 || seq >= plan->batch || layer < 0 || layer >= cfg->n_layers || head < 0 || head >= cfg->n_kv_heads)
    return HKV_EINVAL;
  const UnitDesc& d = lo.units[((size_t)layer * plan->batch + seq) * cfg->n_kv_heads + head];
  if (prompt_rows) *prompt_rows = d.n_prompt_rows;
  if (n_chunks) *n_chunks = d.kind == HKV_DYNAMIC ? d.n_chunks : 0;
  if (k_chunks) *k_chunks = d.kind == HKV_DYNAMIC ? d.k_sel : 0;
  return HKV_OK;
}

int hkv_cache_step_bytes(const hkv_cache* c, int lb, int le, int tail, uint64_t* bytes) {
  int rc = check_range(c, lb, le);
  if (rc != HKV_OK) return rc;
  if (!bytes || tail < 0) return HKV_EINVAL;
  const uint64_t R = (uint64_t)kD * elem_size(c->cfg.dtype);
  const size_t upl = (size_t)c->batch * c->cfg.n_kv_heads;
  uint64_t tot = 0;
  for (size_t u = lb * upl; u < le * upl; ++u) {
    const UnitDesc& d = c->lo.units[u];
    if (d.kind == HKV_STATIC) tot += 2 * R * (uint64_t)(d.n_prompt_rows + tail);
    else {
      // selected chunks' actual rows: k*c, minus what the short last chunk lacks cannot be known on
      // the host (it depends on the selection), so the nominal k*c is used
      if (c->cfg.index_generated) {      // complete chunks of generated tokens are scored and may be among the picks
        const int cs = 1 << d.c_log2, n_gen = tail / cs;
        const int k_now = std::min(d.k_sel, d.n_chunks + n_gen);
        tot += (uint64_t)(d.n_chunks + n_gen) * R + 2 * R * (uint64_t)(k_now * cs + tail % cs);
      } else {
        tot += (uint64_t)d.n_chunks * R + 2 * R * (uint64_t)(d.n_prompt_rows + tail);
      }
    }
  }
  *bytes = tot;
  return HKV_OK;
}

static int locate(const hkv_cache* c, int what, const UnitDesc* d, size_t& off, size_t& bytes) {
  const size_t es = elem_size(c->cfg.dtype);
  const Layout& lo = c->lo;
  const int tail = c->host_tail[d->layer];
  // chunks the unit has now: the prompt's, and with indexed generation the complete chunks of its tail
  const int n_chunks_now = d->n_chunks + (c->cfg.index_generated && d->kind == HKV_DYNAMIC ? tail >> d->c_log2 : 0);
  switch (what) {
    case HKV_X_KEPT_IDX:
      if (d->kind != HKV_STATIC) return HKV_EINVAL;
      off = lo.off_kept + (size_t)d->idx_off * 4; bytes = (size_t)d->n_prompt_rows * 4; return HKV_OK;
    case HKV_X_SCORES:
      if (d->kind != HKV_STATIC) return HKV_EINVAL;
      off = lo.off_scores + (size_t)d->aux_off * 4; bytes = (size_t)d->C * 4; return HKV_OK;
    case HKV_X_CHUNK_SEL:
      if (d->kind != HKV_DYNAMIC) return HKV_EINVAL;
      off = lo.off_sel + (size_t)d->idx_off * 4; bytes = (size_t)std::min(d->k_sel, n_chunks_now) * 4; return HKV_OK;
    case HKV_X_CHUNK_SIGMA:
      if (d->kind != HKV_DYNAMIC) return HKV_EINVAL;
      off = lo.off_sigma + (size_t)d->aux_off * 4; bytes = (size_t)n_chunks_now * 4; return HKV_OK;
    case HKV_X_CHUNK_MEAN:
      if (d->kind != HKV_DYNAMIC) return HKV_EINVAL;
      off = lo.off_mu + (size_t)d->aux_off * kD * es; bytes = (size_t)n_chunks_now * kD * es; return HKV_OK;
    case HKV_X_K_ROWS:
    case HKV_X_V_ROWS: {
      const size_t rows = (size_t)(d->kind == HKV_STATIC ? d->n_prompt_rows : d->C) + tail;
      off = (what == HKV_X_K_ROWS ? lo.off_k : lo.off_v) + (size_t)d->kv_row_off * kD * es;
      bytes = rows * kD * es; return HKV_OK;     // logical size; blocked caches are unpacked by the caller
    }
    default: return HKV_EINVAL;
  }
}

int hkv_cache_decode_shape(const hkv_cache* c, int32_t* tile_rows, int32_t* dynamic_mode) {
  if (!c) return HKV_EINVAL;
  if (tile_rows) *tile_rows = c->lo.tile;
  if (dynamic_mode) *dynamic_mode = c->lo.mode;
  return HKV_OK;
}

int hkv_cache_set_stamps(hkv_cache* c, uint64_t* stamps_dev, int32_t n_records) {
  if (!c || n_records < 0 || (stamps_dev && n_records == 0)) return HKV_EINVAL;
  if (stamps_dev && c->cfg.dtype != HKV_BF16) return HKV_ESHAPE;
  if (reinterpret_cast<uintptr_t>(stamps_dev) & 7u) return HKV_EALIGN;
  c->stamps = stamps_dev;
  c->n_stamps = stamps_dev ? n_records : 0;
  return HKV_OK;
}

int hkv_cache_set_decode_dynamic(hkv_cache* c, int32_t dynamic_mode) {
  if (!c || dynamic_mode < 1 || dynamic_mode > 5) return HKV_EINVAL;
  if (dynamic_mode >= 4 && c->cfg.dtype != HKV_BF16) return HKV_ESHAPE;
  if (c->cfg.index_generated && (dynamic_mode == 2 || dynamic_mode == 5)) return HKV_ESHAPE;
  c->lo.mode = dynamic_mode;
  c->lo.mode_by_rule = false;
  return HKV_OK;
}

int hkv_cache_export(const hkv_cache* c, int what, int seq, int layer, int head, void* dst, size_t bytes,
                     size_t* written, void* stream) {
  const UnitDesc* d = find_unit(c, seq, layer, head);
  if (!d) return HKV_EINVAL;
  size_t off = 0, need = 0;
  int rc = locate(c, what, d, off, need);
  if (rc != HKV_OK) return rc;
  if (written) *written = need;
  if (!dst || bytes < need) return HKV_ENOSPACE;
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return HKV_EHIP;
  if ((what == HKV_X_K_ROWS || what == HKV_X_V_ROWS) && c->cfg.dtype == HKV_BF16) {
    // blocked layout -> plain rows: the prompt rows (device arrays, or the host tier for a dynamic unit of
    // a tiered cache), then the tail rows (always in the device arrays)
    const bool is_k = what == HKV_X_K_ROWS;
    const int tail = c->host_tail[d->layer];
    const int n_prompt = d->kind == HKV_STATIC ? d->n_prompt_rows : d->C;
    const char* prompt_base = static_cast<const char*>(d->kind == HKV_DYNAMIC ? (is_k ? c->cv.k_dyn : c->cv.v_dyn)
                                                                              : (is_k ? c->cv.k_rows : c->cv.v_rows));
    const char* tail_base = static_cast<const char*>(is_k ? c->cv.k_rows : c->cv.v_rows);
    // physical rows [r0, r0 + n) of one array, as whole blocks
    auto fetch = [&](const char* base, int64_t r0, int64_t n, std::vector<uint16_t>& raw, int64_t& first_blk) {
      first_blk = r0 / kBlkRows;
      const int64_t n_blk = n > 0 ? (r0 + n + kBlkRows - 1) / kBlkRows - first_blk : 0;
      raw.resize((size_t)n_blk * kBlkRows * kD);
      if (n_blk == 0) return true;
      return hipMemcpy(raw.data(), base + (size_t)first_blk * kBlkBytes, (size_t)n_blk * kBlkBytes, hipMemcpyDefault) ==
             hipSuccess;
    };
    std::vector<uint16_t> raw_p, raw_t;
    int64_t fb_p = 0, fb_t = 0;
    if (!fetch(prompt_base, d->kv_row_off, n_prompt, raw_p, fb_p)) return HKV_EHIP;
    if (!fetch(tail_base, d->tail_off, tail, raw_t, fb_t)) return HKV_EHIP;
    uint16_t* out = static_cast<uint16_t*>(dst);
    for (int r = 0; r < n_prompt + tail; ++r) {
      const bool in_tail = r >= n_prompt;
      const int64_t pr = in_tail ? d->tail_off + (r - n_prompt) : d->kv_row_off + r;
      const uint16_t* blk = (in_tail ? raw_t.data() : raw_p.data()) +
                            (size_t)(pr / kBlkRows - (in_tail ? fb_t : fb_p)) * (kBlkRows * kD);
      const int e = (int)(pr % kBlkRows);
      for (int dd = 0; dd < kD; ++dd)
        out[(size_t)r * kD + dd] = is_k ? blk[k_piece_index(e, dd >> 3) * 8 + (dd & 7)] : blk[dd * 8 + e];
    }
    return HKV_OK;
  }
  if (need && hipMemcpy(dst, c->arena + off, need, hipMemcpyDeviceToHost) != hipSuccess) return HKV_EHIP;
  return HKV_OK;
}

int hkv_cache_import(hkv_cache* c, int what, int seq, int layer, int head, const void* src, size_t bytes,
                     void* stream) {
  const UnitDesc* d = find_unit(c, seq, layer, head);
  if (!d || !src) return HKV_EINVAL;
  if (what != HKV_X_SCORES && what != HKV_X_CHUNK_SIGMA && what != HKV_X_CHUNK_MEAN) return HKV_EINVAL;
  size_t off = 0, need = 0;
  int rc = locate(c, what, d, off, need);
  if (rc != HKV_OK) return rc;
  if (bytes != need) return HKV_ENOSPACE;
  if (hipStreamSynchronize(static_cast<hipStream_t>(stream)) != hipSuccess) return HKV_EHIP;
  if (need && hipMemcpy(c->arena + off, src, need, hipMemcpyHostToDevice) != hipSuccess) return HKV_EHIP;
  return HKV_OK;
}

// Head types and token budgets of one sequence from its sparsity scores (paper, Section 3.1 threshold and
// Section 3.2, both allocation equations): host arithmetic only.
int hkv_allocate_budgets(int32_t n_heads, const float* scores, float theta, int64_t total_budget, float share_ratio,
                         float alpha, int32_t pad_pow2, uint8_t* head_type, int32_t* budget) {
  if (n_heads < 1 || !scores || !head_type || !budget || total_budget < 0) return HKV_EINVAL;
  if (!(share_ratio >= 0.f) || !(alpha >= 0.f) || !(alpha <= 1.f)) return HKV_EINVAL;
  // every input is checked and every result computed before anything is written: an error leaves the
  // caller's arrays as they were
  int n_stat = 0, n_dyn = 0;
  double stat_sum = 0.0;
  for (int i = 0; i < n_heads; ++i) {
    if (!(scores[i] >= 0.f)) return HKV_EINVAL;                    // NaN or negative
    if (scores[i] >= theta) { ++n_stat; stat_sum += (double)scores[i]; } else ++n_dyn;
  }
  // A ceiling is taken of its argument minus 1e-9: a product that is a whole number up to floating-point
  // error (r = 0.75 of a budget divisible by four) must not creep up to the next integer.
  constexpr double kCeilSlack = 1e-9;
  // type level: B_dyna = ceil(r * B_bar * N_dyna), r clipped so that it cannot exceed the total
  int64_t b_dyn = 0;
  if (n_dyn > 0) {
    const double b_bar = (double)total_budget / n_heads;
    const double r = std::min((double)share_ratio, (double)total_budget / std::max(b_bar * n_dyn, 1e-300));
    b_dyn = std::min<int64_t>(total_budget, (int64_t)std::ceil(r * b_bar * n_dyn - kCeilSlack));
  }
  const int64_t b_stat = total_budget - b_dyn;
  // dynamic heads: uniform share, optionally to the nearest power of two (ties upwards)
  int64_t dyn_each = 0;
  if (n_dyn > 0) {
    const double b = (double)b_dyn / n_dyn;
    if (!pad_pow2) dyn_each = (int64_t)b;
    else if (b <= 1.0) dyn_each = 1;
    else {
      const double lo = std::exp2(std::floor(std::log2(b)));
      dyn_each = (int64_t)((b - lo) < (2.0 * lo - b) ? lo : 2.0 * lo);
    }
  }
  std::vector<int32_t> result((size_t)n_heads);
  for (int i = 0; i < n_heads; ++i) {
    int64_t v;
    if (!(scores[i] >= theta)) v = dyn_each;
    else {
      const double s_norm = stat_sum > 0.0 ? (double)scores[i] / stat_sum : 1.0 / n_stat;
      v = (int64_t)std::ceil((double)alpha * b_stat / n_stat + (1.0 - (double)alpha) * b_stat * s_norm - kCeilSlack);
    }
    if (v > 0x7fffffff) return HKV_ESHAPE;
    if (v < 1) return HKV_EBUDGET;                 // the total is too small to give this head a token: hkv_plan needs >= 1
    result[(size_t)i] = (int32_t)v;
  }
  for (int i = 0; i < n_heads; ++i) {
    head_type[i] = scores[i] >= theta ? HKV_STATIC : HKV_DYNAMIC;
    budget[i] = result[(size_t)i];
  }
  return HKV_OK;
}

}  // extern "C"
