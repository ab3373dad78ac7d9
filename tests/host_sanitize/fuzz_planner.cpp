// Fuzz driver for the host planner of libhkv, built with AddressSanitizer and UndefinedBehaviorSanitizer and run
// on the CPU (no device is touched): seeded random configurations and plans -- valid ones and ones broken in
// one field -- go through hkv_query_sizes, hkv_query_tier_sizes and hkv_plan_unit_info, and what comes back
// is checked against what the header promises (status codes, retained counts, sizes that grow with the
// rows they must hold).  Any sanitizer finding aborts the run; so does the first broken promise.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "hkv.h"

static uint64_t g_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() { g_state = g_state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(g_state >> 33); }
static int rnd_in(int lo, int hi) { return lo + (int)(rnd() % (uint32_t)(hi - lo + 1)); }

#define REQUIRE(cond)                                                                   \
  do { if (!(cond)) { std::fprintf(stderr, "case %d: broken promise: %s (line %d)\n", g_case, #cond, __LINE__); std::exit(3); } } while (0)
static int g_case = 0;

int main(int argc, char** argv) {
  const int n_cases = argc > 1 ? std::atoi(argv[1]) : 400;
  if (argc > 2) g_state ^= (uint64_t)std::atoll(argv[2]);
  int n_ok = 0, n_refused = 0;
  for (g_case = 0; g_case < n_cases; ++g_case) {
    hkv_config cfg{};
    cfg.struct_size = sizeof(hkv_config);
    cfg.abi_version = HKV_ABI_VERSION;
    cfg.n_layers = rnd_in(1, 6);
    cfg.n_kv_heads = rnd_in(1, 4);
    const int G = rnd_in(1, 8);
    cfg.n_q_heads = cfg.n_kv_heads * G;
    cfg.head_dim = 128;
    cfg.dtype = rnd() & 1;
    cfg.window = rnd_in(1, 256 / G);
    cfg.chunk_size = 4 << rnd_in(0, 5);
    cfg.score_causal = rnd() & 1;
    cfg.max_new_tokens = rnd_in(0, 600);
    cfg.softmax_scale = (rnd() & 1) ? 0.f : 0.125f;
    cfg.decode_tile_rows = (cfg.dtype == HKV_BF16 && (rnd() & 3) == 0) ? 32 * rnd_in(4, 128) : 0;
    cfg.decode_dynamic = rnd_in(0, cfg.dtype == HKV_BF16 ? 5 : 3);
    cfg.chunk_score_group = rnd() & 1;
    cfg.index_generated = (cfg.dtype == HKV_BF16 && cfg.decode_dynamic != 2 && cfg.decode_dynamic != 5 && (rnd() & 3) == 0) ? 1 : 0;
    const int B = rnd_in(1, 5);
    std::vector<int32_t> cu(B + 1, 0), chunk(B);
    for (int b = 0; b < B; ++b) {
      cu[b + 1] = cu[b] + rnd_in(cfg.window, cfg.window + 3000);
      chunk[b] = 4 << rnd_in(cfg.dtype == HKV_BF16 ? 1 : 0, 5);
    }
    std::vector<uint8_t> vis((size_t)cu[B]);
    for (auto& x : vis) x = (uint8_t)((rnd() % 10) < 7);
    const size_t n_units = (size_t)B * cfg.n_layers * cfg.n_kv_heads;
    std::vector<uint8_t> type(n_units);
    std::vector<int32_t> budget(n_units);
    for (size_t i = 0; i < n_units; ++i) {
      type[i] = (uint8_t)(rnd() & 1);
      budget[i] = (rnd() % 16 == 0) ? rnd_in(1, 8) : rnd_in(1, 4000);
    }
    hkv_plan plan{};
    plan.batch = B; plan.cu_seqlens = cu.data(); plan.is_visual = vis.data(); plan.head_type = type.data();
    plan.budget = budget.data(); plan.chunk_size = (rnd() & 1) ? chunk.data() : nullptr;
    if (!plan.chunk_size && cfg.dtype == HKV_BF16 && cfg.chunk_size < 8) cfg.chunk_size = 8;

    // break one thing in a third of the cases
    int expect = HKV_OK;
    switch (rnd() % 12) {
      case 0: cfg.head_dim = 64; expect = HKV_ESHAPE; break;
      case 1: budget[rnd() % n_units] = -rnd_in(0, 5); expect = HKV_EBUDGET; break;
      case 2: type[rnd() % n_units] = 2; expect = HKV_EINVAL; break;
      case 3: if (plan.chunk_size) { chunk[rnd() % B] = 24; expect = HKV_ESHAPE; } break;
      default: break;
    }
    size_t cache_bytes = 0, ws_bytes = 0;
    const int rc = hkv_query_sizes(&cfg, &plan, &cache_bytes, &ws_bytes);
    if (expect != HKV_OK) { REQUIRE(rc == expect); ++n_refused; continue; }
    REQUIRE(rc == HKV_OK);
    REQUIRE(cache_bytes > 0 && ws_bytes > 0 && cache_bytes % 256 == 0);
    // per-unit facts: the retained count follows the keep rule of a static head, the chunk counts that of a dynamic one
    size_t rows_total = 0;
    for (int probe = 0; probe < 12; ++probe) {
      const int b = rnd_in(0, B - 1), l = rnd_in(0, cfg.n_layers - 1), h = rnd_in(0, cfg.n_kv_heads - 1);
      int32_t rows = -1, n_chunks = -1, k_chunks = -1;
      REQUIRE(hkv_plan_unit_info(&cfg, &plan, b, l, h, &rows, &n_chunks, &k_chunks) == HKV_OK);
      const size_t pi = ((size_t)b * cfg.n_layers + l) * cfg.n_kv_heads + h;
      const int C = cu[b + 1] - cu[b], w = cfg.window, bud = budget[pi];
      if (type[pi] == HKV_STATIC) {
        int n_txt = 0, n_vis = 0;
        for (int j = cu[b]; j < cu[b + 1] - w; ++j) (vis[j] ? n_vis : n_txt)++;
        int want;
        if (bud < w) want = bud;
        else if (bud - w - n_txt < 0) want = bud;
        else want = w + n_txt + (bud - w - n_txt < n_vis ? bud - w - n_txt : n_vis);
        REQUIRE(rows == want && rows >= 1 && rows <= C && n_chunks == 0 && k_chunks == 0);
      } else {
        const int c = plan.chunk_size ? chunk[b] : cfg.chunk_size;
        const int nc = (C + c - 1) / c, gen = cfg.index_generated ? cfg.max_new_tokens / c : 0;
        int k = bud / c; if (k < 1) k = 1; if (k > nc + gen) k = nc + gen;
        REQUIRE(n_chunks == nc && k_chunks == k && rows == k * c);
      }
      rows_total += (size_t)rows;
    }
    REQUIRE(hkv_plan_unit_info(&cfg, &plan, B, 0, 0, nullptr, nullptr, nullptr) == HKV_EINVAL);
    if (cfg.dtype == HKV_BF16) {
      size_t cb2 = 0, hb = 0, ws2 = 0;
      REQUIRE(hkv_query_tier_sizes(&cfg, &plan, &cb2, &hb, &ws2) == HKV_OK);
      REQUIRE(cb2 <= cache_bytes + (1u << 20) && hb >= 256);
    }
    ++n_ok;
  }
  // budget allocation (host arithmetic) on random score sets
  for (int t = 0; t < 200; ++t) {
    const int n = rnd_in(1, 300);
    std::vector<float> sc(n);
    for (auto& x : sc) x = (float)(rnd() % 1000) / 999.f;
    std::vector<uint8_t> ty(n);
    std::vector<int32_t> bu(n);
    const int rc = hkv_allocate_budgets(n, sc.data(), 0.9f, (int64_t)rnd_in(0, 500) * n, (float)(rnd() % 150) / 100.f,
                                        (float)(rnd() % 101) / 100.f, rnd() & 1, ty.data(), bu.data());
    REQUIRE(rc == HKV_OK || rc == HKV_EBUDGET);
    if (rc == HKV_OK) for (int i = 0; i < n; ++i) REQUIRE(bu[i] >= 1 && ty[i] <= 1);
  }
  std::printf("planner fuzz: %d plans laid out, %d refused as expected, no finding\n", n_ok, n_refused);
  return 0;
}
