"""CPU-only checks of the C-ABI library: it loads, exports every symbol the header declares, and its
host-side validation and planning behave as documented.  No kernel is launched."""
import os
import re

import numpy as np
import pytest

from hkv_synth import make_workload
from oracle import hybridkv_oracle as O
from paper_2604_05887_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(os.path.join(ROOT, "paper_2604_05887_amd", "libhkv.so")):
        from paper_2604_05887_amd.build import build_library
        build_library(verbose=False)
    return B.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "hkv.h")).read()
    declared = set(re.findall(r"HKV_API[^;(]*?\b(hkv_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.hkv_abi_version() == B.HKV_ABI_VERSION
    assert B.hkv_strerror(B.HKV_ESHAPE) == "unsupported shape"


def _cfg(**kw):
    base = dict(n_layers=1, n_q_heads=28, n_kv_heads=4, dtype=B.HKV_F32, window=32, chunk_size=32, max_new_tokens=4)
    base.update(kw)
    return B.make_config(**base)


def _plan(wl, **kw):
    args = dict(cu_seqlens=wl.cu_seqlens, is_visual=wl.is_visual, head_type=wl.head_type, budget=wl.budget,
                chunk_size=wl.chunk_size)
    args.update(kw)
    return B.PlanArrays(**args)


def test_argument_errors_are_reported_on_the_host(lib):
    wl = make_workload(0, shrink=4, steps=1)
    ok = B.hkv_query_sizes(_cfg(), _plan(wl))
    assert ok[0] > 0 and ok[1] > 0

    def status(cfg, plan):
        with pytest.raises(B.HkvError) as ei:
            B.hkv_query_sizes(cfg, plan)
        return ei.value.status

    assert status(_cfg(head_dim=64), _plan(wl)) == B.HKV_ESHAPE
    assert status(_cfg(chunk_score_group=2), _plan(wl)) == B.HKV_EINVAL
    assert status(_cfg(dtype=B.HKV_BF16, decode_tile_rows=100), _plan(wl)) == B.HKV_ESHAPE    # not a multiple of 32
    assert status(_cfg(dtype=B.HKV_BF16, decode_tile_rows=96), _plan(wl)) == B.HKV_ESHAPE     # below 128
    assert status(_cfg(decode_tile_rows=256), _plan(wl)) == B.HKV_ESHAPE                      # fp32 tiles are fixed
    assert status(_cfg(n_q_heads=36), _plan(wl)) == B.HKV_ESHAPE          # group of 9
    assert status(_cfg(n_q_heads=30), _plan(wl)) == B.HKV_ESHAPE          # not divisible
    assert status(_cfg(window=64), _plan(wl)) == B.HKV_ESHAPE             # G * w > 256
    assert status(_cfg(window=0), _plan(wl)) == B.HKV_ESHAPE
    assert status(_cfg(dtype=7), _plan(wl)) == B.HKV_EINVAL
    bad = _cfg(); bad.struct_size = 12
    assert status(bad, _plan(wl)) == B.HKV_EINVAL
    assert status(_cfg(), _plan(wl, chunk_size=np.array([24]))) == B.HKV_ESHAPE       # not a power of two
    b0 = wl.budget.copy(); b0[0, 0, 1] = 0
    assert status(_cfg(), _plan(wl, budget=b0)) == B.HKV_EBUDGET
    ht = wl.head_type.copy(); ht[0, 0, 0] = 3
    assert status(_cfg(), _plan(wl, head_type=ht)) == B.HKV_EINVAL
    assert status(_cfg(), _plan(wl, cu_seqlens=np.array([0, 20]))) == B.HKV_ESHAPE     # prompt shorter than window
    # decode entry point rejects a null cache before touching the device
    assert lib.hkv_decode_attn(None, 0, 1, None, None, None, None, None, 0, None) == B.HKV_EINVAL
    assert lib.hkv_compress(None, 0, 1, None, None, None, None, 0, None) == B.HKV_EINVAL
    assert lib.hkv_cache_call_tiling(None, 0, 1, None, None) == B.HKV_EINVAL


@pytest.mark.parametrize("rule", ["text_exempt", "literal_total"])
def test_planned_rows_match_the_oracle_rule(lib, rule):
    """Retained rows per static head and chunk counts per dynamic head, computed by the library's
    host planner, equal what the oracle's keep rule yields -- for in-regime budgets, budgets below
    text + window, and budgets below the window."""
    wl = make_workload(4, n_layers=2, shrink=8, steps=1, budget_rule=rule)
    budget = wl.budget.copy()
    budget[0, 0, :] = [3, wl.window, 7, 100000][: wl.n_kv_heads]
    cfg = _cfg(n_layers=2, dtype=B.HKV_BF16)
    plan = _plan(wl, budget=budget)
    w = wl.window
    for b in range(wl.batch):
        lo, hi = int(wl.cu_seqlens[b]), int(wl.cu_seqlens[b + 1])
        C = hi - lo
        vis = wl.is_visual[lo:hi]
        n_txt, n_vis = int((vis[: C - w] == 0).sum()), int((vis[: C - w] == 1).sum())
        for l in range(2):
            for h in range(wl.n_kv_heads):
                rows, n_c, k_sel = B.hkv_plan_unit_info(cfg, plan, b, l, h)
                if wl.head_type[b, l, h] == 0:
                    assert rows == O.retained_count(C, w, n_txt, n_vis, int(budget[b, l, h]))
                    assert rows == O.static_keep_set(np.zeros(C), vis, w, int(budget[b, l, h])).size
                else:
                    c = int(wl.chunk_size[b])
                    assert n_c == -(-C // c)
                    assert k_sel == O.n_selected_chunks(int(budget[b, l, h]), c, n_c)
                    assert rows == k_sel * c


def test_cache_size_covers_the_rows_it_promises(lib):
    wl = make_workload(1, n_layers=2, shrink=4, steps=8)
    cfg = _cfg(n_layers=2, dtype=B.HKV_BF16, max_new_tokens=8)
    plan = _plan(wl)
    cache_bytes, ws_bytes = B.hkv_query_sizes(cfg, plan)
    rows = 0
    for l in range(2):
        for h in range(4):
            r, n_c, k = B.hkv_plan_unit_info(cfg, plan, 0, l, h)
            rows += (r if wl.head_type[0, l, h] == 0 else int(wl.seqlens[0])) + 8
    assert cache_bytes >= 2 * rows * 128 * 2
    assert cache_bytes < 2 * rows * 128 * 2 * 1.2 + (1 << 20)


def test_budget_allocation_matches_the_oracle_equations(lib):
    """hkv_allocate_budgets (host arithmetic) against the oracle's type-level split, static-head formula
    and power-of-two padding, on random score sets and on the degenerate head maps."""
    rng = np.random.default_rng(21)
    for trial in range(40):
        n = int(rng.integers(1, 120))
        scores = rng.uniform(0.7, 1.0, n).astype(np.float32)
        if trial == 0:
            scores[:] = 0.95                       # all static
        if trial == 1:
            scores[:] = 0.5                        # all dynamic
        theta = 0.9
        b_total = int(rng.integers(n, 400 * n))
        r, alpha = float(rng.uniform(0.3, 1.2)), float(rng.uniform(0.0, 1.0))
        pad = bool(trial % 2)
        want_types = O.classify_heads(scores, theta)
        stat = want_types == O.STATIC
        b_stat, b_dyn = O.type_level_budgets(b_total, int(stat.sum()), int((~stat).sum()), r)
        want = np.zeros(n, np.int64)
        want[stat] = O.static_head_budgets(b_stat, scores[stat].astype(np.float64), alpha)
        want[~stat] = O.dynamic_head_budget(b_dyn, int((~stat).sum()), pad_pow2=pad)
        if want.min() < 1:                         # a total too small for every head to get a token
            with pytest.raises(B.HkvError) as ei:
                B.hkv_allocate_budgets(scores, theta, b_total, r, alpha, pad)
            assert ei.value.status == B.HKV_EBUDGET
            continue
        types, budget = B.hkv_allocate_budgets(scores, theta, b_total, r, alpha, pad)
        assert np.array_equal(types, want_types)
        assert np.array_equal(budget.astype(np.int64), want), (trial, n, b_total, r, alpha)
    with pytest.raises(B.HkvError):
        B.hkv_allocate_budgets(np.array([0.5, np.nan], np.float32), 0.9, 100, 0.75, 0.5)
    with pytest.raises(B.HkvError):
        B.hkv_allocate_budgets(np.array([0.5], np.float32), 0.9, 100, 0.75, 1.5)


def test_budget_allocation_writes_nothing_on_error(lib):
    """An error return leaves the caller's arrays untouched: a bad score late in the list, and a total
    too small to give every head a token (three dynamic heads, two tokens, no padding)."""
    import ctypes as C
    for scores, total, pad, want in (([0.95, 0.95, 0.5, float("nan")], 100, 1, B.HKV_EINVAL),
                                     ([0.5, 0.5, 0.5], 2, 0, B.HKV_EBUDGET),
                                     ([0.95, 0.5, 0.5], 0, 1, B.HKV_EBUDGET)):
        sc = np.array(scores, np.float32)
        types = np.full(sc.size, 77, np.uint8)
        budget = np.full(sc.size, -5, np.int32)
        st = lib.hkv_allocate_budgets(sc.size, sc.ctypes.data_as(C.POINTER(C.c_float)), 0.9, total, 0.75, 0.5, pad,
                                      types.ctypes.data_as(C.POINTER(C.c_uint8)), budget.ctypes.data_as(C.POINTER(C.c_int32)))
        assert st == want
        assert (types == 77).all() and (budget == -5).all()


def test_head_scores_workspace_and_argument_checks(lib):
    wl = make_workload(1, n_layers=1, shrink=8, tensors=False)
    cfg = B.make_config(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, dtype=B.HKV_BF16, window=wl.window)
    lo, hi = B.hkv_head_scores_workspace_size(cfg, wl.cu_seqlens, wl.is_visual)
    G = wl.n_q_heads // wl.n_kv_heads
    T = int((wl.is_visual == 0).sum())
    C = int(wl.cu_seqlens[-1])
    head_bytes = G * T * ((C + 31) // 32 * 32) * 4
    assert lo >= head_bytes and hi >= wl.n_kv_heads * head_bytes and hi - lo >= (wl.n_kv_heads - 1) * head_bytes
    bad = np.array(wl.is_visual, copy=True); bad[3] = 7
    with pytest.raises(B.HkvError):
        B.hkv_head_scores_workspace_size(cfg, wl.cu_seqlens, bad)


def test_host_tier_sizes_move_exactly_the_dynamic_prompt_rows(lib):
    """Tiered layout: the dynamic heads' prompt rows (whole 8-row blocks, K and V) leave the device
    arena for the host tier; everything else stays.  fp32 caches have no host tier."""
    wl = make_workload(1, n_layers=2, shrink=4, steps=1)
    cfg = _cfg(n_layers=2, dtype=B.HKV_BF16, window=wl.window, max_new_tokens=wl.max_new_tokens)
    plan = _plan(wl)
    dev0, ws0 = B.hkv_query_sizes(cfg, plan)
    dev1, host1, ws1 = B.hkv_query_tier_sizes(cfg, plan)
    assert ws0 == ws1
    C = int(wl.seqlens[0])
    n_dyn = int((wl.head_type == O.DYNAMIC).sum())
    assert n_dyn > 0
    rows = (C + 7) // 8 * 8
    row_bytes = 128 * 2
    assert host1 == 2 * ((n_dyn * rows * row_bytes + 255) // 256 * 256)
    cap = lambda r: (r + wl.max_new_tokens + 7) // 8 * 8
    moved = n_dyn * (cap(rows) - cap(0))
    assert 0 <= (dev0 - dev1) - 2 * moved * row_bytes < 2 * 256        # only alignment padding may differ
    with pytest.raises(B.HkvError) as ei:
        B.hkv_query_tier_sizes(_cfg(n_layers=2, window=wl.window), plan)   # fp32
    assert ei.value.status == B.HKV_ESHAPE
    with pytest.raises(B.HkvError) as ei:
        B.hkv_cache_create_tiered(cfg, plan, None, dev1, None, host1)
    assert ei.value.status == B.HKV_EINVAL


def test_header_is_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """include/hkv.h compiles as C11 with gcc, and a C program linked against libhkv.so can size a
    cache (host-only entry points; no kernel runs)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "abi_check.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "hkv.h"
int main(void) {
  hkv_config cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.struct_size = (uint32_t)sizeof cfg; cfg.abi_version = HKV_ABI_VERSION;
  cfg.n_layers = 1; cfg.n_q_heads = 8; cfg.n_kv_heads = 2; cfg.head_dim = 128; cfg.dtype = HKV_BF16;
  cfg.window = 16; cfg.chunk_size = 8; cfg.max_new_tokens = 4;
  int32_t cu[2] = {0, 64};
  uint8_t vis[64]; for (int i = 0; i < 64; ++i) vis[i] = (uint8_t)(i >= 8 && i < 40);
  uint8_t types[2] = {HKV_STATIC, HKV_DYNAMIC};
  int32_t budget[2] = {32, 16};
  hkv_plan plan; memset(&plan, 0, sizeof plan);
  plan.batch = 1; plan.cu_seqlens = cu; plan.is_visual = vis; plan.head_type = types; plan.budget = budget;
  size_t cache = 0, ws = 0, host = 0;
  int rc = hkv_query_sizes(&cfg, &plan, &cache, &ws);
  if (rc != HKV_OK || cache == 0 || ws == 0) { printf("query failed: %s\n", hkv_strerror(rc)); return 1; }
  rc = hkv_query_tier_sizes(&cfg, &plan, &cache, &host, &ws);
  if (rc != HKV_OK || host == 0) return 2;
  cfg.head_dim = 64;
  if (hkv_query_sizes(&cfg, &plan, &cache, &ws) != HKV_ESHAPE) return 3;
  printf("abi %u ok\n", hkv_abi_version());
  return 0;
}
''')
    exe = tmp_path / "abi_check"
    libdir = os.path.join(ROOT, "paper_2604_05887_amd")
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:libhkv.so", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"],
                   check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert out.strip() == f"abi {B.HKV_ABI_VERSION} ok"
