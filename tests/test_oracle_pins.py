"""Pins for the CPU oracle: every check here compares it against something other
than its own formulas -- an independent library's softmax attention, closed
forms worked by hand, brute-force enumeration, or invariants the paper states.
A dropped term, a transposed operand, a wrong axis or a wrong tie-break in the
oracle fails at least one of them.  CPU only."""
import itertools
import math

import numpy as np
import pytest
import scipy.special
import torch

from oracle import hybridkv_oracle as O
from hkv_synth import bf16_round, make_workload


def _sdpa_f64(q, K, V, scale):
    """Independent reference: torch's scaled_dot_product_attention in float64."""
    qt = torch.from_numpy(np.asarray(q, np.float64))[None]          # [1, G, d]
    Kt = torch.from_numpy(np.asarray(K, np.float64))[None]          # [1, n, d]
    Vt = torch.from_numpy(np.asarray(V, np.float64))[None]
    o = torch.nn.functional.scaled_dot_product_attention(qt, Kt, Vt, scale=scale)
    return o[0].numpy()


# ---------------------------------------------------------------- attention
def test_attention_matches_library_sdpa():
    rng = np.random.default_rng(1)
    q, K, V = rng.standard_normal((7, 128)), rng.standard_normal((300, 128)), rng.standard_normal((300, 128))
    o, p = O.attention(q, K, V, 1 / math.sqrt(128), return_weights=True)
    np.testing.assert_allclose(o, _sdpa_f64(q, K, V, 1 / math.sqrt(128)), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)     # weights sum to 1


def test_attention_hand_worked():
    # logits ln1, ln3 -> weights 1/4, 3/4; values 4 and 8 -> 7
    q = np.array([[1.0]])
    K = np.array([[0.0], [math.log(3.0)]])
    V = np.array([[4.0], [8.0]])
    np.testing.assert_allclose(O.attention(q, K, V, 1.0), [[7.0]], rtol=1e-14)
    # scale enters the logits: scale 2 -> weights 1/10, 9/10 -> 7.6
    np.testing.assert_allclose(O.attention(q, K, V, 2.0), [[7.6]], rtol=1e-14)


def test_attention_permutation_invariant():
    rng = np.random.default_rng(2)
    q, K, V = rng.standard_normal((4, 16)), rng.standard_normal((50, 16)), rng.standard_normal((50, 16))
    perm = rng.permutation(50)
    np.testing.assert_allclose(O.attention(q, K, V, 0.25), O.attention(q, K[perm], V[perm], 0.25),
                               rtol=1e-12, atol=1e-14)


# ---------------------------------------------------------------- window scores
def test_window_scores_hand_worked():
    # G=2 heads, w=2 rows each, d=1, keys 0 and 1, scale 1.
    # rows (logit of key1 - key0): ln2, ln3, ln4, ln1 -> p(key0) = 1/3, 1/4, 1/5, 1/2
    q = np.array([[[math.log(2)], [math.log(3)]], [[math.log(4)], [0.0]]])
    k = np.array([[0.0], [1.0]])
    s = O.window_scores(q, k, 1.0)
    want0 = (1 / 3 + 1 / 4 + 1 / 5 + 1 / 2) / 4
    np.testing.assert_allclose(s, [want0, 1 - want0], rtol=1e-14)


def test_window_scores_single_row_is_library_softmax():
    rng = np.random.default_rng(3)
    q, k = rng.standard_normal((1, 1, 32)), rng.standard_normal((77, 32))
    s = O.window_scores(q, k, 0.3)
    np.testing.assert_allclose(s, scipy.special.softmax((k @ q[0, 0]) * 0.3), rtol=1e-12)


def test_window_scores_sum_to_one_and_uniform_closed_form():
    rng = np.random.default_rng(4)
    q, k = rng.standard_normal((7, 32, 128)), rng.standard_normal((512, 128))
    s = O.window_scores(q, k, 1 / math.sqrt(128))
    assert abs(s.sum() - 1.0) < 1e-12 and (s >= 0).all()
    # zero queries (or identical keys) -> every row uniform -> s_w = 1/C exactly for C a power of two
    s0 = O.window_scores(np.zeros((7, 32, 128)), k, 1 / math.sqrt(128))
    assert (s0 == 1.0 / 512).all()
    s1 = O.window_scores(q, np.tile(k[:1], (512, 1)), 1 / math.sqrt(128))
    np.testing.assert_allclose(s1, 1.0 / 512, rtol=1e-12)


def test_window_scores_dominant_key_is_indicator():
    rng = np.random.default_rng(5)
    u = np.zeros(16); u[3] = 1.0
    q = np.tile(100.0 * u, (2, 4, 1))
    k = 0.01 * rng.standard_normal((40, 16)); k[17] = 10.0 * u
    s = O.window_scores(q, k, 1.0)
    assert s[17] > 1 - 1e-12 and np.argmax(s) == 17


def test_window_scores_causal_closed_form():
    # zero queries: row i is uniform over the keys it may see (C-w+i+1 of them)
    C, w = 12, 4
    s = O.window_scores(np.zeros((3, w, 8)), np.ones((C, 8)), 1.0, causal=True)
    want = np.zeros(C)
    for i in range(w):
        n = C - w + i + 1
        want[:n] += 1.0 / n
    np.testing.assert_allclose(s, want / w, rtol=1e-14)
    assert abs(s.sum() - 1) < 1e-14


# ---------------------------------------------------------------- selection
@pytest.mark.parametrize("seed", range(6))
def test_top_indices_brute_force(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(5, 12))
    # few distinct values -> many ties
    scores = rng.integers(0, 4, size=n).astype(np.float64)
    cand = np.sort(rng.choice(n, size=int(rng.integers(3, n + 1)), replace=False))
    for m in range(0, cand.size + 1):
        got = tuple(O.top_indices(scores, cand, m).tolist())
        best = max(scores[list(c)].sum() for c in itertools.combinations(cand.tolist(), m)) if m else 0.0
        winners = sorted(c for c in itertools.combinations(cand.tolist(), m) if scores[list(c)].sum() == best)
        # maximal total score and, among the maximisers, the lexicographically smallest index set
        assert got == winners[0]


def test_top_indices_all_equal_takes_first():
    assert O.top_indices(np.full(10, 0.5), np.array([1, 3, 4, 8, 9]), 3).tolist() == [1, 3, 4]


def test_select_chunks_ties_and_order():
    sigma = np.array([1.0, 5.0, 5.0, -2.0, 5.0, 0.0])
    assert O.select_chunks(sigma, 2).tolist() == [1, 2]
    assert O.select_chunks(sigma, 4).tolist() == [0, 1, 2, 4]
    assert O.select_chunks(sigma, 6).tolist() == list(range(6))


# ---------------------------------------------------------------- static keep set
def _layout():
    #          0  1  2  3  4  5  6  7  8  9 10 11
    return np.array([0, 1, 1, 0, 1, 1, 1, 0, 1, 0, 0, 0], np.uint8)   # w = 2 -> window {10, 11}


def test_keep_set_three_sets():
    vis = _layout()
    s = np.array([.0, .05, .30, .0, .10, .30, .02, .0, .20, .0, .01, .02])
    # text before window: {0,3,7,9}; budget 2+4+2 -> two best visual; tie .30/.30 -> both; then .20 next
    assert O.static_keep_set(s, vis, 2, 8).tolist() == [0, 2, 3, 5, 7, 9, 10, 11]
    assert O.static_keep_set(s, vis, 2, 9).tolist() == [0, 2, 3, 5, 7, 8, 9, 10, 11]
    # one visual slot and a tie -> lower index wins
    assert O.static_keep_set(s, vis, 2, 7).tolist() == [0, 2, 3, 7, 9, 10, 11]
    # budget covers everything (or more) -> identity
    assert O.static_keep_set(s, vis, 2, 12).tolist() == list(range(12))
    assert O.static_keep_set(s, vis, 2, 50).tolist() == list(range(12))


def test_keep_set_budget_below_text_plus_window():
    vis = _layout()
    s = np.array([.04, .5, .5, .01, .5, .5, .5, .04, .5, .03, .0, .0])
    # budget 4: window + the 2 best historical TEXT tokens (0 and 7 tie at .04 > .03 > .01); no visual
    assert O.static_keep_set(s, vis, 2, 4).tolist() == [0, 7, 10, 11]
    assert O.static_keep_set(s, vis, 2, 3).tolist() == [0, 10, 11]
    assert O.static_keep_set(s, vis, 2, 2).tolist() == [10, 11]
    assert O.static_keep_set(s, vis, 2, 1).tolist() == [11]


@pytest.mark.parametrize("budget", [1, 2, 3, 5, 6, 7, 9, 11, 12, 20])
def test_retained_count_matches_keep_set(budget):
    vis = _layout()
    rng = np.random.default_rng(budget)
    s = rng.random(12)
    kept = O.static_keep_set(s, vis, 2, budget)
    assert kept.size == O.retained_count(12, 2, 4, 6, budget) == min(budget, 12)
    assert (np.diff(kept) > 0).all()


def test_uniform_scores_keep_first_visual():
    wl = make_workload(0, shrink=4)
    C, w = int(wl.seqlens[0]), wl.window
    s = np.full(C, 1.0 / C)
    kept = O.static_keep_set(s, wl.is_visual, w, int(wl.budget[0, 0, 0]))
    vis_hist = np.nonzero(wl.is_visual[: C - w])[0]
    n_txt = (C - w) - vis_hist.size
    m = int(wl.budget[0, 0, 0]) - w - n_txt
    kept_vis = [j for j in kept if j < C - w and wl.is_visual[j]]
    assert kept_vis == vis_hist[:m].tolist()


# ---------------------------------------------------------------- chunks
def test_chunk_means_closed_form_and_ragged_tail():
    # rows 0..9 hold the row index in every column; c = 4 -> means 1.5, 5.5, and the short last chunk 8.5
    k = np.tile(np.arange(10.0)[:, None], (1, 3))
    mu = O.chunk_means(k, 4, "f32")
    np.testing.assert_array_equal(mu, [[1.5] * 3, [5.5] * 3, [8.5] * 3])
    assert O.chunk_rows(np.array([0, 2]), 4, 10).tolist() == [0, 1, 2, 3, 8, 9]


def test_chunk_size_one_reduces_to_token_topk():
    rng = np.random.default_rng(7)
    k = bf16_round(rng.standard_normal((64, 128)).astype(np.float32))
    q = bf16_round(rng.standard_normal((7, 128)).astype(np.float32))
    mu = O.chunk_means(k, 1, "bf16")
    np.testing.assert_array_equal(mu, k.astype(np.float64))          # mean of one row, already bf16
    sigma = O.chunk_scores(q, mu)
    ref = (torch.from_numpy(k).double() @ torch.from_numpy(q).double().sum(0)).numpy()
    np.testing.assert_allclose(sigma, ref, rtol=1e-12)
    assert O.select_chunks(sigma, 5).tolist() == sorted(np.argsort(-ref, kind="stable")[:5].tolist())


def test_n_selected_chunks():
    assert O.n_selected_chunks(128, 32, 64) == 4
    assert O.n_selected_chunks(10, 32, 64) == 1
    assert O.n_selected_chunks(4096, 32, 64) == 64
    assert O.n_selected_chunks(100, 32, 64) == 3


# ---------------------------------------------------------------- rounding
def test_round_to_bf16():
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    x = np.array([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -(1 + 2.0 ** -8), 1 + 2.0 ** -8 + 2.0 ** -40, 0.0, 3.0])
    np.testing.assert_array_equal(O.round_to_dtype(x, "bf16"),
                                  [1.0, 1 + 2.0 ** -6, -1.0, 1 + 2.0 ** -7, 0.0, 3.0])
    # agrees with torch on float32-exact inputs
    rng = np.random.default_rng(8)
    y = rng.standard_normal(10000).astype(np.float32)
    want = torch.from_numpy(y).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_to_dtype(y.astype(np.float64), "bf16"), want)
    np.testing.assert_array_equal(bf16_round(y).astype(np.float64), want)


# ---------------------------------------------------------------- drivers
def _cfg_plan(wl, budget=None):
    cfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                         head_dim=wl.head_dim, window=wl.window, dtype=wl.dtype)
    plan = O.OraclePlan(cu_seqlens=wl.cu_seqlens, head_type=wl.head_type,
                        budget=wl.budget if budget is None else budget, chunk_size=wl.chunk_size)
    return cfg, plan


def test_full_budget_reproduces_full_attention():
    """Budget = whole context on every head: the kept set is the identity, every
    chunk is selected, and the output equals plain softmax attention."""
    wl = make_workload(0, shrink=4, steps=3)
    full = np.full_like(wl.budget, int(wl.seqlens[0]) + 64)
    cfg, plan = _cfg_plan(wl, full)
    cache = O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual)
    C = int(wl.seqlens[0])
    G = cfg.group
    K_all = [[wl.k[0, :, h].astype(np.float64)] for h in range(4)]
    V_all = [[wl.v[0, :, h].astype(np.float64)] for h in range(4)]
    for s in range(wl.steps):
        out, info = O.decode_attn(cache, wl.q_steps[s], wl.k_new[s], wl.v_new[s])
        for h in range(4):
            K_all[h].append(wl.k_new[s][0, 0, h][None].astype(np.float64))
            V_all[h].append(wl.v_new[s][0, 0, h][None].astype(np.float64))
            ref = _sdpa_f64(wl.q_steps[s][0, 0, h * G:(h + 1) * G], np.concatenate(K_all[h]),
                            np.concatenate(V_all[h]), cfg.scale)
            np.testing.assert_allclose(out[0, 0, h * G:(h + 1) * G], ref, rtol=1e-11, atol=1e-13)
    for h in range(4):
        u = cache.units[(0, 0, h)]
        if u.kind == O.STATIC:
            assert u.kept.tolist() == list(range(C))
        else:
            assert info[(0, 0, h)]["sel"].tolist() == list(range(u.mu.shape[0]))
    # and the uncompressed driver agrees with the library on the prompt alone
    outf = O.full_decode_attn(cfg, wl.cu_seqlens, wl.q_steps[0], wl.k, wl.v)
    ref = _sdpa_f64(wl.q_steps[0][0, 0, :G], wl.k[0, :, 0], wl.v[0, :, 0], cfg.scale)
    np.testing.assert_allclose(outf[0, 0, :G], ref, rtol=1e-11, atol=1e-13)


def test_compress_counts_scores_and_planted_tokens():
    wl = make_workload(0)
    cfg, plan = _cfg_plan(wl)
    cache = O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual)
    C, w = int(wl.seqlens[0]), wl.window
    n_txt = int((wl.is_visual[: C - w] == 0).sum())
    for h in range(4):
        u = cache.units[(0, 0, h)]
        if u.kind == O.STATIC:
            assert abs(u.s_w.sum() - 1) < 1e-12
            assert u.kept.size == int(wl.budget[0, 0, h]) == w + n_txt + 154      # retained = budget
            assert set(range(C - w, C)) <= set(u.kept.tolist())                  # window kept
            assert set(np.nonzero(wl.is_visual[: C - w] == 0)[0].tolist()) <= set(u.kept.tolist())
            np.testing.assert_array_equal(u.K, wl.k[0, u.kept, h].astype(np.float64))
            np.testing.assert_array_equal(u.V, wl.v[0, u.kept, h].astype(np.float64))
            planted = wl.planted[(0, 0, h)]
            frac = np.isin(planted, u.kept).mean()
            assert frac > 0.8, frac        # planted keys carry +3 in logit: most of them make the cut
        else:
            assert u.mu.shape == (C // 32, 128) and u.k_sel == 4


def test_decode_dynamic_rows_against_library_attention():
    wl = make_workload(0, shrink=4, steps=2)
    cfg, plan = _cfg_plan(wl)
    cache = O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual)
    out, info = O.decode_attn(cache, wl.q_steps[0], wl.k_new[0], wl.v_new[0])
    G = cfg.group
    for (b, l, h), d in info.items():
        u = cache.units[(b, l, h)]
        assert d["sel"].size == u.k_sel and (np.diff(d["sel"]) > 0).all()
        rows = O.chunk_rows(d["sel"], u.c, u.C)
        assert rows.size == u.k_sel * u.c
        K = np.concatenate([wl.k[l, rows, h], wl.k_new[0][l, b, h][None]]).astype(np.float64)
        V = np.concatenate([wl.v[l, rows, h], wl.v_new[0][l, b, h][None]]).astype(np.float64)
        ref = _sdpa_f64(wl.q_steps[0][l, b, h * G:(h + 1) * G], K, V, cfg.scale)
        np.testing.assert_allclose(out[l, b, h * G:(h + 1) * G], ref, rtol=1e-11, atol=1e-13)


def test_selection_margin_hand_case_and_library_sort():
    # candidates 1, 3, 4, 6 carry 0.5, 0.9, 0.5, 0.7; position 0 holds the largest value but is no candidate
    scores = np.array([9.0, 0.5, 8.0, 0.9, 0.5, 7.0, 0.7])
    cand = np.array([1, 3, 4, 6])
    assert O.selection_margin(scores, cand, 1) == (0.9, 0.7)
    assert O.selection_margin(scores, cand, 2) == (0.7, 0.5)
    assert O.selection_margin(scores, cand, 3) == (0.5, 0.5)          # an exact tie at the cut
    assert O.selection_margin(scores, cand, 0) == (float("inf"), float("-inf"))   # nothing is cut off
    assert O.selection_margin(scores, cand, 4) == (float("inf"), float("-inf"))
    # against a library sort, and against the selection itself: every pick is at least `hi`, every
    # candidate left out at most `lo`
    rng = np.random.default_rng(11)
    for _ in range(50):
        n = int(rng.integers(2, 40))
        sc = rng.integers(0, 6, size=n).astype(np.float64)            # many ties
        cand = np.sort(rng.choice(n, size=int(rng.integers(1, n + 1)), replace=False))
        m = int(rng.integers(1, cand.size + 1))
        hi, lo = O.selection_margin(sc, cand, m)
        if m == cand.size:
            assert (hi, lo) == (float("inf"), float("-inf"))
            continue
        desc = sorted(sc[cand].tolist(), reverse=True)
        assert (hi, lo) == (desc[m - 1], desc[m])
        picked = O.top_indices(sc, cand, m)
        rest = np.setdiff1d(cand, picked)
        assert sc[picked].min() == hi and sc[rest].max() == lo


def test_keep_override_and_sel_override_attend_exactly_the_given_rows():
    """The two hooks the GPU tests use inside a tie band: the oracle must then attend the rows it is
    given, nothing else -- checked with library softmax attention over those rows."""
    wl = make_workload(0, shrink=4, steps=2)
    cfg, plan = _cfg_plan(wl)
    G = cfg.group
    C = int(wl.seqlens[0])
    plain = O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual)
    s_key = next(key for key, u in plain.units.items() if u.kind == O.STATIC)
    d_key = next(key for key, u in plain.units.items() if u.kind == O.DYNAMIC)
    # a keep set of the right size that the scores would never produce: every third position from the start
    n_keep = plain.units[s_key].kept.size
    forced_keep = np.arange(n_keep) * 3 % C
    forced_keep = np.sort(np.unique(forced_keep))
    assert not np.array_equal(forced_keep, plain.units[s_key].kept)
    cache = O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual, keep_override={s_key: forced_keep})
    u = cache.units[s_key]
    np.testing.assert_array_equal(u.kept, forced_keep)
    np.testing.assert_array_equal(u.K, wl.k[0, forced_keep, s_key[2]].astype(np.float64))
    np.testing.assert_array_equal(u.V, wl.v[0, forced_keep, s_key[2]].astype(np.float64))
    np.testing.assert_array_equal(u.s_w, plain.units[s_key].s_w)       # scores are not touched by the hook
    for key, other in cache.units.items():                              # nor is any unit that was not listed
        if key != s_key and other.kind == O.STATIC:
            np.testing.assert_array_equal(other.kept, plain.units[key].kept)
    # forced chunk picks: the two last chunks, which random queries do not single out
    ud = cache.units[d_key]
    n_c = ud.mu.shape[0]
    forced_sel = np.arange(n_c - ud.k_sel, n_c)
    _, info0 = O.decode_attn(O.compress(cfg, plan, wl.q_window, wl.k, wl.v, wl.is_visual),
                             wl.q_steps[0], wl.k_new[0], wl.v_new[0])
    assert not np.array_equal(info0[d_key]["sel"], forced_sel)
    out, info = O.decode_attn(cache, wl.q_steps[0], wl.k_new[0], wl.v_new[0], sel_override={d_key: forced_sel})
    np.testing.assert_array_equal(info[d_key]["sel"], forced_sel)
    np.testing.assert_array_equal(info[d_key]["sigma"], info0[d_key]["sigma"])     # scores untouched
    b, l, h = d_key
    rows = np.concatenate([np.arange(ci * ud.c, min((ci + 1) * ud.c, C)) for ci in forced_sel])
    K = np.concatenate([wl.k[l, rows, h], wl.k_new[0][l, b, h][None]]).astype(np.float64)
    V = np.concatenate([wl.v[l, rows, h], wl.v_new[0][l, b, h][None]]).astype(np.float64)
    np.testing.assert_allclose(out[l, b, h * G:(h + 1) * G], _sdpa_f64(wl.q_steps[0][l, b, h * G:(h + 1) * G], K, V, cfg.scale),
                               rtol=1e-11, atol=1e-13)
    # the static unit with the forced keep set attends those rows + the new token
    b, l, h = s_key
    K = np.concatenate([wl.k[l, forced_keep, h], wl.k_new[0][l, b, h][None]]).astype(np.float64)
    V = np.concatenate([wl.v[l, forced_keep, h], wl.v_new[0][l, b, h][None]]).astype(np.float64)
    np.testing.assert_allclose(out[l, b, h * G:(h + 1) * G], _sdpa_f64(wl.q_steps[0][l, b, h * G:(h + 1) * G], K, V, cfg.scale),
                               rtol=1e-11, atol=1e-13)
    # units that were not listed decide for themselves
    for key, dd in info.items():
        if key != d_key:
            np.testing.assert_array_equal(dd["sel"], info0[key]["sel"])


# ---------------------------------------------------------------- paper arithmetic
def _golden():
    import os
    vals = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_kv_footprint.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                key, val = line.split("=")
                vals[key.strip()] = float(val)
    return vals


def test_paper_byte_model():
    g = _golden()
    per_token_72b = 80 * 8 * 128 * 2 * 2          # layers x KV heads x head_dim x (K,V) x 2 bytes
    assert round(per_token_72b * g["intro_72b_tokens_images"] / 1e9) == g["intro_72b_gb_images"]
    assert round(per_token_72b * g["intro_72b_tokens_video"] / 1e9) == g["intro_72b_gb_video"]
    assert round(g["table3_full_gb"] / g["table3_b10_gb"], 1) == g["claimed_memory_ratio"]
    assert round(g["table3_full_ms"] / g["table3_b10_ms"], 2) == g["claimed_decode_speedup"]


# ---------------------------------------------------------------- head classification (Section 3.1)
def test_sparsity_score_closed_forms():
    rng = np.random.default_rng(5)
    k = rng.standard_normal((40, 8))
    pos = np.arange(5)
    # zero queries: every row is uniform, its k largest entries hold k/C of the mass
    assert abs(O.text_sparsity_score(np.zeros((2, 5, 8)), k, pos, 0.3, 4) - 4 / 40) < 1e-15
    # identical keys: uniform again, whatever the queries
    assert abs(O.text_sparsity_score(rng.standard_normal((3, 5, 8)), np.ones((40, 8)), pos, 0.3, 7) - 7 / 40) < 1e-15
    # k = C keeps everything
    assert abs(O.text_sparsity_score(rng.standard_normal((2, 5, 8)), k, pos, 0.3, 40) - 1.0) < 1e-14
    # one key far above the rest: nearly all mass in the top-1
    kk = np.zeros((40, 1)); kk[17] = 60.0
    assert abs(O.text_sparsity_score(np.ones((1, 3, 1)), kk, np.arange(3), 1.0, 1) - 1.0) < 1e-15
    # the same key only ln(39) above 39 zeros: half of the mass
    kk[17] = math.log(39.0)
    assert abs(O.text_sparsity_score(np.ones((1, 3, 1)), kk, np.arange(3), 1.0, 1) - 0.5) < 1e-15


def test_sparsity_score_hand_worked_rows():
    # d = 1, q = 1, keys ln(1..4): row probabilities 1/10, 2/10, 3/10, 4/10; top-2 sum 7/10
    k = np.log(np.array([[1.0], [2.0], [3.0], [4.0]]))
    assert abs(O.text_sparsity_score(np.ones((1, 1, 1)), k, np.array([3]), 1.0, 2) - 0.7) < 1e-15
    # second row with q = 2: weights 1, 4, 9, 16 over 30; top-2 sum 25/30; mean of the two rows
    q = np.array([[[1.0], [2.0]]])
    assert abs(O.text_sparsity_score(q, k, np.array([2, 3]), 1.0, 2) - 0.5 * (0.7 + 25 / 30)) < 1e-15
    # causal: the token at position 1 sees keys 0..1 only: weights 1/3, 2/3 -> top-2 = 1, top-1 = 2/3
    assert abs(O.text_sparsity_score(np.ones((1, 1, 1)), k, np.array([1]), 1.0, 1, causal=True) - 2 / 3) < 1e-15
    assert abs(O.text_sparsity_score(np.ones((1, 1, 1)), k, np.array([0]), 1.0, 1, causal=True) - 1.0) < 1e-15


def test_sparsity_score_against_sorted_library_softmax():
    rng = np.random.default_rng(6)
    G, T, C, d = 3, 11, 97, 16
    q, k = rng.standard_normal((G, T, d)), rng.standard_normal((C, d))
    pos = np.sort(rng.choice(C, T, replace=False))
    for causal in (False, True):
        want = 0.0
        for g in range(G):
            for t in range(T):
                lg = (k @ q[g, t]) * 0.7
                if causal:
                    lg = lg[: pos[t] + 1]
                p = np.sort(scipy.special.softmax(lg))[::-1]
                want += p[:9].sum()
        got = O.text_sparsity_score(q, k, pos, 0.7, 9, causal=causal)
        assert abs(got - want / (G * T)) < 1e-13
    # grouped heads: the score is the mean of the single-head scores
    singles = [O.text_sparsity_score(q[g:g + 1], k, pos, 0.7, 9) for g in range(G)]
    assert abs(O.text_sparsity_score(q, k, pos, 0.7, 9) - np.mean(singles)) < 1e-14
    # key order does not matter without the mask; more focus positions never lower the score
    perm = rng.permutation(C)
    assert abs(O.text_sparsity_score(q, k[perm], pos, 0.7, 9) - O.text_sparsity_score(q, k, pos, 0.7, 9)) < 1e-13
    vals = [O.text_sparsity_score(q, k, pos, 0.7, kt) for kt in (1, 5, 20, 97)]
    assert all(a < b for a, b in zip(vals, vals[1:])) and all(v >= kt / C - 1e-15 for v, kt in zip(vals, (1, 5, 20, 97)))


def test_focus_count_and_threshold():
    assert O.focus_count(8192) == 410 and O.focus_count(2048) == 103 and O.focus_count(10) == 1 and O.focus_count(40, 0.5) == 20
    types = O.classify_heads(np.array([0.95, 0.9, 0.8999]), 0.9)
    assert types.tolist() == [O.STATIC, O.STATIC, O.DYNAMIC]


def test_head_scores_driver_matches_unit_calls():
    wl = make_workload(0, n_layers=1, shrink=8, steps=1)
    cfg = O.OracleConfig(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128, window=wl.window,
                         dtype=wl.dtype)
    rng = np.random.default_rng(3)
    qp = rng.standard_normal((1, wl.total_tokens, wl.n_q_heads, 128))
    sc = O.head_scores(cfg, wl.cu_seqlens, qp, wl.k, wl.is_visual)
    G = wl.n_q_heads // wl.n_kv_heads
    pos = np.nonzero(wl.is_visual == 0)[0]
    h = 2
    qt = np.stack([qp[0, pos, h * G + g] for g in range(G)])
    want = O.text_sparsity_score(qt, wl.k[0, :, h], pos, cfg.scale, O.focus_count(wl.total_tokens))
    assert sc.shape == (1, 1, wl.n_kv_heads) and abs(sc[0, 0, h] - want) < 1e-15


# ---------------------------------------------------------------- budget allocation (Section 3.2)
def test_type_level_budget_split():
    for b_total, ns, nd, r in [(1000, 3, 5, 0.75), (22932, 56, 56, 0.75), (999, 1, 7, 1.0), (500, 4, 0, 0.75), (64, 0, 4, 0.5)]:
        bs, bd = O.type_level_budgets(b_total, ns, nd, r)
        assert bs + bd == b_total and bs >= 0 and bd >= 0
        if nd:
            exact = r * b_total / (ns + nd) * nd
            assert exact - 1e-9 <= bd < exact + 1
    # r = 1: the dynamic heads get their uniform share
    assert O.type_level_budgets(1200, 2, 4, 1.0) == (400, 800)
    # r above the stated bound is clipped: nothing is left over-committed
    assert O.type_level_budgets(100, 1, 1, 5.0) == (0, 100)


def test_static_head_budgets_invariants():
    rng = np.random.default_rng(8)
    sc = rng.uniform(0.9, 1.0, 17)
    for alpha in (0.0, 0.3, 1.0):
        b = O.static_head_budgets(5000, sc, alpha)
        exact = alpha * 5000 / 17 + (1 - alpha) * 5000 * sc / sc.sum()
        assert np.all(b >= exact - 1e-9) and np.all(b < exact + 1)          # each is a ceiling
        assert 5000 <= b.sum() < 5000 + 17                                   # total exceeds B_stat by < N_stat
    assert np.all(O.static_head_budgets(5000, sc, 1.0) == math.ceil(5000 / 17))           # base budget only
    assert np.all(O.static_head_budgets(340, np.full(17, 0.93), 0.4) == 20)              # equal scores: uniform
    b = O.static_head_budgets(1000, np.array([1.0, 3.0]), 0.0)                            # proportional only
    assert b.tolist() == [250, 750]


def test_dynamic_budget_padding():
    # 10 % of 2048 tokens at r = 0.75 is 153.6 per head: nearest power of two is 128 (four chunks of 32)
    assert O.dynamic_head_budget(round(153.6 * 10), 10) == 128
    assert O.dynamic_head_budget(96 * 3, 3) == 128          # tie between 64 and 128 goes up
    assert O.dynamic_head_budget(95 * 3, 3) == 64
    assert O.dynamic_head_budget(300, 3, pad_pow2=False) == 100
    assert O.dynamic_head_budget(0, 0) == 0


def test_sparsity_score_gaussian_logits_closed_form():
    """Logits that are i.i.d. N(0,1): the top 5 % of the positions carry 1 - Phi(z_0.95 - 1) = 0.2595 of the
    softmax mass in the limit of many keys (the mass of e^x above the 95th percentile of a standard normal)."""
    from scipy.stats import norm
    rng = np.random.default_rng(12)
    C, d = 40000, 16
    q = np.zeros((1, 6, d)); q[0, :, 0] = 1.0                      # unit queries: logit = first key coordinate
    k = rng.standard_normal((C, d))
    got = O.text_sparsity_score(q, k, np.arange(6), 1.0, O.focus_count(C))
    want = 1.0 - norm.cdf(norm.ppf(0.95) - 1.0)
    assert abs(want - 0.2595) < 1e-3 and abs(got - want) < 0.01


# ---------------------------------------------------------------- chunk scoring, other reading for grouped heads
def test_chunk_scores_max_over_group_against_hand_values_and_the_sum_reading():
    """Two query heads pointing in opposite directions cancel in the summed query, so the sum
    reading scores every chunk 0 and picks the lowest ids; the max reading ranks chunks by
    |component|.  Values worked by hand."""
    mu = np.array([[1.0, 0.0], [-3.0, 0.0], [0.5, 2.0], [0.0, -1.0]])
    q = np.array([[1.0, 0.0], [-1.0, 0.0]])
    np.testing.assert_array_equal(O.chunk_scores(q, mu, "sum"), [0.0, 0.0, 0.0, 0.0])
    np.testing.assert_array_equal(O.chunk_scores(q, mu, "max"), [1.0, 3.0, 0.5, 0.0])
    assert O.select_chunks(O.chunk_scores(q, mu, "sum"), 2).tolist() == [0, 1]
    assert O.select_chunks(O.chunk_scores(q, mu, "max"), 2).tolist() == [0, 1]
    assert O.select_chunks(O.chunk_scores(q, mu, "sum"), 1).tolist() == [0]
    assert O.select_chunks(O.chunk_scores(q, mu, "max"), 1).tolist() == [1]
    # one query head: the two readings are the same thing
    rng = np.random.default_rng(5)
    m = rng.standard_normal((37, 16))
    q1 = rng.standard_normal((1, 16))
    np.testing.assert_array_equal(O.chunk_scores(q1, m, "max"), O.chunk_scores(q1, m, "sum"))
    # G copies of one head: max = that head's score, sum = G times it
    q3 = np.repeat(q1, 3, axis=0)
    np.testing.assert_allclose(O.chunk_scores(q3, m, "max"), O.chunk_scores(q1, m, "sum"), rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(O.chunk_scores(q3, m, "sum"), 3 * O.chunk_scores(q1, m, "sum"), rtol=1e-12, atol=1e-14)
    # brute force, and max >= mean of the heads' scores
    q5 = rng.standard_normal((5, 16))
    brute = np.array([max(float(np.dot(q5[g], m[c])) for g in range(5)) for c in range(37)])
    np.testing.assert_allclose(O.chunk_scores(q5, m, "max"), brute, rtol=1e-14)
    assert np.all(O.chunk_scores(q5, m, "max") >= O.chunk_scores(q5, m, "sum") / 5 - 1e-12)
    with pytest.raises(ValueError):
        O.chunk_scores(q5, m, "mean")


# ---------------------------------------------------------------- cumulative focus count (Section 2.1, Eq. 1)
def test_cumulative_focus_hand_case_and_invariants():
    # keys are the unit vectors of R^3 and their negatives; a query picks the keys by its components
    k = np.array([[1.0, 0, 0], [0, 1.0, 0], [0, 0, 1.0], [-1.0, 0, 0], [0, -1.0, 0]])
    q = np.array([[3.0, 2.0, 1.0],     # logits 3, 2, 1, -3, -2 -> top-2 = {0, 1}
                  [-1.0, 5.0, 4.0],    # logits -1, 5, 4, 1, -5 -> top-2 = {1, 2}
                  [0.0, 0.0, 0.0]])    # all equal -> the two lowest positions {0, 1}
    np.testing.assert_array_equal(O.cumulative_focus(q, k, 1.0, 2), [2, 3, 1, 0, 0])
    np.testing.assert_array_equal(O.cumulative_focus(q, k, 1.0, 5), [3] * 5)          # k = C: every token, every step
    # k = 1 is the histogram of the most attended token
    rng = np.random.default_rng(21)
    kk = rng.standard_normal((50, 16))
    qq = rng.standard_normal((200, 16))
    F1 = O.cumulative_focus(qq, kk, 0.25, 1)
    np.testing.assert_array_equal(F1, np.bincount((qq @ kk.T).argmax(axis=1), minlength=50))
    # softmax is increasing, so a library top-k on the logits names the same tokens (distinct values)
    F7 = O.cumulative_focus(qq, kk, 0.25, 7)
    idx = torch.topk(torch.from_numpy(qq @ kk.T), 7, dim=1).indices.numpy()
    np.testing.assert_array_equal(F7, np.bincount(idx.ravel(), minlength=50))
    assert F7.sum() == 200 * 7 and F7.max() <= 200
    # a head that asks the same question at every step focuses on the same tokens every time
    Fs = O.cumulative_focus(np.repeat(qq[:1], 30, axis=0), kk, 0.25, 4)
    assert sorted(set(Fs.tolist())) == [0, 30] and (Fs == 30).sum() == 4
    # the scale does not change the ranking
    np.testing.assert_array_equal(O.cumulative_focus(qq, kk, 1.0, 7), F7)


# ---------------------------------------------------------------- generated tokens in the chunk index (variant)
def _indexed_cfg_plan(wl, budget=None, chunk=None):
    cfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                         head_dim=wl.head_dim, window=wl.window, dtype=wl.dtype, index_generated=True)
    plan = O.OraclePlan(cu_seqlens=wl.cu_seqlens, head_type=wl.head_type,
                        budget=wl.budget if budget is None else budget,
                        chunk_size=wl.chunk_size if chunk is None else chunk)
    return cfg, plan


def test_indexed_generation_equals_the_plain_reading_until_a_chunk_is_complete():
    """With fewer generated tokens than one chunk nothing is indexed yet: same picks, same outputs."""
    wl = make_workload(0, shrink=4, steps=6)                     # chunk 32 > 6 steps
    plain = O.compress(*_cfg_plan(wl), wl.q_window, wl.k, wl.v, wl.is_visual)
    indexed = O.compress(*_indexed_cfg_plan(wl), wl.q_window, wl.k, wl.v, wl.is_visual)
    for s in range(wl.steps):
        a, ia = O.decode_attn(plain, wl.q_steps[s], wl.k_new[s], wl.v_new[s])
        b, ib = O.decode_attn(indexed, wl.q_steps[s], wl.k_new[s], wl.v_new[s])
        np.testing.assert_array_equal(a, b)
        for key in ia:
            np.testing.assert_array_equal(ia[key]["sel"], ib[key]["sel"])


def test_indexed_generation_with_room_for_every_chunk_is_full_attention():
    """A budget that takes every chunk, the generated ones included, must reproduce plain softmax
    attention over the prompt and all generated tokens at every step (library check), while the
    plain reading with the same budget does so too -- the two differ only when chunks are left out."""
    wl = make_workload(0, shrink=4, steps=20)
    chunk = np.full_like(wl.chunk_size, 4)                       # 20 steps complete five chunks
    full = np.full_like(wl.budget, int(wl.seqlens[0]) + 4096)
    cache = O.compress(*_indexed_cfg_plan(wl, full, chunk), wl.q_window, wl.k, wl.v, wl.is_visual)
    G = cache.cfg.group
    dyn = [h for h in range(4) if cache.units[(0, 0, h)].kind == O.DYNAMIC]
    assert dyn
    Ks = {h: [wl.k[0, :, h].astype(np.float64)] for h in dyn}
    Vs = {h: [wl.v[0, :, h].astype(np.float64)] for h in dyn}
    for s in range(wl.steps):
        out, info = O.decode_attn(cache, wl.q_steps[s], wl.k_new[s], wl.v_new[s])
        for h in dyn:
            Ks[h].append(wl.k_new[s][0, 0, h][None].astype(np.float64))
            Vs[h].append(wl.v_new[s][0, 0, h][None].astype(np.float64))
            ref = _sdpa_f64(wl.q_steps[s][0, 0, h * G:(h + 1) * G], np.concatenate(Ks[h]), np.concatenate(Vs[h]),
                            cache.cfg.scale)
            np.testing.assert_allclose(out[0, 0, h * G:(h + 1) * G], ref, rtol=1e-11, atol=1e-13)
            n_c = cache.units[(0, 0, h)].mu.shape[0]
            assert info[(0, 0, h)]["sel"].tolist() == list(range(n_c + s // 4))      # s tokens before this step


def test_indexed_generation_retrieves_a_generated_chunk_and_drops_the_others():
    """One dynamic head, chunk 4, one chunk per step.  The generated keys of steps 0-3 point along e0,
    those of steps 4-7 along e1, the prompt keys are small.  A query along e0 at step 9 must pick the
    first generated chunk (id n_c), attend its four rows, the incomplete rest (token 8) and the new
    token -- and nothing of the second generated chunk."""
    rng = np.random.default_rng(2)
    C, d, c = 16, 8, 4
    cfg = O.OracleConfig(n_layers=1, n_q_heads=1, n_kv_heads=1, head_dim=d, window=4, dtype="f32",
                         index_generated=True)
    plan = O.OraclePlan(cu_seqlens=np.array([0, C], np.int32), head_type=np.array([[[O.DYNAMIC]]], np.uint8),
                        budget=np.array([[[c]]], np.int32), chunk_size=np.array([c], np.int32))
    k = (0.01 * rng.standard_normal((1, C, 1, d))).astype(np.float32)
    v = rng.standard_normal((1, C, 1, d)).astype(np.float32)
    qw = rng.standard_normal((1, 1, 4, 1, d)).astype(np.float32)
    cache = O.compress(cfg, plan, qw, k, v, np.zeros(C, np.uint8))
    u = cache.units[(0, 0, 0)]
    assert u.k_sel == 1 and u.mu.shape[0] == 4
    e = np.eye(d, dtype=np.float32)
    kn = [3 * e[0] if s < 4 else 3 * e[1] if s < 8 else 0.01 * e[2] for s in range(10)]
    vn = [np.full(d, float(s), np.float32) for s in range(10)]
    q = (5 * e[0])[None, None, None, :]
    for s in range(10):
        out, info = O.decode_attn(cache, q, kn[s][None, None, None, :], vn[s][None, None, None, :])
    assert info[(0, 0, 0)]["sel"].tolist() == [4]                 # the first generated chunk
    assert len(u.mu_gen) == 2
    np.testing.assert_allclose(u.mu_gen[0], 3 * e[0], rtol=1e-6)
    rows_k = np.stack(kn[0:4] + kn[8:10]).astype(np.float64)
    rows_v = np.stack(vn[0:4] + vn[8:10]).astype(np.float64)
    ref = _sdpa_f64(q[0, 0], rows_k, rows_v, cfg.scale)
    np.testing.assert_allclose(out[0, 0], ref, rtol=1e-12)
    assert abs(out[0, 0, 0, 0] - 1.5) < 0.05                      # mostly the values 0..3 of the retrieved chunk
