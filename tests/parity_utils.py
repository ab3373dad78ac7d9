"""Shared machinery of the GPU parity tests: runs a workload through libhkv and through the
CPU oracle and compares them unit by unit.

Comparison rules
  * integer results (kept positions, chunk picks, compacted rows) must be bit-exact whenever
    both sides decide on the same values:
      - stage-exact: the oracle's selection routine applied to the device's own fp32 scores must
        reproduce the device's choice exactly, ties included;
      - end-to-end: against the oracle's double-precision scores the sets must be equal unless
        the cut falls inside a tie band (scores within TAU of the threshold), in which case the
        two sets may differ only by tokens inside that band.
  * floating-point results: s_w within SCORE_RTOL of the oracle; attention outputs within
    OUT_TOL[dtype] relative (max-norm per head vector).
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np
import torch

from oracle import hybridkv_oracle as O
from paper_2604_05887_amd import binding as B
from paper_2604_05887_amd import runner

TAU = 1e-5          # relative half-width of the tie band around a selection threshold
SCORE_RTOL = 1e-5   # fp32 MFMA accumulation + exp2 + fp32 column sums vs double
OUT_TOL = {"f32": 1e-5, "bf16": 2e-2}


def oracle_setup(wl, budget=None, head_type=None, causal=False, chunk_score_group="sum", index_generated=False):
    cfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                         head_dim=wl.head_dim, window=wl.window, dtype=wl.dtype, score_causal=causal,
                         chunk_score_group=chunk_score_group, index_generated=index_generated)
    plan = O.OraclePlan(cu_seqlens=wl.cu_seqlens, head_type=wl.head_type if head_type is None else head_type,
                        budget=wl.budget if budget is None else budget, chunk_size=wl.chunk_size)
    return cfg, plan


def assert_summaries_equal(mu_gpu: np.ndarray, mu_ref: np.ndarray, dtype: str, what) -> int:
    """Chunk summaries are formed exactly on the device (double-precision sum and divide, one rounding to
    the cache's type), so they must equal the oracle's.  bf16: bit for bit, always (sums of bf16 values are
    exact in double precision on both sides).  fp32: the two double-precision sums run in different orders
    and can differ in their last bit, which moves the rounded fp32 value only when the mean sits within
    ~1e-16 of a rounding boundary; at most two such elements per unit are tolerated, each by one fp32 ulp.
    Returns the number of unequal elements."""
    assert mu_gpu.shape == mu_ref.shape, (what, mu_gpu.shape, mu_ref.shape)
    bad = mu_gpu != mu_ref
    n_bad = int(bad.sum())
    if dtype == "bf16":
        assert n_bad == 0, f"chunk summaries of {what} differ from the oracle's in {n_bad} elements"
    elif n_bad:
        ulp = np.spacing(np.abs(mu_ref[bad]).astype(np.float32)).astype(np.float64)
        assert n_bad <= 2 and np.all(np.abs(mu_gpu[bad] - mu_ref[bad]) <= ulp), f"chunk summaries of {what} off"
    return n_bad


def candidates_of(is_visual: np.ndarray, w: int, budget: int):
    """(candidate positions, number to select) under the static keep rule."""
    C = is_visual.size
    hist = np.arange(C - w)
    txt = hist[is_visual[: C - w] == 0]
    vis = hist[is_visual[: C - w] == 1]
    if budget < w:
        return np.zeros(0, np.int64), 0
    m = budget - w - txt.size
    if m < 0:
        return txt, budget - w
    return vis, min(m, vis.size)


def check_banded(got: np.ndarray, want: np.ndarray, scores: np.ndarray, cand: np.ndarray, m: int,
                 tau_abs_fn) -> bool:
    """got/want: ascending index sets.  Returns True when they are identical; otherwise asserts that
    they differ only inside the tie band and returns False."""
    assert got.size == want.size, (got.size, want.size)
    if np.array_equal(got, want):
        return True
    hi, lo = O.selection_margin(scores, cand, m)
    band = tau_abs_fn(hi)
    diff = np.setxor1d(got, want)
    s = np.asarray(scores, dtype=np.float64)[diff]
    assert np.all(np.abs(s - hi) <= band), (
        f"sets differ outside the tie band: thr={hi:.9e} next={lo:.9e} band={band:.3e} "
        f"diff={diff[:8]} scores={s[:8]}")
    return False


def compare_compress(wl, dw, ocache, stats: Dict[str, float]) -> Dict[Tuple[int, int, int], np.ndarray]:
    """Checks every unit after hkv_compress.  Returns the keep sets the oracle must adopt where the
    device's differ inside a tie band (empty when everything matched exactly)."""
    overrides = {}
    w = wl.window
    for (b, l, h), u in ocache.units.items():
        lo, hi = int(wl.cu_seqlens[b]), int(wl.cu_seqlens[b + 1])
        vis = wl.is_visual[lo:hi]
        if u.kind == O.STATIC:
            budget = int(ocache.plan.budget[b, l, h])
            rows, _, _ = dw.cache.unit_info(b, l, h)
            assert rows == u.kept.size == O.retained_count(hi - lo, w, int((vis[:hi - lo - w] == 0).sum()),
                                                           int((vis[:hi - lo - w] == 1).sum()), budget)
            s_gpu = dw.cache.export(B.HKV_X_SCORES, b, l, h)
            kept_gpu = dw.cache.export(B.HKV_X_KEPT_IDX, b, l, h).astype(np.int64)
            # scores
            rel = np.abs(s_gpu.astype(np.float64) - u.s_w) / np.maximum(u.s_w, 1e-300)
            big = u.s_w > 1e-30
            stats["score_rel"] = max(stats.get("score_rel", 0.0), float(rel[big].max()))
            assert rel[big].max() <= SCORE_RTOL, f"s_w off by {rel[big].max():.3e} on unit {(b, l, h)}"
            assert abs(float(s_gpu.astype(np.float64).sum()) - 1.0) < 1e-4
            # stage-exact: the oracle's rule on the device's own fp32 scores
            want_stage = O.static_keep_set(s_gpu, vis, w, budget)
            assert np.array_equal(kept_gpu, want_stage), f"selection not exact on unit {(b, l, h)}"
            # end-to-end with tie band
            cand, m = candidates_of(vis, w, budget)
            same = check_banded(kept_gpu, u.kept, u.s_w, cand, m, lambda thr: TAU * thr)
            if not same:
                overrides[(b, l, h)] = kept_gpu
                stats["banded_units"] = stats.get("banded_units", 0) + 1
            # compacted rows are bit-exact copies, ascending position order
            Kc = dw.cache.export(B.HKV_X_K_ROWS, b, l, h)
            Vc = dw.cache.export(B.HKV_X_V_ROWS, b, l, h)
            assert np.array_equal(Kc[: kept_gpu.size], wl.k[l, lo + kept_gpu, h])
            assert np.array_equal(Vc[: kept_gpu.size], wl.v[l, lo + kept_gpu, h])
        else:
            rows, n_c, k_sel = dw.cache.unit_info(b, l, h)
            k_want = u.k_sel
            if ocache.cfg.index_generated:         # room for the chunks generation can complete
                k_want = min(u.k_cap, u.mu.shape[0] + wl.max_new_tokens // u.c)
            assert (n_c, k_sel) == (u.mu.shape[0], k_want) and rows == k_sel * u.c
            mu_gpu = dw.cache.export(B.HKV_X_CHUNK_MEAN, b, l, h).astype(np.float64)
            stats["mu_unequal"] = stats.get("mu_unequal", 0) + assert_summaries_equal(mu_gpu, u.mu, wl.dtype, (b, l, h))
            Kd = dw.cache.export(B.HKV_X_K_ROWS, b, l, h)
            Vd = dw.cache.export(B.HKV_X_V_ROWS, b, l, h)
            assert np.array_equal(Kd[: hi - lo], wl.k[l, lo:hi, h]) and np.array_equal(Vd[: hi - lo], wl.v[l, lo:hi, h])
    return overrides


def run_decode_and_compare(wl, dw, ocache, n_steps: int, stats: Dict[str, float], layer_ranges=None,
                           append: bool = True, oracle_layers=None, layer_ranges_by_step=None):
    """n_steps decode steps on both sides.  Chunk scores and chunk picks are compared with the oracle's own
    (computed from its own chunk summaries); only where a cut falls inside a tie band does the oracle
    adopt the device's picks for the attention that follows.
    layer_ranges_by_step[s], if given and not None, replaces layer_ranges for step s."""
    L, Bn = wl.n_layers, wl.batch
    tdt = runner.torch_dtype(wl.dtype)
    out = torch.empty((L, Bn, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda:0")
    layer_ranges = layer_ranges or [(0, L)]
    G = wl.group
    indexed = ocache.cfg.index_generated
    for s in range(n_steps):
        q = runner.to_device(wl.q_steps[s], wl.dtype)
        kn = runner.to_device(wl.k_new[s], wl.dtype) if append else None
        vn = runner.to_device(wl.v_new[s], wl.dtype) if append else None
        ranges = layer_ranges
        if layer_ranges_by_step is not None and layer_ranges_by_step[s] is not None:
            ranges = layer_ranges_by_step[s]
        for (lb, le) in ranges:
            dw.cache.decode_attn(q[lb:le], None if kn is None else kn[lb:le], None if vn is None else vn[lb:le],
                                 out[lb:le], layer_begin=lb, layer_end=le)
        torch.cuda.synchronize()
        got = runner.to_host_f32(out).astype(np.float64)
        # chunk picks first: they decide which rows the oracle attends
        sel_over = {}
        for key, u in ocache.units.items():
            if u.kind != O.DYNAMIC or (oracle_layers is not None and key[1] not in oracle_layers):
                continue
            b, l, h = key
            sig_gpu = dw.cache.export(B.HKV_X_CHUNK_SIGMA, b, l, h)
            sel_gpu = dw.cache.export(B.HKV_X_CHUNK_SEL, b, l, h).astype(np.int64)
            k_step = u.k_sel
            mu_ref = u.mu
            if indexed:
                # the step saw the chunks complete before it: those of the prompt and of the tokens generated so
                # far (the oracle formed their summaries when its own earlier steps completed them)
                n_gen = (s if append else 0) // u.c
                n_now = u.mu.shape[0] + n_gen
                k_step = min(u.k_cap, n_now)
                if n_gen:
                    mu_ref = np.concatenate([u.mu, np.stack(u.mu_gen[:n_gen])], axis=0)
                sig_gpu, sel_gpu = sig_gpu[:n_now], sel_gpu[:k_step]
            # stage-exact: the oracle's rule on the device's own fp32 scores
            assert np.array_equal(sel_gpu, O.select_chunks(sig_gpu, k_step)), f"chunk top-k not exact on {key}"
            # end to end: scores and picks against the oracle's own summaries, scores and picks
            qh = wl.q_steps[s][l, b, h * G:(h + 1) * G].astype(np.float64)
            group = ocache.cfg.chunk_score_group
            sig_ref = O.chunk_scores(qh, mu_ref, group)
            q_norm = np.linalg.norm(qh.sum(0)) if group == "sum" else np.linalg.norm(qh, axis=1).max()
            scale = q_norm * np.linalg.norm(mu_ref, axis=1).max()
            err = np.abs(sig_gpu - sig_ref).max() / scale
            stats["sigma_err"] = max(stats.get("sigma_err", 0.0), float(err))
            assert err <= 1e-5, f"chunk scores off by {err:.3e} (relative to |q||mu|) on {key}"
            want = O.select_chunks(sig_ref, k_step)
            same = check_banded(sel_gpu, want, sig_ref, np.arange(sig_ref.size), k_step, lambda thr: 1e-5 * scale)
            stats["chunk_picks_compared"] = stats.get("chunk_picks_compared", 0) + 1
            if not same:
                sel_over[key] = sel_gpu
                stats["banded_chunk_picks"] = stats.get("banded_chunk_picks", 0) + 1
            if indexed:
                stats["generated_chunks_picked"] = stats.get("generated_chunks_picked", 0) + int((sel_gpu >= u.mu.shape[0]).sum())
        ref, _ = O.decode_attn(ocache, wl.q_steps[s], wl.k_new[s] if append else None,
                               wl.v_new[s] if append else None, layers=oracle_layers, sel_override=sel_over)
        if oracle_layers is not None:       # the oracle only ran a sample of layers
            got, ref = got[oracle_layers], ref[oracle_layers]
        err = np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        stats["out_err"] = max(stats.get("out_err", 0.0), float(err.max()))
        assert err.max() <= OUT_TOL[wl.dtype], f"step {s}: output off by {err.max():.3e}"
    if indexed:
        # the summaries of the generated chunks themselves: exact means, equal to the oracle's
        for key, u in ocache.units.items():
            if u.kind != O.DYNAMIC or (oracle_layers is not None and key[1] not in oracle_layers) or not u.mu_gen:
                continue
            n_c = u.mu.shape[0]
            got_mu = dw.cache.export(B.HKV_X_CHUNK_MEAN, *key).astype(np.float64)
            assert got_mu.shape[0] == n_c + len(u.mu_gen)
            assert_summaries_equal(got_mu[n_c:], np.stack(u.mu_gen), wl.dtype, ("generated", key))
            stats["generated_chunks_indexed"] = stats.get("generated_chunks_indexed", 0) + len(u.mu_gen)
    return out


def full_pipeline(wl, budget=None, head_type=None, causal=False, n_steps=None, layer_ranges=None, **setup_kw):
    stats: Dict[str, float] = {}
    dw = runner.setup(wl, budget=budget, head_type=head_type, score_causal=int(causal), **setup_kw)
    ocfg, oplan = oracle_setup(wl, budget, head_type, causal,
                               chunk_score_group="max" if setup_kw.get("chunk_score_group", 0) == 1 else "sum",
                               index_generated=bool(setup_kw.get("index_generated", 0)))
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual)
    if layer_ranges:
        for (lb, le) in layer_ranges:
            dw.cache.compress(dw.q_window[lb:le], dw.k[lb:le], dw.v[lb:le], layer_begin=lb, layer_end=le)
    else:
        dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    overrides = compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, keep_override=overrides)
    run_decode_and_compare(wl, dw, ocache, wl.steps if n_steps is None else n_steps, stats, layer_ranges)
    # tails hold the appended rows in order
    steps = wl.steps if n_steps is None else n_steps
    for (b, l, h), u in ocache.units.items():
        Kr = dw.cache.export(B.HKV_X_K_ROWS, b, l, h)
        base = u.kept.size if u.kind == O.STATIC else u.C
        assert Kr.shape[0] == base + steps
        assert np.array_equal(Kr[base:], wl.k_new[:steps, l, b, h])
    dw.cache.close()
    return stats
