"""GPU parity: libhkv (through the C ABI) against the CPU oracle on the same seeded inputs."""
import os

import numpy as np
import pytest
import torch

from hkv_synth import make_workload
from oracle import hybridkv_oracle as O
from paper_2604_05887_amd import binding as B
from paper_2604_05887_amd import runner

import parity_utils as P

pytestmark = pytest.mark.gpu


def _say(name, stats):
    print(f"\n[{name}] " + " ".join(f"{k}={v:.3g}" for k, v in sorted(stats.items())), flush=True)


def _random_shape_seeds():
    """Seeds 0..9 always; HKV_RANDOM_SHAPE_SEEDS="a-b" adds the seeds a..b-1 for a longer run."""
    extra = os.environ.get("HKV_RANDOM_SHAPE_SEEDS", "")
    seeds = list(range(10))
    if extra:
        lo, hi = (int(x) for x in extra.split("-"))
        seeds += [s for s in range(lo, hi) if s not in seeds]
    return seeds


def _random_shape_scale():
    """HKV_RANDOM_SHAPE_SCALE=n multiplies the drawn visual-token counts (longer prompts: more tiles, longer shares)."""
    return max(1, int(os.environ.get("HKV_RANDOM_SHAPE_SCALE", "1")))


def test_cfg0_fp32_end_to_end():
    """Config 0 at full size: compress + 16 decode steps, every unit, every step."""
    wl = make_workload(0)
    stats = P.full_pipeline(wl)
    _say("cfg0", stats)
    assert stats.get("banded_units", 0) == 0      # the seed has no tie-band hits


def test_cfg1_shape_bf16_three_layers():
    wl = make_workload(1, n_layers=3, shrink=4, steps=5)
    stats = P.full_pipeline(wl)
    _say("cfg1/4 L3", stats)


def test_layer_by_layer_calls_match_one_call():
    """Per-layer compress/decode calls (how a model would drive it) give the same bits as one call."""
    wl = make_workload(1, n_layers=3, shrink=8, steps=3)
    outs = []
    for ranges in ([(0, 3)], [(0, 1), (1, 2), (2, 3)], [(0, 2), (2, 3)]):
        dw = runner.setup(wl)
        for (lb, le) in ranges:
            dw.cache.compress(dw.q_window[lb:le], dw.k[lb:le], dw.v[lb:le], layer_begin=lb, layer_end=le)
        out = torch.empty((3, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        res = []
        for s in range(wl.steps):
            q, kn, vn = (runner.to_device(x[s], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
            for (lb, le) in ranges:
                dw.cache.decode_attn(q[lb:le], kn[lb:le], vn[lb:le], out[lb:le], layer_begin=lb, layer_end=le)
            torch.cuda.synchronize()
            res.append(out.clone())
        outs.append(torch.stack(res))
        dw.cache.close()
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


def test_ragged_batch_both_chunk_sizes_and_short_last_chunk():
    """Config 4 shape, shrunk: 16 ragged sequences, chunk sizes 32 and 64, prompt lengths that are
    not multiples of the chunk size, hierarchical ragged budgets."""
    wl = make_workload(4, n_layers=2, shrink=8, steps=3)
    assert len(set(wl.chunk_size.tolist())) == 2 and any(int(c) % 64 for c in wl.seqlens)
    stats = P.full_pipeline(wl)
    _say("cfg4/8 L2", stats)


def test_literal_total_budgets_hit_text_overflow_rule():
    """Budgets read as a fraction of the whole context are smaller than text + window on these
    shapes: the overflow rule (keep window, then best text tokens) decides the keep set."""
    wl = make_workload(1, n_layers=2, shrink=4, steps=2, budget_rule="literal_total")
    C, w = int(wl.seqlens[0]), wl.window
    n_txt = int((wl.is_visual[: C - w] == 0).sum())
    stat = wl.head_type[0] == 0
    assert (wl.budget[0][stat] < w + n_txt).any()
    stats = P.full_pipeline(wl)
    _say("cfg1/4 literal", stats)


def test_group_of_eight_72b_shape():
    wl = make_workload(3, n_layers=2, shrink=16, steps=2)
    assert wl.group == 8
    stats = P.full_pipeline(wl)
    _say("cfg3/16 L2", stats)


@pytest.mark.parametrize("mix", ["all_static", "all_dynamic"])
def test_degenerate_head_maps(mix):
    wl = make_workload(0, shrink=2, steps=2, head_mix=mix)
    stats = P.full_pipeline(wl)
    _say(mix, stats)


def test_tiny_budgets_and_budget_below_window():
    wl = make_workload(0, shrink=4, steps=2)
    budget = wl.budget.copy()
    budget[0, 0, 0] = 5            # below the window: keep the last 5 positions
    budget[0, 0, 1] = wl.window    # exactly the window
    budget[0, 0, 2] = 1            # dynamic: one chunk
    stats = P.full_pipeline(wl, budget=budget)
    _say("tiny budgets", stats)


def test_causal_window_scoring():
    wl = make_workload(0, shrink=2, steps=1)
    stats = P.full_pipeline(wl, causal=True)
    _say("causal", stats)


def test_full_budget_equals_full_attention_and_full_kernel():
    """Budget = whole context: kept set is the identity, all chunks are picked, and the hybrid
    output, the full-KV kernel and textbook attention agree."""
    wl = make_workload(0, shrink=2, steps=1)
    C = int(wl.seqlens[0])
    budget = np.full_like(wl.budget, C)
    dw = runner.setup(wl, budget=budget)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    out_h = torch.empty((1, 1, wl.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
    q = runner.to_device(wl.q_steps[0], wl.dtype)
    dw.cache.decode_attn(q, None, None, out_h)
    for h in range(4):
        if wl.head_type[0, 0, h] == 0:
            assert np.array_equal(dw.cache.export(B.HKV_X_KEPT_IDX, 0, 0, h), np.arange(C))
        else:
            assert np.array_equal(dw.cache.export(B.HKV_X_CHUNK_SEL, 0, 0, h), np.arange(C // 32))
    ws_bytes = B.hkv_full_workspace_size(dw.cfg, wl.cu_seqlens, 1)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    out_f = torch.empty_like(out_h)
    B.hkv_full_decode_attn(dw.cfg, wl.cu_seqlens, 1, q, dw.k, dw.v, out_f, ws, ws_bytes)
    torch.cuda.synchronize()
    ocfg, _ = P.oracle_setup(wl)
    ref = O.full_decode_attn(ocfg, wl.cu_seqlens, wl.q_steps[0], wl.k, wl.v)
    for got in (out_h, out_f):
        g = runner.to_host_f32(got).astype(np.float64)
        err = np.abs(g - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
        assert err.max() <= 1e-5, err.max()
    dw.cache.close()


def test_full_kv_kernel_ragged_batch_bf16():
    wl = make_workload(4, n_layers=2, shrink=8, steps=1)
    cfg = B.make_config(n_layers=2, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, dtype=B.HKV_BF16,
                        window=wl.window, chunk_size=32)
    q, k, v = (runner.to_device(x, "bf16") for x in (wl.q_steps[0], wl.k, wl.v))
    ws_bytes = B.hkv_full_workspace_size(cfg, wl.cu_seqlens, 2)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    out = torch.empty_like(q)
    B.hkv_full_decode_attn(cfg, wl.cu_seqlens, 2, q, k, v, out, ws, ws_bytes)
    torch.cuda.synchronize()
    ocfg, _ = P.oracle_setup(wl)
    ref = O.full_decode_attn(ocfg, wl.cu_seqlens, wl.q_steps[0], wl.k, wl.v)
    g = runner.to_host_f32(out).astype(np.float64)
    err = np.abs(g - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
    assert err.max() <= 2e-2, err.max()


@pytest.mark.parametrize("seed", _random_shape_seeds())
def test_full_kv_kernel_on_seeded_random_shapes(seed):
    """The comparison kernel against textbook attention: group sizes 1 to 8, one to four ragged sequences of 1 to
    ~6000 rows (single rows, lengths around the tile size and its multiples included), one to three layers, bf16
    and fp32."""
    rng = np.random.default_rng(7000 + seed)
    n_kv, G, batch, L = int(rng.choice([1, 2, 4])), int(rng.integers(1, 9)), int(rng.integers(1, 5)), int(rng.integers(1, 4))
    dtype = "f32" if seed % 3 == 2 else "bf16"
    special = [1, 2, 7, 8, 9, 31, 32, 33, 127, 128, 129, 255, 256, 257, 511, 512, 513, 1023, 1024, 1025, 2048, 4096]
    lens = [int(rng.choice(special)) if rng.integers(0, 2) else int(rng.integers(1, 6000)) for _ in range(batch)]
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    n_q = n_kv * G
    from hkv_synth.workloads import bf16_round
    to_dtype = bf16_round if dtype == "bf16" else (lambda x: x.astype(np.float32))
    q, k, v = (to_dtype(rng.standard_normal(shape)) for shape in
               ((L, batch, n_q, 128), (L, int(cu[-1]), n_kv, 128), (L, int(cu[-1]), n_kv, 128)))
    cfg = B.make_config(n_layers=L, n_q_heads=n_q, n_kv_heads=n_kv, dtype=runner.hkv_dtype(dtype), window=1, chunk_size=32)
    qd, kd, vd = (runner.to_device(x, dtype) for x in (q, k, v))
    ws_bytes = B.hkv_full_workspace_size(cfg, cu, L)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0")
    out = torch.empty_like(qd)
    B.hkv_full_decode_attn(cfg, cu, L, qd, kd, vd, out, ws, ws_bytes)
    torch.cuda.synchronize()
    ocfg = O.OracleConfig(n_layers=L, n_q_heads=n_q, n_kv_heads=n_kv, head_dim=128, window=1, dtype=dtype)
    ref = O.full_decode_attn(ocfg, cu, q.astype(np.float64), k.astype(np.float64), v.astype(np.float64))
    g = runner.to_host_f32(out).astype(np.float64)
    err = (np.abs(g - ref).max(axis=-1) / np.abs(ref).max(axis=-1)).max()
    print(f"\n[full KV, random shape {seed}: G{G} kv{n_kv} L{L} {dtype} rows {lens}] max rel err {err:.2e}", flush=True)
    assert err <= (2e-2 if dtype == "bf16" else 1e-5)


def test_selection_stage_with_planted_ties():
    """Feed the device selection kernels oracle-made scores full of exact ties (quantised values):
    kept positions and chunk picks must equal the oracle's, lowest index first."""
    wl = make_workload(0, shrink=2, steps=1)
    dw = runner.setup(wl)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    rng = np.random.default_rng(5)
    C, w = int(wl.seqlens[0]), wl.window
    for levels in (3, 17, 1):
        for h in range(4):
            if wl.head_type[0, 0, h] == 0:
                s = (rng.integers(0, levels, size=C) / 64.0).astype(np.float32)
                dw.cache.import_(B.HKV_X_SCORES, 0, 0, h, s)
        dw.cache.compress_from_scores(dw.k, dw.v)
        for h in range(4):
            if wl.head_type[0, 0, h] == 0:
                s = dw.cache.export(B.HKV_X_SCORES, 0, 0, h)
                want = O.static_keep_set(s, wl.is_visual, w, int(wl.budget[0, 0, h]))
                got = dw.cache.export(B.HKV_X_KEPT_IDX, 0, 0, h)
                assert np.array_equal(got, want), (levels, h)
                Kc = dw.cache.export(B.HKV_X_K_ROWS, 0, 0, h)
                assert np.array_equal(Kc[: want.size], wl.k[0, want, h])
    for levels in (2, 9, 1):
        for h in range(4):
            if wl.head_type[0, 0, h] == 1:
                n_c = dw.cache.unit_info(0, 0, h)[1]
                sig = (rng.integers(-levels, levels, size=n_c) / 8.0).astype(np.float32)
                sig[rng.integers(0, n_c)] = -0.0
                dw.cache.import_(B.HKV_X_CHUNK_SIGMA, 0, 0, h, sig)
        B.hkv_reselect_chunks(dw.cache.handle, 0, 1)
        for h in range(4):
            if wl.head_type[0, 0, h] == 1:
                sig = dw.cache.export(B.HKV_X_CHUNK_SIGMA, 0, 0, h)
                k_sel = dw.cache.unit_info(0, 0, h)[2]
                assert np.array_equal(dw.cache.export(B.HKV_X_CHUNK_SEL, 0, 0, h), O.select_chunks(sig, k_sel))
    dw.cache.close()


@pytest.mark.parametrize("chunk,n_layers", [(8, 4), (32, 4)])
def test_chunk_selection_with_planted_ties_among_many_chunks(chunk, n_layers):
    """Heads with 1024 (or 256) chunks: the picks from imported scores equal the oracle's for k below, at and above
    the limit of the search that starts from the lanes' maxima (32), for scores that are all different, quantised
    to a few levels (most keys tie at the bound: the radix search takes over), all equal, equal at the cut only,
    negative throughout, and with the largest values crowded into a few lanes."""
    wl = make_workload(1, n_layers=n_layers, steps=1)
    wl.chunk_size[:] = chunk
    dyn = [(l, h) for l in range(wl.n_layers) for h in range(wl.n_kv_heads) if wl.head_type[0, l, h] == O.DYNAMIC]
    ks = [5, 32, 33, 64, 200, 17, 31, 1]
    for i, (l, h) in enumerate(dyn):
        wl.budget[0, l, h] = chunk * ks[i % len(ks)]
    dw = runner.setup(wl)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    rng = np.random.default_rng(11)
    n_c = dw.cache.unit_info(0, dyn[0][0], dyn[0][1])[1]
    assert n_c == int(wl.seqlens[0]) // chunk

    def patterns():
        yield "distinct", rng.standard_normal(n_c).astype(np.float32) * 30
        yield "three levels", (rng.integers(-1, 2, size=n_c) / 4.0).astype(np.float32)
        yield "many levels", (rng.integers(-4000, 4000, size=n_c) / 16.0).astype(np.float32)
        yield "all equal", np.full(n_c, 2.5, np.float32)
        x = rng.standard_normal(n_c).astype(np.float32)
        x[np.argsort(x)[-40:-10]] = np.sort(x)[-40]              # thirty values tie across the 17th to 40th place
        yield "ties at the cut", x
        yield "negative", -np.abs(rng.standard_normal(n_c).astype(np.float32)) - 1.0
        x = rng.standard_normal(n_c).astype(np.float32)
        x[64 * np.arange(n_c // 64) + 3] += 50.0                 # the largest values all sit in one lane's registers
        x[64 * np.arange(n_c // 64) + 40] += 49.0
        yield "crowded lanes", x

    for name, sig in patterns():
        for (l, h) in dyn:
            dw.cache.import_(B.HKV_X_CHUNK_SIGMA, 0, l, h, sig)
        B.hkv_reselect_chunks(dw.cache.handle, 0, wl.n_layers)
        for (l, h) in dyn:
            k_sel = dw.cache.unit_info(0, l, h)[2]
            got = dw.cache.export(B.HKV_X_CHUNK_SEL, 0, l, h)
            assert np.array_equal(got, O.select_chunks(sig, k_sel)), (name, l, h, k_sel)
    dw.cache.close()


def test_tail_capacity_and_rewind():
    wl = make_workload(0, shrink=4, steps=3, max_new_tokens=2)
    dw = runner.setup(wl)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    out = torch.empty((1, 1, wl.n_q_heads, 128), dtype=torch.float32, device="cuda:0")
    q, kn, vn = (runner.to_device(x[0], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
    dw.cache.decode_attn(q, kn, vn, out)
    first = out.clone()
    dw.cache.decode_attn(q, kn, vn, out)
    with pytest.raises(B.HkvError) as ei:
        dw.cache.decode_attn(q, kn, vn, out)
    assert ei.value.status == B.HKV_ENOSPACE
    dw.cache.rewind()
    dw.cache.decode_attn(q, kn, vn, out)
    torch.cuda.synchronize()
    assert torch.equal(out, first)      # same state, same bits: the path is deterministic
    dw.cache.close()


def test_cfg1_full_size_sampled_units():
    """Config 1 at full size (28 layers, 8192 tokens) in the launch configuration bench.py times:
    one hkv_compress and one hkv_decode_attn call over all layers.  The oracle runs on a seeded
    sample of layers (all units of those layers, every step)."""
    wl = make_workload(1, steps=4)
    rng = np.random.default_rng(11)
    layers = sorted(rng.choice(wl.n_layers, size=3, replace=False).tolist())
    print(f"\n[cfg1 full] sampled layers {layers}", flush=True)
    dw = runner.setup(wl)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl)
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers)
    _say("cfg1 full", stats)
    dw.cache.close()


@pytest.mark.parametrize("chunk,k_chunks,shrink", [(8, 24, 2), (16, 300, 1), (8, 40, 1), (8, 700, 1)])
def test_many_small_chunks_radix_path(chunk, k_chunks, shrink):
    """Small chunks (the paper's example is 8 tokens) give more than 256 chunks per head: up to 2048 the
    chunk top-k keeps the keys in each wave's registers (8 or 16 per lane here: 512 and 1024 chunks; 32 per
    lane in the next test) and selects by radix over a per-wave histogram; k larger than 256 and k of most
    chunks as well.
    Every decode shape that repeats or owns the selection runs it."""
    wl = make_workload(1, n_layers=2, shrink=shrink, steps=3)
    wl.chunk_size[:] = chunk
    dyn = wl.head_type == 1
    wl.budget[dyn] = chunk * k_chunks
    n_c = -(-int(wl.seqlens[0]) // chunk)
    assert n_c > 256
    for mode in (0, 1, 2, 4, 5):
        stats = P.full_pipeline(wl, decode_dynamic=mode)
        _say(f"chunk {chunk} k {k_chunks} n_c {n_c} mode {mode}", stats)


@pytest.mark.parametrize("n_visual,expect", [(15360, "registers"), (19456, "block")])
def test_chunk_counts_around_the_register_limit(n_visual, expect):
    """8-token chunks on a 16k-token prompt give 2048 chunks per head, the most the register-resident chunk
    top-k takes (32 keys per lane); on a 20k-token prompt 2560, which runs as block-wide radix passes over the
    scores in shared memory."""
    from hkv_synth import workloads as W
    base = dict(W.CONFIGS[1])
    base.update(name=f"chunks_{n_visual}", n_layers=1, n_visual=[n_visual], n_text=[1024], block=n_visual, steps=2, chunk=[8],
                k_chunks=300)
    W.CONFIGS[96] = base
    try:
        wl = make_workload(96, seed=2)
    finally:
        del W.CONFIGS[96]
    n_c = -(-int(wl.seqlens[0]) // 8)
    assert (n_c == 2048) if expect == "registers" else (n_c > 2048)
    for mode in (3, 5):
        stats = P.full_pipeline(wl, decode_dynamic=mode)
        _say(f"n_c {n_c} mode {mode}", stats)


@pytest.mark.parametrize("n_q,n_kv,window,dtype", [(4, 4, 48, "bf16"), (8, 4, 32, "bf16"), (6, 2, 16, "bf16"),
                                                   (8, 2, 64, "bf16"), (10, 2, 8, "bf16"), (12, 2, 20, "bf16"),
                                                   (8, 2, 16, "f32"), (3, 3, 10, "f32"), (16, 2, 24, "f32")])
def test_other_group_sizes_and_windows(n_q, n_kv, window, dtype):
    """Group sizes 1 to 6 and windows that are not 32 (G * w not a multiple of 32 included, and G * w at its
    limit of 256), in the three single-launch decode shapes."""
    from hkv_synth import workloads as W
    base = dict(W.CONFIGS[1])
    base.update(name=f"g{n_q // n_kv}_w{window}_{dtype}", n_layers=2, n_q_heads=n_q, n_kv_heads=n_kv, window=window,
                n_visual=[1200], n_text=[300], block=1200, steps=2, dtype=dtype)
    W.CONFIGS[99] = base
    try:
        wl = make_workload(99, seed=3)
    finally:
        del W.CONFIGS[99]
    for mode in (1, 3, 4) if dtype == "bf16" else (1, 2, 3):
        stats = P.full_pipeline(wl, decode_dynamic=mode)
        _say(f"G{n_q // n_kv} w{window} {dtype} mode {mode}", stats)


def _sep_that_fits(n_visual, n_text, block, sep, window):
    """The drawn separator length, or 0 where the text between the blocks would not leave the window and 16
    more tokens of some prompt outside them."""
    for nv, nt in zip(n_visual, n_text):
        if sep * (max(1, -(-nv // block)) - 1) > nt - window - 16:
            return 0
    return sep


@pytest.mark.parametrize("seed", _random_shape_seeds())
def test_seeded_random_shapes_in_every_decode_shape(seed):
    """Ten shapes drawn from a seeded generator: group sizes 1 to 8, windows from 4 up to the limit of
    G * w = 256, chunk sizes 8 to 128, one to three ragged sequences, prompts of 300 to 2600 tokens, budgets of
    4 % to 45 %, static fractions from none to all, one to three layers, bf16 and fp32; each runs the whole
    chain compress -> decode steps against the oracle in every decode shape its dtype has (automatic
    included), once more with a call per layer."""
    from hkv_synth import workloads as W
    rng = np.random.default_rng(1000 + seed)
    n_kv = int(rng.choice([1, 2, 3, 4]))
    G = int(rng.integers(1, 9))
    window = int(rng.choice([w for w in (4, 8, 12, 16, 24, 32, 48, 64, 128) if G * w <= 256]))
    batch = int(rng.integers(1, 4))
    dtype = "f32" if seed % 5 == 4 else "bf16"
    n_visual = [int(rng.integers(200, 2200)) * _random_shape_scale() for _ in range(batch)]
    n_text = [int(rng.integers(window + 80, 420)) for _ in range(batch)]
    chunk = [int(rng.choice([8, 16, 32, 64, 128])) for _ in range(batch)]
    base = dict(W.CONFIGS[1])
    n_layers, block, sep = int(rng.integers(1, 4)), int(rng.choice([64, 256, 700])), int(rng.choice([0, 4, 16]))
    base.update(name=f"rand{seed}_{dtype}", dtype=dtype, n_layers=n_layers, n_q_heads=G * n_kv, n_kv_heads=n_kv,
                batch=batch, n_visual=n_visual, n_text=n_text, block=block, sep=_sep_that_fits(n_visual, n_text, block, sep, window),
                window=window, chunk=chunk, budget_frac=[float(rng.uniform(0.04, 0.45)) for _ in range(batch)],
                static_frac=float(rng.choice([0.0, 0.25, 0.5, 0.75, 1.0])), steps=3,
                q_mode=str(rng.choice(["normal", "centroid"])))
    W.CONFIGS[97] = base
    try:
        wl = make_workload(97, seed=seed)
    finally:
        del W.CONFIGS[97]
    modes = (0, 1, 2, 3, 4, 5) if dtype == "bf16" else (0, 1, 2, 3)
    for mode in modes:
        stats = P.full_pipeline(wl, decode_dynamic=mode)
        _say(f"random shape {seed}: G{G} kv{n_kv} w{window} B{batch} {dtype} chunks {chunk} mode {mode}", stats)
    stats = P.full_pipeline(wl, layer_ranges=[(l, l + 1) for l in range(wl.n_layers)])
    _say(f"random shape {seed}: a call per layer", stats)


@pytest.mark.parametrize("seed", _random_shape_seeds())
def test_seeded_random_shapes_across_the_variants(seed):
    """Shapes drawn as above (bf16 only), each run with a seeded choice of the switches that change what the
    kernels read or how they are launched: host tier for the dynamic heads, generated tokens in the chunk index,
    the other group reading of the chunk score, causal window scoring, a tile size between 128 and 1024 rows,
    one of the launch shapes the switches allow, and enough steps to complete chunks of generated tokens."""
    from hkv_synth import workloads as W
    rng = np.random.default_rng(5000 + seed)
    n_kv = int(rng.choice([1, 2, 4]))
    G = int(rng.integers(1, 9))
    window = int(rng.choice([w for w in (4, 8, 16, 32, 64) if G * w <= 256]))
    batch = int(rng.integers(1, 4))
    n_visual = [int(rng.integers(200, 2600)) * _random_shape_scale() for _ in range(batch)]
    n_text = [int(rng.integers(window + 80, 420)) for _ in range(batch)]
    chunk = [int(rng.choice([8, 16, 32, 64])) for _ in range(batch)]
    indexed = bool(rng.integers(0, 2))
    base = dict(W.CONFIGS[1])
    n_layers, block, sep = int(rng.integers(1, 4)), int(rng.choice([64, 256, 700])), int(rng.choice([0, 4, 16]))
    base.update(name=f"randv{seed}", dtype="bf16", n_layers=n_layers, n_q_heads=G * n_kv, n_kv_heads=n_kv,
                batch=batch, n_visual=n_visual, n_text=n_text, block=block, sep=_sep_that_fits(n_visual, n_text, block, sep, window),
                window=window, chunk=chunk, budget_frac=[float(rng.uniform(0.04, 0.45)) for _ in range(batch)],
                static_frac=float(rng.choice([0.0, 0.25, 0.5, 0.75])), steps=int(rng.integers(9, 20)) if indexed else 3,
                q_mode=str(rng.choice(["normal", "centroid"])))
    W.CONFIGS[96] = base
    try:
        wl = make_workload(96, seed=seed)
    finally:
        del W.CONFIGS[96]
    kw = dict(host_tier=bool(rng.integers(0, 2)), index_generated=int(indexed), chunk_score_group=int(rng.integers(0, 2)),
              causal=bool(rng.integers(0, 2)), decode_tile_rows=int(rng.choice([0, 128, 160, 288, 512, 1024])))
    modes = [0, 1, 3, 4] if indexed else [0, 1, 2, 3, 4, 5]
    kw["decode_dynamic"] = int(rng.choice(modes))
    per_layer = bool(rng.integers(0, 2))
    stats = P.full_pipeline(wl, layer_ranges=[(l, l + 1) for l in range(wl.n_layers)] if per_layer else None, **kw)
    _say(f"random variant {seed}: G{G} kv{n_kv} w{window} B{batch} chunks {chunk} per_layer={per_layer} {kw}", stats)


def test_chunk_scores_from_their_own_launch_under_the_automatic_rule():
    """Heads with more than 512 chunks (1024 chunks of 8 tokens) in calls whose tiles are all resident at once:
    under the automatic rule the chunk scores come from a launch of their own and the tiles only pick.  The
    whole chain matches the oracle (whole-model calls and a call per layer); the profiled second launch shows
    that the path was taken, and scores, picks and outputs equal those of the explicit single-launch shape
    bit for bit."""
    wl = make_workload(1, n_layers=2, steps=3)
    wl.chunk_size[:] = 8
    wl.budget[wl.head_type == O.DYNAMIC] = 8 * 96
    for ranges in (None, [(0, 1), (1, 2)]):
        stats = P.full_pipeline(wl, decode_tile_rows=1024, layer_ranges=ranges)
        _say(f"scores from their own launch, ranges {ranges}", stats)
    outs, sigmas, picks, second_ms = {}, {}, {}, {}
    for mode in (0, 3):
        dw = runner.setup(wl, decode_tile_rows=1024, decode_dynamic=mode)
        assert dw.cache.decode_shape()[1] == 3
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        q = runner.to_device(wl.q_steps[0], wl.dtype)
        out = torch.zeros_like(q)
        B.hkv_profile_enable(dw.cache.handle, 4)
        dw.cache.decode_attn(q, None, None, out)
        (ms, n_calls) = B.hkv_profile_read(dw.cache.handle)
        B.hkv_profile_disable(dw.cache.handle)
        assert n_calls == 1
        second_ms[mode] = ms[1]
        outs[mode] = out.view(torch.int16).cpu().numpy()
        dyn = [(l, h) for l in range(wl.n_layers) for h in range(wl.n_kv_heads) if wl.head_type[0, l, h] == O.DYNAMIC]
        sigmas[mode] = [dw.cache.export(B.HKV_X_CHUNK_SIGMA, 0, l, h) for l, h in dyn]
        picks[mode] = [dw.cache.export(B.HKV_X_CHUNK_SEL, 0, l, h) for l, h in dyn]
        dw.cache.close()
    assert second_ms[0] > 0.0 and second_ms[3] == 0.0
    assert np.array_equal(outs[0], outs[3])
    for a, b in zip(sigmas[0] + picks[0], sigmas[3] + picks[3]):
        assert np.array_equal(a, b)


@pytest.mark.parametrize("dtype_cfg,mode,tile", [(1, 1, 0), (1, 2, 128), (1, 2, 0), (1, 3, 128), (1, 3, 0), (1, 3, 160), (1, 2, 288), (1, 1, 416), (1, 4, 0), (0, 1, 0), (0, 2, 0), (0, 3, 0)])
def test_both_decode_shapes_for_dynamic_heads(dtype_cfg, mode, tile):
    """Dynamic heads handled by one workgroup each (mode 1), by split-K tiles in a second launch
    (mode 2), by tiles that repeat the selection (mode 3) and by one wide workgroup per head of either
    kind (mode 4, bf16 only) all match the oracle; bf16 (config 1 shape, heads spanning several tiles)
    and fp32 (config 0)."""
    if dtype_cfg == 1:
        wl = make_workload(1, n_layers=3, shrink=2, steps=4)
    else:
        wl = make_workload(0, n_layers=3, steps=4)
    stats = P.full_pipeline(wl, decode_dynamic=mode, decode_tile_rows=tile)
    _say(f"cfg{dtype_cfg} dynamic mode {mode} tile {tile}", stats)


def test_decode_shape_is_reported_and_auto_rule():
    wl = make_workload(1, n_layers=2, shrink=4, steps=1)
    for mode in (1, 2, 3, 4):
        dw = runner.setup(wl, decode_dynamic=mode, upload_prompt=False)
        assert dw.cache.decode_shape()[1] == mode
        dw.cache.close()
    dw = runner.setup(wl, upload_prompt=False)
    tile, mode = dw.cache.decode_shape()
    assert tile in (256, 512, 1024) and mode == 4      # heads of a few hundred rows: one wide workgroup each
    dw.cache.close()
    wl8k = make_workload(1, n_layers=2, steps=1, tensors=False)
    dw = runner.setup(wl8k, upload_prompt=False)
    assert dw.cache.decode_shape()[1] == 3             # long heads, 32-token chunks: summaries are cheap to re-read
    dw.cache.close()
    wl.chunk_size[:] = 8
    wl.budget[wl.head_type == 1] = 1024
    dw = runner.setup(wl, upload_prompt=False, decode_tile_rows=128)
    assert dw.cache.decode_shape() == (128, 2)          # small chunks, many tiles: the selection runs once per head
    dw.cache.close()
    # a serving mix of 16 long prompts: the whole-model call streams (768 equal shares), a call per layer has
    # shares too short for that under the automatic rule and runs as tiles; a caller's explicit choice of the
    # streamed shape is followed for both
    big = make_workload(4, steps=1, tensors=False)
    dw = runner.setup(big, upload_prompt=False)
    assert dw.cache.decode_shape()[1] == 5
    whole, one = dw.cache.call_tiling(), dw.cache.call_tiling(5, 6)
    assert whole[1] == 768 and whole[0] >= 2048
    assert one[0] in (256, 512, 1024) and one[1] > 0
    dw.cache.set_decode_dynamic(5)
    forced = dw.cache.call_tiling(5, 6)
    assert forced[1] == 768 and forced[0] < 2048
    dw.cache.close()


def test_workgroup_time_stamps_of_the_tile_launch():
    """The instrumented instantiation of the tile kernel: every workgroup leaves ordered stamps (start <=
    descriptor <= selection <= done), dynamic tiles have a selection stamp and static ones none, tiles kept
    for tail growth stay empty, and the outputs are bit-equal to the plain kernel's."""
    wl = make_workload(1, n_layers=3, shrink=2, steps=2)
    dw = runner.setup(wl, decode_dynamic=3)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    tdt = runner.torch_dtype(wl.dtype)
    q = runner.to_device(wl.q_steps[0], wl.dtype)
    kn, vn = runner.to_device(wl.k_new[0], wl.dtype), runner.to_device(wl.v_new[0], wl.dtype)
    out_a = torch.empty((wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim), dtype=tdt, device="cuda:0")
    out_b = torch.empty_like(out_a)
    dw.cache.decode_attn(q, kn, vn, out_a)
    torch.cuda.synchronize()
    dw.cache.rewind()
    n_tiles = dw.cache.call_tiling()[1]
    stamps = torch.full((n_tiles + 3, B.HKV_STAMP_WORDS), -1, dtype=torch.int64, device="cuda:0")
    dw.cache.set_stamps(stamps, n_tiles)
    dw.cache.decode_attn(q, kn, vn, out_b)
    torch.cuda.synchronize()
    dw.cache.set_stamps(None)
    assert torch.equal(out_a, out_b)
    st = stamps.cpu().numpy()
    assert np.all(st[n_tiles:] == -1)                       # nothing beyond the records asked for
    rec = st[:n_tiles]
    assert np.all(rec[:, 0] > 0) and np.all(rec[:, 1] >= rec[:, 0]) and np.all(rec[:, 7] == 0)
    reached = rec[:, 3] > 0
    assert reached.sum() >= n_tiles // 2
    dyn = rec[:, 5] == 1
    assert dyn.any() and (~dyn).any()
    assert np.all(rec[dyn & reached, 2] >= rec[dyn & reached, 1]) and np.all(rec[dyn & reached, 3] >= rec[dyn & reached, 2])
    assert np.all(rec[~dyn, 2] == 0) and np.all(rec[~dyn & reached, 3] >= rec[~dyn & reached, 1])
    assert np.all(rec[~dyn, 6] == 0)                        # scores-ready stamp: dynamic tiles only, inside the selection
    assert np.all(rec[dyn & reached, 6] >= rec[dyn & reached, 1]) and np.all(rec[dyn & reached, 6] <= rec[dyn & reached, 2])
    assert np.all(rec[:, 4] % dw.cache.call_tiling()[0] == 0)       # first rows are multiples of the tile size
    span_us = (rec[reached, 3].max() - rec[:, 0].min()) / 100.0
    assert 1.0 < span_us < 1000.0
    with pytest.raises(B.HkvError):
        dw.cache.set_stamps(stamps, 0)
    dw.cache.close()


def test_stream_read_probe_reports_a_plausible_rate():
    buf = torch.full((512 << 20,), 5, dtype=torch.uint8, device="cuda:0")
    torch.cuda.synchronize()
    us = B.hkv_probe_stream_read(buf.data_ptr(), buf.numel(), 64 << 20, 8)
    gbs = (64 << 20) / (us * 1e-6) / 1e9
    print(f"\n[probe] 64 MiB in {us:.2f} us = {gbs:.0f} GB/s", flush=True)
    assert 200.0 < gbs < 8000.0                      # below the HBM peak, above any sane floor
    with pytest.raises(B.HkvError):
        B.hkv_probe_stream_read(buf.data_ptr(), buf.numel(), buf.numel() + (1 << 20), 1)


def test_switching_the_decode_shape_on_a_live_cache():
    """hkv_cache_set_decode_dynamic changes how later steps run, not what they compute."""
    wl = make_workload(1, n_layers=2, shrink=4, steps=3)
    dw = runner.setup(wl)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    q = runner.to_device(wl.q_steps[0], wl.dtype)
    outs = []
    for mode in (1, 2, 3, 4, 5):
        dw.cache.set_decode_dynamic(mode)
        assert dw.cache.decode_shape()[1] == mode
        out = torch.empty((2, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        dw.cache.decode_attn(q, None, None, out)
        torch.cuda.synchronize()
        outs.append(out.float())
    for o in outs[1:]:
        assert (o - outs[0]).abs().max().item() <= 2e-2 * outs[0].abs().max().item()
    with pytest.raises(B.HkvError):
        dw.cache.set_decode_dynamic(6)
    dw.cache.close()
    wl32 = make_workload(0, shrink=4, steps=1)           # the per-unit and streamed shapes exist for bf16 caches only
    dw = runner.setup(wl32, upload_prompt=False)
    for mode in (4, 5):
        with pytest.raises(B.HkvError) as ei:
            dw.cache.set_decode_dynamic(mode)
        assert ei.value.status == B.HKV_ESHAPE
    dw.cache.close()


def test_decode_recorded_in_a_hip_graph_replays_correctly():
    """One recorded step (a call per layer, tail lengths on the device) replayed several times, with eager
    work and synchronisation between the replays, gives on every replay the bits of an eager cache that
    takes the same steps; afterwards the host bookkeeping is back in step and the tails hold the rows."""
    n_rep = 4
    wl = make_workload(1, n_layers=3, shrink=4, steps=2, max_new_tokens=n_rep + 1)
    L = wl.n_layers
    q, kn, vn = (runner.to_device(x[0], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
    eager, rec, warm = runner.setup(wl), runner.setup(wl), runner.setup(wl)
    for dw in (eager, rec, warm):
        dw.cache.compress(dw.q_window, dw.k, dw.v)
    out_e = torch.empty((L, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
    out_g = torch.zeros_like(out_e)
    warm.cache.set_device_tail(True)
    warm.cache.decode_attn(q, kn, vn, out_g)               # first use of the kernels happens outside the recording
    torch.cuda.synchronize()
    rec.cache.set_device_tail(True)
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        sp = torch.cuda.current_stream().cuda_stream
        for l in range(L):
            rec.cache.decode_attn(q[l:l + 1], kn[l:l + 1], vn[l:l + 1], out_g[l:l + 1], layer_begin=l, layer_end=l + 1,
                                  stream=sp)
    torch.cuda.synchronize()
    scratch = torch.randn(1 << 20, device="cuda:0")
    for r in range(n_rep):
        graph.replay()
        torch.cuda.synchronize()
        scratch = scratch * 1.0001 + 1.0                    # the program's own eager work between replays
        eager.cache.decode_attn(q, kn, vn, out_e)
        torch.cuda.synchronize()
        assert torch.equal(out_g, out_e), f"replay {r} differs from the eager step"
    rec.cache.set_device_tail(False)
    for l in range(L):
        for h in range(wl.n_kv_heads):
            a = rec.cache.export(B.HKV_X_K_ROWS, 0, l, h)
            b = eager.cache.export(B.HKV_X_K_ROWS, 0, l, h)
            assert a.shape == b.shape and np.array_equal(a, b)
    # host bookkeeping continues where the device left off: one more eager step on both
    rec.cache.decode_attn(q, kn, vn, out_g)
    eager.cache.decode_attn(q, kn, vn, out_e)
    torch.cuda.synchronize()
    assert torch.equal(out_g, out_e)
    for dw in (eager, rec, warm):
        dw.cache.close()


def _device_head_scores(wl, qp, causal=False, rho=0.05, small_workspace=False):
    cfg = B.make_config(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                        dtype=runner.hkv_dtype(wl.dtype), window=wl.window, score_causal=int(causal))
    lo, hi = B.hkv_head_scores_workspace_size(cfg, wl.cu_seqlens, wl.is_visual)
    nbytes = lo if small_workspace else hi
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    q_dev, k_dev = runner.to_device(qp, wl.dtype), runner.to_device(wl.k, wl.dtype)
    scores = torch.full((wl.n_layers, wl.batch, wl.n_kv_heads), -1.0, dtype=torch.float32, device="cuda:0")
    B.hkv_head_scores(cfg, wl.cu_seqlens, wl.is_visual, wl.n_layers, q_dev, k_dev, rho, scores, ws, nbytes)
    torch.cuda.synchronize()
    return scores.cpu().numpy().transpose(1, 0, 2)          # [batch, L, Hkv] like the oracle


SCORE_ATOL = 5e-5     # fp32 logits (exact bf16/fp32 products, fp32 accumulation of 128 terms), exp2, fp32 sums


@pytest.mark.parametrize("cfg_id,shrink,causal", [(1, 4, False), (1, 4, True), (0, 2, False), (4, 8, False), (4, 8, True)])
def test_head_sparsity_scores_match_the_oracle(cfg_id, shrink, causal):
    """Text-centric sparsity score of every (sequence, layer, KV head) against the float64 oracle: bf16 and
    fp32, one sequence and a ragged batch, with and without the causal option; the head types at the
    paper's threshold agree wherever the score is not within the tolerance of it."""
    from hkv_synth import make_prompt_queries
    wl = make_workload(cfg_id, n_layers=2, shrink=shrink, steps=1)
    qp = make_prompt_queries(wl)
    got = _device_head_scores(wl, qp, causal=causal)
    ocfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128,
                          window=wl.window, dtype=wl.dtype, score_causal=causal)
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual)
    err = np.abs(got - want).max()
    print(f"\n[head scores cfg{cfg_id}/{shrink} causal={causal}] max abs err {err:.2e}; scores {want.min():.3f}..{want.max():.3f}",
          flush=True)
    assert err <= SCORE_ATOL
    clear = np.abs(want - 0.9) > 2 * SCORE_ATOL
    assert np.array_equal(O.classify_heads(got, 0.9)[clear], O.classify_heads(want, 0.9)[clear])
    # the generator's static heads are the sparse ones
    assert np.all(want[wl.head_type == 0] > 0.9) and np.all(want[wl.head_type == 1] < 0.6)


def test_head_scores_do_not_depend_on_the_workspace_size_and_focus_edges():
    from hkv_synth import make_prompt_queries
    wl = make_workload(1, n_layers=1, shrink=8, steps=1)
    qp = make_prompt_queries(wl)
    a = _device_head_scores(wl, qp)
    b = _device_head_scores(wl, qp, small_workspace=True)       # one head per pass
    assert np.array_equal(a, b)
    ocfg = O.OracleConfig(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128, window=wl.window,
                          dtype=wl.dtype)
    full = _device_head_scores(wl, qp, rho=1.0)                 # every position counts: the score is 1
    assert np.abs(full - 1.0).max() <= SCORE_ATOL
    tiny = _device_head_scores(wl, qp, rho=1e-6)                # k = 1: mean of the row maxima
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual, rho=1e-6)
    assert np.abs(tiny - want).max() <= SCORE_ATOL


def test_head_scores_on_short_prompts():
    """Prompts of 120 to 230 tokens (a handful of 32-key tiles, fewer groups of 16 keys than lanes, k = 6 to
    12), three in a batch, bf16 and fp32."""
    from hkv_synth import make_prompt_queries
    from hkv_synth import workloads as W
    for dtype in ("bf16", "f32"):
        base = dict(W.CONFIGS[1])
        base.update(name=f"short_{dtype}", dtype=dtype, n_layers=2, batch=3, n_visual=[8, 40, 100], n_text=[112, 120, 130],
                    block=64, chunk=[8, 8, 8], budget_frac=[0.3, 0.3, 0.3], steps=1)
        W.CONFIGS[95] = base
        try:
            wl = make_workload(95, seed=4)
        finally:
            del W.CONFIGS[95]
        qp = make_prompt_queries(wl)
        ocfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128,
                              window=wl.window, dtype=wl.dtype)
        for rho in (0.05, 0.01):
            got = _device_head_scores(wl, qp, rho=rho)
            want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual, rho=rho)
            err = np.abs(got - want).max()
            print(f"\n[head scores, short prompts {list(map(int, wl.seqlens))} {dtype} rho={rho}] max abs err {err:.2e}", flush=True)
            assert err <= SCORE_ATOL


def test_head_scores_with_runs_of_equal_logits():
    """Equal keys give equal logits: a head whose keys are all the same row (every logit of a row ties, the
    bound from the group maxima admits the whole row and the listed logits no longer fit the registers), a
    head whose first half repeats one key, and two untouched heads; focus fractions on both sides of the
    switch between the scanning and the materialising form."""
    from hkv_synth import make_prompt_queries
    wl = make_workload(1, n_layers=1, shrink=4, steps=1)
    qp = make_prompt_queries(wl)
    k = np.array(wl.k, copy=True)
    C = int(wl.seqlens[0])
    k[0, :, 0, :] = k[0, 7, 0, :]
    k[0, :C // 2, 1, :] = k[0, 11, 1, :]
    wl.k = k
    ocfg = O.OracleConfig(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128, window=wl.window,
                          dtype=wl.dtype)
    for rho in (0.02, 0.05, 0.2):
        got = _device_head_scores(wl, qp, rho=rho)
        want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual, rho=rho)
        err = np.abs(got - want).max()
        print(f"\n[head scores, equal keys, rho={rho}] max abs err {err:.2e}; scores {want.ravel()[:4]}", flush=True)
        assert err <= SCORE_ATOL
        k_top = O.focus_count(C, rho)
        assert abs(want[0, 0, 0] - k_top / C) < 1e-12           # all keys equal: every probability is 1/C


@pytest.mark.parametrize("seed", _random_shape_seeds())
def test_head_scores_on_seeded_random_shapes(seed):
    """Group sizes 1 to 8, one to three ragged prompts of 300 to 4500 tokens with 40 to 400 text tokens, focus
    fractions from 0.005 to 0.4 (both sides of the switch between the scanning and the materialising form),
    with and without the causal option, bf16 and fp32, full and smallest workspace."""
    from hkv_synth import make_prompt_queries
    from hkv_synth import workloads as W
    rng = np.random.default_rng(9000 + seed)
    n_kv, G, batch = int(rng.choice([1, 2, 4])), int(rng.integers(1, 9)), int(rng.integers(1, 4))
    dtype = "f32" if seed % 4 == 3 else "bf16"
    n_visual = [int(rng.integers(260, 4100)) for _ in range(batch)]
    n_text = [int(rng.integers(40, 400)) for _ in range(batch)]
    block = int(rng.choice([256, 700, 5000]))
    base = dict(W.CONFIGS[1])
    base.update(name=f"randh{seed}_{dtype}", dtype=dtype, n_layers=int(rng.integers(1, 3)), n_q_heads=G * n_kv, n_kv_heads=n_kv,
                batch=batch, n_visual=n_visual, n_text=n_text, block=block, sep=0, window=int(rng.choice([8, 16, 32])),
                chunk=[8] * batch, budget_frac=[0.3] * batch, steps=1)
    W.CONFIGS[94] = base
    try:
        wl = make_workload(94, seed=seed)
    finally:
        del W.CONFIGS[94]
    qp = make_prompt_queries(wl)
    rho, causal = float(rng.choice([0.005, 0.02, 0.05, 0.055, 0.08, 0.2, 0.4])), bool(rng.integers(0, 2))
    small = bool(rng.integers(0, 2))
    ocfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128,
                          window=wl.window, dtype=wl.dtype, score_causal=causal)
    got = _device_head_scores(wl, qp, causal=causal, rho=rho, small_workspace=small)
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual, rho=rho)
    err = np.abs(got - want).max()
    print(f"\n[head scores, random shape {seed}: G{G} kv{n_kv} {dtype} C={list(map(int, wl.seqlens))} T={n_text} rho={rho} "
          f"causal={causal} small_ws={small}] max abs err {err:.2e}", flush=True)
    assert err <= SCORE_ATOL


@pytest.mark.parametrize("n_visual,rho", [(9800, 0.05), (19900, 0.05), (40000, 0.05), (9800, 0.1), (19900, 0.1), (40000, 0.1),
                                          (70000, 0.05)])
def test_head_scores_on_long_rows(n_visual, rho):
    """Long rows.  At a focus fraction of 0.05 the rows are scanned on the fly (up to 65536 keys; more group
    maxima per lane and more listed logits per row as the rows grow); at 0.1, and beyond 65536 keys, the
    logits are materialised and the per-row top-k takes its wider register-resident forms (up to 16384 and
    32768 keys) or the form that re-reads the row from memory.  Few text tokens keep the oracle quick."""
    from hkv_synth import make_prompt_queries
    from hkv_synth import workloads as W
    base = dict(W.CONFIGS[1])
    base.update(name=f"long_{n_visual}", n_layers=1, n_visual=[n_visual], n_text=[96], block=n_visual, steps=1)
    W.CONFIGS[98] = base
    try:
        wl = make_workload(98, seed=5)
    finally:
        del W.CONFIGS[98]
    qp = make_prompt_queries(wl)
    got = _device_head_scores(wl, qp, rho=rho)
    ocfg = O.OracleConfig(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128, window=wl.window,
                          dtype=wl.dtype)
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual, rho=rho)
    err = np.abs(got - want).max()
    print(f"\n[head scores C={int(wl.seqlens[0])} rho={rho}] max abs err {err:.2e}", flush=True)
    assert err <= SCORE_ATOL


# ---- host-memory tier for the dynamic heads (Section 3.3: their prompt K/V lives outside GPU memory) ----

@pytest.mark.parametrize("mode,tile", [(1, 0), (2, 0), (3, 0), (3, 128)])
def test_host_tier_matches_the_oracle(mode, tile):
    """The dynamic heads' prompt rows live in page-locked host memory; compression writes them there,
    decode gathers the selected chunks from there.  Same oracle, same tolerances as an untiered cache;
    the exported rows (prompt part from the host tier, tail part from device memory) are compared too."""
    wl = make_workload(1, n_layers=3, shrink=2, steps=4)
    stats = P.full_pipeline(wl, host_tier=True, decode_dynamic=mode, decode_tile_rows=tile)
    _say(f"host tier mode {mode} tile {tile}", stats)


def test_host_tier_ragged_batch_and_layer_ranges():
    wl = make_workload(4, n_layers=2, shrink=8, steps=3)
    stats = P.full_pipeline(wl, host_tier=True, layer_ranges=[(0, 1), (1, 2)])
    _say("host tier cfg4/8", stats)


def test_host_tier_outputs_equal_the_untiered_cache_bit_for_bit():
    """Where the rows live changes no arithmetic: outputs of a tiered and an untiered cache are equal,
    and the device arena shrinks by the dynamic heads' prompt rows."""
    wl = make_workload(1, n_layers=2, shrink=4, steps=6)
    outs, sizes = [], []
    for tier in (False, True):
        dw = runner.setup(wl, host_tier=tier)
        sizes.append((dw.cache.cache_bytes, dw.cache.host_bytes))
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        out = torch.empty((wl.n_layers, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        res = []
        for s in range(wl.steps):
            q, kn, vn = (runner.to_device(x[s], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
            dw.cache.decode_attn(q, kn, vn, out)
            torch.cuda.synchronize()
            res.append(out.clone())
        outs.append(torch.stack(res))
        dw.cache.close()
    assert torch.equal(outs[0], outs[1])
    (dev0, host0), (dev1, host1) = sizes
    n_dyn = int((wl.head_type == O.DYNAMIC).sum())
    C = int(wl.seqlens[0])
    assert host0 == 0 and host1 >= 2 * n_dyn * C * 128 * 2
    assert dev0 - dev1 >= 2 * n_dyn * (C - 8) * 128 * 2          # up to block rounding of the tails


def test_host_tier_rejects_memory_the_device_cannot_address():
    wl = make_workload(1, n_layers=1, shrink=8, steps=1)
    dw = runner.setup(wl, upload_prompt=False)           # supplies cfg and plan
    cb, hb, wb = B.hkv_query_tier_sizes(dw.cfg, dw.plan)
    arena = torch.empty(cb + 256, dtype=torch.uint8, device="cuda:0")
    a = arena[(-arena.data_ptr()) % 256:]
    pageable = torch.empty(hb + 256, dtype=torch.uint8)              # ordinary host memory
    pg = pageable[(-pageable.data_ptr()) % 256:]
    with pytest.raises(B.HkvError) as ei:
        B.hkv_cache_create_tiered(dw.cfg, dw.plan, a, cb, pg, hb)
    assert ei.value.status == B.HKV_EINVAL
    devmem = torch.empty(hb + 256, dtype=torch.uint8, device="cuda:0")   # device memory is no host tier
    dm = devmem[(-devmem.data_ptr()) % 256:]
    with pytest.raises(B.HkvError) as ei:
        B.hkv_cache_create_tiered(dw.cfg, dw.plan, a, cb, dm, hb)
    assert ei.value.status == B.HKV_EINVAL
    pinned = torch.empty(hb + 256, dtype=torch.uint8, pin_memory=True)
    pn = pinned[(-pinned.data_ptr()) % 256:]
    with pytest.raises(B.HkvError) as ei:
        B.hkv_cache_create_tiered(dw.cfg, dw.plan, a, cb, pn, hb - 1)    # too small
    assert ei.value.status == B.HKV_ENOSPACE
    h = B.hkv_cache_create_tiered(dw.cfg, dw.plan, a, cb, pn, hb)
    B.hkv_cache_destroy(h)
    dw.cache.close()
    torch.cuda.synchronize()          # no error left behind by the refused pointers


# ---- other reading of the chunk scoring for grouped query heads ----

@pytest.mark.parametrize("cfg_id,mode", [(1, 3), (1, 1), (1, 2), (0, 3), (4, 0)])
def test_chunk_scores_as_the_largest_over_the_group(cfg_id, mode):
    """chunk_score_group = 1: a chunk's score is the largest of the G query heads' inner products with
    its summary (bf16 and fp32 caches, every launch shape, ragged batch with both chunk sizes)."""
    if cfg_id == 4:
        wl = make_workload(4, n_layers=2, shrink=8, steps=3)
    else:
        wl = make_workload(cfg_id, n_layers=2, shrink=2 if cfg_id == 1 else 1, steps=4)
    stats = P.full_pipeline(wl, chunk_score_group=1, decode_dynamic=mode)
    _say(f"cfg{cfg_id} max-over-group mode {mode}", stats)


def test_the_two_group_readings_pick_different_chunks():
    """The variant is not a no-op: on the same inputs the two readings disagree on some head's picks."""
    wl = make_workload(1, n_layers=2, shrink=4, steps=1)
    picks = []
    for grp in (0, 1):
        dw = runner.setup(wl, chunk_score_group=grp)
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        out = torch.empty((wl.n_layers, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        q, kn, vn = (runner.to_device(x[0], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
        dw.cache.decode_attn(q, kn, vn, out)
        torch.cuda.synchronize()
        picks.append([dw.cache.export(B.HKV_X_CHUNK_SEL, 0, l, h) for l in range(wl.n_layers)
                      for h in range(wl.n_kv_heads) if wl.head_type[0, l, h] == O.DYNAMIC])
        dw.cache.close()
    assert any(not np.array_equal(a, b) for a, b in zip(*picks))


# ---- cumulative focus count of every head (Section 2.1, Eq. 1) ----

def _focus_bounds(q_steps, k, scale, k_top, band_rel):
    """Per token: in how many steps it is surely / possibly among the k_top largest logits, when a
    logit within `band` of the cut may fall on either side (fp32 logits on the device, fp64 here)."""
    q = q_steps.astype(np.float64)
    kk = k.astype(np.float64)
    C = kk.shape[0]
    lo, hi = np.zeros(C, np.int64), np.zeros(C, np.int64)
    for i in range(q.shape[0]):
        lg = (kk @ q[i]) * scale
        if k_top >= C:
            lo += 1
            hi += 1
            continue
        srt = np.sort(lg)[::-1]
        band = band_rel * np.linalg.norm(q[i]) * np.linalg.norm(kk, axis=1).max() * scale
        lo += lg > srt[k_top] + band          # clearly above the first one left out
        hi += lg >= srt[k_top - 1] - band     # not clearly below the last one taken
    return lo, hi


@pytest.mark.parametrize("cfg_id,n_steps,frac", [(1, 24, 0.05), (0, 16, 0.05), (1, 5, 0.3), (1, 3, 1.0)])
def test_cumulative_focus_counts_match_the_oracle(cfg_id, n_steps, frac):
    wl = make_workload(cfg_id, n_layers=2, shrink=4 if cfg_id == 1 else 2, steps=n_steps)
    l, b = 1, 0
    C = int(wl.seqlens[b]) - 3                       # a context length that is no multiple of 32
    cfg = B.make_config(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, dtype=runner.hkv_dtype(wl.dtype),
                        window=wl.window)
    q_host = np.ascontiguousarray(wl.q_steps[:n_steps, l, b])            # [N, Hq, d]
    k_host = np.ascontiguousarray(wl.k[l, :C])                           # [C, Hkv, d]
    q_dev, k_dev = runner.to_device(q_host, wl.dtype), runner.to_device(k_host, wl.dtype)
    lo_b, hi_b = B.hkv_focus_counts_workspace_size(cfg, n_steps, C)
    assert lo_b * wl.n_kv_heads >= hi_b > lo_b
    got = []
    for nbytes in (hi_b, lo_b):                      # all KV heads in one pass / one KV head per pass
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
        counts = torch.full((wl.n_q_heads, C), -7, dtype=torch.int32, device="cuda:0")
        B.hkv_focus_counts(cfg, n_steps, C, q_dev, k_dev, frac, counts, ws, nbytes)
        torch.cuda.synchronize()
        got.append(counts.cpu().numpy().astype(np.int64))
    assert np.array_equal(got[0], got[1])
    F = got[0]
    k_top = O.focus_count(C, frac)
    assert np.all(F.sum(axis=1) == n_steps * k_top) and F.min() >= 0 and F.max() <= n_steps
    scale = 1.0 / np.sqrt(128.0)
    G = wl.group
    exact = 0
    for hq in range(wl.n_q_heads):
        ref = O.cumulative_focus(q_host[:, hq], k_host[:, hq // G], scale, k_top)
        lo, hi = _focus_bounds(q_host[:, hq], k_host[:, hq // G], scale, k_top, 1e-5)
        assert np.all(lo <= ref) and np.all(ref <= hi)                   # the bounds bracket the oracle itself
        assert np.all(lo <= F[hq]) and np.all(F[hq] <= hi), f"head {hq}: counts outside the tie band"
        exact += int(np.array_equal(F[hq], ref))
    print(f"\n[focus cfg{cfg_id}] C={C} k={k_top} steps={n_steps}: {exact}/{wl.n_q_heads} heads bit-equal to the oracle",
          flush=True)
    assert exact >= wl.n_q_heads - 2                 # a near-tie at the cut is rare
    if frac == 1.0:
        assert np.all(F == n_steps)


@pytest.mark.parametrize("seed", _random_shape_seeds())
def test_focus_counts_on_seeded_random_shapes(seed):
    """Group sizes 1 to 8, 1 to 40 decoding steps, contexts of 40 to 9000 tokens, focus fractions from one token to
    everything, bf16 and fp32, full and smallest workspace: the counts lie inside the tie band around the oracle's
    and add up to steps x k."""
    from hkv_synth.workloads import bf16_round
    rng = np.random.default_rng(11000 + seed)
    n_kv, G, n_steps = int(rng.choice([1, 2, 4])), int(rng.integers(1, 9)), int(rng.integers(1, 41))
    C = int(rng.choice([40, 63, 64, 65, 255, 256, 257, 1000, 2048])) if rng.integers(0, 2) else int(rng.integers(40, 9000))
    frac = float(rng.choice([1e-6, 0.01, 0.05, 0.05, 0.3, 1.0]))
    dtype = "f32" if seed % 3 == 1 else "bf16"
    n_q = G * n_kv
    to_dtype = bf16_round if dtype == "bf16" else (lambda x: x.astype(np.float32))
    q_host, k_host = to_dtype(rng.standard_normal((n_steps, n_q, 128))), to_dtype(rng.standard_normal((C, n_kv, 128)))
    cfg = B.make_config(n_layers=1, n_q_heads=n_q, n_kv_heads=n_kv, dtype=runner.hkv_dtype(dtype), window=1)
    q_dev, k_dev = runner.to_device(q_host, dtype), runner.to_device(k_host, dtype)
    lo_b, hi_b = B.hkv_focus_counts_workspace_size(cfg, n_steps, C)
    nbytes = lo_b if rng.integers(0, 2) else hi_b
    ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")
    counts = torch.full((n_q, C), -7, dtype=torch.int32, device="cuda:0")
    B.hkv_focus_counts(cfg, n_steps, C, q_dev, k_dev, frac, counts, ws, nbytes)
    torch.cuda.synchronize()
    F = counts.cpu().numpy().astype(np.int64)
    k_top = O.focus_count(C, frac)
    assert np.all(F.sum(axis=1) == n_steps * k_top) and F.min() >= 0 and F.max() <= n_steps
    scale = 1.0 / np.sqrt(128.0)
    exact = 0
    for hq in range(n_q):
        qd, kd = q_host[:, hq].astype(np.float64), k_host[:, hq // G].astype(np.float64)
        ref = O.cumulative_focus(qd, kd, scale, k_top)
        lo, hi = _focus_bounds(qd, kd, scale, k_top, 1e-5)
        assert np.all(lo <= F[hq]) and np.all(F[hq] <= hi), f"head {hq}: counts outside the tie band"
        exact += int(np.array_equal(F[hq], ref))
    print(f"\n[focus, random shape {seed}: G{G} kv{n_kv} {dtype} C={C} k={k_top} steps={n_steps}] {exact}/{n_q} heads bit-equal",
          flush=True)
    # a head differs from the oracle only where two logits at the cut lie closer than fp32 resolves: about
    # 2e-7 * C of the (head, step) pairs for Gaussian logits
    assert exact >= n_q - 2 - int(4 * 2e-7 * C * n_q * n_steps)


def test_focus_counts_argument_checks():
    cfg = B.make_config(n_layers=1, n_q_heads=28, n_kv_heads=4, dtype=B.HKV_BF16, window=32)
    t = torch.zeros(4096, dtype=torch.uint8, device="cuda:0")
    for args, status in (((0, 100), B.HKV_ESHAPE), ((4, 0), B.HKV_ESHAPE)):
        with pytest.raises(B.HkvError) as ei:
            B.hkv_focus_counts_workspace_size(cfg, *args)
        assert ei.value.status == status
    with pytest.raises(B.HkvError) as ei:
        B.hkv_focus_counts(cfg, 4, 100, t, t, 0.05, t, t, 16)            # workspace too small
    assert ei.value.status == B.HKV_ENOSPACE
    with pytest.raises(B.HkvError) as ei:
        B.hkv_focus_counts(cfg, 4, 100, t, t, 0.0, t, t, 1 << 20)        # fraction out of range
    assert ei.value.status == B.HKV_EINVAL


def test_focus_counts_full_context_and_planted_ties():
    """Config 1's full context (8192 tokens); every key appears twice (positions 2j and 2j+1), so each
    row's cut falls between two exactly equal logits whenever k is odd: the lower position must win."""
    wl = make_workload(1, n_layers=1, steps=8)
    C = int(wl.seqlens[0]) - 1                        # 8191 -> k = ceil(0.05 * 8191) = 410; use a fraction giving an odd k
    frac = 411 / C
    cfg = B.make_config(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, dtype=B.HKV_BF16, window=wl.window)
    q_host = np.ascontiguousarray(wl.q_steps[:8, 0, 0])
    k_host = np.ascontiguousarray(wl.k[0, :C]).copy()
    k_host[1::2] = k_host[0:C - 1:2]
    k_top = O.focus_count(C, frac)
    assert k_top == 411
    q_dev, k_dev = runner.to_device(q_host, "bf16"), runner.to_device(k_host, "bf16")
    _, hi_b = B.hkv_focus_counts_workspace_size(cfg, 8, C)
    ws = torch.empty(hi_b, dtype=torch.uint8, device="cuda:0")
    counts = torch.empty((wl.n_q_heads, C), dtype=torch.int32, device="cuda:0")
    B.hkv_focus_counts(cfg, 8, C, q_dev, k_dev, frac, counts, ws, hi_b)
    torch.cuda.synchronize()
    F = counts.cpu().numpy().astype(np.int64)
    assert np.all(F.sum(axis=1) == 8 * k_top)
    # within a pair the lower position is never behind the upper one, and is ahead at every split cut
    assert np.all(F[:, 0:C - 1:2] >= F[:, 1::2])
    # odd k: one split pair per step, except at steps where the unpaired last token is among the picks
    assert np.all((F[:, 0:C - 1:2] - F[:, 1::2]).sum(axis=1) == 8 - F[:, C - 1])
    G = wl.group
    exact = 0
    for hq in range(0, wl.n_q_heads, 3):
        ref = O.cumulative_focus(q_host[:, hq], k_host[:, hq // G], 1.0 / np.sqrt(128.0), k_top)
        lo, hi = _focus_bounds(q_host[:, hq], k_host[:, hq // G], 1.0 / np.sqrt(128.0), k_top, 1e-5)
        assert np.all(lo <= F[hq]) and np.all(F[hq] <= hi)
        exact += int(np.array_equal(F[hq], ref))
    assert exact >= len(range(0, wl.n_q_heads, 3)) - 1


# ---- degenerate prompts ----

@pytest.mark.parametrize("dtype,chunks", [("bf16", [8, 8, 16, 8]), ("f32", [64, 4, 16, 256])])
def test_degenerate_prompts_in_one_batch(dtype, chunks):
    """A batch whose sequences sit on the edges of the method: a prompt that is exactly the observation
    window (no historical token at all), one with five visual tokens, an ordinary one, and one whose text is
    the window plus a single token; chunk sizes from 4 tokens up to more than the whole prompt (one short
    chunk)."""
    import hkv_synth.workloads as W
    W.CONFIGS[99] = dict(name="degenerate_prompts", dtype=dtype, n_layers=2, n_q_heads=8, n_kv_heads=2, batch=4,
                         n_visual=[0, 5, 300, 120], n_text=[32, 40, 150, 33], block=64, sep=4, window=32,
                         chunk=chunks, budget_frac=[0.5, 0.5, 0.2, 0.2], k_chunks=2, static_frac=0.5,
                         fixed_types=[0, 1], hierarchical=False, steps=3, q_mode="normal")
    try:
        wl = make_workload(99, seed=5)
    finally:
        del W.CONFIGS[99]
    assert wl.seqlens.tolist() == [32, 45, 450, 153]
    for mode in (1, 3) + ((4,) if dtype == "bf16" else ()):
        stats = P.full_pipeline(wl, decode_dynamic=mode)
        _say(f"degenerate prompts {dtype} mode {mode}", stats)


@pytest.mark.parametrize("modality", [0, 1])
def test_prompt_of_a_single_modality(modality):
    """All text (the visual candidate set is empty, budgets fall under the text-overflow rule) and all
    visual (no text to exempt, the window itself is visual)."""
    wl = make_workload(0, shrink=4, steps=2)
    wl.is_visual[:] = modality
    stats = P.full_pipeline(wl)
    _say(f"single modality {modality}", stats)
    wl2 = make_workload(1, n_layers=2, shrink=8, steps=2)
    wl2.is_visual[:] = modality
    stats = P.full_pipeline(wl2)
    _say(f"single modality {modality} bf16", stats)


# ---- one wide workgroup per head, no split-K (decode_dynamic = 4) ----

@pytest.mark.parametrize("case", ["ragged", "g8", "small_chunks", "host_tier", "max_group", "layer_calls"])
def test_one_workgroup_per_head_shape(case):
    """The per-unit launch on the shapes that stress it: ragged batch with both chunk sizes, group of
    eight, many small chunks (radix selection by 768 threads), host tier, the other group reading of the
    chunk score, per-layer calls."""
    kw = dict(decode_dynamic=4)
    if case == "ragged":
        wl = make_workload(4, n_layers=2, shrink=8, steps=3)
    elif case == "g8":
        wl = make_workload(3, n_layers=2, shrink=16, steps=3)
    elif case == "small_chunks":
        wl = make_workload(1, n_layers=2, steps=2)
        wl.chunk_size[:] = 16
        wl.budget[wl.head_type == O.DYNAMIC] = 16 * 300
    elif case == "host_tier":
        wl = make_workload(1, n_layers=2, shrink=2, steps=3)
        kw["host_tier"] = True
    elif case == "max_group":
        wl = make_workload(1, n_layers=2, shrink=2, steps=3)
        kw["chunk_score_group"] = 1
    else:
        wl = make_workload(1, n_layers=3, shrink=4, steps=3)
        kw["layer_ranges"] = [(0, 1), (1, 2), (2, 3)]
    stats = P.full_pipeline(wl, **kw)
    _say(f"per-unit shape, {case}", stats)


# ---- the larger shapes at their full context length (a few layers; the oracle checks a sampled layer) ----

@pytest.mark.parametrize("cfg_id,n_layers,steps,tile", [(2, 2, 3, 1024), (3, 2, 2, 1024), (2, 1, 2, 0)])
def test_full_context_of_the_larger_shapes(cfg_id, n_layers, steps, tile):
    """Config 2 (four 32768-token multi-image prompts, 64-token chunks, decode queries near chunk
    centroids) and config 3 (72B attention shape, one 51200-token video prompt, group of eight) at their
    real per-head sizes: hundreds of chunks per head, and the 1024-row tiles that caches of all their
    layers pick (a cache of two layers would stay at 256 rows)."""
    wl = make_workload(cfg_id, n_layers=n_layers, steps=steps)
    assert int(wl.seqlens.max()) == (32768 if cfg_id == 2 else 51200)
    layers = [n_layers - 1]
    dw = runner.setup(wl, decode_tile_rows=tile)
    tile_used, mode = dw.cache.decode_shape()
    print(f"\n[cfg{cfg_id} full context] tile {tile_used} mode {mode}", flush=True)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl)
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers)
    _say(f"cfg{cfg_id} full context", stats)
    dw.cache.close()


def test_serving_mix_at_full_context_lengths():
    """Config 4 with its real ragged lengths (16 sequences of 4096 to 40960 tokens, both chunk sizes,
    per-sequence budgets), one layer, every unit checked."""
    wl = make_workload(4, n_layers=1, steps=2)
    assert wl.batch == 16 and int(wl.seqlens.max()) > 30000
    stats = P.full_pipeline(wl, decode_tile_rows=1024)
    _say("cfg4 full lengths L1", stats)


# ---- generated tokens in the chunk index (index_generated = 1) ----

@pytest.mark.parametrize("mode,case", [(1, "small_chunks"), (4, "small_chunks"), (3, "small_chunks"), (1, "every_chunk"),
                                       (3, "every_chunk"), (4, "ragged"), (3, "ragged"), (1, "host_tier"),
                                       (3, "host_tier"), (0, "max_group")])
def test_generated_tokens_are_indexed_and_retrieved(mode, case):
    """Dynamic heads retrieve complete chunks of generated tokens like chunks of the prompt; the rest of
    the tail is always attended.  40 steps with 8-token chunks complete five chunks (and carry a head with
    256 prompt chunks over the 256-chunk boundary between the two selection routines); the ragged case
    has 32- and 64-token chunks and runs long enough to complete both kinds."""
    kw = dict(index_generated=1, decode_dynamic=mode)
    if case == "ragged":
        wl = make_workload(4, n_layers=1, shrink=8, steps=66)
    else:
        wl = make_workload(1, n_layers=2, shrink=4, steps=40)
        wl.chunk_size[:] = 8
        dyn = wl.head_type == O.DYNAMIC
        wl.budget[dyn] = 8 * (10 ** 6 if case == "every_chunk" else 100)
        if case == "host_tier":
            kw["host_tier"] = True
        if case == "max_group":
            kw["chunk_score_group"] = 1
    stats = P.full_pipeline(wl, **kw)
    _say(f"indexed generation, {case}, mode {mode}", stats)
    assert stats["generated_chunks_picked"] > 0


def test_indexed_generation_argument_checks_and_device_tail():
    wl = make_workload(1, n_layers=2, shrink=8, steps=20)
    wl.chunk_size[:] = 8
    with pytest.raises(B.HkvError) as ei:
        runner.setup(wl, upload_prompt=False, index_generated=1, decode_dynamic=2)
    assert ei.value.status == B.HKV_ESHAPE
    wl32 = make_workload(0, shrink=4, steps=1)
    with pytest.raises(B.HkvError) as ei:
        runner.setup(wl32, upload_prompt=False, index_generated=1)           # fp32 cache
    assert ei.value.status == B.HKV_ESHAPE
    # tail lengths kept on the device (as a recorded step needs them) give the same bits as host bookkeeping
    outs = []
    for device_tail, mode in ((False, 0), (True, 0), (True, 1), (True, 3), (True, 4)):
        dw = runner.setup(wl, index_generated=1, decode_dynamic=mode)
        assert dw.cache.decode_shape()[1] in (1, 3, 4)
        with pytest.raises(B.HkvError):
            dw.cache.set_decode_dynamic(2)
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        if device_tail:
            dw.cache.set_device_tail(True)
        out = torch.empty((wl.n_layers, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        res = []
        for s in range(wl.steps):
            q, kn, vn = (runner.to_device(x[s], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
            dw.cache.decode_attn(q, kn, vn, out)
            torch.cuda.synchronize()
            res.append(out.clone())
        outs.append(torch.stack(res))
        if device_tail:
            dw.cache.set_device_tail(False)
        dw.cache.close()
    assert torch.equal(outs[0], outs[1])                 # same shape, host or device bookkeeping: same bits
    for o in outs[2:]:                                   # other shapes: same results up to summation order
        assert (o.float() - outs[0].float()).abs().max().item() <= 2e-2 * outs[0].float().abs().max().item()


def test_head_scores_of_sequences_without_text_or_without_visual_tokens():
    """Sequence 0 of the batch has no text token (its heads score 0 by definition: there is no text row
    to average), sequence 1 is all text (every token of the prompt is a row), the others are ordinary."""
    from hkv_synth import make_prompt_queries
    wl = make_workload(4, n_layers=1, shrink=8, steps=1)
    lo0, hi0, hi1 = int(wl.cu_seqlens[0]), int(wl.cu_seqlens[1]), int(wl.cu_seqlens[2])
    wl.is_visual[lo0:hi0] = 1
    wl.is_visual[hi0:hi1] = 0
    qp = make_prompt_queries(wl)
    got = _device_head_scores(wl, qp)
    ocfg = O.OracleConfig(n_layers=1, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128, window=wl.window,
                          dtype=wl.dtype)
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual)
    assert np.all(got[0] == 0.0) and np.all(want[0] == 0.0)
    assert np.abs(got - want).max() <= SCORE_ATOL


@pytest.mark.parametrize("cfg_id,mode", [(1, 3), (1, 2), (1, 1), (0, 3)])
def test_long_generation_grows_tails_across_tile_boundaries(cfg_id, mode):
    """300 decode steps on a short prompt: every head's tail grows through several 128-row tiles that were
    only reserved at first, the appended row lands in a different tile as it goes, and the combination
    takes more tiles every few steps."""
    wl = make_workload(cfg_id, n_layers=1, shrink=8, steps=300)
    kw = dict(decode_dynamic=mode)
    if cfg_id == 1:
        kw["decode_tile_rows"] = 128
    stats = P.full_pipeline(wl, **kw)
    _say(f"300 steps cfg{cfg_id} mode {mode}", stats)


# ---- two tilings in one cache: small whole-model steps take the large tiles, per-layer calls the small ones ----

@pytest.mark.parametrize("mode", [0, 1, 2])
def test_whole_model_call_takes_large_tiles_and_per_layer_calls_small_ones(mode):
    """Config 1 at full size (28 layers, 8192-token prompt): a call over all layers has more 256-row tiles
    than the device has compute units and fewer 1024-row tiles, so it runs the second tiling; a call per
    layer runs the first.  Both are checked against the oracle on sampled layers at every step, with
    the tails growing through both kinds of call in turn."""
    wl = make_workload(1, steps=4)
    assert wl.n_layers == 28
    layers = [0, 13, 27]
    dw = runner.setup(wl, decode_dynamic=mode)       # 0: the default shape (3 here); 1 and 2 take the same tilings
    tile, mode = dw.cache.decode_shape()
    whole = dw.cache.call_tiling()
    one = dw.cache.call_tiling(5, 6)
    print(f"\n[two tilings] cache tile {tile} mode {mode}; whole-model call {whole}, one layer {one}", flush=True)
    assert tile == 256 and whole[0] == 1024 and one[0] == 256 and whole[1] <= 256
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl)
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    per_layer = [(l, l + 1) for l in range(28)]
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers,
                             layer_ranges_by_step=[None, per_layer, None, [(0, 14), (14, 28)]])
    _say("two tilings", stats)
    dw.cache.close()


@pytest.mark.parametrize("variant", ["indexed", "host_tier"])
def test_large_tiles_with_indexed_generation_and_with_the_host_tier(variant):
    """The 1024-row tiling of a whole-model call together with the variants that change what a dynamic tile
    reads: generated tokens in the chunk index (36 steps complete a 32-token chunk in every dynamic head) and
    prompt rows in host memory.  Config 1 at full size, oracle on sampled layers, every step."""
    steps = 36 if variant == "indexed" else 3
    wl = make_workload(1, steps=steps)
    layers = [5, 20]
    kw = dict(index_generated=1) if variant == "indexed" else dict(host_tier=True)
    dw = runner.setup(wl, decode_dynamic=3, **kw)
    whole = dw.cache.call_tiling()
    assert whole[0] == 1024 and whole[1] <= 256
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl, index_generated=variant == "indexed")
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers)
    _say(f"large tiles, {variant}", stats)
    if variant == "indexed":
        assert stats.get("generated_chunks_indexed", 0) > 0
    dw.cache.close()


def test_large_tiles_with_tail_lengths_kept_on_the_device():
    """Whole-model calls of config 1 at full size (the 1024-row tiling), tail lengths read from the device
    counters as a recorded step needs them: the same bits as with host bookkeeping, step after step, and
    the host mirror is back in step afterwards."""
    wl = make_workload(1, steps=5)
    outs = []
    for device_tail in (False, True):
        dw = runner.setup(wl)
        assert dw.cache.call_tiling()[0] == 1024
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        if device_tail:
            dw.cache.set_device_tail(True)
        out = torch.empty((wl.n_layers, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        res = []
        for s in range(wl.steps):
            q, kn, vn = (runner.to_device(x[s], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
            dw.cache.decode_attn(q, kn, vn, out)
            torch.cuda.synchronize()
            res.append(out.clone())
        outs.append(torch.stack(res))
        if device_tail:
            dw.cache.set_device_tail(False)
            Kr = dw.cache.export(B.HKV_X_K_ROWS, 0, 27, 3)
            assert np.array_equal(Kr[-wl.steps:], wl.k_new[:, 27, 0, 3])
        dw.cache.close()
    assert torch.equal(outs[0], outs[1])


# ---- streamed shape: every workgroup walks an equal share of the step's rows (decode_dynamic = 5) ----

@pytest.mark.parametrize("case", ["cfg1", "ragged", "g8", "small_chunks", "host_tier", "max_group", "layer_calls",
                                  "other_ranges", "tiny"])
def test_streamed_shape(case):
    """The streamed launch on the shapes that stress it: heads spanning several workgroups and workgroups
    spanning several heads (config 1 shape), ragged batch with both chunk sizes, group of eight, many small
    chunks (radix selection), host tier, the other group reading of the chunk score, per-layer calls (a
    table per layer), layer ranges that have no table (they run as tiles) mixed with ones that have, and
    a prompt so small that the call is a single workgroup."""
    kw = dict(decode_dynamic=5)
    if case == "cfg1":
        wl = make_workload(1, n_layers=3, shrink=2, steps=4)
    elif case == "ragged":
        wl = make_workload(4, n_layers=2, shrink=8, steps=3)
    elif case == "g8":
        wl = make_workload(3, n_layers=2, shrink=16, steps=3)
    elif case == "small_chunks":
        wl = make_workload(1, n_layers=2, steps=2)
        wl.chunk_size[:] = 16
        wl.budget[wl.head_type == O.DYNAMIC] = 16 * 300
    elif case == "host_tier":
        wl = make_workload(1, n_layers=2, shrink=2, steps=3)
        kw["host_tier"] = True
    elif case == "max_group":
        wl = make_workload(1, n_layers=2, shrink=2, steps=3)
        kw["chunk_score_group"] = 1
    elif case == "layer_calls":
        wl = make_workload(1, n_layers=3, shrink=4, steps=3)
        kw["layer_ranges"] = [(0, 1), (1, 2), (2, 3)]
    elif case == "other_ranges":
        wl = make_workload(1, n_layers=3, shrink=4, steps=3)
        kw["layer_ranges"] = [(0, 2), (2, 3)]
    else:
        wl = make_workload(1, n_layers=1, shrink=32, steps=3)
    stats = P.full_pipeline(wl, **kw)
    _say(f"streamed shape, {case}", stats)


def test_streamed_shape_long_generation_crosses_the_reference_tail_lengths():
    """300 decode steps on a short prompt: the tail outgrows one table's reference length after another
    (every 32 tokens up to 256, then 384), the appended row moves from share to share, and between two
    reference lengths the last share of every head takes the rows the table did not count."""
    wl = make_workload(1, n_layers=1, shrink=8, steps=300)
    stats = P.full_pipeline(wl, decode_dynamic=5)
    _say("streamed shape, 300 steps", stats)


def test_streamed_shape_at_full_size_whole_model_and_per_layer_calls():
    """Config 1 at full size (28 layers, 8192-token prompt, 768 workgroups over 112 heads): whole-model
    calls and per-layer calls in turn, tails growing through both, oracle on sampled layers at every step;
    then the same steps with the tail lengths kept on the device give the same bits."""
    wl = make_workload(1, steps=4)
    layers = [0, 13, 27]
    dw = runner.setup(wl, decode_dynamic=5)
    whole, one = dw.cache.call_tiling(), dw.cache.call_tiling(5, 6)
    print(f"\n[streamed] whole-model call {whole}, one layer {one}", flush=True)
    assert 1 <= one[1] < whole[1] <= 768
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl)
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    per_layer = [(l, l + 1) for l in range(28)]
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers,
                             layer_ranges_by_step=[None, per_layer, None, [(0, 14), (14, 28)]])
    _say("streamed, full size", stats)
    dw.cache.close()
    outs = []
    for device_tail in (False, True):
        dw = runner.setup(wl, decode_dynamic=5)
        dw.cache.compress(dw.q_window, dw.k, dw.v)
        if device_tail:
            dw.cache.set_device_tail(True)
        out = torch.empty((wl.n_layers, 1, wl.n_q_heads, 128), dtype=torch.bfloat16, device="cuda:0")
        res = []
        for s in range(wl.steps):
            q, kn, vn = (runner.to_device(x[s], wl.dtype) for x in (wl.q_steps, wl.k_new, wl.v_new))
            dw.cache.decode_attn(q, kn, vn, out)
            torch.cuda.synchronize()
            res.append(out.clone())
        outs.append(torch.stack(res))
        if device_tail:
            dw.cache.set_device_tail(False)
            Kr = dw.cache.export(B.HKV_X_K_ROWS, 0, 27, 3)
            assert np.array_equal(Kr[-wl.steps:], wl.k_new[:, 27, 0, 3])
        dw.cache.close()
    assert torch.equal(outs[0], outs[1])


@pytest.mark.parametrize("cfg_id,n_layers,steps", [(2, 2, 3), (3, 2, 2), (4, 1, 2)])
def test_streamed_shape_on_the_larger_shapes_at_full_context(cfg_id, n_layers, steps):
    """Configs 2, 3 and 4 at their real per-head sizes through the streamed launch (oracle on one layer)."""
    wl = make_workload(cfg_id, n_layers=n_layers, steps=steps)
    layers = [n_layers - 1]
    dw = runner.setup(wl, decode_dynamic=5)
    print(f"\n[cfg{cfg_id} streamed] call {dw.cache.call_tiling()}", flush=True)
    dw.cache.compress(dw.q_window, dw.k, dw.v)
    torch.cuda.synchronize()
    ocfg, oplan = P.oracle_setup(wl)
    ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers)
    stats = {}
    overrides = P.compare_compress(wl, dw, ocache, stats)
    if overrides:
        ocache = O.compress(ocfg, oplan, wl.q_window, wl.k, wl.v, wl.is_visual, layers=layers, keep_override=overrides)
    P.run_decode_and_compare(wl, dw, ocache, wl.steps, stats, oracle_layers=layers)
    _say(f"cfg{cfg_id} streamed, full context", stats)
    dw.cache.close()


# ---- classification -> allocation -> plan -> compression -> decode, end to end (Sections 3.1 - 3.3) ----

@pytest.mark.parametrize("cfg_id,n_layers,shrink", [(1, 3, 4), (4, 2, 8)])
def test_scores_to_budgets_to_compressed_decode_end_to_end(cfg_id, n_layers, shrink):
    """The whole chain the paper describes, on the device and in the oracle: sparsity scores of the prompt
    (hkv_head_scores) -> head types at theta = 0.9 and top-down budgets (hkv_allocate_budgets, r = 0.75,
    alpha = 0.5, power-of-two dynamic budgets) -> hkv_plan -> hkv_compress -> hkv_decode_attn, against
    head_scores -> classify_heads -> type_level_budgets / static_head_budgets / dynamic_head_budget ->
    compress -> decode_attn.  Head types must agree wherever the score is not within tolerance of theta;
    the allocation is exact on the device's own scores and within one token (a ceiling's flip) of the
    oracle's own chain; compression and decode then run on the allocated plan on both sides."""
    from hkv_synth import make_prompt_queries
    theta, r, alpha, frac = 0.9, 0.75, 0.5, 0.2
    wl = make_workload(cfg_id, n_layers=n_layers, shrink=shrink, steps=3)
    qp = make_prompt_queries(wl)
    got = _device_head_scores(wl, qp)                                   # [batch, L, Hkv] float32 values
    ocfg = O.OracleConfig(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads, head_dim=128,
                          window=wl.window, dtype=wl.dtype)
    want = O.head_scores(ocfg, wl.cu_seqlens, qp, wl.k, wl.is_visual)
    assert np.abs(got - want).max() <= SCORE_ATOL
    n_heads = wl.n_layers * wl.n_kv_heads
    types_dev = np.zeros((wl.batch, wl.n_layers, wl.n_kv_heads), np.uint8)
    budget_dev = np.zeros((wl.batch, wl.n_layers, wl.n_kv_heads), np.int32)
    flips = 0
    for b in range(wl.batch):
        C = int(wl.seqlens[b])
        b_total = int(np.ceil(frac * C)) * n_heads                       # the paper's B_total for this prompt
        t_dev, bud_dev = B.hkv_allocate_budgets(got[b].reshape(-1), theta, b_total, r, alpha, True)

        def oracle_chain(scores):
            types = O.classify_heads(scores, theta)
            stat = types == O.STATIC
            b_stat, b_dyn = O.type_level_budgets(b_total, int(stat.sum()), int((~stat).sum()), r)
            bud = np.zeros(n_heads, np.int64)
            bud[stat] = O.static_head_budgets(b_stat, scores[stat], alpha)
            bud[~stat] = O.dynamic_head_budget(b_dyn, int((~stat).sum()), pad_pow2=True)
            return types, bud

        # stage-exact: the oracle's equations on the device's own scores
        t_stage, bud_stage = oracle_chain(got[b].reshape(-1).astype(np.float32).astype(np.float64))
        assert np.array_equal(t_dev, t_stage) and np.array_equal(bud_dev.astype(np.int64), bud_stage)
        # end to end: the oracle's own scores
        t_own, bud_own = oracle_chain(want[b].reshape(-1))
        clear = np.abs(want[b].reshape(-1) - theta) > 2 * SCORE_ATOL
        assert np.array_equal(t_dev[clear], t_own[clear])
        if np.array_equal(t_dev, t_own):
            diff = np.abs(bud_dev.astype(np.int64) - bud_own)
            assert diff.max() <= 1, "budgets differ by more than a ceiling's flip"
            flips += int((diff != 0).sum())
        types_dev[b] = t_dev.reshape(wl.n_layers, wl.n_kv_heads)
        budget_dev[b] = bud_dev.reshape(wl.n_layers, wl.n_kv_heads)
    # the generator's sparse heads come out static, its diffuse ones dynamic
    assert np.array_equal(types_dev, wl.head_type)
    assert (types_dev == O.STATIC).any() and (types_dev == O.DYNAMIC).any()
    stats = P.full_pipeline(wl, budget=budget_dev, head_type=types_dev)
    stats["budget_ceiling_flips"] = flips
    _say(f"scores -> budgets -> compress -> decode, cfg{cfg_id}/{shrink}", stats)
