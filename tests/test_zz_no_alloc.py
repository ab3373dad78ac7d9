"""GPU check of hkv_decode_attn_noalloc, the decode entry point for callers that cannot allocate device
memory or pass a workspace: its split-K records live in an array inside the library.  Its output must be
that of hkv_decode_attn (same kernels, same order: bit for bit) and within the oracle's tolerance, on
calls in a row that share the library's array -- a larger cache first, then smaller ones and a
sub-range of layers -- and a call whose records do not fit must be refused before anything is enqueued."""
import numpy as np
import pytest
import torch

from hkv_synth import make_workload
from paper_2604_05887_amd import binding as B
from paper_2604_05887_amd import runner

import parity_utils as P
from oracle import hybridkv_oracle as O

pytestmark = pytest.mark.gpu


def _pair(wl, **kw):
    """Two caches of the same prompt, compressed alike: one for each entry point."""
    a, b = runner.setup(wl, **kw), runner.setup(wl, **kw)
    for dw in (a, b):
        dw.cache.compress(dw.q_window, dw.k, dw.v)
    return a, b


def _step_both(wl, a, b, s, layer_begin=0, layer_end=None, append=True):
    le = wl.n_layers if layer_end is None else layer_end
    q = runner.to_device(wl.q_steps[s], wl.dtype)
    kn = runner.to_device(wl.k_new[s], wl.dtype) if append else None
    vn = runner.to_device(wl.v_new[s], wl.dtype) if append else None
    shape = (wl.n_layers, wl.batch, wl.n_q_heads, wl.head_dim)
    out_a = torch.zeros(shape, dtype=runner.torch_dtype(wl.dtype), device="cuda:0")
    out_b = torch.zeros(shape, dtype=runner.torch_dtype(wl.dtype), device="cuda:0")
    sl = slice(layer_begin, le)
    a.cache.decode_attn(q[sl], None if kn is None else kn[sl], None if vn is None else vn[sl], out_a[sl],
                        layer_begin=layer_begin, layer_end=le)
    b.cache.decode_attn_noalloc(q[sl], None if kn is None else kn[sl], None if vn is None else vn[sl], out_b[sl],
                                layer_begin=layer_begin, layer_end=le)
    torch.cuda.synchronize()
    return out_a, out_b


@pytest.mark.parametrize("mode", [3, 1, 2, 5])
def test_noalloc_entry_point_matches_the_workspace_entry_point(mode):
    big = make_workload(1, n_layers=3, shrink=4, steps=4)          # several tiles per head, bf16
    # the second, smaller input: one fp32 layer (far fewer, smaller records); fp32 caches have no streamed shape
    small = make_workload(0, shrink=4, steps=3)
    print(f"\n[noalloc] mode={mode} big={big.name} small={small.name}", flush=True)
    big_a, big_b = _pair(big, decode_dynamic=mode)
    small_a, small_b = _pair(small, decode_dynamic=3 if mode == 5 else mode)
    ocfg, oplan = P.oracle_setup(big)
    ocache = O.compress(ocfg, oplan, big.q_window, big.k, big.v, big.is_visual)
    kept_same = all(np.array_equal(big_b.cache.export(B.HKV_X_KEPT_IDX, *key), u.kept)
                    for key, u in ocache.units.items() if u.kind == O.STATIC)
    for s in range(3):
        # first call: the larger input; second call straight after it: a smaller one (the array still
        # holds the first call's records)
        oa, ob = _step_both(big, big_a, big_b, s)
        assert torch.equal(oa, ob), f"step {s}: big cache differs"
        if kept_same and s == 0:
            ref, info = O.decode_attn(ocache, big.q_steps[s], big.k_new[s], big.v_new[s])
            picks_same = all(np.array_equal(big_b.cache.export(B.HKV_X_CHUNK_SEL, *key), v["sel"])
                             for key, v in info.items())
            if picks_same:
                got = runner.to_host_f32(ob).astype(np.float64)
                err = np.abs(got - ref).max(axis=-1) / np.abs(ref).max(axis=-1)
                assert err.max() <= P.OUT_TOL[big.dtype]
        oa, ob = _step_both(small, small_a, small_b, s)
        assert torch.equal(oa, ob), f"step {s}: small cache differs"
        # a sub-range of the big cache's layers, without an append: smaller again
        oa, ob = _step_both(big, big_a, big_b, s + 1, layer_begin=1, layer_end=2, append=False)
        assert torch.equal(oa, ob), f"step {s}: layer sub-range differs"
    # the caches advanced in lockstep
    for key in [(0, 0, 0), (0, 2, 3)]:
        assert np.array_equal(big_a.cache.export(B.HKV_X_K_ROWS, *key), big_b.cache.export(B.HKV_X_K_ROWS, *key))
    for dw in (big_a, big_b, small_a, small_b):
        dw.cache.close()


def test_noalloc_entry_point_refuses_what_does_not_fit_and_checks_arguments():
    # 64 short prompts x 4 layers x 4 heads, every head keeping everything, 128-row tiles: ~17 K tiles whose
    # records (3648 bytes each) exceed the library's array
    n_seq, L, C = 64, 4, 2048
    cu = np.arange(n_seq + 1, dtype=np.int32) * C
    vis = np.ones(n_seq * C, np.uint8)
    vis[:: 4] = 0
    head_type = np.zeros((n_seq, L, 4), np.uint8)
    budget = np.full((n_seq, L, 4), C, np.int32)
    cfg = B.make_config(n_layers=L, n_q_heads=28, n_kv_heads=4, dtype=B.HKV_BF16, window=32, chunk_size=32,
                        max_new_tokens=8, decode_tile_rows=128, decode_dynamic=3)
    plan = B.PlanArrays(cu, vis, head_type, budget, np.full(n_seq, 32, np.int32))
    cache = B.HybridKVCache(cfg, plan)
    _, n_tiles = cache.call_tiling()
    assert n_tiles * (7 * 512 + 64) > B.HKV_NOALLOC_SCRATCH_BYTES
    q = torch.zeros((L, n_seq, 28, 128), dtype=torch.bfloat16, device="cuda:0")
    out = torch.zeros_like(q)
    with pytest.raises(B.HkvError) as ei:
        cache.decode_attn_noalloc(q, None, None, out)
    assert ei.value.status == B.HKV_ENOSPACE
    # one layer of it fits the array, but the cache has not been compressed: refused as out of order
    _, n_tiles1 = cache.call_tiling(0, 1)
    assert n_tiles1 * (7 * 512 + 64) <= B.HKV_NOALLOC_SCRATCH_BYTES
    with pytest.raises(B.HkvError) as ei:
        cache.decode_attn_noalloc(q[:1], None, None, out[:1], layer_begin=0, layer_end=1)
    assert ei.value.status == B.HKV_ESTATE
    with pytest.raises(B.HkvError) as ei:
        cache.decode_attn_noalloc(q[:1], q[:1], None, out[:1], layer_begin=0, layer_end=1)
    assert ei.value.status == B.HKV_EINVAL
    cache.close()
