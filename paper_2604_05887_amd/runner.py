"""Moves a synthetic workload (hkv_synth.Workload, host numpy arrays) onto the GPU and wires it
to the C ABI.  Memory plumbing only: no step of the method is computed here."""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Dict, Optional, Sequence

import numpy as np
import torch

from . import binding as B


def torch_dtype(dtype: str):
    return torch.bfloat16 if dtype == "bf16" else torch.float32


def hkv_dtype(dtype: str) -> int:
    return B.HKV_BF16 if dtype == "bf16" else B.HKV_F32


def to_device(x: np.ndarray, dtype: str, device="cuda:0") -> torch.Tensor:
    """float32 host array whose values are exact in `dtype` -> device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32))
    return t.to(device=device, dtype=torch_dtype(dtype)).contiguous()


def to_host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


@dataclass
class DeviceWorkload:
    cfg: B.hkv_config
    plan: B.PlanArrays
    cache: B.HybridKVCache
    q_window: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    dtype: str


def setup(wl, device="cuda:0", budget: Optional[np.ndarray] = None, head_type: Optional[np.ndarray] = None,
          score_causal: int = 0, upload_prompt: bool = True, decode_tile_rows: int = 0,
          decode_dynamic: int = 0, host_tier: bool = False, chunk_score_group: int = 0,
          index_generated: int = 0) -> DeviceWorkload:
    cfg = B.make_config(n_layers=wl.n_layers, n_q_heads=wl.n_q_heads, n_kv_heads=wl.n_kv_heads,
                        dtype=hkv_dtype(wl.dtype), window=wl.window, chunk_size=int(wl.chunk_size[0]),
                        max_new_tokens=wl.max_new_tokens, score_causal=score_causal,
                        decode_tile_rows=decode_tile_rows, decode_dynamic=decode_dynamic,
                        chunk_score_group=chunk_score_group, index_generated=index_generated)
    plan = B.PlanArrays(wl.cu_seqlens, wl.is_visual, wl.head_type if head_type is None else head_type,
                        wl.budget if budget is None else budget, wl.chunk_size)
    cache = B.HybridKVCache(cfg, plan, device=device, host_tier=host_tier)
    if upload_prompt:
        qw, k, v = (to_device(wl.q_window, wl.dtype, device), to_device(wl.k, wl.dtype, device),
                    to_device(wl.v, wl.dtype, device))
    else:
        qw = k = v = None
    return DeviceWorkload(cfg=cfg, plan=plan, cache=cache, q_window=qw, k=k, v=v, dtype=wl.dtype)


def tune_decode_dynamic(caches: Sequence, step_fn: Callable[[object, int], None], modes=(1, 2, 3, 4, 5), steps: int = 24,
                        warmup: int = 6) -> Dict[int, float]:
    """Time the ways a decode step can run on the caller's own caches and keep the fastest on all of
    them (mode 4 exists for bf16 caches only and is skipped elsewhere).  step_fn(cache_holder, i) issues one step WITHOUT appending (k_new = None),
    so the caches come out unchanged; the caches are visited in rotation, as a benchmark that defeats the
    memory-side cache does.  Returns {mode: microseconds per step}."""
    result: Dict[int, float] = {}
    for m in modes:
        if m >= 4 and caches[0].cfg.dtype != B.HKV_BF16:
            continue
        try:
            for c in caches:
                c.cache.set_decode_dynamic(m)
        except B.HkvError:            # a shape this cache does not support
            continue
        for i in range(warmup):
            step_fn(caches[i % len(caches)], i)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(steps):
            step_fn(caches[(warmup + i) % len(caches)], i)
        e1.record()
        torch.cuda.synchronize()
        result[m] = e0.elapsed_time(e1) / steps * 1e3
    best = min(result, key=result.get)
    for c in caches:
        c.cache.set_decode_dynamic(best)
    return result
