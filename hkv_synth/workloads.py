"""Seeded synthetic workloads shaped like the paper's Qwen2.5-VL runs.

The paper measures on multimodal prompts (tens of images, or 64 video frames,
plus a text instruction; Section 4 "Tasks and Models", Table 3).  Those data
sets and the model weights are not available here, so every tensor is drawn
from a seeded generator with the same shapes, token layout (text prefix,
visual blocks, text suffix ending in the observation window), head-type mix
and budget structure.  Nothing in this module evaluates the method: it only
produces inputs (Q/K/V values, modality mask, head types, per-head budgets).

Budgets follow the top-down allocation of Section 3.2 (type-level split, then
score-proportional static budgets, power-of-two dynamic budgets) driven by
*synthetic* head importance weights, because the real weights come from head
classification, which is upstream of the hot path.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional

import numpy as np

STATIC = 0
DYNAMIC = 1
HEAD_DIM = 128


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); returns float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((bits >> np.uint32(16)) & np.uint32(1))
    out = ((bits + bias) & np.uint32(0xFFFF0000)).view(np.float32)
    return out.reshape(x.shape)


def _cast(x: np.ndarray, dtype: str) -> np.ndarray:
    return bf16_round(x) if dtype == "bf16" else np.ascontiguousarray(x, dtype=np.float32)


def token_layout(n_visual: int, n_text: int, block: int, sep: int, prefix: int = 64) -> np.ndarray:
    """Modality mask for one prompt: 1 = visual token, 0 = text token.

    Layout: `prefix` text tokens, then visual blocks of `block` tokens with
    `sep` text tokens between consecutive blocks (sep = 0 for video frames),
    then the remaining text as a suffix (which holds the observation window).
    """
    n_blocks = max(1, math.ceil(n_visual / block))
    n_sep = sep * (n_blocks - 1)
    prefix = min(prefix, max(0, n_text - n_sep - 1))
    suffix = n_text - prefix - n_sep
    if suffix < 0:
        raise ValueError("not enough text tokens for the requested layout")
    parts: List[np.ndarray] = [np.zeros(prefix, np.uint8)]
    left = n_visual
    for bi in range(n_blocks):
        n = min(block, left)
        parts.append(np.ones(n, np.uint8))
        left -= n
        if bi + 1 < n_blocks:
            parts.append(np.zeros(sep, np.uint8))
    parts.append(np.zeros(suffix, np.uint8))
    out = np.concatenate(parts)
    assert out.size == n_visual + n_text and int(out.sum()) == n_visual
    return out


def pow2_nearest(x: float) -> int:
    """Nearest power of two in linear distance, ties upwards (>= 1)."""
    if x <= 1:
        return 1
    lo = 1 << int(math.floor(math.log2(x)))
    hi = lo * 2
    return lo if (x - lo) < (hi - x) else hi


# ----------------------------------------------------------------------------
# Named configurations (the five shapes the benchmark description lists).
# ----------------------------------------------------------------------------
CONFIGS: Dict[int, dict] = {
    0: dict(name="cfg0_tiny_f32", dtype="f32", n_layers=1, n_q_heads=28, n_kv_heads=4, batch=1,
            n_visual=[1536], n_text=[512], block=1536, sep=16, window=32, chunk=[32],
            budget_frac=[0.10], k_chunks=4, static_frac=0.5, fixed_types=[0, 0, 1, 1],
            hierarchical=False, steps=16, q_mode="normal"),
    1: dict(name="cfg1_qwen7b_8k_bf16", dtype="bf16", n_layers=28, n_q_heads=28, n_kv_heads=4, batch=1,
            n_visual=[6656], n_text=[1536], block=6656, sep=16, window=32, chunk=[32],
            budget_frac=[0.10], k_chunks=None, static_frac=0.5, fixed_types=None,
            hierarchical=True, steps=128, q_mode="normal"),
    2: dict(name="cfg2_multi_image_32k_bf16", dtype="bf16", n_layers=28, n_q_heads=28, n_kv_heads=4, batch=4,
            n_visual=[30720] * 4, n_text=[2048] * 4, block=1536, sep=16, window=32, chunk=[64] * 4,
            budget_frac=[0.10] * 4, k_chunks=8, static_frac=0.5, fixed_types=None,
            hierarchical=True, steps=16, q_mode="centroid"),
    3: dict(name="cfg3_video_72b_bf16", dtype="bf16", n_layers=80, n_q_heads=64, n_kv_heads=8, batch=1,
            n_visual=[48000], n_text=[3200], block=750, sep=0, window=32, chunk=[64],
            budget_frac=[0.05], k_chunks=16, static_frac=0.4, fixed_types=None,
            hierarchical=True, steps=16, q_mode="normal"),
    4: dict(name="cfg4_serving_mix_bf16", dtype="bf16", n_layers=28, n_q_heads=28, n_kv_heads=4, batch=16,
            n_visual=None, n_text=None, block=1536, sep=16, window=32, chunk=None,
            budget_frac=None, k_chunks=None, static_frac=0.5, fixed_types=None,
            hierarchical=True, steps=256, q_mode="normal"),
}


@dataclass
class Workload:
    name: str
    dtype: str                      # "f32" | "bf16": values are exactly representable in it
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    batch: int
    seqlens: np.ndarray             # [batch] int32
    cu_seqlens: np.ndarray          # [batch+1] int32
    chunk_size: np.ndarray          # [batch] int32, power of two
    is_visual: np.ndarray           # [total_tokens] uint8
    head_type: np.ndarray           # [batch, n_layers, n_kv_heads] uint8 (0 static, 1 dynamic)
    budget: np.ndarray              # [batch, n_layers, n_kv_heads] int32 tokens
    budget_rule: str
    budget_frac: np.ndarray         # [batch] nominal fraction
    max_new_tokens: int
    steps: int
    q_window: np.ndarray            # [L, batch, w, Hq, d] float32
    k: np.ndarray                   # [L, total_tokens, Hkv, d] float32
    v: np.ndarray                   # [L, total_tokens, Hkv, d] float32
    q_steps: np.ndarray             # [steps, L, batch, Hq, d]
    k_new: np.ndarray               # [steps, L, batch, Hkv, d]
    v_new: np.ndarray               # [steps, L, batch, Hkv, d]
    planted: Dict[tuple, np.ndarray] = field(default_factory=dict)  # (b,l,h) -> planted positions
    seed: int = 0

    @property
    def total_tokens(self) -> int:
        return int(self.cu_seqlens[-1])

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


def allocate_budgets(rng: np.random.Generator, *, rule: str, hierarchical: bool, head_type: np.ndarray,
                     n_ctx: int, n_text_hist: int, n_vis_hist: int, window: int, frac: float,
                     chunk: int, k_chunks: Optional[int], alpha: float = 0.5, r: float = 0.75) -> np.ndarray:
    """Per-(layer, KV head) token budgets for one sequence (Section 3.2, Eq. 4-5).

    rule = "text_exempt": window and historical text are always complete and the
      nominal fraction applies to the visual tokens of static heads;
    rule = "literal_total": the nominal fraction is the total retained fraction of
      the whole context, split by Eq. 4 (r) and Eq. 5 (alpha).
    Head importance (the normalised sparsity score of Eq. 5) is synthetic:
    layer weights ~ Dirichlet(1), head weights ~ Dirichlet(1) within a layer.
    """
    n_layers, n_heads = head_type.shape
    stat = head_type == STATIC
    n_stat, n_dyn = int(stat.sum()), int((~stat).sum())
    budget = np.zeros((n_layers, n_heads), np.int64)

    # synthetic normalised importance over all static heads (sums to 1)
    s_tilde = np.zeros((n_layers, n_heads))
    if n_stat:
        if hierarchical:
            lam = rng.dirichlet(np.ones(n_layers))
            for l in range(n_layers):
                idx = np.nonzero(stat[l])[0]
                if idx.size:
                    s_tilde[l, idx] = lam[l] * rng.dirichlet(np.ones(idx.size))
            s_tilde /= s_tilde.sum()
        else:
            s_tilde[stat] = 1.0 / n_stat

    if k_chunks is None:
        dyn_tokens = pow2_nearest(r * math.ceil(frac * n_ctx))
    else:
        dyn_tokens = k_chunks * chunk
    dyn_tokens = max(chunk, min(dyn_tokens, (n_ctx // chunk) * chunk if n_ctx >= chunk else chunk))

    if rule == "text_exempt":
        b_stat = n_stat * math.ceil(frac * n_vis_hist)
        for l in range(n_layers):
            for h in range(n_heads):
                if stat[l, h]:
                    m = math.ceil(alpha * b_stat / n_stat - 1e-9 + (1 - alpha) * b_stat * s_tilde[l, h])
                    m = min(m, n_vis_hist)
                    budget[l, h] = window + n_text_hist + m
                else:
                    budget[l, h] = dyn_tokens
    elif rule == "literal_total":
        b_bar = math.ceil(frac * n_ctx)
        b_total = b_bar * (n_stat + n_dyn)
        b_stat = b_total - n_dyn * dyn_tokens
        for l in range(n_layers):
            for h in range(n_heads):
                if stat[l, h]:
                    b = math.ceil(alpha * b_stat / n_stat - 1e-9 + (1 - alpha) * b_stat * s_tilde[l, h])
                    budget[l, h] = max(1, min(b, n_ctx))
                else:
                    budget[l, h] = dyn_tokens
    else:
        raise ValueError(rule)
    return budget.astype(np.int32)


def make_workload(cfg_id: int, seed: Optional[int] = None, *, budget_rule: str = "text_exempt",
                  n_layers: Optional[int] = None, steps: Optional[int] = None,
                  shrink: int = 1, budget_frac: Optional[float] = None,
                  head_mix: Optional[str] = None, max_new_tokens: Optional[int] = None,
                  tensors: bool = True) -> Workload:
    """Build configuration `cfg_id` (0..4).

    `n_layers`, `steps` and `shrink` (divide every sequence's visual/text counts by
    it) give smaller variants with the same structure for parity tests.
    `head_mix` in {"all_static", "all_dynamic"} overrides the head-type map.
    `tensors=False` builds only the layout, head types and budgets (Q/K/V fields are None): the
    benchmark then draws the large configurations' tensors on the device.
    """
    c = dict(CONFIGS[cfg_id])
    seed = cfg_id if seed is None else seed
    rng = np.random.default_rng(np.random.SeedSequence([0x48594B56, cfg_id, seed]))
    L = n_layers or c["n_layers"]
    Hq, Hkv, d = c["n_q_heads"], c["n_kv_heads"], HEAD_DIM
    G = Hq // Hkv
    B = c["batch"]
    w = c["window"]
    n_steps = steps if steps is not None else c["steps"]
    dtype = c["dtype"]

    if cfg_id == 4:
        ctx = rng.integers(4096, 40960, size=B, endpoint=True)
        vfrac = rng.uniform(0.6, 0.9, size=B)
        n_vis = np.round(ctx * vfrac).astype(np.int64)
        n_txt = ctx - n_vis
        chunk = rng.choice([32, 64], size=B)
        fracs = rng.uniform(0.05, 0.20, size=B)
    else:
        n_vis = np.array(c["n_visual"], np.int64)
        n_txt = np.array(c["n_text"], np.int64)
        chunk = np.array(c["chunk"], np.int64)
        fracs = np.array(c["budget_frac"], np.float64)
    if budget_frac is not None:
        fracs = np.full(B, budget_frac)
    if shrink > 1:
        n_vis = np.maximum(n_vis // shrink, 64)
        n_txt = np.maximum(n_txt // shrink, w + 80)
    block = max(16, c["block"] // shrink) if shrink > 1 else c["block"]

    masks = [token_layout(int(n_vis[b]), int(n_txt[b]), block, c["sep"]) for b in range(B)]
    seqlens = np.array([m.size for m in masks], np.int32)
    cu = np.zeros(B + 1, np.int32)
    cu[1:] = np.cumsum(seqlens)
    is_visual = np.concatenate(masks)
    total = int(cu[-1])

    # head types
    head_type = np.zeros((B, L, Hkv), np.uint8)
    for b in range(B):
        if head_mix == "all_static":
            head_type[b] = STATIC
        elif head_mix == "all_dynamic":
            head_type[b] = DYNAMIC
        elif c["fixed_types"] is not None:
            head_type[b, :, :] = np.array(c["fixed_types"], np.uint8)[None, :]
        elif abs(c["static_frac"] - 0.5) < 1e-9:
            for l in range(L):
                perm = rng.permutation(Hkv)
                head_type[b, l, perm[Hkv // 2:]] = DYNAMIC
        else:
            flat = np.full(L * Hkv, DYNAMIC, np.uint8)
            n_stat = int(round(c["static_frac"] * L * Hkv))
            flat[rng.permutation(L * Hkv)[:n_stat]] = STATIC
            head_type[b] = flat.reshape(L, Hkv)

    # budgets
    budget = np.zeros((B, L, Hkv), np.int32)
    for b in range(B):
        m = masks[b]
        C = m.size
        hist = m[: C - w]
        budget[b] = allocate_budgets(
            rng, rule=budget_rule, hierarchical=c["hierarchical"], head_type=head_type[b], n_ctx=C,
            n_text_hist=int((hist == 0).sum()), n_vis_hist=int((hist == 1).sum()), window=w,
            frac=float(fracs[b]), chunk=int(chunk[b]), k_chunks=c["k_chunks"])

    if not tensors:
        return Workload(
            name=c["name"] + (f"_shrink{shrink}" if shrink > 1 else "") + (f"_L{L}" if L != c["n_layers"] else ""),
            dtype=dtype, n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, window=w, batch=B,
            seqlens=seqlens, cu_seqlens=cu, chunk_size=chunk.astype(np.int32), is_visual=is_visual,
            head_type=head_type, budget=budget, budget_rule=budget_rule, budget_frac=fracs,
            max_new_tokens=max_new_tokens if max_new_tokens is not None else max(n_steps, 1), steps=n_steps,
            q_window=None, k=None, v=None, q_steps=None, k_new=None, v_new=None, planted={}, seed=seed)

    # tensors
    def normal(shape):
        return rng.standard_normal(shape, dtype=np.float32)

    k = normal((L, total, Hkv, d))
    v = normal((L, total, Hkv, d))
    q_window = normal((L, B, w, Hq, d))
    planted: Dict[tuple, np.ndarray] = {}
    for b in range(B):
        m = masks[b]
        C = m.size
        vis_pos = np.nonzero(m[: C - w])[0]
        n_plant = int(round(0.05 * vis_pos.size))
        for l in range(L):
            for h in range(Hkv):
                if head_type[b, l, h] != STATIC or n_plant == 0:
                    continue
                u = rng.standard_normal(d)
                u = (u / np.linalg.norm(u)).astype(np.float32)
                pos = np.sort(rng.choice(vis_pos, size=n_plant, replace=False))
                k[l, cu[b] + pos, h, :] += 3.0 * u
                q_window[l, b, :, h * G:(h + 1) * G, :] += math.sqrt(d) * u
                planted[(b, l, h)] = pos
    k = _cast(k, dtype)
    v = _cast(v, dtype)
    q_window = _cast(q_window, dtype)

    q_steps = normal((n_steps, L, B, Hq, d))
    if c["q_mode"] == "centroid":
        for b in range(B):
            C = int(seqlens[b])
            cs = int(chunk[b])
            n_c = (C + cs - 1) // cs
            for l in range(L):
                for h in range(Hkv):
                    if head_type[b, l, h] != DYNAMIC:
                        continue
                    picks = rng.integers(0, n_c, size=n_steps)
                    for s in range(n_steps):
                        lo = cu[b] + picks[s] * cs
                        hi = min(cu[b] + C, lo + cs)
                        cen = k[l, lo:hi, h, :].mean(axis=0, dtype=np.float64).astype(np.float32)
                        q_steps[s, l, b, h * G:(h + 1) * G, :] = cen + 0.5 * q_steps[s, l, b, h * G:(h + 1) * G, :]
    q_steps = _cast(q_steps, dtype)
    k_new = _cast(normal((n_steps, L, B, Hkv, d)), dtype)
    v_new = _cast(normal((n_steps, L, B, Hkv, d)), dtype)

    return Workload(
        name=c["name"] + (f"_shrink{shrink}" if shrink > 1 else "") + (f"_L{L}" if L != c["n_layers"] else ""),
        dtype=dtype, n_layers=L, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, window=w, batch=B,
        seqlens=seqlens, cu_seqlens=cu, chunk_size=chunk.astype(np.int32), is_visual=is_visual,
        head_type=head_type, budget=budget, budget_rule=budget_rule, budget_frac=fracs,
        max_new_tokens=max_new_tokens if max_new_tokens is not None else max(n_steps, 1), steps=n_steps,
        q_window=q_window, k=k, v=v, q_steps=q_steps, k_new=k_new, v_new=v_new, planted=planted, seed=seed)


def make_prompt_queries(wl: Workload, seed: int = 0, sharp_gain: float = 2.5) -> np.ndarray:
    """Queries of the whole prompt, [L, total_tokens, Hq, d] (float32 holding dtype-exact values), for the
    head-classification step that runs before the compression.

    N(0,1) everywhere; on the query heads of KV heads marked static in the workload, the text tokens'
    queries additionally point at that head's planted keys (along the mean planted key, which is the
    planted direction up to noise), so that their attention concentrates on about 5 % of the visual
    tokens and the head comes out sparse; the other heads stay diffuse.  Needs wl.k and wl.planted.
    """
    rng = np.random.default_rng([0x48594B51, int(wl.seed if wl.seed is not None else 0), int(seed)])
    L, Hq, Hkv, d = wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim
    G = Hq // Hkv
    total = int(wl.cu_seqlens[-1])
    q = rng.standard_normal((L, total, Hq, d), dtype=np.float32)
    for (b, l, h), pos in wl.planted.items():
        if pos.size == 0:
            continue
        s0, s1 = int(wl.cu_seqlens[b]), int(wl.cu_seqlens[b + 1])
        direction = wl.k[l, s0 + pos, h, :].astype(np.float64).mean(axis=0)
        direction /= np.linalg.norm(direction)
        text = s0 + np.nonzero(wl.is_visual[s0:s1] == 0)[0]
        q[l, text[:, None], np.arange(h * G, (h + 1) * G)[None, :], :] += (sharp_gain * math.sqrt(d) * direction).astype(np.float32)
    return _cast(q, wl.dtype)
