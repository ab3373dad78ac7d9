"""CPU oracle for the HybridKV hot path (test infrastructure, not the product).

A plain, slow, double-precision restatement of what the paper defines for
hybrid KV-cache compression (Section 3.3 and Appendix A) and of the decode
attention that runs over the compressed cache.  Only tests, the smoke check and
the benchmark's cpu_baseline leg may use it; the HIP library never does, and
this file shares no code, tables or helpers with it.

Every routine works on one (sequence, layer, KV head) unit at a time, in the
order and notation of the paper:

  * window_scores      Appendix A, the two equations for S_w and s_w
                       (observation-window softmax attention, averaged rows)
  * static_keep_set    Appendix A, static heads: the retained set is the union
                       of the window, the historical text and the Top-M
                       historical visual tokens
  * chunk_means        Appendix A, dynamic heads: a chunk's summary is the mean
                       of its key vectors
  * chunk_scores       Appendix A, dynamic heads: a chunk is scored by the dot
                       product of the query with its summary
  * select_chunks      Appendix A, dynamic heads: how many chunks are loaded
                       follows from the head's budget and the chunk size
  * attention          ordinary softmax attention over the retained rows
                       (Section 3.3: static and dynamic parts share one buffer
                       and are attended together)

  * text_sparsity_score  Section 3.1, text-centric attention S_text and the
                       sparsity score S_{l,h} (sum of each text row's top-k
                       probabilities, averaged over text rows)
  * cumulative_focus   Section 2.1, Eq. 1: how often each context token is among a
                       head's k most attended tokens over N decoding steps
  * classify_heads     Section 3.1, threshold theta on S_{l,h}
  * type_level_budgets / static_head_budgets
                       Section 3.2, the two allocation equations

Where the paper is silent the reading taken is written next to the code
(grouped-query heads, ties, budgets smaller than text + window, ragged last
chunk, rounding of the chunk metadata); the same list is in the design notes.

Pinning status.  window_scores, static_keep_set, top_indices, chunk_means,
chunk_scores, select_chunks, attention and the compress/decode drivers are
pinned by tests that do not restate their formulas: textbook softmax attention
from an independent library at full budget, closed forms (uniform scores,
rational softmax values worked by hand), brute-force subset enumeration,
chunk size 1, permutation invariance and count invariants.  The paper prints no
worked numeric example for this path, so beyond those pins the actual values of
s_w and of the attention outputs are "parity unpinned".
text_sparsity_score is pinned by closed forms (uniform rows give k/C, k = C
gives 1, a one-hot row gives 1), by a sort-based restatement on random inputs
and by hand-worked rational softmax rows; the budget equations by their printed
invariants (type budgets add up to the total, r = 1 and equal scores give the
uniform split, every ceiling is at most one token above its argument).
selection_margin is pinned by a hand case and by its relation to a library sort; the
keep_override / sel_override hooks of the drivers by library softmax attention over
hand-chosen rows.
The indexed-generation variant of decode_attn is pinned by its reductions (no complete
chunk: the plain reading; room for every chunk: library softmax attention over everything)
and a hand-built retrieval case.
cumulative_focus is pinned by a hand-worked case, by the argmax histogram for
k = 1, by a library top-k on the logits, and by its count invariants.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np

STATIC = 0
DYNAMIC = 1


# ----------------------------------------------------------------------------
# value rounding
# ----------------------------------------------------------------------------
def round_to_dtype(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 values to `dtype` ("f32" or "bf16"), nearest-even, in ONE step.

    bf16 keeps 8 significand bits (7 stored); going through float32 first could
    round twice, so the bf16 case works on the float64 bit pattern directly.
    """
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32).astype(np.float64)
    if dtype != "bf16":
        raise ValueError(dtype)
    a = np.abs(x)
    if np.any((a != 0) & (a < 2.0 ** -126)) or np.any(a > 3.38e38):
        raise ValueError("value outside the bf16 normal range")
    bits = np.ascontiguousarray(x).view(np.uint64)
    drop = np.uint64(45)                       # 52 stored float64 bits -> 7 stored bf16 bits
    half_minus_one = np.uint64((1 << 44) - 1)
    odd = (bits >> drop) & np.uint64(1)
    rounded = (bits + half_minus_one + odd) & ~np.uint64((1 << 45) - 1)
    return rounded.view(np.float64).reshape(x.shape)


# ----------------------------------------------------------------------------
# selection with the lowest-index tie-break
# ----------------------------------------------------------------------------
def top_indices(scores: np.ndarray, candidates: np.ndarray, m: int) -> np.ndarray:
    """The m candidate positions with the largest scores; equal scores go to the
    lower position.  `candidates` is an ascending index array.  Returns the chosen
    positions in ascending order.  Comparisons are exact in the scores' own type."""
    candidates = np.asarray(candidates, dtype=np.int64)
    if m <= 0:
        return np.zeros(0, np.int64)
    if m >= candidates.size:
        return candidates.copy()
    vals = np.asarray(scores)[candidates]
    # stable sort by descending value: among equal values the ascending candidate order survives
    order = np.argsort(-vals, kind="stable")
    return np.sort(candidates[order[:m]])


def selection_margin(scores: np.ndarray, candidates: np.ndarray, m: int) -> Tuple[float, float]:
    """(value of the m-th largest candidate, value of the (m+1)-th), for judging how
    close a selection is to a tie.  (+inf, -inf) when nothing is cut off."""
    candidates = np.asarray(candidates, dtype=np.int64)
    if m <= 0 or m >= candidates.size:
        return float("inf"), float("-inf")
    vals = np.sort(np.asarray(scores, dtype=np.float64)[candidates])[::-1]
    return float(vals[m - 1]), float(vals[m])


# ----------------------------------------------------------------------------
# prefill: static heads
# ----------------------------------------------------------------------------
def window_scores(q_win: np.ndarray, k: np.ndarray, scale: float, causal: bool = False) -> np.ndarray:
    """Relevance vector s_w over all C prompt tokens (Appendix A, S_w and s_w).

    q_win : [G, w, d]  queries of the last w prompt positions for the G query heads
            that share this KV head (the paper writes one head; with grouped-query
            attention the rows of all G heads are averaged together),
    k     : [C, d]     keys of the whole prompt.
    S_w = softmax(Q[C-w:C] K^T * scale) row by row over ALL C keys; s_w is the
    mean of its rows.  `causal` masks key j > C-w+i for window row i (the paper
    prints no mask; the default follows the paper).
    """
    q = np.asarray(q_win, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    G, w, d = q.shape
    C = kk.shape[0]
    logits = np.einsum("gid,jd->gij", q, kk) * scale            # [G, w, C]
    if causal:
        j = np.arange(C)[None, None, :]
        i = np.arange(w)[None, :, None]
        logits = np.where(j > C - w + i, -np.inf, logits)
    logits = logits - logits.max(axis=2, keepdims=True)
    e = np.exp(logits)
    S_w = e / e.sum(axis=2, keepdims=True)                        # each row sums to 1
    return S_w.reshape(G * w, C).sum(axis=0) / (G * w)


def retained_count(C: int, w: int, n_text_hist: int, n_vis_hist: int, budget: int) -> int:
    """How many prompt tokens a static head keeps under `budget` (a total count that
    includes the window and the historical text, Appendix A)."""
    if budget < w:
        return max(int(budget), 0)
    m = budget - w - n_text_hist
    if m < 0:
        return int(budget)
    return int(w + n_text_hist + min(m, n_vis_hist))


def static_keep_set(s_w: np.ndarray, is_visual: np.ndarray, w: int, budget: int) -> np.ndarray:
    """Ascending prompt positions a static head keeps (Appendix A, static heads).

    Keep = window (last w positions) + every text token before the window +
    the Top-M visual tokens before the window by s_w, M = budget - w - #text.
    Outside the paper's regime (the budget does not even cover window + text)
    text keeps its priority over visual tokens (Section 3.3): M = 0 and the
    budget that is left after the window goes to the historical text tokens with
    the largest s_w; a budget below w keeps the last `budget` positions.
    """
    is_visual = np.asarray(is_visual).astype(bool)
    C = is_visual.size
    hist = np.arange(C - w)
    win = np.arange(C - w, C)
    txt = hist[~is_visual[: C - w]]
    vis = hist[is_visual[: C - w]]
    if budget < w:
        return np.arange(C - max(int(budget), 0), C)
    m = budget - w - txt.size
    if m < 0:
        top_txt = top_indices(s_w, txt, budget - w)
        return np.sort(np.concatenate([top_txt, win]))
    top_vis = top_indices(s_w, vis, min(m, vis.size))
    return np.sort(np.concatenate([txt, top_vis, win]))


# ----------------------------------------------------------------------------
# prefill: dynamic heads
# ----------------------------------------------------------------------------
def chunk_means(k: np.ndarray, c: int, dtype: str) -> np.ndarray:
    """Chunk metadata: the mean key vector of each fixed-size chunk of the prompt
    (Appendix A, dynamic heads).  The last chunk may be shorter and is averaged
    over the rows it has.  The index is stored in the KV dtype, so the mean is
    rounded once to it."""
    kk = np.asarray(k, dtype=np.float64)
    C, d = kk.shape
    n_c = (C + c - 1) // c
    mu = np.zeros((n_c, d))
    for ci in range(n_c):
        rows = kk[ci * c: min((ci + 1) * c, C)]
        mu[ci] = rows.sum(axis=0) / rows.shape[0]
    return round_to_dtype(mu, dtype)


def chunk_scores(q: np.ndarray, mu: np.ndarray, group: str = "sum") -> np.ndarray:
    """Inner product of the step's query with every chunk's metadata (Appendix A).
    One selection is made per cached (KV) head; the paper writes one query vector
    and is silent on grouped-query heads.  group="sum" (the default reading): the G
    query heads of the group are summed into one query vector first.  group="max":
    every query head scores every chunk and a chunk takes the largest of its G
    scores (a chunk that matters to any one head of the group ranks high).
    No scaling in either (it cannot change ranks); with G = 1 the two coincide."""
    qq = np.asarray(q, dtype=np.float64)                          # [G, d]
    m = np.asarray(mu, dtype=np.float64)                          # [n_c, d]
    if group == "sum":
        return m @ qq.sum(axis=0)                                 # [n_c]
    if group == "max":
        return (m @ qq.T).max(axis=1)                             # [n_c]
    raise ValueError(group)


def n_selected_chunks(budget: int, c: int, n_c: int) -> int:
    """Chunks loaded per step = per-head budget / chunk size (Appendix A), at least
    one, at most all."""
    return int(min(max(1, budget // c), n_c))


def select_chunks(sigma: np.ndarray, k_sel: int) -> np.ndarray:
    """The k_sel chunks with the largest score, ties to the lower chunk id, ascending."""
    return top_indices(sigma, np.arange(np.asarray(sigma).size), k_sel)


def chunk_rows(sel: np.ndarray, c: int, C: int) -> np.ndarray:
    """Prompt positions covered by the selected chunks, ascending."""
    rows = [np.arange(ci * c, min((ci + 1) * c, C)) for ci in np.asarray(sel, dtype=np.int64)]
    return np.concatenate(rows) if rows else np.zeros(0, np.int64)


# ----------------------------------------------------------------------------
# decode
# ----------------------------------------------------------------------------
def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float,
              return_weights: bool = False):
    """softmax(q K^T * scale) V for the G query heads of one KV head.
    q [G, d], K [n, d], V [n, d] -> [G, d]."""
    q = np.asarray(q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    logits = (q @ K.T) * scale
    logits = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    p = e / e.sum(axis=1, keepdims=True)
    o = p @ V
    return (o, p) if return_weights else o


# ----------------------------------------------------------------------------
# head classification and budget allocation (upstream of the compression)
# ----------------------------------------------------------------------------
def focus_count(C: int, rho: float = 0.05) -> int:
    """k = ceil(rho * C): how many positions of a row count as its focus (Section 2.1 states
    k = ceil(0.05 C) for the focus count; the sparsity score of Section 3.1 names no k and is read
    with the same one)."""
    return max(1, min(C, int(np.ceil(rho * C - 1e-12))))


def text_sparsity_score(q_text: np.ndarray, k: np.ndarray, text_pos: np.ndarray, scale: float, k_top: int,
                        causal: bool = False) -> float:
    """Text-centric sparsity score of one KV head (Section 3.1).

    q_text  : [G, T, d]  queries of the T text tokens of the prompt for the G query heads that share
              this KV head (the paper writes one head; with grouped-query attention the rows of all
              G heads are averaged together, as for s_w),
    k       : [C, d]     keys of the whole prompt,
    text_pos: [T]        prompt positions of those text tokens (used by `causal` only).
    S_text = softmax(Q_text K^T * scale) row by row over all C keys (as printed: no mask; `causal`
    lets text token at position p see keys j <= p).  Each row contributes the sum of its k_top
    largest probabilities; the score is the mean over all G*T rows.
    """
    q = np.asarray(q_text, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    G, T, d = q.shape
    C = kk.shape[0]
    if T == 0:
        return 0.0
    total = 0.0
    for g in range(G):
        logits = (q[g] @ kk.T) * scale                                # [T, C]
        if causal:
            j = np.arange(C)[None, :]
            logits = np.where(j > np.asarray(text_pos)[:, None], -np.inf, logits)
        logits = logits - logits.max(axis=1, keepdims=True)
        e = np.exp(logits)
        p = e / e.sum(axis=1, keepdims=True)
        kt = min(k_top, C)
        top = np.partition(p, C - kt, axis=1)[:, C - kt:]             # the kt largest of every row
        total += float(np.sort(top, axis=1).sum())                    # ascending order: small terms first
    return total / (G * T)


def classify_heads(scores: np.ndarray, theta: float) -> np.ndarray:
    """Head types from sparsity scores (Section 3.1): static where S >= theta, dynamic below."""
    return np.where(np.asarray(scores, dtype=np.float64) >= theta, STATIC, DYNAMIC).astype(np.uint8)


def type_level_budgets(b_total: int, n_stat: int, n_dyn: int, r: float) -> Tuple[int, int]:
    """Split of the total token budget between the head types (Section 3.2, first equation):
    B_dyna = ceil(r * B_bar * N_dyna) with B_bar = B_total / (N_stat + N_dyna); B_stat is the rest.
    r is clipped to the bound the paper states, r <= B_total / (B_bar * N_dyna).
    (Here and in static_head_budgets the ceiling is taken of the value minus 1e-9: a product that is a
    whole number up to floating-point error, such as 0.75 of a budget divisible by four, stays there.)"""
    n = n_stat + n_dyn
    if n == 0 or n_dyn == 0:
        return int(b_total), 0
    b_bar = b_total / n
    r_eff = min(r, b_total / (b_bar * n_dyn))
    b_dyn = min(int(b_total), int(np.ceil(r_eff * b_bar * n_dyn - 1e-9)))
    return int(b_total) - b_dyn, b_dyn


def static_head_budgets(b_stat: int, scores: np.ndarray, alpha: float) -> np.ndarray:
    """Budgets of the static heads (Section 3.2, second equation): scores are L1-normalised over all
    static heads; b = ceil(alpha * B_stat / N_stat + (1 - alpha) * B_stat * S_norm)."""
    sc = np.asarray(scores, dtype=np.float64).reshape(-1)
    n = sc.size
    if n == 0:
        return np.zeros(0, np.int64)
    tot = sc.sum()
    s_norm = sc / tot if tot > 0 else np.full(n, 1.0 / n)
    return np.ceil(alpha * b_stat / n + (1.0 - alpha) * b_stat * s_norm - 1e-9).astype(np.int64)


def dynamic_head_budget(b_dyn: int, n_dyn: int, pad_pow2: bool = True) -> int:
    """Uniform budget of a dynamic head (Section 3.2); `pad_pow2` applies the paper's padding to the
    nearest power of two (nearest in linear distance, ties upwards)."""
    if n_dyn == 0:
        return 0
    b = b_dyn / n_dyn
    if not pad_pow2:
        return int(b)
    if b <= 1:
        return 1
    lo = 2 ** int(np.floor(np.log2(b)))
    hi = 2 * lo
    return int(lo if (b - lo) < (hi - b) else hi)


# ----------------------------------------------------------------------------
# drivers over all (sequence, layer, KV head) units
# ----------------------------------------------------------------------------
@dataclass
class OracleConfig:
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    window: int
    dtype: str = "f32"              # dtype of Q/K/V (their values are exact in it)
    score_causal: bool = False
    softmax_scale: float = 0.0      # 0 -> 1/sqrt(head_dim)
    chunk_score_group: str = "sum"  # how the G query heads of a group score a chunk: "sum" or "max"
    index_generated: bool = False   # dynamic heads: generated tokens are chunked and retrieved like the prompt

    @property
    def scale(self) -> float:
        return self.softmax_scale if self.softmax_scale > 0 else 1.0 / np.sqrt(self.head_dim)

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads


@dataclass
class OraclePlan:
    cu_seqlens: np.ndarray          # [batch+1]
    head_type: np.ndarray           # [batch, L, Hkv]
    budget: np.ndarray              # [batch, L, Hkv]
    chunk_size: np.ndarray          # [batch]

    @property
    def batch(self) -> int:
        return len(self.cu_seqlens) - 1


@dataclass
class OracleUnit:
    kind: int
    C: int
    # static
    s_w: Optional[np.ndarray] = None
    kept: Optional[np.ndarray] = None
    # dynamic
    c: int = 0
    k_sel: int = 0
    k_cap: int = 0                       # budget // c before it is capped by the number of chunks
    mu: Optional[np.ndarray] = None
    mu_gen: List[np.ndarray] = field(default_factory=list)   # index_generated: means of the complete chunks of generated tokens
    # rows the head attends: static -> compacted rows; dynamic -> the full prompt
    K: Optional[np.ndarray] = None
    V: Optional[np.ndarray] = None
    K_tail: List[np.ndarray] = field(default_factory=list)
    V_tail: List[np.ndarray] = field(default_factory=list)


@dataclass
class OracleCache:
    cfg: OracleConfig
    plan: OraclePlan
    units: Dict[Tuple[int, int, int], OracleUnit]


def compress(cfg: OracleConfig, plan: OraclePlan, q_window: np.ndarray, k: np.ndarray, v: np.ndarray,
             is_visual: np.ndarray, layers: Optional[range] = None,
             keep_override: Optional[Dict[Tuple[int, int, int], np.ndarray]] = None) -> OracleCache:
    """Prefill compression of every unit.

    q_window [L, B, w, Hq, d]; k, v [L, total_tokens, Hkv, d]; is_visual [total_tokens].
    `keep_override` replaces the computed keep set of the listed static units (used
    when a test needs oracle and device to attend the same rows inside a tie band).
    """
    G, w = cfg.group, cfg.window
    units: Dict[Tuple[int, int, int], OracleUnit] = {}
    layers = range(cfg.n_layers) if layers is None else layers
    for b in range(plan.batch):
        lo, hi = int(plan.cu_seqlens[b]), int(plan.cu_seqlens[b + 1])
        C = hi - lo
        vis = np.asarray(is_visual[lo:hi])
        for l in layers:
            for h in range(cfg.n_kv_heads):
                kk = np.asarray(k[l, lo:hi, h, :], dtype=np.float64)
                vv = np.asarray(v[l, lo:hi, h, :], dtype=np.float64)
                budget = int(plan.budget[b, l, h])
                if int(plan.head_type[b, l, h]) == STATIC:
                    qw = np.asarray(q_window[l, b, :, h * G:(h + 1) * G, :], dtype=np.float64)  # [w, G, d]
                    s_w = window_scores(np.transpose(qw, (1, 0, 2)), kk, cfg.scale, cfg.score_causal)
                    kept = static_keep_set(s_w, vis, w, budget)
                    if keep_override is not None and (b, l, h) in keep_override:
                        kept = np.asarray(keep_override[(b, l, h)], dtype=np.int64)
                    units[(b, l, h)] = OracleUnit(kind=STATIC, C=C, s_w=s_w, kept=kept,
                                                  K=kk[kept], V=vv[kept])
                else:
                    c = int(plan.chunk_size[b])
                    mu = chunk_means(kk, c, cfg.dtype)
                    units[(b, l, h)] = OracleUnit(kind=DYNAMIC, C=C, c=c, mu=mu,
                                                  k_sel=n_selected_chunks(budget, c, mu.shape[0]),
                                                  k_cap=max(1, budget // c),
                                                  K=kk, V=vv)
    return OracleCache(cfg=cfg, plan=plan, units=units)


def decode_attn(cache: OracleCache, q: np.ndarray, k_new: Optional[np.ndarray], v_new: Optional[np.ndarray],
                layers: Optional[range] = None,
                sel_override: Optional[Dict[Tuple[int, int, int], np.ndarray]] = None):
    """One decode step.  q [L, B, Hq, d]; k_new, v_new [L, B, Hkv, d] or None.

    New tokens are appended uncompressed to every head's tail and always attended.
    Static heads attend their kept rows + tail; dynamic heads score chunks, pick
    the top ones and attend those chunks' rows + tail.
    cfg.index_generated (a variant for long generations; the paper generates little and
    says nothing of it): on dynamic heads the generated tokens are cut into chunks of c in
    order of generation; a chunk that was complete before the step carries the mean of its
    keys as metadata (same rounding as the prompt's) and competes with the prompt's chunks
    for the budget // c places (capped by the number of chunks there are); the incomplete
    rest and the step's own token are always attended.  Static heads are unchanged.
    `sel_override` replaces the computed chunk picks of the listed dynamic units (used
    when a test needs oracle and device to attend the same rows inside a tie band).
    Returns (out [L, B, Hq, d] float64, info) where info[(b,l,h)] holds sigma/sel
    for dynamic units.
    """
    cfg = cache.cfg
    G = cfg.group
    layers = range(cfg.n_layers) if layers is None else layers
    out = np.zeros((cfg.n_layers, cache.plan.batch, cfg.n_q_heads, cfg.head_dim))
    info: Dict[Tuple[int, int, int], dict] = {}
    for b in range(cache.plan.batch):
        for l in layers:
            for h in range(cfg.n_kv_heads):
                u = cache.units[(b, l, h)]
                t_before = len(u.K_tail)
                if k_new is not None:
                    u.K_tail.append(np.asarray(k_new[l, b, h, :], dtype=np.float64))
                    u.V_tail.append(np.asarray(v_new[l, b, h, :], dtype=np.float64))
                qh = np.asarray(q[l, b, h * G:(h + 1) * G, :], dtype=np.float64)
                tail_from = 0                       # first tail row that is attended unconditionally
                if u.kind == STATIC:
                    K_rows, V_rows = u.K, u.V
                else:
                    mu = u.mu
                    n_gen = 0
                    if cfg.index_generated:
                        # the generated tokens present before this step, in chunks of c in order of generation;
                        # complete chunks compete with the prompt's chunks, the incomplete rest is always attended
                        n_gen = t_before // u.c
                        if n_gen:
                            mu = np.concatenate([mu, np.stack(u.mu_gen[:n_gen])], axis=0)
                        tail_from = n_gen * u.c
                    sigma = chunk_scores(qh, mu, cfg.chunk_score_group)
                    k_step = min(u.k_cap, mu.shape[0]) if cfg.index_generated else u.k_sel
                    sel = select_chunks(sigma, k_step)
                    if sel_override is not None and (b, l, h) in sel_override:
                        sel = np.asarray(sel_override[(b, l, h)], dtype=np.int64)
                    n_c = u.mu.shape[0]
                    rows = chunk_rows(sel[sel < n_c], u.c, u.C)
                    K_rows, V_rows = u.K[rows], u.V[rows]
                    for g in sel[sel >= n_c] - n_c:                  # selected chunks of generated tokens
                        K_rows = np.concatenate([K_rows, np.stack(u.K_tail[g * u.c:(g + 1) * u.c])], axis=0)
                        V_rows = np.concatenate([V_rows, np.stack(u.V_tail[g * u.c:(g + 1) * u.c])], axis=0)
                    info[(b, l, h)] = dict(sigma=sigma, sel=sel)
                    if cfg.index_generated and k_new is not None and len(u.K_tail) % u.c == 0:
                        # this step's token completes a chunk: its metadata joins the index for the next step
                        done = np.stack(u.K_tail[-u.c:])
                        u.mu_gen.append(round_to_dtype(done.sum(axis=0) / u.c, cfg.dtype))
                if len(u.K_tail) > tail_from:
                    K_rows = np.concatenate([K_rows, np.stack(u.K_tail[tail_from:])], axis=0)
                    V_rows = np.concatenate([V_rows, np.stack(u.V_tail[tail_from:])], axis=0)
                out[l, b, h * G:(h + 1) * G, :] = attention(qh, K_rows, V_rows, cfg.scale)
    return out, info


def head_scores(cfg: OracleConfig, cu_seqlens: np.ndarray, q_prompt: np.ndarray, k: np.ndarray,
                is_visual: np.ndarray, rho: float = 0.05, layers: Optional[range] = None) -> np.ndarray:
    """Sparsity score of every (sequence, layer, KV head): q_prompt [L, total_tokens, Hq, d] (queries of
    the whole prompt; only the text tokens' rows are used), k [L, total_tokens, Hkv, d].
    Returns [batch, L, Hkv] (zeros for layers not asked for)."""
    G = cfg.group
    B = len(cu_seqlens) - 1
    out = np.zeros((B, cfg.n_layers, cfg.n_kv_heads))
    for b in range(B):
        s0, s1 = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        C = s1 - s0
        text_pos = np.nonzero(np.asarray(is_visual[s0:s1]) == 0)[0]
        k_top = focus_count(C, rho)
        for l in (layers if layers is not None else range(cfg.n_layers)):
            for h in range(cfg.n_kv_heads):
                qt = np.stack([q_prompt[l, s0:s1][text_pos, h * G + g] for g in range(G)])      # [G, T, d]
                out[b, l, h] = text_sparsity_score(qt, k[l, s0:s1, h], text_pos, cfg.scale, k_top, cfg.score_causal)
    return out


def cumulative_focus(q_steps: np.ndarray, k: np.ndarray, scale: float, k_top: int) -> np.ndarray:
    """Cumulative focus count of one attention head (Section 2.1, Eq. 1).

    q_steps [N, d]: the head's query at each of N decoding steps; k [C, d]: the keys of the context.
    At step i the attention score vector over the context is a_i = softmax(q_i K^T * scale); token j
    scores a point when it is among the k_top largest entries of a_i (equal entries go to the lower
    position, as everywhere else here; the paper does not say).  F_j is the number of steps at which
    j scored.  Returns int64 [C]."""
    q = np.asarray(q_steps, dtype=np.float64)
    kk = np.asarray(k, dtype=np.float64)
    C = kk.shape[0]
    F = np.zeros(C, np.int64)
    pos = np.arange(C)
    for i in range(q.shape[0]):
        logits = (kk @ q[i]) * scale
        e = np.exp(logits - logits.max())
        a = e / e.sum()
        F[top_indices(a, pos, min(k_top, C))] += 1
    return F


def full_decode_attn(cfg: OracleConfig, cu_seqlens: np.ndarray, q: np.ndarray, k: np.ndarray, v: np.ndarray,
                     layers: Optional[range] = None) -> np.ndarray:
    """Uncompressed decode attention: every head attends all rows of its sequence.
    q [L, B, Hq, d]; k, v [L, total_tokens, Hkv, d]."""
    G = cfg.group
    layers = range(cfg.n_layers) if layers is None else layers
    B = len(cu_seqlens) - 1
    out = np.zeros((cfg.n_layers, B, cfg.n_q_heads, cfg.head_dim))
    for b in range(B):
        lo, hi = int(cu_seqlens[b]), int(cu_seqlens[b + 1])
        for l in layers:
            for h in range(cfg.n_kv_heads):
                out[l, b, h * G:(h + 1) * G, :] = attention(
                    q[l, b, h * G:(h + 1) * G, :], k[l, lo:hi, h, :], v[l, lo:hi, h, :], cfg.scale)
    return out
