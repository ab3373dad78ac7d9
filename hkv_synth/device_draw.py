"""The workload recipe of hkv_synth.workloads drawn directly on the GPU, for the configurations whose
tensors are too large to generate on the host in a benchmark run (tens of GB).

Same shapes, layouts, plans and value structure as make_workload(): K, V, Q ~ N(0,1) rounded to the
workload's dtype; on static heads a seeded 5 % of the historical visual positions get K += 3 u (u a unit
vector per unit) and the window queries of that group get + sqrt(d) u; decode queries of dynamic heads are
drawn around a seeded chunk centroid where the configuration says so.  Only the random stream differs
(the device's generator instead of NumPy's), so these tensors are not bit-identical to the host ones;
parity tests use the host generator.  Input generation only: nothing of the method is computed here.
"""
from __future__ import annotations

import math

import numpy as np

from .workloads import CONFIGS, DYNAMIC, STATIC, Workload


def _cfg_of(wl: Workload) -> dict:
    for c in CONFIGS.values():
        if wl.name.startswith(c["name"]):
            return c
    return {}


def draw_device_tensors(wl: Workload, n_inputs: int, device="cuda:0", seed: int = 0):
    """Returns (q_window [L,B,w,Hq,d], k, v [L,total,Hkv,d], q_steps [n,L,B,Hq,d], k_new, v_new [n,L,B,Hkv,d])
    as device tensors of the workload's dtype."""
    import torch

    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    L, B, Hq, Hkv, d, w = wl.n_layers, wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window
    G = Hq // Hkv
    total = wl.total_tokens
    gen = torch.Generator(device=device)
    gen.manual_seed(0x48594B56 + 1000 * int(seed) + sum(ord(ch) for ch in wl.name))

    def randn(*shape):
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)

    cu = [int(x) for x in wl.cu_seqlens]
    vis_hist = []                     # per sequence: absolute token indices of the visual tokens before the window
    for b in range(B):
        m = np.asarray(wl.is_visual[cu[b]:cu[b + 1] - w])
        vis_hist.append(torch.from_numpy(cu[b] + np.nonzero(m)[0]).to(device))

    k = torch.empty((L, total, Hkv, d), dtype=tdt, device=device)
    v = torch.empty((L, total, Hkv, d), dtype=tdt, device=device)
    qw = torch.empty((L, B, w, Hq, d), dtype=tdt, device=device)
    for l in range(L):
        kl, ql = randn(total, Hkv, d), randn(B, w, Hq, d)
        for b in range(B):
            n_vis = int(vis_hist[b].numel())
            n_plant = int(round(0.05 * n_vis))
            if n_plant == 0:
                continue
            for h in range(Hkv):
                if wl.head_type[b, l, h] != STATIC:
                    continue
                u = randn(d)
                u = u / u.norm()
                pos = vis_hist[b][torch.randperm(n_vis, generator=gen, device=device)[:n_plant]]
                kl[pos, h, :] += 3.0 * u
                ql[b, :, h * G:(h + 1) * G, :] += math.sqrt(d) * u
        k[l] = kl.to(tdt)
        qw[l] = ql.to(tdt)
        v[l] = randn(total, Hkv, d).to(tdt)
        del kl, ql

    q_steps = torch.empty((n_inputs, L, B, Hq, d), dtype=tdt, device=device)
    k_new = torch.empty((n_inputs, L, B, Hkv, d), dtype=tdt, device=device)
    v_new = torch.empty((n_inputs, L, B, Hkv, d), dtype=tdt, device=device)
    centroid = _cfg_of(wl).get("q_mode") == "centroid"
    for s in range(n_inputs):
        q_steps[s] = randn(L, B, Hq, d).to(tdt)
        k_new[s] = randn(L, B, Hkv, d).to(tdt)
        v_new[s] = randn(L, B, Hkv, d).to(tdt)
    if centroid:
        for b in range(B):
            C, cs = cu[b + 1] - cu[b], int(wl.chunk_size[b])
            n_c = (C + cs - 1) // cs
            offs = torch.arange(cs, device=device)
            for l in range(L):
                for h in range(Hkv):
                    if wl.head_type[b, l, h] != DYNAMIC:
                        continue
                    picks = torch.randint(0, n_c, (n_inputs,), generator=gen, device=device)
                    rows = picks[:, None] * cs + offs[None, :]                    # [n, cs]
                    ok = (rows < C).to(torch.float32)
                    rows = rows.clamp(max=C - 1) + cu[b]
                    kk = k[l, rows.reshape(-1), h, :].to(torch.float32).reshape(n_inputs, cs, d)
                    cen = (kk * ok[:, :, None]).sum(1) / ok.sum(1, keepdim=True)  # [n, d]
                    noise = q_steps[:, l, b, h * G:(h + 1) * G, :].to(torch.float32)
                    q_steps[:, l, b, h * G:(h + 1) * G, :] = (cen[:, None, :] + 0.5 * noise).to(tdt)
    return qw, k, v, q_steps, k_new, v_new
