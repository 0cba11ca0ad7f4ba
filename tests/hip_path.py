"""Test-side helpers: run a Workload through the C-ABI library, and through the oracle."""
import copy

import numpy as np
import torch

from paper_2605_24832_amd import AttnParams, Plan, inputs


def params_of(w, **kw):
    args = dict(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                page_size=w.page_size, block_size=w.block_size, num_pages=w.num_pages,
                max_pages_per_req=w.block_table.shape[1], mask_mode=w.mask_mode,
                kv_layout=w.kv_layout)
    args.update(kw)
    return AttnParams(**args)


def params_of_geometry(Hq, Hkv, D, P, B, num_pages, max_pages, **kw):
    return AttnParams(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P, block_size=B,
                      num_pages=num_pages, max_pages_per_req=max_pages, **kw)


def run_hip(w, *, tuning=None, out_dtype=0, append=True, validate_table=True, q_pos=None, step=False, **kw):
    """plan_update -> kv_append -> attn_forward on the workload's device tensors
    (``step=True``: after the sizing plan_update, one attn_step call does all three).

    Returns (out tensor on device, plan).  The pools of ``w`` are modified by the append.
    """
    assert w.q.is_cuda
    p = params_of(w, out_dtype=out_dtype, **kw)
    plan = Plan(p, device=w.q.device.index or 0)
    if tuning:
        plan.set_tuning(**tuning)
    ws_bytes = plan.plan_update(w.cu_q, w.prefix_len, w.block_start,
                                w.block_table if validate_table else None)
    bt = torch.as_tensor(w.block_table, device=w.q.device)
    ws = torch.empty(max(ws_bytes, 16) // 4 + 4, dtype=torch.float32, device=w.q.device)
    # poison the outputs and scratch: every byte the library reports must be one it wrote
    ws.fill_(float("nan"))
    out = torch.full((w.total_q, w.num_q_heads, w.head_dim), float("nan"),
                     dtype=torch.float32 if out_dtype == 1 else torch.bfloat16, device=w.q.device)
    pos = None if q_pos is None else torch.as_tensor(np.asarray(q_pos, dtype=np.int32), device=w.q.device)
    if step:
        plan.attn_step(w.cu_q, w.prefix_len, w.block_start, w.block_table if validate_table else None,
                       w.q, w.k_new, w.v_new, w.k_pool, w.v_pool, bt, out, ws, q_pos=pos)
    else:
        if append:
            plan.kv_append(w.k_pool, w.v_pool, w.k_new, w.v_new, bt)
        plan.attn_forward(w.q, w.k_pool, w.v_pool, bt, out, ws, q_pos=pos)
    torch.cuda.synchronize()
    return out, plan


def oracle_params(oracle, w, **kw):
    args = dict(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                page_size=w.page_size, block_size=w.block_size,
                max_pages_per_req=w.block_table.shape[1], mask_mode=w.mask_mode,
                kv_layout=w.kv_layout)
    args.update(kw)
    return oracle.make_params(**args)


def host_bits(w):
    return {k: inputs.to_bits(getattr(w, k)) for k in ("q", "k_new", "v_new", "k_pool", "v_pool")}


def run_oracle(oracle, w, bits=None, requests=None, kv_heads=None, q_pos=None, **kw):
    """Oracle output for the whole batch, or for a subset of requests and/or kv-head groups.

    A request's rows do not depend on the rest of the batch and a kv-head group
    does not depend on the other groups (both pinned in the oracle's own tests),
    so subsets give exactly the rows of the full computation.
    Returns (out f64 [T_sel, Hq_sel, D], token index array, query head index array).
    """
    b = host_bits(w) if bits is None else bits
    Hq, Hkv, D = w.num_q_heads, w.num_kv_heads, w.head_dim
    G = Hq // Hkv
    req = np.arange(w.batch) if requests is None else np.asarray(requests)
    kvh = np.arange(Hkv) if kv_heads is None else np.asarray(kv_heads)
    tok = np.concatenate([np.arange(w.cu_q[i], w.cu_q[i + 1]) for i in req]) if len(req) else \
        np.zeros(0, dtype=np.int64)
    qh = np.concatenate([np.arange(g * G, (g + 1) * G) for g in kvh])
    q = b["q"].reshape(-1, Hq, D)[tok][:, qh]
    kn = b["k_new"].reshape(-1, Hkv, D)[tok][:, kvh]
    vn = b["v_new"].reshape(-1, Hkv, D)[tok][:, kvh]
    kp, vp = b["k_pool"], b["v_pool"]
    tile = w.page_size * D
    p = oracle_params(oracle, w, num_q_heads=len(qh), num_kv_heads=len(kvh),
                      k_stride_page=Hkv * tile, v_stride_page=Hkv * tile, **kw)
    if len(kvh) != Hkv:
        # gather the selected heads into a dense pool copy
        kp = np.ascontiguousarray(kp.reshape(-1, Hkv, tile)[:, kvh])
        vp = np.ascontiguousarray(vp.reshape(-1, Hkv, tile)[:, kvh])
        p.k_stride_page = p.v_stride_page = len(kvh) * tile
    cu = np.zeros(len(req) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(w.chunk[req])
    out = oracle.chunked_attention(p, cu, w.prefix_len[req], w.block_start[req],
                                   w.block_table[req], q, kn, vn, kp, vp,
                                   q_pos=None if q_pos is None else np.asarray(q_pos, dtype=np.int32)[tok])
    return out, tok, qh


def clone_workload(w, device=None):
    w2 = copy.copy(w)
    for k in ("q", "k_new", "v_new", "k_pool", "v_pool"):
        t = getattr(w, k)
        setattr(w2, k, t.clone() if device is None else t.to(device).clone())
    return w2


def check_close(got, ref, max_tol=1e-2, mean_tol=1e-3, what=""):
    got = np.asarray(got, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    assert err.max() <= max_tol, f"{what}: max abs err {err.max():.3e} > {max_tol}"
    assert err.mean() <= mean_tol, f"{what}: mean abs err {err.mean():.3e} > {mean_tol}"
    return err.max(), err.mean()
