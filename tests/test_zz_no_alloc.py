"""optimus_attn_forward_static (the entry point that allocates nothing: split-KV partials in the
library's static device scratch) against optimus_attn_forward with a caller workspace: same plan,
same kernels, so the outputs must be bit-identical, and both must meet the oracle's bar.  Two
calls in a row, the second with a smaller input, so that whatever the first call left in the
shared scratch is seen not to matter; then a plan that needs more than the scratch is refused."""
import numpy as np
import pytest
import torch

from paper_2605_24832_amd import OptimusError, Plan, inputs, static_scratch_bytes
from tests import hip_path as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both_ways(oracle, w, tuning):
    bits = hp.host_bits(w)                       # before the append
    plan = Plan(hp.params_of(w), device=0)
    plan.set_tuning(**tuning)
    ws_bytes = plan.plan_update(w.cu_q, w.prefix_len, w.block_start, w.block_table)
    assert 0 < ws_bytes <= static_scratch_bytes()
    assert plan.num_merge_items() > 0            # the scratch is really used
    bt = torch.as_tensor(w.block_table, device=DEV)
    ws = torch.full((ws_bytes // 4 + 4,), float("nan"), dtype=torch.float32, device=DEV)
    out_ws = torch.full_like(w.q, float("nan"))
    out_st = torch.full_like(w.q, float("nan"))
    plan.kv_append(w.k_pool, w.v_pool, w.k_new, w.v_new, bt)
    plan.attn_forward(w.q, w.k_pool, w.v_pool, bt, out_ws, ws)
    plan.attn_forward_static(w.q, w.k_pool, w.v_pool, bt, out_st)
    torch.cuda.synchronize()
    assert torch.equal(out_ws.view(torch.int16), out_st.view(torch.int16))
    ref, _, _ = hp.run_oracle(oracle, w, bits=bits)
    mx, mean = hp.check_close(out_st.float().cpu().numpy(), ref, what="forward_static")
    print(f"  items={plan.num_work_items()} merges={plan.num_merge_items()} workspace={ws_bytes} B "
          f"max={mx:.2e} mean={mean:.2e}", flush=True)
    plan.close()


def test_static_scratch_forward_matches_workspace_forward(oracle_mod):
    print("no-alloc forward", flush=True)
    kw = dict(num_q_heads=16, num_kv_heads=4, head_dim=128, page_size=16, block_size=32, device=DEV)
    tuning = dict(target_items=1 << 20, min_split_tokens=64, max_split_tokens=128)
    big = inputs.make_workload("static_big", seed=301, prefix_len=[3000, 700, 1500, 64, 2222],
                               chunk=[4, 32, 1, 20, 9], block_inner=[0] * 5, **kw)
    small = inputs.make_workload("static_small", seed=302, prefix_len=[333, 90], chunk=[2, 17],
                                 block_inner=[0, 0], **kw)
    both_ways(oracle_mod, big, tuning)
    both_ways(oracle_mod, small, tuning)         # smaller input right after: stale partials beyond it stay unread


def test_static_scratch_forward_refuses_what_does_not_fit():
    # three requests of 128 query rows per kv head over 32K keys, cut as finely as the planner
    # allows (16 tiles per item at this row count): about 100 MB of partials
    w = inputs.make_workload("static_too_big", seed=303, num_q_heads=32, num_kv_heads=8, head_dim=128,
                             page_size=64, block_size=32, prefix_len=[32768] * 3, chunk=[32] * 3,
                             block_inner=[0] * 3, poison=False, device=DEV)
    plan = Plan(hp.params_of(w), device=0)
    plan.set_tuning(target_items=1 << 20, min_split_tokens=32, max_split_tokens=32)
    ws_bytes = plan.plan_update(w.cu_q, w.prefix_len, w.block_start, w.block_table)
    assert ws_bytes > static_scratch_bytes()
    out = torch.zeros_like(w.q)
    bt = torch.as_tensor(w.block_table, device=DEV)
    with pytest.raises(OptimusError) as e:
        plan.attn_forward_static(w.q, w.k_pool, w.v_pool, bt, out)
    assert e.value.status == -8
    torch.cuda.synchronize()
    assert float(out.float().abs().sum()) == 0.0  # nothing was launched
    plan.close()
