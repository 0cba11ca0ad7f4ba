"""GPU parity: the HIP path, called through the C ABI, against the fp64 CPU oracle.

Bar: bf16 in, fp32 accumulate, bf16 out: max |err| <= 1e-2 and mean |err| <= 1e-3 over
the outputs of a case; pool contents after the append and everything derived from the
block table bit-exact.
"""
import numpy as np
import pytest
import torch

from paper_2605_24832_amd import inputs
from tests import hip_path as hp

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _say(msg):
    print(msg, flush=True)


def full_parity(oracle, w, what, **kw):
    bits = hp.host_bits(w)  # before the append
    out, plan = hp.run_hip(w, **kw)
    ref, _, _ = hp.run_oracle(oracle, w, bits=bits, **{k: v for k, v in kw.items() if k == "mask_mode"})
    mx, mean = hp.check_close(out.float().cpu().numpy(), ref, what=what)
    _say(f"{what}: items={plan.num_work_items()} merges={plan.num_merge_items()} "
         f"max={mx:.2e} mean={mean:.2e}")
    # append bit-exactness against the oracle's scatter
    p = hp.oracle_params(oracle, w)
    kp, vp = bits["k_pool"].copy(), bits["v_pool"].copy()
    oracle.kv_append(p, w.cu_q, w.prefix_len, w.block_table, bits["k_new"], bits["v_new"], kp, vp)
    np.testing.assert_array_equal(inputs.to_bits(w.k_pool), kp)
    np.testing.assert_array_equal(inputs.to_bits(w.v_pool), vp)
    return out, plan


def test_config0_tiny(oracle_mod):
    _say("config0")
    w = inputs.make_config(0, device=DEV)
    full_parity(oracle_mod, w, "config0")


@pytest.mark.parametrize("c", [4, 8, 16, 32])
def test_config1_mha_batch1(oracle_mod, c):
    _say(f"config1 c={c}")
    w = inputs.make_config(1, device=DEV, chunk=c)
    _, plan = full_parity(oracle_mod, w, f"config1 c={c}")
    assert plan.num_merge_items() > 0  # batch 1 must split the KV range to fill the chip


@pytest.mark.parametrize("c", [1, 2, 3, 5, 6, 7, 22, 31, 32])
def test_arbitrary_chunk_sizes(oracle_mod, c):
    """Any chunk size, not only 1 or the block size (Sec. 6); Sec. 7.4 reports 6 and 22."""
    _say(f"chunk {c}")
    w = inputs.make_workload("chunks", seed=100 + c, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[200, 77, 1000],
                             chunk=[c, c, c], block_inner=[0, 0, 0], device=DEV)
    full_parity(oracle_mod, w, f"chunk {c}")


def test_ragged_edge_cases(oracle_mod):
    """L=0, c=0, one-key tail tiles, tile-aligned lengths, a request with one key in total."""
    _say("ragged edges")
    L = [0, 0, 31, 32, 33, 63, 64, 65, 16, 15, 1, 0, 511, 96]
    c = [1, 5, 1, 1, 1, 1, 1, 1, 0, 1, 31, 0, 1, 32]
    w = inputs.make_workload("edges", seed=7, num_q_heads=8, num_kv_heads=4, head_dim=128,
                             page_size=16, block_size=32, prefix_len=L, chunk=c,
                             block_inner=[0] * len(L), device=DEV)
    out, _ = full_parity(oracle_mod, w, "ragged edges")
    # L=0, c=1: the only key is the token itself
    t = int(w.cu_q[0])
    g = w.num_q_heads // w.num_kv_heads
    np.testing.assert_array_equal(out[t].float().cpu().numpy(),
                                  w.v_new[t].float().cpu().numpy().repeat(g, axis=0))


@pytest.mark.parametrize("P", [16, 32, 64, 128])
@pytest.mark.parametrize("D", [64, 128])
def test_page_sizes_and_head_dims(oracle_mod, P, D):
    _say(f"P={P} D={D}")
    w = inputs.make_workload("pd", seed=11 + P + D, num_q_heads=6, num_kv_heads=2, head_dim=D,
                             page_size=P, block_size=32, prefix_len=[300, 45, 129, 0],
                             chunk=[7, 32, 1, 3], block_inner=[0, 0, 0, 0], device=DEV)
    full_parity(oracle_mod, w, f"P={P} D={D}")


def test_gqa7_many_q_tiles(oracle_mod):
    """G=7, c=32 -> 224 rows per kv head: four q tiles, odd head grouping."""
    _say("gqa7")
    w = inputs.make_workload("gqa7", seed=13, num_q_heads=28, num_kv_heads=4, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[700, 130], chunk=[32, 9],
                             block_inner=[0, 0], device=DEV)
    full_parity(oracle_mod, w, "gqa7")


@pytest.mark.parametrize("Hq,Hkv,D,P", [(12, 2, 128, 16), (32, 2, 64, 32), (16, 1, 128, 64), (24, 2, 64, 16)])
def test_wide_row_tiles(oracle_mod, Hq, Hkv, D, P):
    """Every row-tile class of the wide body: 33..64, 65..128, 129..192, 193..256 rows and more than 256 rows
    (several row tiles), unsplit and split, with ragged key tails."""
    _say(f"wide rows Hq={Hq} Hkv={Hkv} D={D} P={P}")
    G = Hq // Hkv
    chunks = sorted({-(-r // G) for r in (33, 64, 65, 128, 129, 192, 193, 256, 257, 300, 512)} - {0})
    chunks = [c for c in chunks if c <= 64]
    L = [37 + 61 * k for k in range(len(chunks))]
    w = inputs.make_workload("wide", seed=41 + Hq, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                             page_size=P, block_size=64, prefix_len=L, chunk=chunks,
                             block_inner=[0] * len(L), device=DEV)
    full_parity(oracle_mod, w, "wide rows")
    w2 = inputs.make_workload("wide", seed=41 + Hq, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                              page_size=P, block_size=64, prefix_len=L, chunk=chunks,
                              block_inner=[0] * len(L), device=DEV)
    full_parity(oracle_mod, w2, "wide rows split",
                tuning=dict(target_items=1 << 20, min_split_tokens=64, max_split_tokens=64))


@pytest.mark.parametrize("P", [16, 64])
def test_wide_rows_long_unsplit_key_range(oracle_mod, P):
    """One work item per (request, kv head) walks more than 64 pages: the wide kernel's page
    register is refilled on the way; chunk 40 x G 4 = 160 rows (a full and a partial row tile)."""
    _say(f"wide rows, long unsplit range, P={P}")
    L = [16 * 150 + 5, 64 * 70 + 33] if P == 16 else [64 * 70 + 33, 64 * 130 + 1]
    w = inputs.make_workload("wide_long", seed=77 + P, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=P, block_size=64, prefix_len=L, chunk=[40, 24],
                             block_inner=[0, 0], device=DEV)
    _, plan = full_parity(oracle_mod, w, "wide long",
                          tuning=dict(target_items=1, min_split_tokens=1 << 20, max_split_tokens=1 << 20))
    assert plan.num_merge_items() == 0


@pytest.mark.parametrize("P", [16, 32, 64, 128])
@pytest.mark.parametrize("D", [64, 128])
def test_wide_only_batches(oracle_mod, D, P):
    """Batches in which every (request, kv head) pair has more than 32 query rows, so that only
    the wide body runs: key ranges of 1..8 tiles and longer (every prologue and tail case of its
    staging ring), ragged row tiles (72, 104, 136 and 264 rows), an empty request in between;
    default plan, forced splits, fp32 output and mask mode 1."""
    _say(f"wide-only D={D} P={P}")
    L = [0, 30, 70, 100, 140, 170, 200, 230, 50, 1000, 2077, 333]
    c = [9, 9, 9, 9, 9, 9, 9, 9, 0, 13, 17, 33]
    kw = dict(seed=300 + D + P, num_q_heads=16, num_kv_heads=2, head_dim=D, page_size=P,
              block_size=64, prefix_len=L, chunk=c, block_inner=[0] * len(L), device=DEV)
    # the smallest share of keys the planner gives an item grows with the rows of the largest
    # pair (264 here), so only the two long requests can be split
    split = dict(target_items=1 << 20, min_split_tokens=64, max_split_tokens=64)
    for name, tuning in (("default", None), ("split", split)):
        w = inputs.make_workload("wide_only", **kw)
        _, plan = full_parity(oracle_mod, w, f"wide-only {name}", tuning=tuning)
        assert plan.num_merge_items() > 0
    w = inputs.make_workload("wide_only", **kw)
    bits = hp.host_bits(w)
    out, _ = hp.run_hip(w, out_dtype=1)
    ref, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
    mx, mean = hp.check_close(out.cpu().numpy(), ref, max_tol=5e-3, mean_tol=5e-4, what="wide-only fp32")
    _say(f"wide-only fp32: max={mx:.2e} mean={mean:.2e}")
    kw1 = dict(kw, block_size=32, block_inner=[0, 30, 6, 4, 12, 10, 8, 6, 18, 8, 29, 13], mask_mode=1)
    for tuning in (None, split):
        w = inputs.make_workload("wide_only_m1", **kw1)
        full_parity(oracle_mod, w, "wide-only mask mode 1", tuning=tuning)


def test_forced_splits_and_merge(oracle_mod):
    """Tiny split size: many partials per row, including splits some waves get no tile of."""
    _say("forced splits")
    w = inputs.make_workload("splits", seed=17, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[1000, 50, 333], chunk=[4, 20, 1],
                             block_inner=[0, 0, 0], device=DEV)
    for split in (32, 64, 96):
        w2 = hp.clone_workload(w)
        _, plan = full_parity(oracle_mod, w2, f"split {split}",
                              tuning=dict(target_items=1 << 20, min_split_tokens=split,
                                          max_split_tokens=split))
        assert plan.num_merge_items() > 0
    # and no split at all
    w2 = hp.clone_workload(w)
    _, plan = full_parity(oracle_mod, w2, "unsplit",
                          tuning=dict(target_items=1, min_split_tokens=1 << 20, max_split_tokens=1 << 20))
    assert plan.num_merge_items() == 0


def test_fp32_output(oracle_mod):
    _say("fp32 out")
    w = inputs.make_config(0, device=DEV)
    bits = hp.host_bits(w)
    out, _ = hp.run_hip(w, out_dtype=1)
    ref, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
    mx, mean = hp.check_close(out.cpu().numpy(), ref, max_tol=5e-3, mean_tol=5e-4, what="fp32 out")
    _say(f"fp32 out: max={mx:.2e} mean={mean:.2e}")


def test_block_causal_mode(oracle_mod):
    """mask_mode 1: chunks that cross a block boundary, block-causal inside the chunk."""
    _say("mask mode 1")
    w = inputs.make_workload("obs", seed=19, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[100, 40, 0, 500],
                             chunk=[32, 32, 20, 7], block_inner=[20, 0, 0, 30], mask_mode=1,
                             device=DEV)
    full_parity(oracle_mod, w, "mask mode 1")
    w2 = inputs.make_workload("obs", seed=19, num_q_heads=8, num_kv_heads=2, head_dim=128,
                              page_size=16, block_size=32, prefix_len=[100, 40, 0, 500],
                              chunk=[32, 32, 20, 7], block_inner=[20, 0, 0, 30], mask_mode=1,
                              device=DEV)
    full_parity(oracle_mod, w2, "mask mode 1 split",
                tuning=dict(target_items=1 << 20, min_split_tokens=32, max_split_tokens=32))


@pytest.mark.parametrize("split", [0, 32])
def test_block_causal_mode_with_explicit_positions(oracle_mod, split):
    """mask_mode 1 with the sequence positions of the chunk tokens (Sec. 4.4: the chunk is the
    positions not yet decoded, with holes where tokens were decoded out of order): every body
    (7, 20 and 32 tokens x 4 heads per kv head = 28, 80, 128 rows; 2 x 4 = 8 rows), chunks that
    cross a block boundary, a block origin that is not a multiple of the block size."""
    _say(f"mask mode 1, explicit positions, split {split}")
    B = 32
    L = np.array([100, 40, 0, 500, 77])
    d_in = np.array([20, 0, 0, 30, 13])
    c = np.array([32, 20, 7, 2, 32])
    w = inputs.make_workload("obs_pos", seed=59, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=B, prefix_len=L, chunk=c, block_inner=d_in,
                             mask_mode=1, device=DEV)
    rng = np.random.RandomState(59)
    pos = []
    for i in range(len(L)):
        s = int(L[i] - d_in[i])
        # the chunk = the first c_i not decoded positions among the 2B after the origin: a random
        # subset of d_in positions is decoded (cached), the chunk skips them
        decoded = set(rng.choice(2 * B, size=int(d_in[i]), replace=False).tolist())
        free = [s + x for x in range(3 * B) if x not in decoded]
        pos += free[:int(c[i])]
    tuning = None if split == 0 else dict(target_items=1 << 20, min_split_tokens=split, max_split_tokens=split)
    bits = hp.host_bits(w)
    out, plan = hp.run_hip(w, q_pos=pos, tuning=tuning)
    ref, _, _ = hp.run_oracle(oracle_mod, w, bits=bits, q_pos=pos)
    mx, mean = hp.check_close(out.float().cpu().numpy(), ref, what="explicit positions")
    _say(f"explicit positions: items={plan.num_work_items()} merges={plan.num_merge_items()} max={mx:.2e} mean={mean:.2e}")
    # the positions matter: the contiguous reading gives a different result on this input
    ref_contig, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
    assert np.abs(ref - ref_contig).max() > 1e-2
    # contiguous positions through the same entry point reproduce the default path bit for bit
    w2 = inputs.make_workload("obs_pos", seed=59, num_q_heads=8, num_kv_heads=2, head_dim=128,
                              page_size=16, block_size=B, prefix_len=L, chunk=c, block_inner=d_in,
                              mask_mode=1, device=DEV)
    contig = np.concatenate([np.arange(ci) + Li for Li, ci in zip(L, c)])
    o_a, _ = hp.run_hip(w2, q_pos=contig, tuning=tuning)
    w3 = inputs.make_workload("obs_pos", seed=59, num_q_heads=8, num_kv_heads=2, head_dim=128,
                              page_size=16, block_size=B, prefix_len=L, chunk=c, block_inner=d_in,
                              mask_mode=1, device=DEV)
    o_b, _ = hp.run_hip(w3, tuning=tuning)
    assert torch.equal(o_a, o_b)


def test_strided_interleaved_pool(oracle_mod):
    """K and V tiles interleaved in one allocation: page/head strides twice the dense ones."""
    _say("strided pool")
    w = inputs.make_workload("strided", seed=23, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[150, 61], chunk=[5, 16],
                             block_inner=[0, 0], device=DEV)
    tile = w.page_size * w.head_dim
    Hkv = w.num_kv_heads
    both = torch.full((w.num_pages, Hkv, 2, tile), float("nan"), dtype=torch.bfloat16, device=DEV)
    both[:, :, 0] = w.k_pool
    both[:, :, 1] = w.v_pool
    bits = hp.host_bits(w)
    ref, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
    w.k_pool = both.view(-1)[0:]
    w.v_pool = both.view(-1)[tile:]
    out, _ = hp.run_hip(w, k_stride_page=2 * Hkv * tile, v_stride_page=2 * Hkv * tile,
                        k_stride_head=2 * tile, v_stride_head=2 * tile)
    hp.check_close(out.float().cpu().numpy(), ref, what="strided pool")


def test_gpu_invariants(oracle_mod):
    """Page reshuffle and NaN tails leave the GPU output bit-identical; chunk permutation
    permutes it within tolerance."""
    _say("invariants")
    kw = dict(seed=29, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, block_size=32,
              prefix_len=[300, 37], chunk=[6, 11], block_inner=[0, 0], device=DEV)
    clean = inputs.make_workload("inv", poison=False, **kw)
    dirty = inputs.make_workload("inv", poison=True, **kw)
    o_clean, _ = hp.run_hip(clean)
    o_dirty, _ = hp.run_hip(dirty)
    assert torch.isfinite(o_dirty.float()).all()
    assert torch.equal(o_clean, o_dirty)
    # reshuffle physical pages
    base = inputs.make_workload("inv", poison=True, **kw)
    rng = np.random.RandomState(1)
    perm = rng.permutation(base.num_pages)
    inv = torch.as_tensor(np.argsort(perm), device=DEV)
    shuf = hp.clone_workload(base)
    shuf.k_pool = base.k_pool[inv].contiguous()
    shuf.v_pool = base.v_pool[inv].contiguous()
    bt = base.block_table.copy()
    bt[bt >= 0] = perm[bt[bt >= 0]]
    shuf.block_table = bt
    o_shuf, _ = hp.run_hip(shuf)
    assert torch.equal(o_shuf, o_dirty)
    # permute chunk tokens
    pm = np.concatenate([rng.permutation(6), 6 + rng.permutation(11)])
    pt = torch.as_tensor(pm, device=DEV)
    permd = inputs.make_workload("inv", poison=True, **kw)
    permd.q, permd.k_new, permd.v_new = permd.q[pt].contiguous(), permd.k_new[pt].contiguous(), \
        permd.v_new[pt].contiguous()
    o_perm, _ = hp.run_hip(permd)
    hp.check_close(o_perm.float().cpu().numpy(), o_dirty[pt].double().cpu().numpy(), what="perm")


def test_constant_v_and_single_token_decode(oracle_mod):
    _say("constant V")
    w = inputs.make_workload("cv", seed=31, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[500, 40], chunk=[1, 1],
                             block_inner=[0, 0], poison=False, device=DEV)
    v0 = torch.linspace(-1.5, 2.0, 128, device=DEV).to(torch.bfloat16)
    inputs.v_tile_view(w.v_pool, 16, 128, 1)[:] = v0.view(1, 1, 128, 1)
    w.v_new[:] = v0
    out, _ = hp.run_hip(w)
    err = (out.float() - v0.float()).abs().max().item()
    assert err <= 2.0 * 2 ** -8, err  # one bf16 rounding of |v| <= 2


def test_append_overwrites_provisional_slots(oracle_mod):
    """Chunk KV is provisional: after commit the final KV of the same tokens is written over
    the same slots (Sec. 4.1).  A second append to the same slots must win, bit for bit,
    and attention must then see the new rows."""
    _say("overwrite")
    kw = dict(seed=43, num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16, block_size=32,
              prefix_len=[70, 9], chunk=[5, 12], block_inner=[0, 0], device=DEV)
    w = inputs.make_workload("ow", **kw)
    bits0 = hp.host_bits(w)
    hp.run_hip(w)                                  # first append: provisional rows
    # second pass over the same slots with different K/V (the "committed" rows)
    g = torch.Generator(device=DEV); g.manual_seed(99)
    w.k_new = torch.randn(w.k_new.shape, generator=g, device=DEV).to(torch.bfloat16)
    w.v_new = torch.randn(w.v_new.shape, generator=g, device=DEV).to(torch.bfloat16)
    out, _ = hp.run_hip(w)
    bits1 = hp.host_bits(w)
    kp, vp = bits0["k_pool"].copy(), bits0["v_pool"].copy()
    p = hp.oracle_params(oracle_mod, w)
    oracle_mod.kv_append(p, w.cu_q, w.prefix_len, w.block_table, bits1["k_new"], bits1["v_new"], kp, vp)
    np.testing.assert_array_equal(bits1["k_pool"], kp)
    np.testing.assert_array_equal(bits1["v_pool"], vp)
    ref, _, _ = hp.run_oracle(oracle_mod, w, bits=dict(bits0, k_new=bits1["k_new"], v_new=bits1["v_new"]))
    hp.check_close(out.float().cpu().numpy(), ref, what="overwrite")


def test_one_call_step(oracle_mod):
    """optimus_attn_step = plan_update + kv_append + attn_forward: same outputs and pool bytes as
    the three calls (here: against the oracle), with explicit positions in the block-causal
    mode, and the refusal of a workspace that is too small for the new plan."""
    _say("one-call step")
    kw = dict(seed=61, num_q_heads=28, num_kv_heads=4, head_dim=128, page_size=16, block_size=32,
              prefix_len=[700, 90, 1500, 15, 333, 64, 4000], chunk=[1, 2, 4, 8, 16, 32, 5],
              block_inner=[0] * 7, device=DEV)
    w = inputs.make_workload("step", **kw)
    _, plan = full_parity(oracle_mod, w, "step", step=True)
    assert plan.num_merge_items() > 0
    w = inputs.make_workload("step_obs", **dict(kw, mask_mode=1, chunk=[1, 2, 40, 8, 16, 70, 5]))
    full_parity(oracle_mod, w, "step mask mode 1", step=True)
    # too small a workspace: error after planning, nothing launched (the output stays poisoned)
    w = inputs.make_workload("step", **kw)
    p = hp.params_of(w)
    from paper_2605_24832_amd import OptimusError, Plan
    plan = Plan(p, device=0)
    bt = torch.as_tensor(w.block_table, device=DEV)
    out = torch.full_like(w.q, float("nan"))
    with pytest.raises(OptimusError) as e:
        plan.attn_step(w.cu_q, w.prefix_len, w.block_start, w.block_table, w.q, w.k_new, w.v_new,
                       w.k_pool, w.v_pool, bt, out, torch.empty(4, dtype=torch.float32, device=DEV))
    assert e.value.status == -8
    torch.cuda.synchronize()
    assert torch.isnan(out.float()).all()


def test_step_on_premarshalled_descriptors_and_buffers(oracle_mod):
    """Plan.attn_step_bound (HostBatch + DeviceBuffers resolved once) is the same library call as
    attn_step: equal outputs and pools bit for bit, and descriptors rewritten in place between
    two iterations are what the second iteration uses (checked against the oracle)."""
    _say("bound step")
    from paper_2605_24832_amd import DeviceBuffers, HostBatch, Plan
    kw = dict(seed=67, num_q_heads=16, num_kv_heads=2, head_dim=128, page_size=16, block_size=32,
              device=DEV)
    L1, c1 = [760, 90, 1500, 15], [1, 8, 4, 16]
    L2, c2 = [701, 98, 1504, 31], [3, 2, 16, 1]          # same batch, other lengths and chunks
    w1 = inputs.make_workload("bound", prefix_len=L1, chunk=c1, block_inner=[0] * 4,
                              max_pages_per_req=100, **kw)
    w2 = inputs.make_workload("bound", prefix_len=L2, chunk=c2, block_inner=[0] * 4,
                              max_pages_per_req=100, **kw)
    assert w2.num_pages <= w1.num_pages   # the plan is created for w1's pool
    p = hp.params_of(w1)
    plan = Plan(p, device=0)
    ws = torch.empty(1 << 22, dtype=torch.float32, device=DEV)
    host = HostBatch(w1.cu_q, w1.prefix_len, w1.block_start, w1.block_table)
    # iteration 1 on w1's tensors
    bits1 = hp.host_bits(w1)
    out1 = torch.full_like(w1.q, float("nan"))
    bt1 = torch.as_tensor(w1.block_table, device=DEV)
    plan.attn_step_bound(host, DeviceBuffers(w1.q, w1.k_new, w1.v_new, w1.k_pool, w1.v_pool, bt1, out1, ws))
    ref1, _, _ = hp.run_oracle(oracle_mod, w1, bits=bits1)
    hp.check_close(out1.float().cpu().numpy(), ref1, what="bound step 1")
    wa = inputs.make_workload("bound", prefix_len=L1, chunk=c1, block_inner=[0] * 4,
                              max_pages_per_req=100, **kw)
    out_a, _ = hp.run_hip(wa, step=True)
    assert torch.equal(out1, out_a)
    np.testing.assert_array_equal(inputs.to_bits(w1.k_pool), inputs.to_bits(wa.k_pool))   # NaN poison: bits
    np.testing.assert_array_equal(inputs.to_bits(w1.v_pool), inputs.to_bits(wa.v_pool))
    # iteration 2: the same HostBatch rewritten in place, w2's tensors
    host.cu_q[:] = w2.cu_q
    host.prefix_len[:] = w2.prefix_len
    host.block_start[:] = w2.block_start
    host.block_table[:] = w2.block_table
    with pytest.raises(AttributeError):
        host.cu_q = np.zeros(5, dtype=np.int32)
    bits2 = hp.host_bits(w2)
    out2 = torch.full_like(w2.q, float("nan"))
    bt2 = torch.as_tensor(w2.block_table, device=DEV)
    plan.attn_step_bound(host, DeviceBuffers(w2.q, w2.k_new, w2.v_new, w2.k_pool, w2.v_pool, bt2, out2, ws))
    ref2, _, _ = hp.run_oracle(oracle_mod, w2, bits=bits2)
    mx, mean = hp.check_close(out2.float().cpu().numpy(), ref2, what="bound step 2")
    _say(f"bound step 2: max={mx:.2e} mean={mean:.2e}")


@pytest.mark.parametrize("R", [191, 192, 193, 400])
def test_append_run_list_in_the_argument_block_or_in_memory(oracle_mod, R):
    """Up to 192 append runs travel in the kernel's argument block, longer lists are read from
    memory: both sides of the limit (one run per request here), pools bit-exact, outputs to
    the bar."""
    _say(f"append runs R={R}")
    rng = np.random.RandomState(R)
    L = rng.randint(0, 200, size=R)
    w = inputs.make_workload("runs", seed=500 + R, num_q_heads=4, num_kv_heads=2, head_dim=64,
                             page_size=16, block_size=32, prefix_len=L, chunk=[1] * R,
                             block_inner=L % 32, device=DEV)
    full_parity(oracle_mod, w, f"append runs R={R}")


def test_empty_batches():
    _say("empty")
    w = inputs.make_workload("empty", seed=37, num_q_heads=8, num_kv_heads=2, head_dim=128,
                             page_size=16, block_size=32, prefix_len=[50, 20], chunk=[0, 0],
                             device=DEV)
    out, plan = hp.run_hip(w)
    assert out.shape[0] == 0 and plan.num_work_items() == 0
    from paper_2605_24832_amd import Plan
    plan = Plan(hp.params_of(w), device=0)
    assert plan.plan_update([0], [], []) == 0
    plan.attn_forward(None, None, None, None, None)  # no-op on an empty plan


def test_config2_gqa_continuous_batching(oracle_mod):
    """Every output of the full-size launch against the oracle (all 64 requests, all heads)."""
    _say("config2")
    w = inputs.make_config(2, device=DEV)
    _, plan = full_parity(oracle_mod, w, "config2")
    assert plan.num_merge_items() > 0


def test_config3_high_load(oracle_mod):
    """Every output of the full-size launch against the oracle (all 256 requests, all heads)."""
    _say("config3")
    w = inputs.make_config(3, device=DEV)
    assert w.k_pool.numel() * 2 > (1 << 31)  # the pool crosses the 32-bit byte-offset range
    full_parity(oracle_mod, w, "config3")


@pytest.mark.parametrize("chunk", [64, 128, None])
def test_config4_long_context(oracle_mod, chunk):
    """Every output of the full-size launch against the oracle: all 4 requests, all 8 kv heads
    (the oracle needs a few seconds per variant on the machine's host cores)."""
    _say(f"config4 chunk={chunk}")
    w = inputs.make_config(4, device=DEV, chunk=chunk)
    assert w.extra["peaked_positions"] > 0
    full_parity(oracle_mod, w, f"config4 chunk={chunk}")


def test_fp32_output_all_bodies(oracle_mod):
    """fp32 output from every body (split-wave, lds-tile, wide; unsplit and merged), tighter bar:
    without the bf16 store only the bf16 rounding of P is left."""
    _say("fp32 out, all bodies")
    kw = dict(seed=53, num_q_heads=16, num_kv_heads=2, head_dim=128, page_size=16, block_size=32,
              prefix_len=[900, 333, 1200, 64], chunk=[2, 7, 32, 16], block_inner=[0, 0, 0, 0], device=DEV)
    for tuning in (None, dict(target_items=1 << 20, min_split_tokens=128, max_split_tokens=128)):
        w = inputs.make_workload("fp32", **kw)
        bits = hp.host_bits(w)
        out, plan = hp.run_hip(w, out_dtype=1, tuning=tuning)
        ref, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
        mx, mean = hp.check_close(out.cpu().numpy(), ref, max_tol=5e-3, mean_tol=5e-4, what="fp32 out")
        _say(f"fp32 out: merges={plan.num_merge_items()} max={mx:.2e} mean={mean:.2e}")


def test_one_plan_over_many_updates(oracle_mod):
    """One plan object across decoding iterations whose descriptors grow and shrink (Sec. 4.4:
    the chunk size is re-chosen every iteration): after every plan_update the whole step is
    compared with the oracle and the pools bit for bit.  Covers the staging ring (more updates
    than slots), appends with and without a pending upload, and the growth of the plan's device
    buffer while earlier kernels are still queued."""
    _say("plan reuse")
    from paper_2605_24832_amd import Plan
    rng = np.random.RandomState(77)
    Hq, Hkv, D, P, B = 8, 2, 128, 16, 32
    R_max, max_pages = 24, 80
    num_pages = R_max * max_pages
    g = torch.Generator(device=DEV); g.manual_seed(78)
    k_pool = torch.randn((num_pages, Hkv, P * D), generator=g, device=DEV).to(torch.bfloat16)
    v_pool = torch.randn((num_pages, Hkv, P * D), generator=g, device=DEV).to(torch.bfloat16)
    table = rng.permutation(num_pages).astype(np.int32).reshape(R_max, max_pages)
    plan = Plan(hp.params_of_geometry(Hq, Hkv, D, P, B, num_pages, max_pages), device=0)
    p_or = oracle_mod.make_params(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P,
                                  block_size=B, max_pages_per_req=max_pages)
    batches = [2, 24, 5, 1, 17, 24, 3, 9]          # shrinking and growing work lists
    for it, R in enumerate(batches):
        blocks = rng.randint(0, 36, size=R)
        d_in = rng.randint(0, B, size=R)
        c = np.array([rng.randint(0, B - d + 1) for d in d_in])
        if it == 3:
            c[:] = 0                                # an iteration without any chunk token
        L = (blocks * B + d_in).astype(np.int32)
        cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
        T = int(cu[-1])
        q = torch.randn((T, Hq, D), generator=g, device=DEV).to(torch.bfloat16)
        k_new = torch.randn((T, Hkv, D), generator=g, device=DEV).to(torch.bfloat16)
        v_new = torch.randn((T, Hkv, D), generator=g, device=DEV).to(torch.bfloat16)
        bt_h = table[:R]
        kb, vb = inputs.to_bits(k_pool), inputs.to_bits(v_pool)   # pools before this iteration
        # iterations 5 and 6 keep the descriptors of a repeated step: plan once, run twice
        ws_bytes = plan.plan_update(cu, L, (L - d_in).astype(np.int32), bt_h)
        bt = torch.as_tensor(bt_h, device=DEV)
        ws = torch.full((max(ws_bytes, 16) // 4 + 4,), float("nan"), dtype=torch.float32, device=DEV)
        out = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device=DEV)
        reps = 2 if it in (5, 6) else 1
        for _ in range(reps):                       # the second pass appends without a pending upload
            plan.kv_append(k_pool, v_pool, k_new, v_new, bt)
            plan.attn_forward(q, k_pool, v_pool, bt, out, ws)
        torch.cuda.synchronize()
        _say(f"  iteration {it}: R={R} T={T} items={plan.num_work_items()} merges={plan.num_merge_items()}")
        if T:
            ref = oracle_mod.chunked_attention(p_or, cu, L, (L - d_in).astype(np.int32), bt_h,
                                               inputs.to_bits(q), inputs.to_bits(k_new),
                                               inputs.to_bits(v_new), kb, vb)
            hp.check_close(out.float().cpu().numpy(), ref, what=f"plan reuse, iteration {it}")
        oracle_mod.kv_append(p_or, cu, L, bt_h, inputs.to_bits(k_new), inputs.to_bits(v_new), kb, vb)
        np.testing.assert_array_equal(inputs.to_bits(k_pool), kb)
        np.testing.assert_array_equal(inputs.to_bits(v_pool), vb)
    plan.close()


@pytest.mark.parametrize("seed", range(24))
def test_random_small_workloads(oracle_mod, seed):
    """Seeded random shapes, descriptors and planner tunings (every body, every page size,
    both mask modes, splits of any size): full parity against the oracle."""
    rng = np.random.RandomState(9000 + seed)
    D = int(rng.choice([64, 128]))
    P = int(rng.choice([16, 32, 64, 128]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 4, 7, 8]))
    B = int(rng.choice([32, 64, 128]))
    mask_mode = int(rng.choice([0, 1]))
    R = int(rng.randint(1, 6))
    d_in = rng.randint(0, B, size=R)                                  # cached tokens inside the block
    if mask_mode == 0:
        c = np.array([rng.randint(0, B - d + 1) for d in d_in])      # chunk stays in the block
    else:
        c = rng.randint(0, B + 1, size=R)                             # may cross into the next block
    if c.sum() == 0:
        c[0] = 1                                                      # d_in < B: one token always fits
    blocks_before = rng.randint(0, 2000 // B, size=R)
    L = blocks_before * B + d_in
    _say(f"random seed={seed} D={D} P={P} Hq={Hkv * G} Hkv={Hkv} B={B} mask={mask_mode} L={L.tolist()} c={c.tolist()}")
    w = inputs.make_workload("rnd", seed=7000 + seed, num_q_heads=Hkv * G, num_kv_heads=Hkv, head_dim=D,
                             page_size=P, block_size=B, prefix_len=L, chunk=c, block_inner=d_in,
                             mask_mode=mask_mode, device=DEV)
    split = int(rng.choice([0, 32, 64, 256, 1024]))
    tuning = None if split == 0 else dict(target_items=1 << 20, min_split_tokens=split, max_split_tokens=split)
    full_parity(oracle_mod, w, f"random {seed}", tuning=tuning)
