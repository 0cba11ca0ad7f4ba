"""Pins of the fp64 CPU oracle against things other than itself.

The paper prints no worked numeric example for the attention step, so the
oracle is pinned to: an independent numpy brute force with an explicit mask
matrix, PyTorch's scaled_dot_product_attention in fp64 on the dense special
case, the textbook single-token decode attention (c_i = 1), closed forms
(constant V, zero Q, peaked Q, shift invariance, sum-to-one), and structural
invariants (chunk permutation, GQA replication, page reshuffle, page size,
ragged batching, NaN tails, block-start inertness, split-and-merge algebra).
"""
import copy

import numpy as np
import pytest
import torch

from paper_2605_24832_amd import inputs
from tests import bruteforce


def bits_of(w):
    return {k: inputs.to_bits(getattr(w, k)) for k in ("q", "k_new", "v_new", "k_pool", "v_pool")}


def oracle_params(oracle, w, **kw):
    args = dict(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                page_size=w.page_size, block_size=w.block_size,
                max_pages_per_req=w.block_table.shape[1], mask_mode=w.mask_mode,
                kv_layout=w.kv_layout)
    args.update(kw)
    return oracle.make_params(**args)


def run_oracle(oracle, w, bits=None, q_pos=None, **kw):
    b = bits_of(w) if bits is None else bits
    p = oracle_params(oracle, w, **kw)
    return oracle.chunked_attention(p, w.cu_q, w.prefix_len, w.block_start, w.block_table, b["q"],
                                    b["k_new"], b["v_new"], b["k_pool"], b["v_pool"], q_pos=q_pos)


def small(seed=1, **kw):
    args = dict(num_q_heads=4, num_kv_heads=2, head_dim=16, page_size=4, block_size=8,
                prefix_len=[5, 0, 13, 8], chunk=[3, 2, 1, 0])
    args.update(kw)
    return inputs.make_workload("small", seed=seed, **args)


def f64_to_bf16_bits(x):
    return inputs.to_bits(torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ---------------------------------------------------------------- brute force

@pytest.mark.parametrize("kv_layout", [0, 1])
@pytest.mark.parametrize("mask_mode", [0, 1])
def test_matches_numpy_bruteforce(oracle_mod, kv_layout, mask_mode):
    # mode 1 needs chunks that cross a block boundary to exercise the mask
    w = small(seed=3, kv_layout=kv_layout, mask_mode=mask_mode, prefix_len=[5, 0, 13, 8, 30],
              chunk=[3, 2, 1, 0, 7], block_inner=[5, 0, 5, 0, 6] if mask_mode else None)
    got = run_oracle(oracle_mod, w)
    ref = bruteforce.attention(w, bits_of(w))
    assert got.shape == ref.shape
    assert np.isfinite(got).all()
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


def test_block_causal_mask_changes_result_when_chunk_crosses_block(oracle_mod):
    w0 = small(seed=4, prefix_len=[6], chunk=[6], block_inner=[6], mask_mode=0)
    a = run_oracle(oracle_mod, w0, mask_mode=0)
    b = run_oracle(oracle_mod, w0, mask_mode=1)
    # queries 0,1 sit in the first block (positions 6,7) and lose keys 2..5
    assert np.abs(a[:2] - b[:2]).max() > 1e-3
    # queries 2.. sit in the second block and see everything in both modes
    np.testing.assert_array_equal(a[2:], b[2:])


def test_explicit_positions_contiguous_case_and_mode_0(oracle_mod):
    """Positions that follow the cached tokens of the block contiguously give the default
    block-causal result bit for bit; in mode 0 positions are not looked at."""
    w = small(seed=5, prefix_len=[13, 6, 20], chunk=[7, 8, 5], block_inner=[5, 6, 4], mask_mode=1)
    pos = np.concatenate([np.arange(c) + L for L, c in zip(w.prefix_len, w.chunk)]).astype(np.int32)
    np.testing.assert_array_equal(run_oracle(oracle_mod, w, q_pos=pos), run_oracle(oracle_mod, w))
    rng = np.random.RandomState(5)
    anywhere = (w.block_start.repeat(w.chunk) + rng.randint(0, 40, size=len(pos))).astype(np.int32)
    np.testing.assert_array_equal(run_oracle(oracle_mod, w, q_pos=anywhere, mask_mode=0),
                                  run_oracle(oracle_mod, w, mask_mode=0))


def test_explicit_positions_hand_worked_holes(oracle_mod):
    """Block size 4, block origin 6 (not a multiple of the block size), one cached token inside
    the block.  Chunk tokens at sequence positions 7, 9, 10, 12: offsets 1, 3, 4, 6 from the
    origin, i.e. blocks 0, 0, 1, 1.  Queries 0, 1 see chunk keys 0, 1; queries 2, 3 see all four.
    The contiguous reading would put them at offsets 1, 2, 3, 4 (blocks 0, 0, 0, 1)."""
    w = small(seed=6, block_size=4, prefix_len=[7], chunk=[4], block_inner=[1], mask_mode=1)
    assert w.block_start[0] == 6
    pos = np.array([7, 9, 10, 12], dtype=np.int32)
    table = [[1, 1, 0, 0],
             [1, 1, 0, 0],
             [1, 1, 1, 1],
             [1, 1, 1, 1]]
    got = run_oracle(oracle_mod, w, q_pos=pos)
    ref = bruteforce.attention(w, bits_of(w), chunk_mask={0: table})
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert np.abs(got - run_oracle(oracle_mod, w)).max() > 1e-3   # not the contiguous reading
    # later positions in an earlier block of the chunk order: visibility follows the positions,
    # not the order of the chunk tokens
    pos2 = np.array([12, 7, 10, 9], dtype=np.int32)                # blocks 1, 0, 1, 0
    table2 = [[1, 1, 1, 1],
              [0, 1, 0, 1],
              [1, 1, 1, 1],
              [0, 1, 0, 1]]
    got2 = run_oracle(oracle_mod, w, q_pos=pos2)
    ref2 = bruteforce.attention(w, bits_of(w), chunk_mask={0: table2})
    np.testing.assert_allclose(got2, ref2, rtol=0, atol=1e-12)


def test_bruteforce_scale_argument(oracle_mod):
    w = small(seed=5)
    got = run_oracle(oracle_mod, w, scale=0.37)
    ref = bruteforce.attention(w, bits_of(w), scale=0.37)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- library routine

@pytest.mark.parametrize("mask_mode", [0, 1])
def test_matches_torch_sdpa_fp64(oracle_mod, mask_mode):
    Hq, Hkv, D, B = 6, 2, 32, 8
    w = inputs.make_workload("sdpa", seed=7, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D,
                             page_size=4, block_size=B, prefix_len=[19, 4], chunk=[5, 7],
                             block_inner=[3, 4], mask_mode=mask_mode, kv_layout=1)
    got = run_oracle(oracle_mod, w)
    b = bits_of(w)
    G = Hq // Hkv
    for i in range(w.batch):
        a, e = int(w.cu_q[i]), int(w.cu_q[i + 1])
        c, L = e - a, int(w.prefix_len[i])
        q = torch.as_tensor(bruteforce.bf16_bits_to_f64(b["q"]).reshape(-1, Hq, D)[a:e]).permute(1, 0, 2)
        Ks, Vs = [], []
        for h in range(Hq):
            Kc, Vc = bruteforce.logical_kv(w, b["k_pool"], b["v_pool"], i, h // G)
            kn = bruteforce.bf16_bits_to_f64(b["k_new"]).reshape(-1, Hkv, D)[a:e, h // G]
            vn = bruteforce.bf16_bits_to_f64(b["v_new"]).reshape(-1, Hkv, D)[a:e, h // G]
            Ks.append(np.concatenate([Kc, kn]))
            Vs.append(np.concatenate([Vc, vn]))
        K = torch.as_tensor(np.stack(Ks))
        V = torch.as_tensor(np.stack(Vs))
        mask = None
        if mask_mode == 1:
            d_in = L - int(w.block_start[i])
            blk = (d_in + np.arange(c)) // B
            m = np.ones((c, L + c), dtype=bool)
            m[:, L:] = blk[None, :] <= blk[:, None]
            mask = torch.as_tensor(m)
        ref = torch.nn.functional.scaled_dot_product_attention(
            q[None], K[None], V[None], attn_mask=mask, is_causal=False)[0]
        np.testing.assert_allclose(got[a:e], ref.permute(1, 0, 2).numpy(), rtol=0, atol=1e-12)


def test_single_token_chunk_is_decode_attention(oracle_mod):
    """c_i = 1: one query over L_i cached keys plus itself, the textbook decode step."""
    w = small(seed=8, prefix_len=[11, 6], chunk=[1, 1])
    got = run_oracle(oracle_mod, w)
    b = bits_of(w)
    Hq, Hkv, D = w.num_q_heads, w.num_kv_heads, w.head_dim
    q = bruteforce.bf16_bits_to_f64(b["q"]).reshape(-1, Hq, D)
    kn = bruteforce.bf16_bits_to_f64(b["k_new"]).reshape(-1, Hkv, D)
    vn = bruteforce.bf16_bits_to_f64(b["v_new"]).reshape(-1, Hkv, D)
    for i in range(2):
        for h in range(Hq):
            g = h // (Hq // Hkv)
            Kc, Vc = bruteforce.logical_kv(w, b["k_pool"], b["v_pool"], i, g)
            K = np.vstack([Kc, kn[i, g][None]])
            V = np.vstack([Vc, vn[i, g][None]])
            s = K @ q[i, h] / np.sqrt(D)
            p = np.exp(s - s.max())
            p /= p.sum()
            np.testing.assert_allclose(got[i, h], p @ V, rtol=0, atol=1e-12)


# ---------------------------------------------------------------- closed forms

def test_softmax_rows_sum_to_one_and_are_nonnegative(oracle_mod):
    w = small(seed=9)
    b = bits_of(w)
    p = oracle_params(oracle_mod, w)
    for (i, j, h) in [(0, 0, 0), (0, 2, 3), (1, 1, 2), (2, 0, 1)]:
        pr = oracle_mod.attention_probs(p, w.cu_q, w.prefix_len, w.block_start, w.block_table,
                                        b["q"], b["k_new"], b["v_new"], b["k_pool"], b["v_pool"],
                                        i, j, h)
        assert len(pr) == w.prefix_len[i] + w.chunk[i]
        assert (pr >= 0).all()
        assert abs(pr.sum() - 1.0) < 1e-14


def test_probs_times_v_is_output(oracle_mod):
    w = small(seed=10)
    b = bits_of(w)
    p = oracle_params(oracle_mod, w)
    out = run_oracle(oracle_mod, w)
    i, j, h = 2, 0, 3
    g = h // 2
    pr = oracle_mod.attention_probs(p, w.cu_q, w.prefix_len, w.block_start, w.block_table, b["q"],
                                    b["k_new"], b["v_new"], b["k_pool"], b["v_pool"], i, j, h)
    _, Vc = bruteforce.logical_kv(w, b["k_pool"], b["v_pool"], i, g)
    a, e = w.cu_q[i], w.cu_q[i + 1]
    vn = bruteforce.bf16_bits_to_f64(b["v_new"]).reshape(-1, 2, 16)[a:e, g]
    np.testing.assert_allclose(out[a + j, h], pr @ np.vstack([Vc, vn]), rtol=0, atol=1e-13)


def test_constant_v_returns_v(oracle_mod):
    w = small(seed=11, poison=False)
    v0 = torch.linspace(-1.5, 2.0, w.head_dim).to(torch.bfloat16)
    P, D = w.page_size, w.head_dim
    inputs.v_tile_view(w.v_pool, P, D, w.kv_layout)[:] = (
        v0.view(1, 1, D, 1) if w.kv_layout == 1 else v0.view(1, 1, 1, D))
    w.v_new[:] = v0
    out = run_oracle(oracle_mod, w)
    ref = v0.to(torch.float64).numpy()
    assert out.shape[0] == w.total_q
    np.testing.assert_allclose(out, np.broadcast_to(ref, out.shape), rtol=0, atol=1e-14)


def test_zero_query_gives_mean_of_visible_values(oracle_mod):
    w = small(seed=12)
    w.q.zero_()
    out = run_oracle(oracle_mod, w)
    b = bits_of(w)
    vn = bruteforce.bf16_bits_to_f64(b["v_new"]).reshape(-1, 2, 16)
    for i in range(w.batch):
        a, e = int(w.cu_q[i]), int(w.cu_q[i + 1])
        for h in range(4):
            _, Vc = bruteforce.logical_kv(w, b["k_pool"], b["v_pool"], i, h // 2)
            mean = np.vstack([Vc, vn[a:e, h // 2]]).mean(axis=0)
            for t in range(a, e):
                np.testing.assert_allclose(out[t, h], mean, rtol=0, atol=1e-14)


def test_shift_invariance_of_keys(oracle_mod):
    """Adding one vector u to every visible key adds q.u to every score of a row."""
    w = small(seed=13, poison=False, prefix_len=[9], chunk=[3], head_dim=16)
    base = run_oracle(oracle_mod, w)
    # values that stay exactly representable in bf16 after the shift: multiples of 1/8, small
    for t in (w.k_pool, w.k_new):
        t.copy_((torch.round(t.float() * 8) / 8).clamp(-3, 3).to(torch.bfloat16))
    u = (torch.arange(16) % 5 - 2).float() / 4
    ref = run_oracle(oracle_mod, w)
    P, D = w.page_size, w.head_dim
    kt = inputs.k_tile_view(w.k_pool, P, D, w.kv_layout)
    kt += u.view(D // 8, 1, 8).to(torch.bfloat16)
    w.k_new += u.to(torch.bfloat16)
    got = run_oracle(oracle_mod, w)
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-12)
    assert np.abs(ref - base).max() > 0  # the rounding step did change the data


def test_peaked_query_selects_one_value(oracle_mod):
    w = small(seed=14, prefix_len=[12], chunk=[2], poison=False)
    b = bits_of(w)
    Kc, Vc = bruteforce.logical_kv(w, b["k_pool"], b["v_pool"], 0, 1)
    n_star = 7
    qv = torch.as_tensor(Kc[n_star] * 64.0).to(torch.bfloat16)
    w.q[0, 2] = qv  # head 2 -> kv head 1
    out = run_oracle(oracle_mod, w)
    s = (np.vstack([Kc]) @ qv.double().numpy()) / 4.0
    assert s[n_star] - np.delete(s, n_star).max() > 40  # the construction is peaked enough
    np.testing.assert_allclose(out[0, 2], Vc[n_star], rtol=0, atol=1e-12)


# ---------------------------------------------------------------- structural invariants

def test_chunk_permutation_permutes_outputs(oracle_mod):
    w = small(seed=15, prefix_len=[10, 3], chunk=[5, 4])
    ref = run_oracle(oracle_mod, w)
    perm = np.array([3, 0, 4, 1, 2, 5 + 2, 5 + 3, 5 + 0, 5 + 1])
    w2 = copy.copy(w)
    pt = torch.as_tensor(perm)
    w2.q, w2.k_new, w2.v_new = w.q[pt], w.k_new[pt], w.v_new[pt]
    got = run_oracle(oracle_mod, w2)
    np.testing.assert_allclose(got, ref[perm], rtol=0, atol=1e-13)


def test_gqa_equals_replicated_mha(oracle_mod):
    w = small(seed=16, num_q_heads=6, num_kv_heads=2)
    ref = run_oracle(oracle_mod, w)
    G = 3
    w2 = copy.copy(w)
    w2.num_kv_heads = 6
    w2.k_new = w.k_new.repeat_interleave(G, dim=1)
    w2.v_new = w.v_new.repeat_interleave(G, dim=1)
    w2.k_pool = w.k_pool.repeat_interleave(G, dim=1).contiguous()
    w2.v_pool = w.v_pool.repeat_interleave(G, dim=1).contiguous()
    got = run_oracle(oracle_mod, w2)
    np.testing.assert_array_equal(got, ref)


def test_page_reshuffle_is_bit_identical(oracle_mod):
    w = small(seed=17)
    ref = run_oracle(oracle_mod, w)
    rng = np.random.RandomState(0)
    perm = rng.permutation(w.num_pages)          # new_id = perm[old_id]
    inv = np.argsort(perm)
    w2 = copy.copy(w)
    w2.k_pool = w.k_pool[torch.as_tensor(inv)].contiguous()
    w2.v_pool = w.v_pool[torch.as_tensor(inv)].contiguous()
    bt = w.block_table.copy()
    bt[bt >= 0] = perm[bt[bt >= 0]]
    w2.block_table = bt
    got = run_oracle(oracle_mod, w2)
    np.testing.assert_array_equal(got, ref)


def logical_to_pool(K_rows, V_rows, Hkv, P, D, kv_layout):
    """Pack logical rows ``[n, Hkv, D]`` into in-order pages (test-side, numpy)."""
    n = K_rows.shape[0]
    pages = (n + P - 1) // P
    kp = np.full((max(pages, 1), Hkv, P * D), inputs.BF16_NAN_BITS, dtype=np.uint16)
    vp = kp.copy()
    for t in range(n):
        pg, sl = t // P, t % P
        for g in range(Hkv):
            if kv_layout == 0:
                kp[pg, g].reshape(P, D)[sl] = K_rows[t, g]
                vp[pg, g].reshape(P, D)[sl] = V_rows[t, g]
            else:
                kp[pg, g].reshape(D // 8, P, 8)[:, sl, :] = K_rows[t, g].reshape(D // 8, 8)
                vp[pg, g].reshape(D, P)[:, sl] = V_rows[t, g]
    return kp, vp


@pytest.mark.parametrize("kv_layout", [0, 1])
def test_page_size_and_layout_do_not_matter(oracle_mod, kv_layout):
    Hq, Hkv, D, L, c = 4, 2, 16, 21, 3
    rng = np.random.RandomState(18)
    rows = lambda n, h: f64_to_bf16_bits(rng.standard_normal((n, h, D)))
    Kr, Vr = rows(L, Hkv), rows(L, Hkv)
    q, kn, vn = rows(c, Hq), rows(c, Hkv), rows(c, Hkv)
    outs = []
    for P in (2, 4, 16, 32):
        kp, vp = logical_to_pool(Kr, Vr, Hkv, P, D, kv_layout)
        pages = kp.shape[0]
        need = (L + c + P - 1) // P
        bt = np.full((1, max(need, pages)), -1, dtype=np.int32)
        bt[0, :pages] = np.arange(pages)
        p = oracle_mod.make_params(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P,
                                   block_size=32, max_pages_per_req=bt.shape[1], kv_layout=kv_layout)
        outs.append(oracle_mod.chunked_attention(p, [0, c], [L], [L], bt, q, kn, vn, kp, vp))
    for o in outs[1:]:
        np.testing.assert_array_equal(o, outs[0])
    # and against a direct dense computation from the logical rows
    K = np.concatenate([bruteforce.bf16_bits_to_f64(Kr), bruteforce.bf16_bits_to_f64(kn)])
    V = np.concatenate([bruteforce.bf16_bits_to_f64(Vr), bruteforce.bf16_bits_to_f64(vn)])
    qf = bruteforce.bf16_bits_to_f64(q)
    for h in range(Hq):
        S = qf[:, h] @ K[:, h // 2].T / 4.0
        E = np.exp(S - S.max(axis=1, keepdims=True))
        np.testing.assert_allclose(outs[0][:, h], (E / E.sum(1, keepdims=True)) @ V[:, h // 2],
                                   rtol=0, atol=1e-12)


def test_request_alone_equals_request_in_batch(oracle_mod):
    w = small(seed=19, prefix_len=[5, 9, 13], chunk=[3, 2, 4])
    full = run_oracle(oracle_mod, w)
    b = bits_of(w)
    for i in range(3):
        a, e = int(w.cu_q[i]), int(w.cu_q[i + 1])
        p = oracle_params(oracle_mod, w)
        alone = oracle_mod.chunked_attention(
            p, [0, e - a], w.prefix_len[i:i + 1], w.block_start[i:i + 1], w.block_table[i:i + 1],
            b["q"].reshape(-1, 4, 16)[a:e], b["k_new"].reshape(-1, 2, 16)[a:e],
            b["v_new"].reshape(-1, 2, 16)[a:e], b["k_pool"], b["v_pool"])
        np.testing.assert_array_equal(alone, full[a:e])


def test_nan_tails_and_unused_pages_do_not_leak(oracle_mod):
    clean = small(seed=20, poison=False)
    dirty = small(seed=20, poison=True)
    assert torch.isnan(dirty.k_pool.float()).any() and not torch.isnan(clean.k_pool.float()).any()
    a = run_oracle(oracle_mod, clean)
    b = run_oracle(oracle_mod, dirty)
    assert np.isfinite(b).all()
    np.testing.assert_array_equal(a, b)


def test_block_start_is_inert_in_mode_0(oracle_mod):
    w = small(seed=21, prefix_len=[13, 6], chunk=[2, 2])
    ref = run_oracle(oracle_mod, w)
    for d_in in ([0, 0], [5, 6], [3, 1]):
        w2 = copy.copy(w)
        w2.block_start = (w.prefix_len - np.array(d_in)).astype(np.int32)
        np.testing.assert_array_equal(run_oracle(oracle_mod, w2), ref)


def test_empty_chunks_and_empty_prefix(oracle_mod):
    w = small(seed=22, prefix_len=[0, 7, 0], chunk=[4, 0, 1])
    out = run_oracle(oracle_mod, w)
    assert out.shape == (5, 4, 16)
    ref = bruteforce.attention(w, bits_of(w))
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)
    # L=0, c=1: the only key is the query's own token -> output is its V row
    vn = bruteforce.bf16_bits_to_f64(bits_of(w)["v_new"]).reshape(-1, 2, 16)
    for h in range(4):
        np.testing.assert_allclose(out[4, h], vn[4, h // 2], rtol=0, atol=1e-15)


# ---------------------------------------------------------------- split / merge algebra

@pytest.mark.parametrize("cuts", [[0, 16], [0, 5, 16], [0, 1, 2, 9, 16], [0, 4, 4, 16]])
def test_merge_of_any_partition_equals_unsplit(oracle_mod, cuts):
    w = small(seed=23, prefix_len=[13], chunk=[3], mask_mode=0)
    b = bits_of(w)
    p = oracle_params(oracle_mod, w)
    full = run_oracle(oracle_mod, w)
    i, j, h = 0, 1, 3
    parts = [oracle_mod.partial_row(p, w.cu_q, w.prefix_len, w.block_start, w.block_table, b["q"],
                                    b["k_new"], b["v_new"], b["k_pool"], b["v_pool"], i, j, h, lo, hi)
             for lo, hi in zip(cuts[:-1], cuts[1:])]
    o = oracle_mod.merge_partials(np.stack([x[0] for x in parts]), np.array([x[1] for x in parts]),
                                  np.array([x[2] for x in parts]))
    np.testing.assert_allclose(o, full[j, h], rtol=0, atol=1e-13)
    # an empty range is the identity element: m = -inf, l = 0
    for (o_part, m, l), lo, hi in zip(parts, cuts[:-1], cuts[1:]):
        if lo == hi:
            assert m == -np.inf and l == 0.0 and not o_part.any()


def test_merge_against_direct_formula():
    import oracle
    rng = np.random.RandomState(24)
    S, D = 5, 8
    # build partials from a known score/value list
    s = rng.standard_normal(40) * 3
    V = rng.standard_normal((40, D))
    cuts = [0, 3, 11, 12, 30, 40]
    o_part, m, l = [], [], []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        mm = s[lo:hi].max()
        e = np.exp(s[lo:hi] - mm)
        o_part.append(e @ V[lo:hi]); m.append(mm); l.append(e.sum())
    got = oracle.merge_partials(np.array(o_part), np.array(m), np.array(l))
    e = np.exp(s - s.max())
    np.testing.assert_allclose(got, (e / e.sum()) @ V, rtol=0, atol=1e-14)


# ---------------------------------------------------------------- append step

@pytest.mark.parametrize("kv_layout", [0, 1])
def test_kv_append_matches_host_scatter_bit_exact(oracle_mod, kv_layout):
    w = small(seed=25, kv_layout=kv_layout, prefix_len=[5, 0, 13, 7], chunk=[3, 2, 4, 0])
    b = bits_of(w)
    kp, vp = b["k_pool"].copy(), b["v_pool"].copy()
    p = oracle_params(oracle_mod, w)
    oracle_mod.kv_append(p, w.cu_q, w.prefix_len, w.block_table, b["k_new"], b["v_new"], kp, vp)
    # independent scatter with numpy views
    P, D, Hkv = w.page_size, w.head_dim, w.num_kv_heads
    ek, ev = b["k_pool"].copy(), b["v_pool"].copy()
    kn = b["k_new"].reshape(-1, Hkv, D)
    vn = b["v_new"].reshape(-1, Hkv, D)
    for i in range(w.batch):
        for j in range(int(w.chunk[i])):
            n = int(w.prefix_len[i]) + j
            pg, sl = int(w.block_table[i, n // P]), n % P
            t = int(w.cu_q[i]) + j
            for g in range(Hkv):
                if kv_layout == 0:
                    ek[pg, g].reshape(P, D)[sl] = kn[t, g]
                    ev[pg, g].reshape(P, D)[sl] = vn[t, g]
                else:
                    ek[pg, g].reshape(D // 8, P, 8)[:, sl, :] = kn[t, g].reshape(D // 8, 8)
                    ev[pg, g].reshape(D, P)[:, sl] = vn[t, g]
    np.testing.assert_array_equal(kp, ek)
    np.testing.assert_array_equal(vp, ev)
    assert (kp != b["k_pool"]).any()


def test_append_then_treat_chunk_as_cached_gives_same_keys(oracle_mod):
    """After the append, a one-token chunk placed after L+c cached tokens sees exactly the
    keys the original chunk saw plus itself; with a hugely negative self score the output
    must equal the original chunk's row computed with the same query."""
    Hq = Hkv = 2
    D = 16
    w = small(seed=26, num_q_heads=Hq, num_kv_heads=Hkv, prefix_len=[9], chunk=[3], poison=True)
    b = bits_of(w)
    p = oracle_params(oracle_mod, w)
    ref = run_oracle(oracle_mod, w)
    kp, vp = b["k_pool"].copy(), b["v_pool"].copy()
    oracle_mod.kv_append(p, w.cu_q, w.prefix_len, w.block_table, b["k_new"], b["v_new"], kp, vp)
    # new request: L' = 12 cached (9 + appended 3), chunk = 1 token whose key is -64*q (score << 0)
    j = 1
    q1 = b["q"].reshape(-1, Hq, D)[j:j + 1]
    qf = bruteforce.bf16_bits_to_f64(q1)[0]
    kself = (-64.0 * qf)[None]
    for h in range(Hq):
        assert (qf[h] @ kself[0, h]) / 4.0 < -100
    k1 = f64_to_bf16_bits(kself)
    v1 = f64_to_bf16_bits(np.zeros((1, Hkv, D)))
    # 9+3 = 12 = 3 full pages of 4; slot 12 needs a 4th page: take the spare (unreferenced) one
    spare = sorted(set(range(w.num_pages)) - set(w.block_table.ravel().tolist()))
    assert spare
    bt = np.concatenate([w.block_table, np.array([[spare[0]]], dtype=np.int32)], axis=1)
    p2 = oracle_params(oracle_mod, w, max_pages_per_req=bt.shape[1])
    out = oracle_mod.chunked_attention(p2, [0, 1], [12], [12], bt, q1, k1, v1, kp, vp)
    np.testing.assert_allclose(out[0], ref[j], rtol=0, atol=1e-12)
