"""optimus_kv_write: a prompt's K/V reach the pool layout through the C ABI (Sec. 4.2 prefix
caching; Sec. 6), in several unaligned pieces, and attention over a prefix written this way
matches the oracle fed the same logical rows in the plain [page, head, slot, d] layout."""
import numpy as np
import pytest
import torch

from paper_2605_24832_amd import Plan, inputs, kv_write
from tests import hip_path as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
NAN = 0x7FC0


def plain_pool(rows, table, num_pages, Hkv, P, D):
    """Layout 0, written out with its own index formula: slot n of request i is row
    pool[table[i][n // P], head, n % P, :]."""
    pool = np.full((num_pages, Hkv, P, D), NAN, dtype=np.uint16)
    for i, r in enumerate(rows):
        for n in range(r.shape[0]):
            pool[table[i][n // P], :, n % P, :] = r[n]
    return pool.reshape(num_pages, Hkv, P * D)


@pytest.mark.parametrize("Hq,Hkv,D,P", [(8, 2, 128, 16), (6, 3, 64, 64), (4, 1, 128, 128)])
def test_prefix_written_through_the_library(oracle_mod, Hq, Hkv, D, P):
    print(f"kv_write Hq={Hq} Hkv={Hkv} D={D} P={P}", flush=True)
    rng = np.random.RandomState(500 + P)
    B = 32
    L = np.array([300, 45, 129, 1000, 0, 8], dtype=np.int32)
    c = np.array([7, 32, 1, 3, 5, 0], dtype=np.int32)
    R = len(L)
    pages = -(-(L + c) // P)
    max_pages = int(pages.max()) + 1
    num_pages = int(pages.sum()) + 7
    perm = rng.permutation(num_pages).astype(np.int32)
    table = np.full((R, max_pages), -1, dtype=np.int32)
    off = 0
    for i in range(R):
        table[i, :pages[i]] = perm[off:off + pages[i]]
        off += pages[i]
    g = torch.Generator(device=DEV); g.manual_seed(600 + P)
    rnd = lambda *shape: torch.randn(shape, generator=g, device=DEV).to(torch.bfloat16)
    k_rows = [rnd(int(n), Hkv, D) for n in L]
    v_rows = [rnd(int(n), Hkv, D) for n in L]
    params = hp.params_of_geometry(Hq, Hkv, D, P, B, num_pages, max_pages)
    nan = torch.tensor(float("nan"), dtype=torch.bfloat16, device=DEV)
    k_pool = nan.repeat(num_pages * Hkv * P * D).view(num_pages, Hkv, P * D)
    v_pool = k_pool.clone()
    bt = torch.as_tensor(table, device=DEV)
    # each prefix in up to three pieces with unaligned boundaries (also inside a group of 8 slots)
    for i in range(R):
        n = int(L[i])
        cuts = sorted({0, n} | set(rng.randint(0, n + 1, size=2).tolist())) if n else [0, 0]
        for a, b in zip(cuts[:-1], cuts[1:]):
            kv_write(params, k_pool, v_pool, k_rows[i][a:b].contiguous(), v_rows[i][a:b].contiguous(), bt, i, a)
    kv_write(params, k_pool, v_pool, k_rows[0][:0], v_rows[0][:0], bt, 0, 3)      # n = 0: no-op
    torch.cuda.synchronize()

    # bit-exact against the oracle's scatter (layout 1): the prefixes as "chunks" appended at slot 0
    p1 = oracle_mod.make_params(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P,
                                block_size=B, max_pages_per_req=max_pages)
    kp1 = np.full((num_pages, Hkv, P * D), NAN, dtype=np.uint16)
    vp1 = kp1.copy()
    cu_L = np.concatenate([[0], np.cumsum(L)]).astype(np.int32)
    cat = lambda rows: np.concatenate([inputs.to_bits(r) for r in rows])
    oracle_mod.kv_append(p1, cu_L, np.zeros(R, dtype=np.int32), table, cat(k_rows), cat(v_rows), kp1, vp1)
    np.testing.assert_array_equal(inputs.to_bits(k_pool), kp1)
    np.testing.assert_array_equal(inputs.to_bits(v_pool), vp1)

    # one decoding step on top; the oracle reads the same logical rows from the plain layout
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    T = int(cu[-1])
    q, k_new, v_new = rnd(T, Hq, D), rnd(T, Hkv, D), rnd(T, Hkv, D)
    d_in = np.minimum(L % B, B - c)
    s = (L - d_in).astype(np.int32)
    plan = Plan(params, device=0)
    ws_bytes = plan.plan_update(cu, L, s, table)
    ws = torch.empty(max(ws_bytes, 16) // 4 + 4, dtype=torch.float32, device=DEV)
    out = torch.full((T, Hq, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    plan.kv_append(k_pool, v_pool, k_new, v_new, bt)
    plan.attn_forward(q, k_pool, v_pool, bt, out, ws)
    torch.cuda.synchronize()
    p0 = oracle_mod.make_params(num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P,
                                block_size=B, max_pages_per_req=max_pages, kv_layout=0)
    kp0 = plain_pool([inputs.to_bits(r) for r in k_rows], table, num_pages, Hkv, P, D)
    vp0 = plain_pool([inputs.to_bits(r) for r in v_rows], table, num_pages, Hkv, P, D)
    ref = oracle_mod.chunked_attention(p0, cu, L, s, table, inputs.to_bits(q), inputs.to_bits(k_new),
                                       inputs.to_bits(v_new), kp0, vp0)
    mx, mean = hp.check_close(out.float().cpu().numpy(), ref, what="attention over a written prefix")
    print(f"  max={mx:.2e} mean={mean:.2e}", flush=True)


def test_kv_write_keeps_the_callers_device_and_rejects_bad_ranges():
    from paper_2605_24832_amd import OptimusError
    params = hp.params_of_geometry(4, 2, 64, 16, 32, 8, 2)
    z = torch.zeros((8, 2, 16 * 64), dtype=torch.bfloat16, device=DEV)
    src = torch.zeros((40, 2, 64), dtype=torch.bfloat16, device=DEV)
    bt = torch.zeros((1, 2), dtype=torch.int32, device=DEV)
    assert torch.cuda.current_device() == 0
    with pytest.raises(OptimusError) as e:
        kv_write(params, z, z, src, src, bt, 0, 0)          # 40 slots need 3 pages, the row has 2
    assert e.value.status == -6
    with pytest.raises(OptimusError) as e:
        kv_write(params, z, z, src[:4], src[:4], bt, 0, -1)
    assert e.value.status == -1
    # an entry outside the pool: that page's tokens are skipped, nothing is written out of bounds
    bad = torch.tensor([[99, 3]], dtype=torch.int32, device=DEV)
    kp, vp = z.clone(), z.clone()
    one = torch.ones((20, 2, 64), dtype=torch.bfloat16, device=DEV)
    kv_write(params, kp, vp, one, one, bad, 0, 0)
    torch.cuda.synchronize()
    assert kp[3].float().sum().item() == 4 * 2 * 64 and kp[:3].float().sum().item() == 0
    assert torch.cuda.current_device() == 0
