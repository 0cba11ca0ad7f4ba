"""One decoding iteration end to end through the C ABI, twice in a row, against the oracles:
reorganisation (chunk from the decoded map, Sec. 4.4) -> plan, KV append, attention (Sec. 4,
Sec. 6) -> commit on synthetic logits (Sec. 2.3) -> decoded map updated with the committed
positions -> next reorganisation.  Integer results identical, attention within the tolerance."""
import numpy as np
import pytest
import torch

from paper_2605_24832_amd import (commit_forward, commit_params, inputs,
                                  reorg_forward)
from tests import hip_path as hp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_reorg(dec, s, want):
    R, B = dec.shape
    t = lambda a, dt: torch.as_tensor(np.ascontiguousarray(a), dtype=dt, device=DEV)
    mk = lambda n: torch.full((n,), -1, dtype=torch.int32, device=DEV)
    cap = int(np.minimum(want, B).sum())
    chunk, cu, L, pos, slot, req = mk(R), mk(R + 1), mk(R), mk(cap), mk(cap), mk(cap)
    reorg_forward(t(dec, torch.uint8), t(s, torch.int32), t(want, torch.int32), chunk, cu, L, pos, slot, req)
    torch.cuda.synchronize()
    n = int(cu[-1])
    return {k: v.cpu().numpy() for k, v in dict(chunk=chunk, cu_q=cu, prefix_len=L, q_pos=pos[:n],
                                                 kv_slot=slot[:n], token_req=req[:n]).items()}


def test_two_decoding_iterations(oracle_mod):
    print("decode iteration chain", flush=True)
    R, B, V = 6, 32, 1000
    dec, s, want = inputs.make_decode_state(R, B, seed=123, chunk_choices=(2, 4, 8, 16), max_context=1024)
    dec_ref = dec.copy()
    for it in range(2):
        # ---- chunk selection by position
        got = gpu_reorg(dec, s, want)
        ref = oracle_mod.reorganise(dec_ref, s, want)
        for k in ref:
            np.testing.assert_array_equal(got[k], ref[k], err_msg=f"iteration {it}: {k}")
        c, L = got["chunk"], got["prefix_len"]
        if c.sum() == 0:
            break
        # ---- attention step on a workload with exactly these descriptors
        w = inputs.make_workload(f"iter{it}", seed=500 + it, num_q_heads=8, num_kv_heads=2, head_dim=64,
                                 page_size=16, block_size=B, prefix_len=L, chunk=c, block_inner=L - s,
                                 device=DEV)
        np.testing.assert_array_equal(w.cu_q, got["cu_q"])
        np.testing.assert_array_equal(w.block_start, s)
        bits = hp.host_bits(w)
        out, _ = hp.run_hip(w)
        ref_out, _, _ = hp.run_oracle(oracle_mod, w, bits=bits)
        hp.check_close(out.float().cpu().numpy(), ref_out, what=f"iteration {it}")
        # the chunk's K/V went to the slots the reorganisation announced
        kview = inputs.k_tile_view(w.k_pool, 16, 64, 1)       # [pages, Hkv, D/8, P, 8]
        for tkn, (i, slot) in enumerate(zip(got["token_req"], got["kv_slot"])):
            page = int(w.block_table[i, slot // 16])
            assert torch.equal(kview[page, 0, :, slot % 16, :].reshape(-1), w.k_new[tkn, 0])
        # ---- commit on synthetic logits, per-request progress rule
        T = int(c.sum())
        x = inputs.make_logits(T, V, seed=900 + it, device=DEV)
        p = commit_params(T, V, x.shape[1], 0.9, R, 1)
        tok = torch.empty(T, dtype=torch.int32, device=DEV)
        conf = torch.empty(T, dtype=torch.float32, device=DEV)
        com = torch.empty(T, dtype=torch.int32, device=DEV)
        commit_forward(p, x, torch.as_tensor(got["cu_q"], device=DEV), tok, conf, com)
        torch.cuda.synchronize()
        rt, rc, rcom = oracle_mod.commit(inputs.to_bits(x), V, 0.9, got["cu_q"], 1)
        np.testing.assert_array_equal(tok.cpu().numpy(), rt)
        clear = np.abs(rc - 0.9) > 1e-4          # positions whose flag does not hang on rounding
        assert clear.all(), "synthetic logits put a confidence on the threshold: change the seed"
        np.testing.assert_array_equal(com.cpu().numpy(), rcom)
        # ---- every request with a chunk advanced; mark the committed positions decoded
        com_h = com.cpu().numpy().astype(bool)
        for i in range(R):
            lo, hi = got["cu_q"][i], got["cu_q"][i + 1]
            assert hi == lo or com_h[lo:hi].any()
        rows, cols = got["token_req"][com_h], (got["q_pos"] - s[got["token_req"]])[com_h]
        assert (dec[rows, cols] == 0).all()
        dec[rows, cols] = 1
        dec_ref[rows, cols] = 1
