"""GPU parity of the commit step against its fp64 oracle.

Tokens (argmax over exact bf16 values, first index on ties) must match exactly.  Confidences
must agree to 2e-5 relative (fp32 sums of up to 152K exponentials).  Commit flags must be
identical wherever the oracle's confidence is farther than that from the threshold; the few
borderline positions only have to be consistent with the GPU's own confidence."""
import numpy as np
import pytest
import torch

from paper_2605_24832_amd import commit_forward, commit_params, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
REL = 2e-5


def run_gpu(x, vocab, thr, cu_q=None, min_commit=0):
    T = x.shape[0]
    p = commit_params(T, vocab, x.shape[1], thr, 0 if cu_q is None else len(cu_q) - 1, min_commit)
    tok = torch.full((T,), -7, dtype=torch.int32, device=DEV)
    conf = torch.full((T,), float("nan"), dtype=torch.float32, device=DEV)
    com = torch.full((T,), -7, dtype=torch.int32, device=DEV)
    cu = None if cu_q is None else torch.as_tensor(np.asarray(cu_q, dtype=np.int32), device=DEV)
    commit_forward(p, x, cu, tok, conf, com)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), conf.cpu().numpy(), com.cpu().numpy()


def check(oracle, x, vocab, thr, cu_q=None, min_commit=0):
    tok, conf, com = run_gpu(x, vocab, thr, cu_q, min_commit)
    rt, rc, rcom = oracle.commit(inputs.to_bits(x), vocab, thr, cu_q, min_commit)
    np.testing.assert_array_equal(tok, rt)
    np.testing.assert_allclose(conf, rc, rtol=REL, atol=0)
    assert ((tok >= 0) & (tok < vocab)).all()
    thr32 = np.float64(np.float32(thr))
    clear = np.abs(rc - thr32) > REL * thr32
    if cu_q is None or min_commit == 0:
        np.testing.assert_array_equal(com[clear], rcom[clear])
        border = ~clear
        np.testing.assert_array_equal(com[border], (conf[border] > np.float32(thr)).astype(np.int32))
    else:
        # per request: identical when no position of the request is borderline
        for i in range(len(cu_q) - 1):
            lo, hi = cu_q[i], cu_q[i + 1]
            if clear[lo:hi].all():
                np.testing.assert_array_equal(com[lo:hi], rcom[lo:hi])
            elif hi > lo:
                assert com[lo:hi].sum() >= 1
    return tok, conf, com


@pytest.mark.parametrize("T,V", [(1, 1), (3, 7), (5, 2048), (17, 2049), (64, 32000), (40, 151936)])
def test_commit_matches_oracle(oracle_mod, T, V):
    print(f"commit T={T} V={V}", flush=True)
    x = inputs.make_logits(T, V, seed=50 + T, device=DEV)
    _, conf, com = check(oracle_mod, x, V, 0.9)
    if T >= 17:
        assert 0 < com.sum() < T


def test_commit_padded_rows_and_per_request_rule(oracle_mod):
    print("commit per request", flush=True)
    V, stride = 5003, 5120
    c = [4, 0, 32, 1, 7, 20]
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    x = inputs.make_logits(int(cu[-1]), V, seed=61, row_stride=stride, device=DEV)
    for mc in (0, 1):
        check(oracle_mod, x, V, 0.9, cu, mc)
    # nothing can pass a threshold of 1: every non-empty request commits exactly its best token
    tok, conf, com = check(oracle_mod, x, V, 1.0, cu, 1)
    for i in range(len(c)):
        lo, hi = cu[i], cu[i + 1]
        assert com[lo:hi].sum() == (1 if hi > lo else 0)


def test_commit_full_size(oracle_mod):
    """The benchmark shape: 604 chunk tokens (config 3) x a 151936-entry vocabulary."""
    print("commit full size", flush=True)
    w = inputs.make_config(3, device="cpu", scale_down=256)  # descriptors only matter here
    rng = np.random.RandomState(inputs.BASE_SEED + 3)
    rng.randint(1024, 8193, size=256)
    c = rng.choice([1, 2, 4], size=256)
    cu = np.concatenate([[0], np.cumsum(c)]).astype(np.int32)
    x = inputs.make_logits(int(cu[-1]), 151936, seed=62, device=DEV)
    check(oracle_mod, x, 151936, 0.9, cu, 1)


def test_commit_masked_entries_and_one_token_requests(oracle_mod):
    """-inf and NaN logits are entries that cannot be chosen: whole aligned 8-entry pieces of them
    before the first finite entry (the running maximum is still -inf there), runs spanning many
    threads' pieces, a single finite entry, fully masked rows; one-token requests under the
    progress rule, one of them fully masked (its token is the forced fallback)."""
    print("commit masked entries", flush=True)
    V = 20000
    x = inputs.make_logits(12, V, seed=71, device=DEV)
    ninf, nan = float("-inf"), float("nan")
    x[0, :4096] = ninf
    x[1, 8:16384] = ninf
    x[2, 10000:] = ninf            # the padding beyond V is NaN already
    x[3, :V - 1] = ninf
    x[4, ::2] = ninf
    x[5, :V] = ninf
    x[6, :8192] = nan
    x[7, 1::3] = nan
    x[8, :V] = nan
    x[9, 5:9000] = nan
    x[9, 9000:15000] = ninf
    x[10, :V] = ninf
    cu = [0, 1, 2, 5, 6, 9, 10, 11, 12]          # rows 5, 10 (fully masked) are one-token requests
    for mc in (0, 1):
        tok, conf, com = check(oracle_mod, x, V, 0.9, cu, mc)
        assert np.isfinite(conf).all()
        assert conf[5] == 0 and conf[8] == 0 and conf[10] == 0 and tok[5] == 0
        assert tok[3] == V - 1 and conf[3] == 1.0
    assert com[5] == 1 and com[10] == 1          # forced: the only token of their requests
