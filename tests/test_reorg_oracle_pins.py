"""Pins of the step-wise reorganisation oracle (Sec. 4.4) against what the method fixes: the
contiguous-chunk special case the attention path uses, an independent numpy formulation,
invariants, and a full decode of a block in which every position is decoded exactly once."""
import numpy as np

from paper_2605_24832_amd import inputs


def test_prefix_decoded_block_gives_the_contiguous_chunk(oracle_mod):
    # first d positions decoded: the chunk is positions d..d+c-1, cached length = block start + d,
    # KV slot = sequence position (the layout the attention step's descriptors assume)
    B = 32
    for d, want in [(0, 4), (5, 8), (30, 8), (32, 4), (0, 32), (0, 40)]:
        dec = np.zeros((1, B), np.uint8)
        dec[0, :d] = 1
        r = oracle_mod.reorganise(dec, [96], [want])
        c = min(want, B - d)
        assert r["chunk"].tolist() == [c] and r["cu_q"].tolist() == [0, c]
        assert r["prefix_len"].tolist() == [96 + d]
        assert r["q_pos"].tolist() == list(range(96 + d, 96 + d + c))
        assert r["kv_slot"].tolist() == r["q_pos"].tolist()
        assert r["token_req"].tolist() == [0] * c


def test_hand_worked_holes(oracle_mod):
    # block of 8 at position 16: decoded = positions 1, 2, 5.  Undecoded: 0, 3, 4, 6, 7.
    dec = np.array([[0, 1, 1, 0, 0, 1, 0, 0]], np.uint8)
    r = oracle_mod.reorganise(dec, [16], [3])
    assert r["q_pos"].tolist() == [16, 19, 20]
    assert r["prefix_len"].tolist() == [19]          # 16 cached before the block + 3 decoded
    assert r["kv_slot"].tolist() == [19, 20, 21]
    r = oracle_mod.reorganise(dec, [16], [9])
    assert r["q_pos"].tolist() == [16, 19, 20, 22, 23] and r["chunk"].tolist() == [5]
    r = oracle_mod.reorganise(dec, [16], [0])
    assert r["chunk"].tolist() == [0] and len(r["q_pos"]) == 0 and r["prefix_len"].tolist() == [19]


def test_against_numpy_formulation_and_invariants(oracle_mod):
    for seed, R, B in [(1, 7, 32), (2, 64, 32), (3, 33, 64), (4, 5, 200), (5, 16, 4)]:
        dec, s, want = inputs.make_decode_state(R, B, seed=seed, chunk_choices=(0, 1, 2, 4, 8, 32, 300))
        r = oracle_mod.reorganise(dec, s, want)
        pos, req, slot, chunk = [], [], [], []
        for i in range(R):
            und = np.flatnonzero(dec[i] == 0)[:want[i]]
            pos += (s[i] + und).tolist()
            req += [i] * len(und)
            L = s[i] + int(dec[i].astype(bool).sum())
            slot += (L + np.arange(len(und))).tolist()
            chunk.append(len(und))
            assert r["prefix_len"][i] == L
        assert r["q_pos"].tolist() == pos and r["token_req"].tolist() == req
        assert r["kv_slot"].tolist() == slot and r["chunk"].tolist() == chunk
        assert r["cu_q"].tolist() == np.concatenate([[0], np.cumsum(chunk)]).tolist()
        # invariants: positions strictly increase inside a request, lie in the block, were undecoded;
        # slots never reach past the block's end
        for i in range(R):
            lo, hi = r["cu_q"][i], r["cu_q"][i + 1]
            p = r["q_pos"][lo:hi] - s[i]
            assert (np.diff(p) > 0).all() and ((p >= 0) & (p < B)).all() and (dec[i, p] == 0).all()
            assert (r["kv_slot"][lo:hi] < s[i] + B).all()


def test_block_is_decoded_exactly_once_over_the_steps(oracle_mod):
    # every step commits a random non-empty subset of each chunk; the block finishes with every
    # position chosen for commit exactly once and the cached length equal to the block's end
    rng = np.random.RandomState(9)
    R, B = 6, 32
    dec = np.zeros((R, B), np.uint8)
    s = (np.arange(R) * B).astype(np.int32)
    times = np.zeros((R, B), int)
    for step in range(10 * B):
        r = oracle_mod.reorganise(dec, s, rng.choice([1, 2, 4, 8], size=R))
        if r["cu_q"][-1] == 0:
            break
        for i in range(R):
            p = r["q_pos"][r["cu_q"][i]:r["cu_q"][i + 1]] - s[i]
            if len(p):
                take = p[rng.uniform(size=len(p)) < 0.5]
                take = p[:1] if len(take) == 0 else take
                times[i, take] += 1
                dec[i, take] = 1
    assert (times == 1).all()
    r = oracle_mod.reorganise(dec, s, [4] * R)
    assert r["prefix_len"].tolist() == (s + B).tolist() and r["cu_q"][-1] == 0


def test_empty_batch(oracle_mod):
    r = oracle_mod.reorganise(np.zeros((0, 32), np.uint8), [], [])
    assert r["cu_q"].tolist() == [0] and len(r["q_pos"]) == 0
