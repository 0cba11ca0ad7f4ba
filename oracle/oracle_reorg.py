"""CPU oracle of the step-wise reorganisation of streaming chunked decoding (Optimus
Sec. 4.4: at every step the chunk positions are re-chosen from the tokens decoded so far and
the chunk inputs are rebuilt; Sec. 7.2: streaming stays inside the current block).

TEST INFRASTRUCTURE ONLY: plain Python loops, no code shared with the HIP path.

Reading (the paper gives no pseudo-code): the chunk of a request is the first c not yet
decoded positions of its current block, in sequence order, where c is the chunk size the
scheduler asked for, cut to the number of positions still undecoded.  The decoded positions of
the block are already cached, so the request's cached length is block_start + (number of
decoded positions), and chunk token j goes to KV slot cached_length + j.
"""
import numpy as np


def reorganise(decoded, block_start, chunk_req):
    """decoded: uint8 [R, B] (1 = decoded); block_start, chunk_req: int [R].

    Returns dict of int32 arrays: chunk [R], cu_q [R+1], prefix_len [R], and per chunk token
    q_pos, kv_slot, token_req [T]."""
    decoded = np.asarray(decoded)
    R, B = decoded.shape
    chunk, prefix_len, q_pos, kv_slot, token_req = [], [], [], [], []
    for i in range(R):
        want = int(chunk_req[i])
        n_dec = 0
        for b in range(B):
            n_dec += 1 if decoded[i, b] else 0
        L = int(block_start[i]) + n_dec
        taken = 0
        for b in range(B):
            if taken >= want:
                break
            if not decoded[i, b]:
                q_pos.append(int(block_start[i]) + b)
                kv_slot.append(L + taken)
                token_req.append(i)
                taken += 1
        chunk.append(taken)
        prefix_len.append(L)
    cu_q = [0]
    for c in chunk:
        cu_q.append(cu_q[-1] + c)
    as32 = lambda x: np.asarray(x, dtype=np.int32)
    return dict(chunk=as32(chunk), cu_q=as32(cu_q), prefix_len=as32(prefix_len), q_pos=as32(q_pos),
                kv_slot=as32(kv_slot), token_req=as32(token_req))
