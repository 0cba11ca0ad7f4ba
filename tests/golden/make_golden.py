"""Writes tests/golden/tiny_config0.json: the fp64 oracle's output for BASELINE configs[0] (the
tiny single-request case) on CPU-generated inputs.  Calls only the oracle and the seeded input
generator; run from the repository root:  python tests/golden/make_golden.py"""
import hashlib
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2605_24832_amd import inputs  # noqa: E402  (seeded generators only)

ROWS = [(t, h) for t in range(8) for h in range(4)]     # every (chunk token, query head) row is stored


def compute():
    oracle.build()
    w = inputs.make_config(0, device="cpu")
    bits = {k: inputs.to_bits(getattr(w, k)) for k in ("q", "k_new", "v_new", "k_pool", "v_pool")}
    p = oracle.make_params(num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim,
                           page_size=w.page_size, block_size=w.block_size,
                           max_pages_per_req=w.block_table.shape[1], mask_mode=w.mask_mode,
                           kv_layout=w.kv_layout)
    out = oracle.chunked_attention(p, w.cu_q, w.prefix_len, w.block_start, w.block_table, bits["q"],
                                   bits["k_new"], bits["v_new"], bits["k_pool"], bits["v_pool"])
    digest = hashlib.sha256(b"".join(np.ascontiguousarray(bits[k]).tobytes() for k in sorted(bits))).hexdigest()
    return w, out, digest


def main():
    w, out, digest = compute()
    doc = {
        "what": "oracle output (fp64) of BASELINE configs[0]: Hq=Hkv=4, D=64, prefix 128, chunk 8, P=16",
        "inputs_sha256": digest,
        "rows": [{"token": t, "head": h, "values": [repr(float(x)) for x in out[t, h]]} for t, h in ROWS],
        "sum_of_all_outputs": repr(float(out.sum())),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_config0.json")
    with open(path, "w") as f:
        json.dump(doc, f, indent=1)
    print("wrote", path)


if __name__ == "__main__":
    main()
