"""Seeded synthetic inputs for the chunked block-diffusion attention step.

This module only *makes data*: descriptors (ragged chunk sizes, cached
lengths, block origins, block tables) and bf16 N(0,1) tensors laid out in a
paged pool.  It holds none of the attention arithmetic and is the one thing
the HIP path and the CPU oracle have in common: both consume the buffers it
returns.

The shapes follow the serving regimes the paper describes (Optimus Sec. 7:
batch 1..256, block size 32, chunk sizes 1..32 chosen per iteration, contexts
of 0.1K..8K tokens, a 32K long-context case); the paper's datasets and model
weights are not used, only their shapes.

Pool layouts (``kv_layout``), per (page, kv head) tile of ``P*D`` elements:
  0: K and V as ``[P, D]``
  1: K as ``[D/8, P, 8]`` (8-element groups of the head dim, slot-major inside
     a group), V as ``[D, P]`` (slot-contiguous)
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 248320
BF16_NAN_BITS = 0x7FC0


@dataclass
class Workload:
    name: str
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    page_size: int
    block_size: int
    kv_layout: int
    mask_mode: int
    num_pages: int
    max_pages_per_req: int
    cu_q: np.ndarray          # int32 [R+1]
    prefix_len: np.ndarray    # int32 [R]
    block_start: np.ndarray   # int32 [R]
    block_table: np.ndarray   # int32 [R, max_pages_per_req], unused entries -1
    q: torch.Tensor           # bf16 [T, Hq, D]
    k_new: torch.Tensor       # bf16 [T, Hkv, D]
    v_new: torch.Tensor       # bf16 [T, Hkv, D]
    k_pool: torch.Tensor      # bf16 [num_pages, Hkv, P*D]
    v_pool: torch.Tensor      # bf16 [num_pages, Hkv, P*D]
    extra: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return len(self.prefix_len)

    @property
    def total_q(self) -> int:
        return int(self.cu_q[-1])

    @property
    def chunk(self) -> np.ndarray:
        return np.diff(self.cu_q)

    def kv_bytes(self) -> int:
        """K and V bytes of all visible keys (cached + chunk), each read once."""
        n = int((self.prefix_len.astype(np.int64) + self.chunk).sum())
        return 2 * 2 * self.num_kv_heads * self.head_dim * n

    def qo_bytes(self) -> int:
        return 2 * 2 * self.total_q * self.num_q_heads * self.head_dim

    def flops(self) -> int:
        c = self.chunk.astype(np.int64)
        n = self.prefix_len.astype(np.int64) + c
        return int(4 * self.num_q_heads * self.head_dim * (c * n).sum())

    def host_bits(self, t: torch.Tensor) -> np.ndarray:
        """bf16 tensor -> contiguous numpy uint16 bit patterns on the host."""
        return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().cpu().view(torch.int16).numpy().view(np.uint16)


def _randn_bf16(shape, gen: torch.Generator, device) -> torch.Tensor:
    """fp32 N(0,1) rounded to bf16 (round-to-nearest-even), generated in slabs."""
    n0 = shape[0]
    out = torch.empty(shape, dtype=torch.bfloat16, device=device)
    if n0 == 0:
        return out
    per = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    slab = max(1, (1 << 26) // max(per, 1))
    for a in range(0, n0, slab):
        b = min(n0, a + slab)
        x = torch.randn((b - a,) + tuple(shape[1:]), generator=gen, device=device,
                        dtype=torch.float32)
        out[a:b] = x.to(torch.bfloat16)
    return out


def k_tile_view(k_pool: torch.Tensor, P: int, D: int, kv_layout: int) -> torch.Tensor:
    """View ``[pages, Hkv, P*D]`` so that the slot axis is explicit.

    layout 0 -> ``[pages, Hkv, P, D]``;  layout 1 -> ``[pages, Hkv, D/8, P, 8]``.
    """
    n, h, _ = k_pool.shape
    return k_pool.view(n, h, P, D) if kv_layout == 0 else k_pool.view(n, h, D // 8, P, 8)


def v_tile_view(v_pool: torch.Tensor, P: int, D: int, kv_layout: int) -> torch.Tensor:
    """layout 0 -> ``[pages, Hkv, P, D]``;  layout 1 -> ``[pages, Hkv, D, P]``."""
    n, h, _ = v_pool.shape
    return v_pool.view(n, h, P, D) if kv_layout == 0 else v_pool.view(n, h, D, P)


def make_workload(name: str, *, seed: int, num_q_heads: int, num_kv_heads: int, head_dim: int,
                  page_size: int, block_size: int, prefix_len, chunk, block_inner=None,
                  shuffle_pages: bool = True, spare_frac: float = 0.1, kv_layout: int = 1,
                  mask_mode: int = 0, poison: bool = True, peaked_frac: float = 0.0,
                  max_pages_per_req: int | None = None, device="cpu") -> Workload:
    """Build one ragged batch.

    ``prefix_len[i]`` = L_i cached tokens, ``chunk[i]`` = c_i query tokens,
    ``block_inner[i]`` = d_i cached tokens already inside the current block
    (default ``min(L_i mod B, B - c_i)``); the block origin is s_i = L_i - d_i.
    Request i owns ``ceil((L_i + c_i)/P)`` pages.  With ``poison`` every slot
    at or beyond L_i in a request's pages and every unreferenced page holds
    bf16 NaN, so nothing outside the key set can leak into an output unseen.
    ``peaked_frac`` > 0 doubles the K rows of that fraction of positions (same
    positions for all heads) to make some softmax rows peaked.
    """
    device = torch.device(device)
    rng = np.random.RandomState(seed)
    L = np.asarray(prefix_len, dtype=np.int64)
    c = np.asarray(chunk, dtype=np.int64)
    R = len(L)
    B, P, D, Hq, Hkv = block_size, page_size, head_dim, num_q_heads, num_kv_heads
    if block_inner is None:
        d_in = np.minimum(L % B, np.maximum(B - c, 0))
    else:
        d_in = np.asarray(block_inner, dtype=np.int64)
    s = L - d_in
    cu_q = np.zeros(R + 1, dtype=np.int32)
    cu_q[1:] = np.cumsum(c)
    T = int(cu_q[-1])
    pages_per_req = (L + c + P - 1) // P
    total_pages = int(pages_per_req.sum())
    num_pages = total_pages + int(np.ceil(total_pages * spare_frac)) if shuffle_pages else total_pages
    num_pages = max(num_pages, 1)
    perm = rng.permutation(num_pages) if shuffle_pages else np.arange(num_pages)
    mp = int(pages_per_req.max()) if R else 1
    mp = max(mp, 1) if max_pages_per_req is None else max_pages_per_req
    block_table = np.full((R, mp), -1, dtype=np.int32)
    off = 0
    for i in range(R):
        n = int(pages_per_req[i])
        block_table[i, :n] = perm[off:off + n]
        off += n

    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    q = _randn_bf16((T, Hq, D), gen, device)
    k_new = _randn_bf16((T, Hkv, D), gen, device)
    v_new = _randn_bf16((T, Hkv, D), gen, device)
    k_pool = _randn_bf16((num_pages, Hkv, P * D), gen, device)
    v_pool = _randn_bf16((num_pages, Hkv, P * D), gen, device)
    kt = k_tile_view(k_pool, P, D, kv_layout)
    vt = v_tile_view(v_pool, P, D, kv_layout)
    slot_axis_k = 2 if kv_layout == 0 else 3
    slot_axis_v = 2 if kv_layout == 0 else 3

    extra = {}
    if peaked_frac > 0.0:
        # Bernoulli per logical position; cached positions act on the pool rows,
        # chunk positions on k_new.  Doubling is exact in bf16.
        pg_idx, sl_idx = [], []
        new_idx = []
        for i in range(R):
            hit = rng.random_sample(int(L[i] + c[i])) < peaked_frac
            pos = np.nonzero(hit)[0]
            cached = pos[pos < L[i]]
            pg_idx.append(block_table[i, cached // P])
            sl_idx.append(cached % P)
            new_idx.append(cu_q[i] + (pos[pos >= L[i]] - L[i]))
        pg = torch.as_tensor(np.concatenate(pg_idx), dtype=torch.long, device=device)
        sl = torch.as_tensor(np.concatenate(sl_idx), dtype=torch.long, device=device)
        if kv_layout == 0:
            kt[pg, :, sl, :] = kt[pg, :, sl, :] * 2
        else:
            kt[pg, :, :, sl, :] = kt[pg, :, :, sl, :] * 2
        ni = torch.as_tensor(np.concatenate(new_idx), dtype=torch.long, device=device)
        if len(ni):
            k_new[ni] = k_new[ni] * 2
        extra["peaked_positions"] = int(len(pg) + len(ni))

    if poison:
        nan = torch.tensor(float("nan"), dtype=torch.bfloat16, device=device)
        used = np.zeros(num_pages, dtype=bool)
        used[block_table[block_table >= 0]] = True
        unused = torch.as_tensor(np.nonzero(~used)[0], dtype=torch.long, device=device)
        if len(unused):
            k_pool[unused] = nan
            v_pool[unused] = nan
        for i in range(R):
            # every slot >= L_i of the request's pages (chunk slots are written by the append step)
            first = int(L[i] // P)
            for pi in range(first, int(pages_per_req[i])):
                page = int(block_table[i, pi])
                lo = int(L[i] - pi * P) if pi == first else 0
                if lo >= P:
                    continue
                kt[page].narrow(slot_axis_k - 1, lo, P - lo).fill_(float("nan"))
                vt[page].narrow(slot_axis_v - 1, lo, P - lo).fill_(float("nan"))

    return Workload(name=name, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=D, page_size=P,
                    block_size=B, kv_layout=kv_layout, mask_mode=mask_mode, num_pages=num_pages,
                    max_pages_per_req=mp, cu_q=cu_q, prefix_len=L.astype(np.int32),
                    block_start=s.astype(np.int32), block_table=block_table, q=q, k_new=k_new,
                    v_new=v_new, k_pool=k_pool, v_pool=v_pool, extra=extra)


CONFIG_NAMES = ("tiny", "mha_b1", "gqa_cb64", "highload_b256", "longctx_b4")


def make_config(k: int, *, device="cpu", chunk: int | None = None, scale_down: int = 1,
                kv_layout: int = 1) -> Workload:
    """The five benchmark configurations, seed ``BASE_SEED + k``.

    ``chunk`` fixes the chunk size where the configuration sweeps it (k=1: one
    of 4/8/16/32, default 32; k=4: 64 or 128, default a seeded mix) and makes
    the mixed batch of k=2 uniform (a diagnostic variant, not a benchmark line).
    ``scale_down`` > 1 divides batch (k=2,3) or cached length (k=1,4) so the
    same recipe gives a case the CPU oracle finishes in seconds.
    """
    seed = BASE_SEED + k
    rng = np.random.RandomState(seed)
    if k == 0:
        return make_workload("tiny", seed=seed, num_q_heads=4, num_kv_heads=4, head_dim=64,
                             page_size=16, block_size=32, prefix_len=[128], chunk=[8],
                             shuffle_pages=False, kv_layout=kv_layout, device=device)
    if k == 1:
        c = 32 if chunk is None else chunk
        return make_workload(f"mha_b1_c{c}", seed=seed, num_q_heads=32, num_kv_heads=32,
                             head_dim=128, page_size=16, block_size=32,
                             prefix_len=[2048 // scale_down], chunk=[c], shuffle_pages=False,
                             kv_layout=kv_layout, device=device)
    if k == 2:
        R = max(1, 64 // scale_down)
        L = rng.randint(512, 4096 + 1, size=R)
        c = rng.choice([1, 2, 4, 8, 16, 32], size=R)
        if chunk is not None:      # same lengths and pages, one chunk size: isolates one kernel body
            c = np.full(R, chunk)
        return make_workload("gqa_cb64" if chunk is None else f"gqa_cb64_c{chunk}", seed=seed, num_q_heads=28, num_kv_heads=4, head_dim=128,
                             page_size=16, block_size=32, prefix_len=L, chunk=c,
                             shuffle_pages=True, kv_layout=kv_layout, device=device)
    if k == 3:
        R = max(1, 256 // scale_down)
        L = rng.randint(1024, 8192 + 1, size=R)
        c = rng.choice([1, 2, 4], size=R)
        return make_workload("highload_b256", seed=seed, num_q_heads=32, num_kv_heads=8,
                             head_dim=128, page_size=16, block_size=32, prefix_len=L, chunk=c,
                             shuffle_pages=True, kv_layout=kv_layout, device=device)
    if k == 4:
        R = 4
        L = np.full(R, 32768 // scale_down)
        c = rng.choice([64, 128], size=R) if chunk is None else np.full(R, chunk)
        tag = "mix" if chunk is None else f"c{chunk}"
        return make_workload(f"longctx_b4_{tag}", seed=seed, num_q_heads=32, num_kv_heads=8,
                             head_dim=128, page_size=64, block_size=128, prefix_len=L, chunk=c,
                             block_inner=np.zeros(R, dtype=np.int64), shuffle_pages=True,
                             peaked_frac=0.01, kv_layout=kv_layout, device=device)
    raise ValueError(f"config index {k} not in 0..4")


def make_logits(num_tokens: int, vocab: int, *, seed: int, row_stride: int | None = None,
                max_margin: float | None = None, device="cpu") -> torch.Tensor:
    """bf16 logits ``[T, row_stride]`` for the commit step: N(0,1) noise plus, per row, one
    winner raised by a margin drawn uniformly from [0, max_margin] (default ln V + 6: the
    noise sums to about V * e^0.5, so the winner's probability sweeps 0..1), so that confidences
    cover (0, 1) and a fair share exceeds the 0.9 threshold of the paper's setup.  Entries
    beyond ``vocab`` (row padding) are NaN: they must never be looked at."""
    device = torch.device(device)
    stride = (vocab + 7) // 8 * 8 if row_stride is None else row_stride
    if max_margin is None:
        max_margin = float(np.log(vocab) + 6.0)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    x = torch.full((num_tokens, stride), float("nan"), dtype=torch.bfloat16, device=device)
    x[:, :vocab] = _randn_bf16((num_tokens, vocab), gen, device)
    rng = np.random.RandomState(seed)
    win = torch.as_tensor(rng.randint(0, vocab, size=num_tokens), device=device)
    margin = torch.as_tensor(rng.uniform(0.0, max_margin, size=num_tokens), device=device)
    rows = torch.arange(num_tokens, device=device)
    x[rows, win] = (x[rows, win].float() + margin.float()).to(torch.bfloat16)
    return x


def make_decode_state(batch: int, block_size: int, *, seed: int, decoded_fraction=None,
                      chunk_choices=(1, 2, 4, 8, 16, 32), max_context: int = 8192):
    """Decode state of ``batch`` requests in the middle of a block, for the step-wise
    reorganisation: a uint8 ``[batch, block_size]`` decoded map (every request draws its own
    decoded fraction from [0, 1] unless one is given; confident positions are decoded out of
    order, so the map has holes), the block's start position (a multiple of the block size) and
    the chunk size asked for.  Returns numpy arrays ``(decoded, block_start, chunk_req)``."""
    rng = np.random.RandomState(seed)
    frac = rng.uniform(0.0, 1.0, size=batch) if decoded_fraction is None else \
        np.full(batch, float(decoded_fraction))
    decoded = (rng.uniform(size=(batch, block_size)) < frac[:, None]).astype(np.uint8)
    blocks = max(1, max_context // block_size)
    block_start = (rng.randint(0, blocks, size=batch) * block_size).astype(np.int32)
    chunk_req = rng.choice(list(chunk_choices), size=batch).astype(np.int32)
    return decoded, block_start, chunk_req
