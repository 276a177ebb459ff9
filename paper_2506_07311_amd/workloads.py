"""Seeded synthetic inputs shaped like the paper's workloads.

This module only DRAWS inputs: random K/V pools, random physical page
permutations, block tables, lengths and queries.  It holds none of the
method's arithmetic (no scatter, no gather, no attention) and is the only
module that both the GPU-side tests/benchmark and the CPU oracle's tests use.

The paper measured LLaMA-7B prompts from WikiText-103 and LongBench
(Sec. III-A); attention cost and correctness depend only on tensor shapes and
page structure, so seeded N(0,1) tensors with those shapes stand in for them.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch


@dataclass
class PagedWorkload:
    name: str
    dtype: torch.dtype
    page_size: int
    num_pages: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    scale: float
    causal: bool
    k_cache: torch.Tensor          # [NP, P, Hkv, d]; contexts resident, unused slots poisoned
    v_cache: torch.Tensor
    block_table: torch.Tensor      # int32 [B, MB], -1 where unused
    seq_lens: torch.Tensor         # int32 [B], lengths INCLUDING the step's appended tokens
    q: torch.Tensor                # [total_q, Hq, d]
    cu_q_lens: torch.Tensor        # int32 [B+1]
    k_new: torch.Tensor            # [T, Hkv, d] tokens the step appends
    v_new: torch.Tensor
    seq_ids: torch.Tensor          # int32 [T]
    positions: torch.Tensor        # int32 [T]
    seq_lens_host: List[int] = field(default_factory=list)
    q_lens_host: List[int] = field(default_factory=list)

    @property
    def batch(self) -> int:
        return len(self.seq_lens_host)

    @property
    def max_seq_len(self) -> int:
        return max(self.seq_lens_host) if self.seq_lens_host else 0

    @property
    def max_q_len(self) -> int:
        return max(self.q_lens_host) if self.q_lens_host else 0

    @property
    def total_q(self) -> int:
        return int(sum(self.q_lens_host))

    @property
    def kv_bytes_per_token(self) -> int:
        return 2 * self.num_kv_heads * self.head_dim * self.k_cache.element_size()

    def logical_kv_bytes(self) -> int:
        """K and V bytes of the valid tokens of every sequence (aliased pages counted per reader)."""
        return int(sum(self.seq_lens_host)) * self.kv_bytes_per_token


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host numpy view of a tensor; bf16 is returned as its uint16 bit patterns."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def _randn(shape, dtype, device, gen):
    # fp32 draw rounded once to the storage type, so every consumer sees the same bits
    return torch.randn(shape, generator=gen, device=device, dtype=torch.float32).to(dtype)


def _randn_big(shape, dtype, device, gen, chunk_pages=8192):
    """Same as _randn for a pool too large to hold an fp32 temporary of."""
    out = torch.empty(shape, dtype=dtype, device=device)
    for p0 in range(0, shape[0], chunk_pages):
        p1 = min(shape[0], p0 + chunk_pages)
        out[p0:p1] = torch.randn((p1 - p0,) + tuple(shape[1:]), generator=gen, device=device,
                                 dtype=torch.float32).to(dtype)
    return out


def make_workload(name: str, *, seq_lens: List[int], q_lens: Optional[List[int]] = None,
                  append_lens: Optional[List[int]] = None,
                  num_q_heads: int, num_kv_heads: int, head_dim: int, page_size: int,
                  dtype: torch.dtype = torch.bfloat16, causal: bool = False,
                  pool_factor: float = 2.0, num_pages: Optional[int] = None,
                  share_group: int = 0, share_prefix_tokens: int = 0,
                  poison: bool = True, identity_pages: bool = False,
                  seed: int = 0, device: str = "cpu", scale: Optional[float] = None) -> PagedWorkload:
    """Draw one workload.

    seq_lens    -- context length of every sequence AFTER this step's append.
    q_lens      -- queries per sequence (default 1 = decode); the queries are the LAST q_len positions.
    append_lens -- tokens appended this step per sequence (default = q_lens); they occupy the last positions.
    share_group / share_prefix_tokens -- sequences g*share_group .. +share_group-1 alias the same physical
                   pages for their first floor(min(len-1, share_prefix_tokens) / P) logical blocks (whole
                   pages only, so every sequence's last page stays private).
    poison      -- fill every slot no valid token maps to (unused pages, the tail of each last page)
                   with NaN, so a kernel that reads outside the mask is caught.
    identity_pages -- block tables use pages 0,1,2,... in order (a contiguous layout) instead of a
                   random permutation.
    """
    B = len(seq_lens)
    P = page_size
    q_lens = list(q_lens) if q_lens is not None else [1 if L > 0 else 0 for L in seq_lens]
    append_lens = list(append_lens) if append_lens is not None else list(q_lens)
    assert len(q_lens) == B and len(append_lens) == B
    gen = torch.Generator(device=device)
    gen.manual_seed(1000 + seed)
    rng = np.random.default_rng(2000 + seed)

    nblocks = [(L + P - 1) // P for L in seq_lens]
    max_blocks = max(nblocks + [1])
    # logical -> physical page draw
    shared_blocks = [0] * B
    if share_group > 1 and share_prefix_tokens > 0:
        for s, L in enumerate(seq_lens):
            shared_blocks[s] = max(0, min(L - 1, share_prefix_tokens)) // P
    n_groups = (B + share_group - 1) // share_group if share_group > 1 else 0
    group_prefix_blocks = [0] * n_groups
    for s in range(B):
        if share_group > 1:
            g = s // share_group
            group_prefix_blocks[g] = max(group_prefix_blocks[g], shared_blocks[s])
    used = sum(group_prefix_blocks) + sum(nb - sb for nb, sb in zip(nblocks, shared_blocks))
    if num_pages is None:
        num_pages = max(1, int(math.ceil(used * pool_factor)))
    assert num_pages >= used, "pool too small"
    perm = np.arange(num_pages, dtype=np.int64) if identity_pages else rng.permutation(num_pages)
    table = np.full((B, max_blocks), -1, dtype=np.int32)
    cursor = 0
    group_pages = []
    for g in range(n_groups):
        group_pages.append(perm[cursor:cursor + group_prefix_blocks[g]])
        cursor += group_prefix_blocks[g]
    for s in range(B):
        sb = shared_blocks[s]
        if sb:
            table[s, :sb] = group_pages[s // share_group][:sb]
        own = nblocks[s] - sb
        table[s, sb:nblocks[s]] = perm[cursor:cursor + own]
        cursor += own
    assert cursor == used

    shape = (num_pages, P, num_kv_heads, head_dim)
    big = num_pages * P * num_kv_heads * head_dim > (1 << 28)
    draw = _randn_big if big else _randn
    k_cache = draw(shape, dtype, device, gen)
    v_cache = draw(shape, dtype, device, gen)
    if poison:
        live = np.zeros(num_pages, dtype=bool)
        live[perm[:used]] = True
        dead = torch.from_numpy(np.nonzero(~live)[0]).to(device)
        if dead.numel():
            k_cache.index_fill_(0, dead, float("nan"))
            v_cache.index_fill_(0, dead, float("nan"))
        for s, L in enumerate(seq_lens):
            tail = L % P
            if L > 0 and tail:
                pg = int(table[s, nblocks[s] - 1])
                k_cache[pg, tail:] = float("nan")
                v_cache[pg, tail:] = float("nan")

    total_q = int(sum(q_lens))
    q = _randn((total_q, num_q_heads, head_dim), dtype, device, gen)
    cu = np.zeros(B + 1, dtype=np.int32)
    np.cumsum(np.asarray(q_lens, dtype=np.int64), out=cu[1:])
    T = int(sum(append_lens))
    k_new = _randn((T, num_kv_heads, head_dim), dtype, device, gen)
    v_new = _randn((T, num_kv_heads, head_dim), dtype, device, gen)
    seq_ids = np.concatenate([np.full(a, s, dtype=np.int32) for s, a in enumerate(append_lens)]
                             + [np.zeros(0, dtype=np.int32)])
    positions = np.concatenate([np.arange(L - a, L, dtype=np.int32) for L, a in zip(seq_lens, append_lens)]
                               + [np.zeros(0, dtype=np.int32)])

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device)

    return PagedWorkload(
        name=name, dtype=dtype, page_size=P, num_pages=num_pages, num_q_heads=num_q_heads,
        num_kv_heads=num_kv_heads, head_dim=head_dim,
        scale=float(scale if scale is not None else 1.0 / math.sqrt(head_dim)), causal=causal,
        k_cache=k_cache, v_cache=v_cache, block_table=dev(table),
        seq_lens=dev(np.asarray(seq_lens, dtype=np.int32)), q=q, cu_q_lens=dev(cu),
        k_new=k_new, v_new=v_new, seq_ids=dev(seq_ids), positions=dev(positions),
        seq_lens_host=list(map(int, seq_lens)), q_lens_host=list(map(int, q_lens)))


def restrict(w: PagedWorkload, seqs: List[int], device: Optional[str] = None) -> PagedWorkload:
    """The same workload cut down to the sequences ``seqs``: only the physical pages they map to are kept
    (copied, re-numbered 0..n-1 in ascending page order, aliases preserved) together with their block-table
    rows, lengths, queries and appended tokens.  Plain tensor indexing; used to hand the CPU oracle whole
    sequences of a workload whose pool is too large to copy to the host."""
    seqs = list(seqs)
    idx = torch.tensor(seqs, dtype=torch.long, device=w.block_table.device)
    bt = w.block_table[idx]
    live = bt >= 0
    pages = torch.unique(bt[live]).long()
    remap = torch.full((w.num_pages,), -1, dtype=torch.int32, device=bt.device)
    remap[pages] = torch.arange(pages.numel(), dtype=torch.int32, device=bt.device)
    bt2 = torch.where(live, remap[bt.clamp(min=0).long()], bt)
    cu = w.cu_q_lens.cpu().numpy()
    rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in seqs] + [np.zeros(0, dtype=np.int64)]).astype(np.int64)
    q_lens = [w.q_lens_host[s] for s in seqs]
    cu2 = np.zeros(len(seqs) + 1, dtype=np.int32)
    np.cumsum(np.asarray(q_lens, dtype=np.int64), out=cu2[1:])
    ids = w.seq_ids.cpu().numpy()
    sel = np.nonzero(np.isin(ids, seqs))[0]
    order = {s: i for i, s in enumerate(seqs)}
    new_ids = np.asarray([order[int(x)] for x in ids[sel]], dtype=np.int32)
    dev = device or str(w.q.device)

    def pick(t, index):
        return t[torch.as_tensor(index, dtype=torch.long, device=t.device)].to(dev)

    return PagedWorkload(
        name=w.name + "_sub", dtype=w.dtype, page_size=w.page_size, num_pages=int(pages.numel()),
        num_q_heads=w.num_q_heads, num_kv_heads=w.num_kv_heads, head_dim=w.head_dim, scale=w.scale, causal=w.causal,
        k_cache=w.k_cache[pages].to(dev), v_cache=w.v_cache[pages].to(dev), block_table=bt2.to(dev),
        seq_lens=w.seq_lens[idx].to(dev), q=pick(w.q, rows), cu_q_lens=torch.from_numpy(cu2).to(dev),
        k_new=pick(w.k_new, sel), v_new=pick(w.v_new, sel), seq_ids=torch.from_numpy(new_ids).to(dev),
        positions=pick(w.positions, sel), seq_lens_host=[w.seq_lens_host[s] for s in seqs], q_lens_host=q_lens)


def log_uniform_lengths(n: int, lo: int, hi: int, seed: int) -> List[int]:
    """n lengths with ln(len) uniform on [ln lo, ln hi], rounded to integers."""
    rng = np.random.default_rng(3000 + seed)
    u = rng.uniform(math.log(lo), math.log(hi), size=n)
    return [int(min(hi, max(lo, round(math.exp(x))))) for x in u]


def config(n: int, *, device: str = "cpu", context: Optional[int] = None, page_size: Optional[int] = None,
           shrink: int = 1, poison: bool = True, head_dim: Optional[int] = None,
           heads: Optional[tuple] = None) -> PagedWorkload:
    """The five benchmark workloads (1-based), three jagged-batch workloads (6-8) and the paper's own model shape (9-10).  ``shrink`` divides context lengths
    (and config 4's length range) for cases the CPU oracle must finish in seconds; ``head_dim`` overrides the 128 of
    the 16-bit workloads (2-8); ``heads`` = (query heads, KV heads) overrides workload 5's 64 / 8 (the per-GPU shape
    of a tensor-parallel shard has few KV heads)."""
    hd = head_dim or 128
    if n == 1:   # single-sequence fp32 decode, 8 of 64 pages used
        L = context or 128
        return make_workload("cfg1_fp32_single_decode", seq_lens=[L], num_q_heads=8, num_kv_heads=8,
                             head_dim=64, page_size=page_size or 16, dtype=torch.float32,
                             num_pages=max(64, 8 * ((L + 15) // 16)), seed=1, device=device, poison=poison)
    if n == 2:   # batched GQA decode, bf16
        L = context or 2048
        return make_workload(f"cfg2_bf16_gqa_decode_L{L}", seq_lens=[L] * 8, num_q_heads=32, num_kv_heads=8,
                             head_dim=hd, page_size=page_size or 16, seed=2, device=device, poison=poison)
    if n == 3:   # causal prefill, bf16; every token is appended this step
        S = context or max(16, 2048 // shrink)
        return make_workload(f"cfg3_bf16_causal_prefill_S{S}", seq_lens=[S] * 4, q_lens=[S] * 4,
                             num_q_heads=32, num_kv_heads=8, head_dim=hd, page_size=page_size or 16,
                             causal=True, seed=3, device=device, poison=poison)
    if n == 4:   # mixed-length decode with shared prefixes
        hi = max(128, 32768 // shrink)
        lens = log_uniform_lengths(64, 64, hi, seed=4)
        return make_workload(f"cfg4_bf16_mixed_decode_max{hi}", seq_lens=lens, num_q_heads=32, num_kv_heads=8,
                             head_dim=hd, page_size=page_size or 16, share_group=8,
                             share_prefix_tokens=max(16, 1024 // shrink), seed=4, device=device, poison=poison)
    if n == 5:   # long-context split-KV decode
        L = context or max(64, 131072 // shrink)
        P = page_size or 16
        hq, hkv = heads or (64, 8)
        return make_workload(f"cfg5_bf16_long_decode_L{L}_P{P}", seq_lens=[L] * 16, num_q_heads=hq,
                             num_kv_heads=hkv, head_dim=hd, page_size=P, seed=5, device=device, poison=poison)
    # Jagged-batch workloads of the prefill entry point (Sec. III-B: ragged queries described by prefix sums).
    if n == 6:   # chat growth: one 1024-token chunk appended behind 31744 cached tokens (1k -> 32k incremental)
        L = context or max(128, 32768 // shrink)
        chunk = max(16, 1024 // shrink)
        return make_workload(f"cfg6_bf16_chunked_prefill_{chunk}_on_{L - chunk}", seq_lens=[L], q_lens=[chunk],
                             num_q_heads=32, num_kv_heads=8, head_dim=hd, page_size=page_size or 16, causal=True,
                             seed=6, device=device, poison=poison)
    if n in (7, 8):   # config 4's length mix; 7: four sequences prefill 512 tokens while sixty decode; 8: four
        hi = max(128, 32768 // shrink)            # speculative tokens per sequence
        lens = log_uniform_lengths(64, 64, hi, seed=4)
        if n == 7:
            q_lens = [min(L, max(2, 512 // shrink)) if s % 16 == 5 else 1 for s, L in enumerate(lens)]
        else:
            q_lens = [min(L, 4) for L in lens]
        return make_workload(f"cfg{n}_bf16_jagged_max{hi}", seq_lens=lens, q_lens=q_lens, num_q_heads=32,
                             num_kv_heads=8, head_dim=hd, page_size=page_size or 16, causal=True, seed=n,
                             device=device, poison=poison)
    # The model the paper measures on (Sec. IV-A): one LLaMA-7B layer -- 32 heads without grouping, head_dim 128, fp16 --
    # with the page size the paper settles on (64 tokens, Sec. III-B) and one sequence, prompts of 128 to 2048 tokens
    # (Sec. IV-B).  9: one decode step at context L; 10: the prompt's causal prefill.
    if n in (9, 10):
        L = context or max(16, 2048 // shrink)
        return make_workload(f"cfg{n}_fp16_llama7b_layer_L{L}", seq_lens=[L], q_lens=[L] if n == 10 else None,
                             num_q_heads=32, num_kv_heads=32, head_dim=hd, page_size=page_size or 64,
                             dtype=torch.float16, causal=(n == 10), seed=n, device=device, poison=poison)
    raise ValueError(f"no config {n}")
