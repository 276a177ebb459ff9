"""A serving loop driven by the library's KV page manager on the GPU (Algorithm 1 Reserve + Assign; Sec. III-B),
against the oracle driven by the manager model.  The two sides never exchange page ids or cache contents: the
library path uses the pool's device-resident table, the oracle path the model's table and a host cache of its own;
only the seeded K/V/Q inputs are common.  Attention outputs depend on the logical contents alone, so they must
agree within the stated tolerance whatever pages each side picked."""
import numpy as np
import pytest
import torch

from oracle.page_manager import OutOfPages, PageManagerModel
from paper_2506_07311_amd import binding as pa
from paper_2506_07311_amd import workloads as W
from tests.parity import assert_close, to_f64

pytestmark = pytest.mark.gpu

P, HKV, HQ, D = 16, 2, 8, 128
PAGES, MAX_SEQS, MAX_BLOCKS = 40, 6, 32
DT = torch.bfloat16


class Loop:
    def __init__(self, oracle, seed=0):
        self.oracle = oracle
        self.dev = torch.device("cuda:0")
        self.gen = torch.Generator().manual_seed(seed)
        self.table = torch.zeros((MAX_SEQS, MAX_BLOCKS), dtype=torch.int32, device=self.dev)
        self.pool = pa.pa_pool_create(PAGES, P, MAX_SEQS, MAX_BLOCKS, self.table)
        self.model = PageManagerModel(PAGES, P, MAX_SEQS, MAX_BLOCKS)
        nan = float("nan")     # unwritten slots are poison: a read of one shows up as a non-finite output
        self.k = torch.full((PAGES, P, HKV, D), nan, dtype=DT, device=self.dev)
        self.v = torch.full((PAGES, P, HKV, D), nan, dtype=DT, device=self.dev)
        self.ok = W.to_numpy(torch.full((PAGES, P, HKV, D), nan, dtype=DT)).copy()
        self.ov = self.ok.copy()
        self.lens = [0] * MAX_SEQS
        self.scale = D ** -0.5

    def close(self):
        pa.pa_pool_destroy(self.pool)

    def rand(self, *shape):
        return torch.randn(shape, generator=self.gen, dtype=torch.float32).to(DT)

    def model_table(self):
        t = np.zeros((MAX_SEQS, MAX_BLOCKS), dtype=np.int32)
        for s, row in enumerate(self.model.rows):
            t[s, :len(row)] = row
        return t

    def append(self, seq, n):
        """n new tokens for seq at positions len .. len+n-1, through both managers and both append paths."""
        pos0 = self.lens[seq]
        kn, vn = self.rand(n, HKV, D), self.rand(n, HKV, D)
        ids = np.full(n, seq, dtype=np.int32)
        pos = np.arange(pos0, pos0 + n, dtype=np.int32)
        self.model.reserve(seq, pos0 + n)
        self.oracle.kv_append(self.ok, self.ov, W.to_numpy(kn), W.to_numpy(vn), ids, pos, self.model_table())
        pa.pa_pool_reserve(self.pool, seq, pos0 + n)
        pa.paged_kv_append(self.k, self.v, kn.to(self.dev), vn.to(self.dev), torch.from_numpy(ids).to(self.dev),
                           torch.from_numpy(pos).to(self.dev), self.table)
        self.lens[seq] = pos0 + n

    def attend(self, q_lens, what):
        """q_lens[s] trailing queries per sequence (0 = not in this step), bottom-right causal."""
        cu = np.zeros(MAX_SEQS + 1, dtype=np.int32)
        np.cumsum(q_lens, out=cu[1:])
        q = self.rand(int(cu[-1]), HQ, D)
        lens = np.array([l if n else 0 for l, n in zip(self.lens, q_lens)], dtype=np.int32)
        ref, _ = self.oracle.attention(self.ok, self.ov, W.to_numpy(q), self.model_table(), lens, self.scale,
                                       causal=True, cu_q_lens=cu)
        lens_d = torch.from_numpy(lens).to(self.dev)
        if max(q_lens) == 1:
            # decode entry point: one query row per table row; rows of sequences not in this step have length 0
            live = [s for s, n in enumerate(q_lens) if n]
            q_all = torch.zeros((MAX_SEQS, HQ, D), dtype=DT)
            q_all[live] = q
            out = pa.paged_attention_decode(self.k, self.v, q_all.to(self.dev), self.table, lens_d, int(lens.max()),
                                            self.scale)[live]
        else:
            out = pa.paged_attention_prefill(self.k, self.v, q.to(self.dev), torch.from_numpy(cu).to(self.dev),
                                             int(max(q_lens)), self.table, lens_d, int(lens.max()), self.scale, True)
        torch.cuda.synchronize()
        assert_close(to_f64(out), ref, DT, what)

    def check_state(self, what):
        torch.cuda.synchronize()
        dev_rows = self.table.cpu().numpy()
        rows = [pa.pa_pool_get_row(self.pool, s) for s in range(MAX_SEQS)]
        for s, row in enumerate(rows):
            assert len(row) == self.model.num_blocks(s), what
            assert list(dev_rows[s, :len(row)]) == row, f"{what}: device table row {s} is stale"
            assert (dev_rows[s, len(row):] == -1).all(), f"{what}: device table row {s} keeps released entries"
        assert pa.pa_pool_num_free(self.pool) == self.model.num_free(), what
        groups = {}
        for s, row in enumerate(rows):
            for b, page in enumerate(row):
                groups.setdefault(page, []).append((s, b))
        assert sorted(sorted(g) for g in groups.values()) == self.model.sharing(), what
        for page, g in groups.items():
            assert pa.pa_pool_refcount(self.pool, page) == len(g), what


def test_serving_loop_with_growth_release_sharing_and_copy_on_write(oracle):
    lp = Loop(oracle)
    try:
        # admit three prompts, prefill them together
        for s, n in [(0, 37), (1, 100), (2, 16)]:
            lp.append(s, n)
        lp.attend([37, 100, 16, 0, 0, 0], "prefill of three prompts")
        lp.check_state("after admit")
        # decode: every live sequence grows by one token per step (crossing page boundaries at 48 and 112 ...)
        for step in range(12):
            for s in (0, 1, 2):
                lp.append(s, 1)
            if step % 4 == 3:
                lp.attend([1, 1, 1, 0, 0, 0], f"decode step {step}")
        lp.check_state("after decode")
        # sequence 3 forks from sequence 1 at a page boundary and continues on its own pages
        lp.model.share_prefix(3, 1, 96)
        pa.pa_pool_share_prefix(lp.pool, 3, 1, 96)
        lp.lens[3] = 96
        lp.append(3, 5)
        lp.check_state("after fork")
        lp.attend([0, 1, 0, 5, 0, 0], "fork: parent decodes, child prefills its suffix")
        # sequence 4 shares two pages of sequence 0 but keeps only 20 tokens of them: its next token lands in
        # the shared second page, so that page is copied first
        lp.model.share_prefix(4, 0, 32)
        pa.pa_pool_share_prefix(lp.pool, 4, 0, 32)
        lp.lens[4] = 20
        old = lp.model.rows[4][1]
        assert lp.model.make_writable(4, 20)
        new = lp.model.rows[4][1]
        lp.ok[new], lp.ov[new] = lp.ok[old], lp.ov[old]
        pa.pa_pool_make_writable(lp.pool, lp.k, lp.v, 4, 20)
        lp.append(4, 3)                                    # positions 20..22 overwrite the COPY only
        assert not lp.model.make_writable(4, 21)
        pa.pa_pool_make_writable(lp.pool, lp.k, lp.v, 4, 21)   # private now: nothing happens
        lp.check_state("after copy-on-write")
        lp.attend([1, 0, 0, 0, 3, 0], "copy-on-write: the parent still sees its own tokens 20..22")
        # the parent of the fork ends: its private pages come back at once, the shared ones stay for the child
        free_before = pa.pa_pool_num_free(lp.pool)
        lp.model.release(1)
        pa.pa_pool_release(lp.pool, 1)
        lp.lens[1] = 0
        assert pa.pa_pool_num_free(lp.pool) == free_before + 1     # 7 blocks, 6 of them shared
        lp.check_state("after release of the parent")
        # a request the pool cannot hold is refused and changes nothing
        with pytest.raises(OutOfPages):
            lp.model.reserve(5, MAX_BLOCKS * P)
        with pytest.raises(pa.PagedAttnError):
            pa.pa_pool_reserve(lp.pool, 5, MAX_BLOCKS * P)
        lp.check_state("after a refused reservation")
        # a new prompt takes recycled pages; everyone still alive attends correctly
        lp.append(5, 150)
        lp.append(1, 9)
        lp.attend([1, 9, 1, 1, 1, 150], "mixed step on recycled pages")
        lp.check_state("after reuse")
        for s in range(MAX_SEQS):
            lp.model.release(s)
            pa.pa_pool_release(lp.pool, s)
        lp.check_state("after everything ended")
        assert pa.pa_pool_num_free(lp.pool) == PAGES
    finally:
        lp.close()


def test_row_updates_keep_call_order_on_the_stream(oracle):
    """A release enqueued right behind an attention call must not disturb it: the row copies carry the values of
    their own call, not whatever the host mirror holds when the stream gets to them."""
    lp = Loop(oracle, seed=3)
    try:
        lp.append(0, 200)
        lp.append(1, 64)
        q = lp.rand(2, HQ, D)
        lens = np.array([200, 64, 0, 0, 0, 0], dtype=np.int32)
        cu = np.array([0, 1, 2, 2, 2, 2, 2], dtype=np.int32)
        ref, _ = oracle.attention(lp.ok, lp.ov, W.to_numpy(q), lp.model_table(), lens, lp.scale, causal=True,
                                  cu_q_lens=cu)
        lens_d = torch.from_numpy(lens).to(lp.dev)
        qd = q.to(lp.dev)
        torch.cuda.synchronize()
        outs = []
        for _ in range(20):       # reserve/release churn of another sequence between attention calls, no syncs
            pa.pa_pool_reserve(lp.pool, 2, 160)
            outs.append(pa.paged_attention_prefill(lp.k, lp.v, qd, torch.from_numpy(cu).to(lp.dev), 1, lp.table,
                                                   lens_d, 200, lp.scale, True))
            pa.pa_pool_release(lp.pool, 2)
        pa.pa_pool_release(lp.pool, 1)
        pa.pa_pool_reserve(lp.pool, 3, 64)
        torch.cuda.synchronize()
        for o in outs:
            assert_close(to_f64(o), ref, DT, "attention between pool updates")
    finally:
        lp.close()


def test_row_updates_survive_many_wraps_of_the_staging_ring():
    """Far more row entries than the pinned staging ring holds are pushed through it without a host wait in
    between; the device table must end up equal to the host rows."""
    dev = torch.device("cuda:0")
    max_seqs, max_blocks, pages = 4, 20000, 70000
    table = torch.zeros((max_seqs, max_blocks), dtype=torch.int32, device=dev)
    pool = pa.pa_pool_create(pages, 16, max_seqs, max_blocks, table)
    try:
        for it in range(30):                       # 30 * 3 * ~18000 entries = 1.6 M > 4 x 65536
            for s in range(3):
                pa.pa_pool_reserve(pool, s, 16 * (18000 + 100 * s + it))
            if it < 29:
                for s in range(3):
                    pa.pa_pool_release(pool, s)
        pa.pa_pool_reserve(pool, 3, 16 * 70)       # one short row behind the long ones
        torch.cuda.synchronize()
        got = table.cpu().numpy()
        for s in range(max_seqs):
            row = pa.pa_pool_get_row(pool, s)
            assert list(got[s, :len(row)]) == row
            assert (got[s, len(row):] == -1).all()
        assert pa.pa_pool_num_free(pool) == pages - sum(pa.pa_pool_num_blocks(pool, s) for s in range(max_seqs))
    finally:
        pa.pa_pool_destroy(pool)
