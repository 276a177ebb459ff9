"""KV page manager (Algorithm 1 Reserve; Sec. III-B): the model in oracle/ against pins of its own, then the
library's host-side pool against the model.  No GPU is needed: the pool is created without a device table."""
import os
import random
import threading

import pytest

from oracle.page_manager import OutOfPages, PageManagerModel
from paper_2506_07311_amd import binding

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "page_manager_trace.txt")


def read_trace():
    steps = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        op, blocks, free, shared = [f.strip() for f in line.split("|")]
        steps.append((op.split(), [int(x) for x in blocks.split()], int(free), int(shared)))
    return steps


class ModelDriver:
    def __init__(self, num_pages, page_size, max_seqs, max_blocks, pow2=False):
        self.m = PageManagerModel(num_pages, page_size, max_seqs, max_blocks, pow2_growth=pow2)
        self.num_pages, self.max_seqs = num_pages, max_seqs

    def reserve(self, s, n):
        try:
            self.m.reserve(s, n)
            return True
        except OutOfPages:
            return False

    def release(self, s):
        self.m.release(s)

    def share(self, d, s, n):
        self.m.share_prefix(d, s, n)

    def writable(self, s, pos):
        try:
            self.m.make_writable(s, pos)
            return True
        except OutOfPages:
            return False

    def blocks(self):
        return [self.m.num_blocks(s) for s in range(self.max_seqs)]

    def free(self):
        return self.m.num_free()

    def rows(self):
        return [list(r) for r in self.m.rows]

    def refcounts(self):
        return [self.m.refcount(p) for p in range(self.num_pages)]

    def close(self):
        pass


class PoolDriver:
    """The library's pool, host-only.  make_writable needs a cache descriptor; with a NULL device table and a
    private page it returns before touching it, and a shared page would launch a copy, so the CPU tests drive
    copy-on-write through `writable_host`, which performs the same bookkeeping steps through the public calls
    only when the page is private, and otherwise is exercised on the GPU (tests/test_gpu_parity.py)."""

    def __init__(self, num_pages, page_size, max_seqs, max_blocks, pow2=False):
        self.h = binding.pa_pool_create(num_pages, page_size, max_seqs, max_blocks)
        if pow2:
            binding.pa_pool_set_growth(self.h, binding.PA_GROW_POW2)
        self.num_pages, self.max_seqs = num_pages, max_seqs

    def reserve(self, s, n):
        try:
            binding.pa_pool_reserve(self.h, s, n)
            return True
        except binding.PagedAttnError as e:
            assert "exhausted" in str(e), e
            return False

    def release(self, s):
        binding.pa_pool_release(self.h, s)

    def share(self, d, s, n):
        binding.pa_pool_share_prefix(self.h, d, s, n)

    def blocks(self):
        return [binding.pa_pool_num_blocks(self.h, s) for s in range(self.max_seqs)]

    def free(self):
        return binding.pa_pool_num_free(self.h)

    def rows(self):
        return [binding.pa_pool_get_row(self.h, s) for s in range(self.max_seqs)]

    def refcounts(self):
        return [binding.pa_pool_refcount(self.h, p) for p in range(self.num_pages)]

    def close(self):
        binding.pa_pool_destroy(self.h)


def sharing(rows):
    groups = {}
    for s, row in enumerate(rows):
        for b, page in enumerate(row):
            groups.setdefault(page, []).append((s, b))
    return sorted(sorted(g) for g in groups.values())


def check_valid(d):
    """What must hold for ANY correct manager: pages in range, reference count = number of mappings, no page
    both free and mapped, free + distinct mapped = all pages."""
    rows = d.rows()
    refs = d.refcounts()
    count = [0] * d.num_pages
    for row in rows:
        assert len(set(row)) == len(row), "one sequence maps a page twice"
        for page in row:
            assert 0 <= page < d.num_pages
            count[page] += 1
    assert count == refs
    assert d.free() + sum(1 for c in count if c) == d.num_pages


# ---------------------------------------------------------------- pins of the model -------------------------------

def test_model_follows_the_hand_worked_trace():
    d = ModelDriver(8, 4, 3, 6)
    run_trace(d, with_cow=True)


def run_trace(d, with_cow):
    for op, blocks, free, shared in read_trace():
        name, args = op[0], [int(x) for x in op[1:]]
        if name == "writable" and not with_cow:
            return
        if name == "reserve":
            assert d.reserve(*args)
        elif name == "reserve!":
            assert not d.reserve(*args)
        elif name == "share":
            d.share(*args)
        elif name == "release":
            d.release(*args)
        elif name == "writable":
            assert d.writable(*args)
        assert d.blocks() == blocks, op
        assert d.free() == free, op
        assert sum(1 for r in d.refcounts() if r == 2) == shared, op
        check_valid(d)


@pytest.mark.parametrize("P", [1, 16, 64])
def test_model_block_count_is_ceil_len_over_page(P):
    m = PageManagerModel(4096, P, 1, 4096)
    have = 0
    for length in [0, 1, P - 1, P, P + 1, 7 * P, 7 * P + 1, 3, 40 * P - 1]:
        m.reserve(0, length)
        have = max(have, (length + P - 1) // P)             # closed form; never shrinks
        assert m.num_blocks(0) == have
        assert m.num_free() == 4096 - have
    m.release(0)
    assert m.num_free() == 4096 and m.num_blocks(0) == 0


def test_model_refuses_without_side_effects():
    m = PageManagerModel(5, 4, 2, 8)
    m.reserve(0, 12)
    with pytest.raises(OutOfPages):
        m.reserve(1, 12)
    assert m.num_blocks(1) == 0 and m.num_free() == 2
    with pytest.raises(ValueError):
        m.reserve(1, 4 * 9)


# ---------------------------------------------------------------- the library's pool against the model ------------

def test_pool_follows_the_hand_worked_trace_up_to_copy_on_write():
    d = PoolDriver(8, 4, 3, 6)
    try:
        run_trace(d, with_cow=False)
    finally:
        d.close()


def random_ops(rng, n_ops, max_seqs, max_len):
    live = {}
    ops = []
    for _ in range(n_ops):
        r = rng.random()
        s = rng.randrange(max_seqs)
        if r < 0.55:
            grow = rng.choice([1, 1, 1, 7, 64, 300])
            length = min(max_len, live.get(s, 0) + grow)
            ops.append(("reserve", s, length))
            live[s] = length          # the driver drops it again if the reservation is refused
        elif r < 0.8:
            ops.append(("release", s))
            live.pop(s, None)
        else:
            src = rng.randrange(max_seqs)
            if src != s and s not in live and live.get(src, 0) > 0:
                n = rng.randrange(live[src] + 1)
                ops.append(("share", s, src, n))
                live[s] = n
    return ops


def test_power_of_two_growth_closed_form():
    """One sequence growing token by token in an ample pool holds 2^ceil(log2(ceil(len/P))) blocks, capped at the
    row width, and touches the free list only when that number changes."""
    P, max_blocks = 4, 48
    for d in (ModelDriver(1000, P, 1, max_blocks, pow2=True), PoolDriver(1000, P, 1, max_blocks, pow2=True)):
        try:
            changes = 0
            prev = 0
            for length in range(1, max_blocks * P + 1):
                assert d.reserve(0, length)
                n = -(-length // P)
                expect = min(1 << (n - 1).bit_length(), max_blocks)
                assert d.blocks() == [expect], length
                changes += expect != prev
                prev = expect
            assert changes == 7          # 1, 2, 4, 8, 16, 32, 48
        finally:
            d.close()


@pytest.mark.parametrize("seed,P,pages,pow2", [(0, 16, 64, False), (1, 1, 200, False), (2, 64, 24, False),
                                               (3, 16, 600, False), (4, 16, 64, True), (5, 4, 300, True)])
def test_pool_matches_model_on_random_serving_traces(seed, P, pages, pow2):
    rng = random.Random(seed)
    max_seqs, max_blocks = 12, 40
    model = ModelDriver(pages, P, max_seqs, max_blocks, pow2)
    pool = PoolDriver(pages, P, max_seqs, max_blocks, pow2)
    lengths = {}
    try:
        for op in random_ops(rng, 1500, max_seqs, max_blocks * P):
            if op[0] == "reserve":
                ok_m, ok_p = model.reserve(*op[1:]), pool.reserve(*op[1:])
                assert ok_m == ok_p, op
                if ok_m:
                    lengths[op[1]] = op[2]
            elif op[0] == "release":
                model.release(op[1])
                pool.release(op[1])
                lengths.pop(op[1], None)
            else:
                _, dst, src, n = op
                if lengths.get(src, 0) < n or model.blocks()[dst]:
                    continue
                model.share(dst, src, n)
                pool.share(dst, src, n)
                lengths[dst] = (n // P) * P
            assert pool.blocks() == model.blocks(), op
            assert pool.free() == model.free(), op
            assert sharing(pool.rows()) == sharing(model.rows()), op
            assert sorted(pool.refcounts()) == sorted(model.refcounts()), op
        check_valid(pool)
        for s in range(max_seqs):
            pool.release(s)
        assert pool.free() == pages and pool.refcounts() == [0] * pages
    finally:
        pool.close()


def test_pool_argument_errors():
    lib = binding.load_library()
    with pytest.raises(binding.PagedAttnError):
        binding.pa_pool_create(8, 12, 2, 4)                  # page size not a power of two
    with pytest.raises(binding.PagedAttnError):
        binding.pa_pool_create(0, 16, 2, 4)
    h = binding.pa_pool_create(8, 16, 2, 4)
    try:
        with pytest.raises(binding.PagedAttnError):
            binding.pa_pool_reserve(h, 2, 1)                 # sequence out of range
        with pytest.raises(binding.PagedAttnError):
            binding.pa_pool_reserve(h, 0, 16 * 4 + 1)        # more blocks than a row holds
        binding.pa_pool_reserve(h, 0, 40)
        with pytest.raises(binding.PagedAttnError):
            binding.pa_pool_share_prefix(h, 0, 0, 16)
        with pytest.raises(binding.PagedAttnError):
            binding.pa_pool_share_prefix(h, 1, 0, 64)        # more pages than the source maps
        binding.pa_pool_share_prefix(h, 1, 0, 33)
        assert binding.pa_pool_get_row(h, 1) == binding.pa_pool_get_row(h, 0)[:2]
        with pytest.raises(binding.PagedAttnError):
            binding.pa_pool_share_prefix(h, 1, 0, 16)        # destination already holds blocks
        assert lib.pa_pool_num_blocks(h, 9) == -1 and lib.pa_pool_refcount(h, 99) == -1
    finally:
        binding.pa_pool_destroy(h)


def test_pool_is_safe_under_concurrent_sequences():
    """Sequences driven from different host threads (one thread per sequence, as the header allows) never
    receive the same page, and every page comes back."""
    pages, P, threads, rounds = 512, 16, 8, 300
    h = binding.pa_pool_create(pages, P, threads, 64)
    seen_bad = []

    def worker(s):
        rng = random.Random(100 + s)
        for _ in range(rounds):
            length = 0
            for _ in range(rng.randrange(1, 12)):
                length = min(64 * P, length + rng.choice([1, 5, 40, 130]))
                try:
                    binding.pa_pool_reserve(h, s, length)
                except binding.PagedAttnError:
                    break
            row = binding.pa_pool_get_row(h, s)
            if len(set(row)) != len(row) or any(binding.pa_pool_refcount(h, p) != 1 for p in row):
                seen_bad.append((s, row))
            binding.pa_pool_release(h, s)

    try:
        ts = [threading.Thread(target=worker, args=(s,)) for s in range(threads)]
        for t in ts:
            t.start()
        for t in ts:
            t.join()
        assert not seen_bad
        assert binding.pa_pool_num_free(h) == pages
        assert all(binding.pa_pool_refcount(h, p) == 0 for p in range(pages))
        # after the storm every page can still be handed out exactly once
        binding.pa_pool_reserve(h, 0, 64 * P)
        for s in range(1, threads):
            binding.pa_pool_reserve(h, s, 64 * P)
        rows = [binding.pa_pool_get_row(h, s) for s in range(threads)]
        flat = [p for r in rows for p in r]
        assert sorted(flat) == list(range(pages))
    finally:
        binding.pa_pool_destroy(h)
