"""Pins for the CPU oracle: what the paper and the mathematics fix, independent of the oracle itself.

The paper prints no worked numeric example, so the oracle is pinned by
  * hand-worked instances of Algorithm 1's index translation (tests/golden/alg1_translation.txt),
  * a pure-Python brute force with on-the-fly translation (tests/bruteforce.py) on tiny inputs,
  * closed forms (one key, zero query, equal keys, dominant key, weights sum to 1, lse of equal scores),
  * a library special case (torch scaled_dot_product_attention in fp64 on contiguous inputs),
  * invariants (page permutation, pool size, aliased vs copied prefix, gather o append = identity,
    causal prefill row i = decode at length i+1, LSE merge of any split, masked slots never matter).
"""
import math
import os

import numpy as np
import pytest
import torch

from paper_2506_07311_amd import workloads as W
from tests import bruteforce

HERE = os.path.dirname(os.path.abspath(__file__))


def np_inputs(w):
    return dict(k_cache=W.to_numpy(w.k_cache), v_cache=W.to_numpy(w.v_cache), q=W.to_numpy(w.q),
                block_table=W.to_numpy(w.block_table), seq_lens=W.to_numpy(w.seq_lens),
                cu_q_lens=W.to_numpy(w.cu_q_lens))


def run_attention(oracle, w, **kw):
    a = np_inputs(w)
    return oracle.attention(a["k_cache"], a["v_cache"], a["q"], a["block_table"], a["seq_lens"], w.scale,
                            causal=w.causal, cu_q_lens=a["cu_q_lens"], **kw)


def widen(a):
    from oracle import bf16_bits_to_f64
    return bf16_bits_to_f64(a) if a.dtype == np.uint16 else a.astype(np.float64)


# ----------------------------------------------------------------------------- Algorithm 1 golden
def golden_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "alg1_translation.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            P, table, t, p = [x.strip() for x in line.split("|")]
            rows.append((int(P), [int(x) for x in table.split()], int(t), int(p)))
    return rows


@pytest.mark.parametrize("P,table,t,expect", golden_rows())
def test_append_lands_in_hand_worked_slot(oracle, P, table, t, expect):
    """Algorithm 1, Assign: the token written at position t must land in flat slot p (hand-worked)."""
    NP, Hkv, d = 10, 2, 4
    k = np.zeros((NP, P, Hkv, d), dtype=np.float32)
    v = np.zeros_like(k)
    k_new = np.full((1, Hkv, d), 5.0, dtype=np.float32)
    v_new = np.full((1, Hkv, d), -7.0, dtype=np.float32)
    bt = np.array([[9] * len(table), table], dtype=np.int32)       # sequence 1 carries the table
    oracle.kv_append(k, v, k_new, v_new, [1], [t], bt)
    flat_k = k.reshape(NP * P, Hkv * d)
    flat_v = v.reshape(NP * P, Hkv * d)
    hit = np.nonzero(flat_k.any(axis=1))[0]
    assert hit.tolist() == [expect]
    assert (flat_k[expect] == 5.0).all() and (flat_v[expect] == -7.0).all()
    assert np.count_nonzero(flat_v.any(axis=1)) == 1


@pytest.mark.parametrize("P,table,t,expect", golden_rows())
def test_gather_reads_hand_worked_slot(oracle, P, table, t, expect):
    """Algorithm 1, Gather: row t of the gathered sequence is the content of flat slot p."""
    NP, Hkv, d = 10, 2, 4
    k = np.arange(NP * P * Hkv * d, dtype=np.float32).reshape(NP, P, Hkv, d)
    v = -k
    bt = np.array([table], dtype=np.int32)
    L = t + 1
    gk, gv = oracle.kv_gather(k, v, bt, [L])
    assert gk.shape == (L, Hkv, d)
    np.testing.assert_array_equal(gk[t].ravel(), k.reshape(NP * P, -1)[expect])
    np.testing.assert_array_equal(gv[t].ravel(), v.reshape(NP * P, -1)[expect])


def test_head_major_layout_same_logical_content(oracle):
    """The strided descriptor: a [NP,Hkv,P,d] pool holding the same tokens gathers identically."""
    rng = np.random.default_rng(0)
    NP, P, Hkv, d = 6, 4, 3, 8
    k = rng.standard_normal((NP, P, Hkv, d)).astype(np.float32)
    v = rng.standard_normal((NP, P, Hkv, d)).astype(np.float32)
    bt = np.array([[4, 1, 5], [0, 2, 3]], dtype=np.int32)
    lens = [11, 9]
    a = oracle.kv_gather(k, v, bt, lens)
    b = oracle.kv_gather(np.ascontiguousarray(k.transpose(0, 2, 1, 3)),
                         np.ascontiguousarray(v.transpose(0, 2, 1, 3)), bt, lens, head_major=True)
    np.testing.assert_array_equal(a[0], b[0])
    np.testing.assert_array_equal(a[1], b[1])


# ----------------------------------------------------------------------------- append / gather invariants
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_gather_after_append_is_identity_and_pool_untouched(oracle, dtype):
    w = W.make_workload("t", seq_lens=[37, 5, 64, 1], q_lens=[37, 5, 64, 1], num_q_heads=4, num_kv_heads=2,
                        head_dim=8, page_size=8, dtype=dtype, seed=11, poison=False)
    a = np_inputs(w)
    k, v = a["k_cache"].copy(), a["v_cache"].copy()
    sentinel = 0x7FC1 if k.dtype == np.uint16 else np.float32(-12345.5)
    k[...] = sentinel
    v[...] = sentinel
    k_new, v_new = W.to_numpy(w.k_new), W.to_numpy(w.v_new)
    oracle.kv_append(k, v, k_new, v_new, W.to_numpy(w.seq_ids), W.to_numpy(w.positions), a["block_table"])
    gk, gv = oracle.kv_gather(k, v, a["block_table"], a["seq_lens"])
    np.testing.assert_array_equal(gk, k_new)       # every token was appended in order, so gather == input
    np.testing.assert_array_equal(gv, v_new)
    written = int(sum(w.seq_lens_host))
    untouched_k = np.count_nonzero((k == sentinel).all(axis=(2, 3)))
    assert untouched_k == k.shape[0] * k.shape[1] - written
    assert np.count_nonzero((v == sentinel).all(axis=(2, 3))) == untouched_k


def test_append_last_writer_wins_and_errors(oracle):
    k = np.zeros((4, 2, 1, 2), dtype=np.float32)
    v = np.zeros_like(k)
    bt = np.array([[2, 0]], dtype=np.int32)
    k_new = np.array([[[1, 1]], [[2, 2]]], dtype=np.float32)
    oracle.kv_append(k, v, k_new, k_new, [0, 0], [3, 3], bt)
    assert (k[0, 1, 0] == 2).all()
    with pytest.raises(ValueError):
        oracle.kv_append(k, v, k_new, k_new, [0, 0], [3, 4], bt)          # beyond the table
    with pytest.raises(ValueError):
        oracle.kv_append(k, v, k_new, k_new, [0, 0], [0, 1], np.array([[7, 0]], dtype=np.int32))  # bad page
    with pytest.raises(ValueError):
        oracle.kv_gather(np.zeros((4, 3, 1, 2), np.float32), np.zeros((4, 3, 1, 2), np.float32), bt, [2])  # P=3


# ----------------------------------------------------------------------------- brute force
CASES = [
    # lens, q_lens, Hq, Hkv, d, P, causal
    ([5], None, 1, 1, 3, 1, False),
    ([9, 4], None, 4, 2, 4, 2, False),
    ([7, 1, 6], None, 4, 1, 2, 4, False),
    ([6, 9], [6, 9], 2, 2, 3, 4, True),
    ([8, 5, 3], [3, 5, 1], 4, 2, 4, 2, True),
    ([9, 7], [4, 2], 3, 3, 2, 4, False),
    ([4, 0, 3], [1, 0, 1], 2, 1, 4, 2, False),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("case", CASES)
def test_oracle_matches_python_brute_force(oracle, case, dtype):
    lens, q_lens, Hq, Hkv, d, P, causal = case
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d,
                        page_size=P, dtype=dtype, causal=causal, seed=hash((tuple(lens), Hq, d)) % 1000,
                        poison=True, scale=0.7)
    a = np_inputs(w)
    out, lse, wts = run_attention(oracle, w, return_weights=True)
    is_bf16 = dtype == torch.bfloat16
    bo, bl, bw = bruteforce.attention(a["k_cache"].tolist(), a["v_cache"].tolist(), a["q"].tolist(),
                                      a["block_table"].tolist(), lens, a["cu_q_lens"].tolist(), w.scale,
                                      causal, is_bf16)
    if w.total_q == 0:
        return
    np.testing.assert_allclose(out, np.array(bo), rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse, np.array(bl), rtol=0, atol=1e-12)
    for r in range(w.total_q):
        for h in range(Hq):
            n = len(bw[r][h])
            np.testing.assert_allclose(wts[r, h, :n], bw[r][h], rtol=0, atol=1e-13)
            assert (wts[r, h, n:] == 0).all()


# ----------------------------------------------------------------------------- closed forms
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_one_token_context_returns_v_exactly(oracle, dtype):
    w = W.make_workload("t", seq_lens=[1, 1, 1], num_q_heads=4, num_kv_heads=2, head_dim=16, page_size=4,
                        dtype=dtype, seed=3)
    out, lse = run_attention(oracle, w)
    a = np_inputs(w)
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    v = widen(gv)                                        # [3, Hkv, d]
    for h in range(4):
        np.testing.assert_array_equal(out[:, h, :], v[:, h // 2, :])
    # lse of a single key is its score
    k, q = widen(gk), widen(a["q"])
    for h in range(4):
        np.testing.assert_allclose(lse[:, h], w.scale * (q[:, h, :] * k[:, h // 2, :]).sum(-1), rtol=1e-14)


def test_zero_query_gives_mean_of_allowed_values_and_lse_log_n(oracle):
    w = W.make_workload("t", seq_lens=[13, 6], q_lens=[4, 6], num_q_heads=2, num_kv_heads=1, head_dim=8,
                        page_size=4, dtype=torch.float32, causal=True, seed=5)
    w.q.zero_()
    out, lse = run_attention(oracle, w)
    a = np_inputs(w)
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    v0, v1 = gv[:13, 0].astype(np.float64), gv[13:, 0].astype(np.float64)
    for i in range(4):            # queries of sequence 0 sit at positions 9..12
        n = 13 - 4 + i + 1
        np.testing.assert_allclose(out[i, 0], v0[:n].mean(0), rtol=0, atol=1e-14)
        assert abs(lse[i, 1] - math.log(n)) < 1e-14
    for i in range(6):
        np.testing.assert_allclose(out[4 + i, 1], v1[:i + 1].mean(0), rtol=0, atol=1e-14)
        assert abs(lse[4 + i, 0] - math.log(i + 1)) < 1e-14


def test_equal_keys_give_mean_and_lse_shift(oracle):
    w = W.make_workload("t", seq_lens=[10], num_q_heads=2, num_kv_heads=2, head_dim=4, page_size=2,
                        dtype=torch.float32, seed=6, poison=False)
    w.k_cache[:] = torch.tensor([0.5, -1.0, 2.0, 0.25])
    out, lse = run_attention(oracle, w)
    a = np_inputs(w)
    _, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    q = a["q"].astype(np.float64)
    for h in range(2):
        np.testing.assert_allclose(out[0, h], gv[:, h].astype(np.float64).mean(0), atol=1e-14)
        c = w.scale * float(q[0, h] @ np.array([0.5, -1.0, 2.0, 0.25]))
        assert abs(lse[0, h] - (c + math.log(10))) < 1e-13


def test_dominant_key_selects_its_value_row(oracle):
    w = W.make_workload("t", seq_lens=[12], num_q_heads=1, num_kv_heads=1, head_dim=4, page_size=4,
                        dtype=torch.float32, seed=7, poison=False, scale=1.0)
    w.q[:] = torch.tensor([1.0, 0.0, 0.0, 0.0])
    w.k_cache.zero_()
    bt = w.block_table[0].tolist()
    w.k_cache[bt[7 // 4], 7 % 4, 0, 0] = 60.0     # key 7 scores 60, everything else 0
    out, lse, wts = run_attention(oracle, w, return_weights=True)
    v7 = w.v_cache[bt[1], 3, 0].double().numpy()
    np.testing.assert_allclose(out[0, 0], v7, atol=1e-20 + 12 * math.exp(-60) * 10)
    assert abs(wts[0, 0, 7] - 1.0) < 1e-20 + 12 * math.exp(-60)
    assert abs(lse[0, 0] - 60.0) < 1e-13


@pytest.mark.parametrize("causal", [False, True])
def test_weights_sum_to_one_and_mask_is_zero(oracle, causal):
    w = W.make_workload("t", seq_lens=[33, 17, 2], q_lens=[5, 17, 1], num_q_heads=4, num_kv_heads=2,
                        head_dim=16, page_size=8, dtype=torch.bfloat16, causal=causal, seed=8)
    out, lse, wts = run_attention(oracle, w, return_weights=True)
    assert np.abs(wts.sum(-1) - 1.0).max() < 1e-14
    assert (wts >= 0).all()
    row = 0
    for s, (L, Tq) in enumerate(zip(w.seq_lens_host, w.q_lens_host)):
        for i in range(Tq):
            n = (L - Tq + i + 1) if causal else L
            assert (wts[row, :, n:] == 0).all() and (wts[row, :, :n] > 0).all()
            row += 1


# ----------------------------------------------------------------------------- library special case
@pytest.mark.parametrize("causal,Hq,Hkv", [(False, 4, 4), (True, 4, 4), (True, 8, 2), (False, 6, 3)])
def test_matches_torch_sdpa_fp64_on_contiguous_inputs(oracle, causal, Hq, Hkv):
    S, d, P = 40, 16, 8
    w = W.make_workload("t", seq_lens=[S, S], q_lens=[S, S], num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d,
                        page_size=P, dtype=torch.float32, causal=causal, seed=9, identity_pages=True,
                        pool_factor=1.0, poison=False)
    out, _ = run_attention(oracle, w)
    # identity pages: the pool reshaped IS the contiguous [B, S, Hkv, d] tensor
    k = w.k_cache.reshape(2, S, Hkv, d).double().permute(0, 2, 1, 3)
    v = w.v_cache.reshape(2, S, Hkv, d).double().permute(0, 2, 1, 3)
    q = w.q.reshape(2, S, Hq, d).double().permute(0, 2, 1, 3)
    G = Hq // Hkv
    ref = torch.nn.functional.scaled_dot_product_attention(
        q, k.repeat_interleave(G, dim=1), v.repeat_interleave(G, dim=1), is_causal=causal, scale=w.scale)
    ref = ref.permute(0, 2, 1, 3).reshape(2 * S, Hq, d).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-12)


# ----------------------------------------------------------------------------- invariants
def _relayout(oracle, w, num_pages, seed, alias_from=None):
    """Re-house the same logical sequences in a new pool under a new random page permutation.
    Returns numpy (k_cache, v_cache, block_table)."""
    a = np_inputs(w)
    P = w.page_size
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    rng = np.random.default_rng(seed)
    perm = rng.permutation(num_pages)
    k = np.full((num_pages, P) + gk.shape[1:], np.nan, dtype=np.float32)
    v = np.full_like(k, np.nan)
    if gk.dtype == np.uint16:
        k = np.full((num_pages, P) + gk.shape[1:], 0x7FC0, dtype=np.uint16)
        v = k.copy()
    bt = np.full_like(a["block_table"], -1)
    cur, row = 0, 0
    for s, L in enumerate(w.seq_lens_host):
        for b in range((L + P - 1) // P):
            pg = perm[cur]
            cur += 1
            bt[s, b] = pg
            n = min(P, L - b * P)
            k[pg, :n] = gk[row + b * P: row + b * P + n]
            v[pg, :n] = gv[row + b * P: row + b * P + n]
        row += L
    return k, v, bt


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_result_independent_of_page_permutation_and_pool_size(oracle, dtype):
    w = W.make_workload("t", seq_lens=[45, 16, 3, 31], q_lens=[2, 16, 1, 1], num_q_heads=4, num_kv_heads=2,
                        head_dim=8, page_size=4, dtype=dtype, causal=True, seed=12)
    a = np_inputs(w)
    base = run_attention(oracle, w)
    for num_pages, seed in [(30, 1), (97, 2), (400, 3)]:
        k, v, bt = _relayout(oracle, w, num_pages, seed)
        o, l = oracle.attention(k, v, a["q"], bt, a["seq_lens"], w.scale, causal=True, cu_q_lens=a["cu_q_lens"])
        np.testing.assert_array_equal(o, base[0])       # same values in the same order: bit-identical
        np.testing.assert_array_equal(l, base[1])


def test_aliased_prefix_pages_equal_copied_pages(oracle):
    w = W.make_workload("t", seq_lens=[70, 41, 33, 90], num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=8,
                        dtype=torch.bfloat16, seed=13, share_group=4, share_prefix_tokens=32)
    a = np_inputs(w)
    bt = a["block_table"]
    assert (bt[:, :4] == bt[0, :4]).all(), "generator should alias the 4 prefix pages"
    aliased = run_attention(oracle, w)
    k, v, bt2 = _relayout(oracle, w, 80, 5)             # every sequence gets private copies
    assert len(set(bt2[bt2 >= 0].tolist())) == (bt2 >= 0).sum()
    copied = oracle.attention(k, v, a["q"], bt2, a["seq_lens"], w.scale)
    np.testing.assert_array_equal(aliased[0], copied[0])
    np.testing.assert_array_equal(aliased[1], copied[1])


def test_causal_prefill_row_equals_decode_at_that_length(oracle):
    S = 21
    w = W.make_workload("t", seq_lens=[S], q_lens=[S], num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        dtype=torch.float32, causal=True, seed=14)
    a = np_inputs(w)
    full, full_lse = run_attention(oracle, w)
    for i in [0, 1, 3, 4, 12, S - 1]:
        o, l = oracle.attention(a["k_cache"], a["v_cache"], a["q"][i:i + 1], a["block_table"], [i + 1], w.scale)
        np.testing.assert_array_equal(o[0], full[i])
        np.testing.assert_array_equal(l[0], full_lse[i])


def test_lse_merge_of_any_two_way_split_equals_unsplit(oracle):
    """Pins the split-KV merge identity: attention over keys [0,c) and [c,L) merged by LSE weights."""
    L, P = 29, 4
    w = W.make_workload("t", seq_lens=[L], num_q_heads=2, num_kv_heads=1, head_dim=8, page_size=P,
                        dtype=torch.float32, seed=15)
    a = np_inputs(w)
    whole, whole_lse = run_attention(oracle, w)
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], [L])
    for c in [1, 4, 13, 28]:
        parts = []
        for lo, hi in [(0, c), (c, L)]:
            n = hi - lo
            nb = (n + P - 1) // P
            k = np.zeros((nb, P, 1, 8), np.float32)
            v = np.zeros_like(k)
            k.reshape(nb * P, 1, 8)[:n] = gk[lo:hi]
            v.reshape(nb * P, 1, 8)[:n] = gv[lo:hi]
            parts.append(oracle.attention(k, v, a["q"], np.arange(nb, dtype=np.int32)[None], [n], w.scale))
        for h in range(2):
            o, l = oracle.merge_partials(np.stack([parts[0][0][0, h], parts[1][0][0, h]]),
                                         [parts[0][1][0, h], parts[1][1][0, h]])
            np.testing.assert_allclose(o, whole[0, h], rtol=0, atol=1e-14)
            assert abs(l - whole_lse[0, h]) < 1e-13
    # an empty partial contributes nothing
    o, l = oracle.merge_partials(np.stack([whole[0, 0], np.full(8, 123.0)]), [whole_lse[0, 0], -np.inf])
    np.testing.assert_array_equal(o, whole[0, 0])
    assert l == whole_lse[0, 0]


def test_masked_slots_never_matter(oracle):
    """Unused pages, the tail of the last page and (causal) future keys may hold anything."""
    w = W.make_workload("t", seq_lens=[19, 7], q_lens=[3, 7], num_q_heads=2, num_kv_heads=2, head_dim=4,
                        page_size=8, dtype=torch.float32, causal=True, seed=16, poison=True)
    assert torch.isnan(w.k_cache).any()
    out, lse = run_attention(oracle, w)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    w2 = W.make_workload("t", seq_lens=[19, 7], q_lens=[3, 7], num_q_heads=2, num_kv_heads=2, head_dim=4,
                         page_size=8, dtype=torch.float32, causal=True, seed=16, poison=False)
    out2, lse2 = run_attention(oracle, w2)
    np.testing.assert_array_equal(out, out2)
    np.testing.assert_array_equal(lse, lse2)


def test_empty_sequence_gives_zero_and_minus_inf(oracle):
    w = W.make_workload("t", seq_lens=[0, 5], q_lens=[1, 1], num_q_heads=2, num_kv_heads=1, head_dim=4,
                        page_size=4, dtype=torch.float32, seed=17)
    out, lse = run_attention(oracle, w)
    assert (out[0] == 0).all() and (lse[0] == -np.inf).all()
    assert np.isfinite(out[1]).all() and np.isfinite(lse[1]).all()


def test_gqa_maps_consecutive_query_heads_to_one_kv_head(oracle):
    """kv head = floor(h / G): heads 0..G-1 with identical queries give identical outputs, head G differs."""
    w = W.make_workload("t", seq_lens=[11], num_q_heads=6, num_kv_heads=2, head_dim=4, page_size=4,
                        dtype=torch.float32, seed=18)
    w.q[:] = w.q[:, :1, :]
    out, _ = run_attention(oracle, w)
    np.testing.assert_array_equal(out[0, 0], out[0, 1])
    np.testing.assert_array_equal(out[0, 0], out[0, 2])
    np.testing.assert_array_equal(out[0, 3], out[0, 5])
    assert np.abs(out[0, 0] - out[0, 3]).max() > 1e-3
