"""Pins for the oracle's fp16 input path and its mask / score modifications (sliding window, document mask, soft cap,
linear position bias), independent of the oracle:
  * binary16 widening against numpy's float16 -> float64 on all 65536 bit patterns,
  * a dense reference built with numpy index arithmetic and scipy's softmax / logsumexp on contiguous inputs
    (explicit [Tq, len] mask and bias matrices, no shared code path),
  * special cases that reduce to the unmodified attention or to a closed form.
"""
import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

from paper_2506_07311_amd import workloads as W


def np_inputs(w):
    return dict(k_cache=W.to_numpy(w.k_cache), v_cache=W.to_numpy(w.v_cache), q=W.to_numpy(w.q),
                block_table=W.to_numpy(w.block_table), seq_lens=W.to_numpy(w.seq_lens),
                cu_q_lens=W.to_numpy(w.cu_q_lens))


def run(oracle, w, **kw):
    a = np_inputs(w)
    return oracle.attention(a["k_cache"], a["v_cache"], a["q"], a["block_table"], a["seq_lens"], w.scale,
                            causal=w.causal, cu_q_lens=a["cu_q_lens"], **kw)


def to64(t):
    return t.double().numpy()


def test_binary16_widening_matches_numpy_on_every_bit_pattern(oracle):
    h = np.arange(65536, dtype=np.uint16).view(np.float16)
    got = oracle.widen(h)
    ref = h.astype(np.float64)
    nan = np.isnan(ref)
    assert (np.isnan(got) == nan).all()
    assert (got[~nan] == ref[~nan]).all()
    assert (np.signbit(got[~nan]) == np.signbit(ref[~nan])).all()


def dense_reference(w, window=0, softcap=0.0, slopes=None, docs=None, prefix=None, prefix_bias=0.0):
    """Contiguous-layout reference: identity pages, so sequence s occupies pool rows [start_s, start_s + len)."""
    assert w.page_size * w.num_pages >= sum(w.seq_lens_host)
    Hq, Hkv, d = w.num_q_heads, w.num_kv_heads, w.head_dim
    G = Hq // Hkv
    K = to64(w.k_cache.float()).reshape(-1, Hkv, d)
    V = to64(w.v_cache.float()).reshape(-1, Hkv, d)
    Q = to64(w.q.float())
    bt = W.to_numpy(w.block_table)
    outs, lses = [], []
    q0 = 0
    for s, (L, Tq) in enumerate(zip(w.seq_lens_host, w.q_lens_host)):
        start = int(bt[s, 0]) * w.page_size if L else 0
        pos = np.arange(L - Tq, L)[:, None]                  # [Tq, 1]
        j = np.arange(L)[None, :]                            # [1, L]
        mask = np.ones((Tq, L), dtype=bool)
        if w.causal:
            mask &= j <= pos
        if window > 0:
            mask &= np.abs(j - pos) < window
        if docs is not None:
            dd = np.asarray(docs[s][:L])
            mask &= dd[None, :] == dd[np.arange(L - Tq, L)][:, None]
        if prefix is not None:                                # prefix-LM: bidirectional prefix, causal remainder
            mask &= (j <= pos) | (j < prefix[s])
        for h in range(Hq):
            x = w.scale * Q[q0:q0 + Tq, h] @ K[start:start + L, h // G].T
            if softcap > 0:
                x = softcap * np.tanh(x / softcap)
            if slopes is not None:
                x = x + slopes[h] * (j - pos)
            if prefix is not None:
                x = x + prefix_bias * (j < prefix[s])
            x = np.where(mask, x, -np.inf)
            any_key = mask.any(axis=1)
            p = np.zeros_like(x)
            p[any_key] = softmax(x[any_key], axis=1)
            o = p @ V[start:start + L, h // G]
            ls = np.full(Tq, -np.inf)
            ls[any_key] = logsumexp(x[any_key], axis=1)
            outs.append((q0, h, o))
            lses.append((q0, h, ls))
        q0 += Tq
    out = np.zeros((w.total_q, Hq, d))
    lse = np.zeros((w.total_q, Hq))
    for (r0, h, o), (_, _, ls) in zip(outs, lses):
        out[r0:r0 + o.shape[0], h] = o
        lse[r0:r0 + o.shape[0], h] = ls
    return out, lse


def contiguous_workload(dtype, causal, seed=0):
    # identity pages with whole pages per sequence: sequence s starts at its first page
    return W.make_workload("t", seq_lens=[37, 16, 50], q_lens=[37, 3, 1], num_q_heads=6, num_kv_heads=3, head_dim=16,
                           page_size=8, dtype=dtype, causal=causal, seed=seed, identity_pages=True, poison=False,
                           scale=0.6)


def doc_ids_for(w, seed):
    rng = np.random.default_rng(seed)
    width = max(w.seq_lens_host) + 3
    ids = np.zeros((w.batch, width), dtype=np.int32)
    for s in range(w.batch):
        cuts = np.sort(rng.integers(0, width, size=3))
        ids[s] = np.searchsorted(cuts, np.arange(width), side="right")
    return ids


@pytest.mark.parametrize("dtype", [torch.float32, torch.float16, torch.bfloat16])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("mods", [
    dict(),
    dict(window=5),
    dict(window=1),
    dict(softcap=1.5),
    dict(slopes=True),
    dict(docs=True),
    dict(window=9, softcap=2.0, slopes=True, docs=True),
])
def test_oracle_matches_dense_numpy_reference(oracle, dtype, causal, mods):
    w = contiguous_workload(dtype, causal, seed=11)
    slopes = np.array([2.0 ** -(h + 1) for h in range(w.num_q_heads)]) if mods.get("slopes") else None
    docs = doc_ids_for(w, 5) if mods.get("docs") else None
    kw = dict(window=mods.get("window", 0), softcap=mods.get("softcap", 0.0), alibi_slopes=slopes, doc_ids=docs)
    out, lse = run(oracle, w, **kw)
    ref_o, ref_l = dense_reference(w, window=kw["window"], softcap=kw["softcap"], slopes=slopes, docs=docs)
    np.testing.assert_allclose(out, ref_o, rtol=0, atol=1e-12)
    finite = np.isfinite(ref_l)
    assert (np.isfinite(lse) == finite).all()
    np.testing.assert_allclose(lse[finite], ref_l[finite], rtol=0, atol=1e-12)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("extra", [dict(), dict(window=9, softcap=2.0, slopes=True, docs=True)])
@pytest.mark.parametrize("bias", [0.0, 0.75])
def test_prefix_lm_family_matches_dense_numpy_reference(oracle, dtype, extra, bias):
    """The user-defined pair of the extension point (visible: j <= pos or j < prefix_len; score: + bias on prefix
    keys), alone and on top of the built-in hooks, against explicit mask and bias matrices."""
    w = contiguous_workload(dtype, False, seed=12)
    prefix = np.array([20, 0, 50], dtype=np.int32)           # inside, empty, and covering the whole sequence
    slopes = np.array([2.0 ** -(h + 1) for h in range(w.num_q_heads)]) if extra.get("slopes") else None
    docs = doc_ids_for(w, 6) if extra.get("docs") else None
    kw = dict(window=extra.get("window", 0), softcap=extra.get("softcap", 0.0), alibi_slopes=slopes, doc_ids=docs)
    out, lse = run(oracle, w, prefix_lens=prefix, prefix_bias=bias, **kw)
    ref_o, ref_l = dense_reference(w, window=kw["window"], softcap=kw["softcap"], slopes=slopes, docs=docs,
                                   prefix=prefix, prefix_bias=bias)
    np.testing.assert_allclose(out, ref_o, rtol=0, atol=1e-12)
    finite = np.isfinite(ref_l)
    assert (np.isfinite(lse) == finite).all()
    np.testing.assert_allclose(lse[finite], ref_l[finite], rtol=0, atol=1e-12)


def test_prefix_lm_special_cases(oracle):
    """A prefix of length 0 is the causal mask; a prefix that covers the sequence is no mask at all; a bias on a
    prefix that covers every visible key shifts lse by the bias and leaves the output alone."""
    w = contiguous_workload(torch.float32, False, seed=13)
    causal_w = contiguous_workload(torch.float32, True, seed=13)
    zero = np.zeros(w.batch, dtype=np.int32)
    full = np.array(w.seq_lens_host, dtype=np.int32)
    o_causal, l_causal = run(oracle, causal_w)
    o_zero, l_zero = run(oracle, w, prefix_lens=zero)
    np.testing.assert_array_equal(o_zero, o_causal)
    np.testing.assert_array_equal(l_zero, l_causal)
    o_plain, l_plain = run(oracle, w)
    o_full, l_full = run(oracle, w, prefix_lens=full)
    np.testing.assert_array_equal(o_full, o_plain)
    np.testing.assert_array_equal(l_full, l_plain)
    o_b, l_b = run(oracle, w, prefix_lens=full, prefix_bias=1.25)
    np.testing.assert_allclose(o_b, o_plain, rtol=0, atol=1e-13)
    np.testing.assert_allclose(l_b, l_plain + 1.25, rtol=0, atol=1e-12)


def test_neutral_modifications_change_nothing(oracle):
    w = W.make_workload("t", seq_lens=[45, 7], q_lens=[20, 7], num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        dtype=torch.float32, causal=True, seed=2)
    base_o, base_l = run(oracle, w)
    same_doc = np.full((2, 45), 7, dtype=np.int32)
    for kw in (dict(window=45), dict(window=10 ** 6), dict(alibi_slopes=np.zeros(4)), dict(doc_ids=same_doc)):
        o, l = run(oracle, w, **kw)
        np.testing.assert_array_equal(o, base_o)
        np.testing.assert_array_equal(l, base_l)
    o, l = run(oracle, w, softcap=1e7)                   # x - cap*tanh(x/cap) ~ x^3 / (3 cap^2)
    np.testing.assert_allclose(o, base_o, rtol=0, atol=1e-12)


@pytest.mark.parametrize("kw", [dict(window=1), dict(alibi_slopes=np.full(4, 1e4)),
                                dict(doc_ids=np.arange(2 * 45, dtype=np.int32).reshape(2, 45))])
def test_modifications_that_leave_only_the_own_position(oracle, kw):
    """Causal attention restricted to the query's own token returns that token's value row exactly (a window of
    one; a bias of -1e4 per step into the past; every token its own document)."""
    w = W.make_workload("t", seq_lens=[45, 7], q_lens=[20, 7], num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        dtype=torch.float32, causal=True, seed=4)
    out, _ = run(oracle, w, **kw)
    a = np_inputs(w)
    _, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    v = gv.astype(np.float64)
    rows = [(s0 + L - Tq + i) for s0, L, Tq in ((0, 45, 20), (45, 7, 7)) for i in range(Tq)]
    for r, src in enumerate(rows):
        for h in range(4):
            np.testing.assert_allclose(out[r, h], v[src, h // 2], rtol=0, atol=1e-300 if "alibi_slopes" not in kw
                                       else 1e-12)


def test_sliding_window_equals_attention_over_the_truncated_context(oracle):
    """Decode with a window of w tokens = plain decode over the last w tokens re-housed as a sequence of their own."""
    L, win = 61, 17
    w = W.make_workload("t", seq_lens=[L], num_q_heads=4, num_kv_heads=2, head_dim=8, page_size=4,
                        dtype=torch.float32, seed=8, identity_pages=True, poison=False)
    out, lse = run(oracle, w, window=win)
    a = np_inputs(w)
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    pages = (win + 3) // 4
    k2 = np.zeros((pages, 4, 2, 8), dtype=np.float32)
    v2 = np.zeros_like(k2)
    k2.reshape(-1, 2, 8)[:win] = gk[L - win:]
    v2.reshape(-1, 2, 8)[:win] = gv[L - win:]
    o2, l2 = oracle.attention(k2, v2, a["q"], np.arange(pages, dtype=np.int32)[None, :], np.array([win], np.int32),
                              w.scale)
    np.testing.assert_allclose(out, o2, rtol=0, atol=1e-14)
    np.testing.assert_allclose(lse, l2, rtol=0, atol=1e-14)


def test_position_bias_is_a_per_key_shift_for_a_single_query(oracle):
    """For one query, slope*(j - pos) differs from slope*j by a constant, which softmax ignores: the output equals
    plain attention with the bias folded into an extra key/query dimension (q_extra = slope/scale, k_extra = j)."""
    L, d = 23, 8
    w = W.make_workload("t", seq_lens=[L], num_q_heads=2, num_kv_heads=2, head_dim=d, page_size=4,
                        dtype=torch.float32, seed=10, identity_pages=True, poison=False, scale=0.5)
    slopes = np.array([0.25, 0.03125])
    out, _ = run(oracle, w, alibi_slopes=slopes)
    a = np_inputs(w)
    gk, gv = oracle.kv_gather(a["k_cache"], a["v_cache"], a["block_table"], a["seq_lens"])
    pages = (L + 3) // 4
    k2 = np.zeros((pages, 4, 2, d + 8), dtype=np.float32)
    v2 = np.zeros_like(k2)
    k2.reshape(-1, 2, d + 8)[:L, :, :d] = gk
    k2.reshape(-1, 2, d + 8)[:L, :, d] = np.arange(L, dtype=np.float32)[:, None]
    v2.reshape(-1, 2, d + 8)[:L, :, :d] = gv
    q2 = np.zeros((1, 2, d + 8), dtype=np.float32)
    q2[0, :, :d] = a["q"][0]
    q2[0, :, d] = (slopes / w.scale).astype(np.float32)      # exact: powers of two
    o2, _ = oracle.attention(k2, v2, q2, np.arange(pages, dtype=np.int32)[None, :], np.array([L], np.int32), w.scale)
    np.testing.assert_allclose(out, o2[:, :, :d], rtol=0, atol=1e-13)
