"""Helpers shared by the GPU parity tests: run one workload through the C-ABI library and through
the CPU oracle, and compare under the stated tolerances."""
import numpy as np
import torch

from paper_2506_07311_amd import workloads as W

# Tolerances (both measures must hold):
#   max-abs  = max |g - r|
#   max-rel  = max |g - r| / max(|r|, rms(r))   -- floored at the reference tensor's RMS so that zero
#              crossings do not blow the ratio up and an all-zero output cannot pass on max-abs alone
# bf16 I/O with fp32 accumulation: 1e-2 / 2e-2.  fp32 I/O: 1e-5 / 1e-5.
# fp16 I/O with fp32 accumulation: the output's own rounding is 2^-11 relative (4.9e-4 at |out| = 1, 2e-3 at 4);
# softmax weights enter the matrix cores with the same 2^-11: 2e-3 / 4e-3 (a fifth of the bf16 bound, as the
# formats' mantissas suggest: 2^-11 vs 2^-8 would allow an eighth).
TOL = {torch.bfloat16: (1e-2, 2e-2), torch.float32: (1e-5, 1e-5), torch.float16: (2e-3, 4e-3)}


def errors(got: np.ndarray, ref: np.ndarray):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    diff = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    denom = np.maximum(np.abs(ref), max(rms, 1e-30))
    return (float(diff.max()) if diff.size else 0.0), (float((diff / denom).max()) if diff.size else 0.0)


def assert_close(got, ref, dtype, what="", tol=None):
    assert np.isfinite(np.asarray(got, dtype=np.float64)).all(), f"{what}: non-finite GPU output"
    max_abs, max_rel = errors(got, ref)
    tol_abs, tol_rel = tol or TOL[dtype]
    assert max_abs <= tol_abs and max_rel <= tol_rel, \
        f"{what}: max-abs {max_abs:.3e} (tol {tol_abs}), max-rel {max_rel:.3e} (tol {tol_rel})"
    return max_abs, max_rel


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().double().cpu().numpy()


def oracle_step(oracle, w: W.PagedWorkload, append=True, mods=None):
    """Append (Algorithm 1, Assign) then attention on host copies.  Returns (k_cache, v_cache, out, lse).
    mods: dict with any of window, softcap, alibi_slopes (numpy [Hq]), doc_ids (numpy int32 [B, stride]),
    prefix_lens (numpy int32 [B]) and prefix_bias (the prefix-LM user modification)."""
    k, v = W.to_numpy(w.k_cache).copy(), W.to_numpy(w.v_cache).copy()
    bt = W.to_numpy(w.block_table)
    if append and w.seq_ids.numel():
        oracle.kv_append(k, v, W.to_numpy(w.k_new), W.to_numpy(w.v_new), W.to_numpy(w.seq_ids),
                         W.to_numpy(w.positions), bt)
    out, lse = oracle.attention(k, v, W.to_numpy(w.q), bt, W.to_numpy(w.seq_lens), w.scale, causal=w.causal,
                                cu_q_lens=W.to_numpy(w.cu_q_lens), **(mods or {}))
    return k, v, out, lse


def gpu_step(pa, w: W.PagedWorkload, append=True, prefill=None, with_lse=True, mods=None, step_call=False):
    """Append then attention through the C-ABI binding, in place on the workload's pools.  ``step_call``: a decode
    step goes through the single paged_decode_step call instead of paged_kv_append + paged_attention_decode."""
    kw = {}
    if mods:
        dev = w.q.device
        kw = dict(window=mods.get("window", 0), softcap=mods.get("softcap", 0.0))
        if mods.get("alibi_slopes") is not None:
            kw["alibi_slopes"] = torch.tensor(np.asarray(mods["alibi_slopes"]), dtype=torch.float32, device=dev)
        if mods.get("doc_ids") is not None:
            kw["doc_ids"] = torch.tensor(np.asarray(mods["doc_ids"]), dtype=torch.int32, device=dev)
        if mods.get("prefix_lens") is not None:
            from paper_2506_07311_amd import binding
            prefix = torch.tensor(np.asarray(mods["prefix_lens"]), dtype=torch.int32, device=dev)
            kw["user_mod"] = binding.PA_MOD_PREFIX_LM
            kw["user_data"] = binding.prefix_lm_data(prefix, mods.get("prefix_bias", 0.0))
    if prefill is None:
        prefill = w.causal or w.max_q_len > 1 or w.total_q != w.batch
    step_call = step_call and append and not prefill and w.k_new.shape[0] == w.batch
    if append and w.seq_ids.numel() and not step_call:
        pa.paged_kv_append(w.k_cache, w.v_cache, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
    lse = torch.full((w.total_q, w.num_q_heads), float("nan"), dtype=torch.float32, device=w.q.device) \
        if with_lse else None
    # the workspace's contents are unspecified on entry: poison it (all-ones bytes: NaN as float, -1 as int), so a
    # partial that is read without having been written shows up
    ws = torch.full((pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.total_q,
                                                        w.max_seq_len),), 0xFF, dtype=torch.uint8, device=w.q.device)
    kw["workspace"] = ws
    if step_call:
        out = pa.paged_decode_step(w.k_cache, w.v_cache, w.k_new, w.v_new, w.q, w.block_table, w.seq_lens,
                                   w.max_seq_len, w.scale, lse=lse, **kw)
    elif prefill and mods:
        out = pa.paged_attention_prefill_mod(w.k_cache, w.v_cache, w.q, w.cu_q_lens, w.max_q_len, w.block_table,
                                             w.seq_lens, w.max_seq_len, w.scale, w.causal, lse=lse, **kw)
    elif prefill:
        out = pa.paged_attention_prefill(w.k_cache, w.v_cache, w.q, w.cu_q_lens, w.max_q_len, w.block_table,
                                         w.seq_lens, w.max_seq_len, w.scale, w.causal, lse=lse, **kw)
    elif mods:
        out = pa.paged_attention_decode_mod(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len,
                                            w.scale, lse=lse, **kw)
    else:
        out = pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len,
                                        w.scale, lse=lse, **kw)
    torch.cuda.synchronize()
    return out, lse


def _bits(a):
    # NaN-poisoned slots compare by bit pattern
    return a.view(np.uint32) if a.dtype == np.float32 else a.view(np.uint16) if a.dtype == np.float16 else a


def check_step(pa, oracle, w: W.PagedWorkload, what="", prefill=None, seqs=None, tol=None, mods=None,
               step_call=False):
    """Full parity of one step: pools bit-exact after the append, attention within tolerance (both measures over
    the whole compared output tensor).  With ``seqs`` the oracle sees only those sequences (their pages copied out
    BEFORE the GPU path runs); the GPU path always runs the whole workload."""
    # the oracle runs first, on host copies taken before the GPU path touches the pools
    ref_w = w if seqs is None else W.restrict(w, seqs, device="cpu")
    assert mods is None or seqs is None
    k_ref, v_ref, o_ref, lse_ref = oracle_step(oracle, ref_w, mods=mods)
    out, lse = gpu_step(pa, w, prefill=prefill, mods=mods, step_call=step_call)
    after = w if seqs is None else W.restrict(w, seqs, device="cpu")
    assert np.array_equal(_bits(W.to_numpy(after.k_cache)), _bits(k_ref)), f"{what}: K pool differs after append"
    assert np.array_equal(_bits(W.to_numpy(after.v_cache)), _bits(v_ref)), f"{what}: V pool differs after append"
    got, got_lse = to_f64(out), to_f64(lse)
    if seqs is not None:
        cu = W.to_numpy(w.cu_q_lens)
        rows = np.concatenate([np.arange(cu[s], cu[s + 1]) for s in seqs])
        got, got_lse = got[rows], got_lse[rows]
    res = assert_close(got, o_ref, w.dtype, what + " out", tol=tol)
    empty = ~np.isfinite(lse_ref)
    assert (got_lse[empty] == -np.inf).all(), f"{what}: lse of empty rows must be -inf"
    if (~empty).any():
        lse_tol = 1e-4 if w.dtype == torch.float32 else 1e-3
        assert np.abs(got_lse[~empty] - lse_ref[~empty]).max() <= lse_tol, f"{what}: lse"
    return res


def check_step_in_groups(pa, oracle, w: W.PagedWorkload, what="", group=4, tol=None, step_call=False):
    """check_step over EVERY sequence of a workload whose pools are too large to copy to the host in one piece: the
    oracle sees the sequences group by group (host copies of their pages, taken BEFORE the GPU path runs), the GPU
    path runs the whole workload once, and the two measures are taken over the whole output tensor."""
    refs = []
    for g in range(0, w.batch, group):
        seqs = list(range(g, min(w.batch, g + group)))
        refs.append((seqs,) + oracle_step(oracle, W.restrict(w, seqs, device="cpu")))
    out, lse = gpu_step(pa, w, step_call=step_call)
    for seqs, k_ref, v_ref, _, _ in refs:
        after = W.restrict(w, seqs, device="cpu")
        assert np.array_equal(_bits(W.to_numpy(after.k_cache)), _bits(k_ref)), f"{what}: K pool differs after append"
        assert np.array_equal(_bits(W.to_numpy(after.v_cache)), _bits(v_ref)), f"{what}: V pool differs after append"
    o_ref = np.concatenate([r[3] for r in refs])
    lse_ref = np.concatenate([r[4] for r in refs])
    got, got_lse = to_f64(out), to_f64(lse)
    assert got.shape == o_ref.shape
    res = assert_close(got, o_ref, w.dtype, what + " out", tol=tol)
    lse_tol = 1e-4 if w.dtype == torch.float32 else 1e-3
    assert np.abs(got_lse - lse_ref).max() <= lse_tol, f"{what}: lse"
    return res
