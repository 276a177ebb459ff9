"""CPU oracle for attention over a paged KV cache -- TEST INFRASTRUCTURE ONLY.

Thin ctypes/numpy wrapper over ``paged_oracle.c`` (plain C, fp64): Algorithm 1's
Assign / Gather index translation and masked softmax attention by its direct
definition.  Only the tests, the smoke check and the benchmark's CPU-baseline
leg may import this package; the GPU library never does, and this package
imports nothing from it.

Arrays are numpy, on the host.  bf16 data travels as ``uint16`` bit patterns
(numpy has no bfloat16); fp32 as ``float32``; fp16 as ``float16``.  Caches are ``[NP, P, Hkv, d]``
arrays (token-major, Algorithm 1's flat slot p = page * P + o) unless
``head_major=True`` says ``[NP, Hkv, P, d]``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpaged_oracle.so")
_lib = None

F32, BF16, F16 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile paged_oracle.c with gcc into libpaged_oracle.so (in-tree)."""
    src = os.path.join(_HERE, "paged_oracle.c")
    hdr = os.path.join(_HERE, "paged_oracle.h")
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= max(os.path.getmtime(src), os.path.getmtime(hdr))):
        return _LIB_PATH
    # -O3 without -march=native: the built checker travels with the tree to a host with another CPU; ISO C mode keeps
    # floating-point contraction off, so the arithmetic is the source's whatever the optimisation level.
    cmd = ["gcc", "-O3", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", _LIB_PATH, src, "-lm"]
    subprocess.run(cmd, check=True, cwd=_HERE)
    return _LIB_PATH


class _Cache(ctypes.Structure):
    _fields_ = [("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("page_stride", ctypes.c_int64), ("token_stride", ctypes.c_int64),
                ("head_stride", ctypes.c_int64),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB_PATH)
        for name in ("oracle_kv_append", "oracle_kv_gather", "oracle_attention",
                     "oracle_merge_partials", "oracle_num_threads", "oracle_attention_mod", "oracle_widen"):
            getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.uint16:
        return BF16
    if a.dtype == np.float16:
        return F16
    raise TypeError(f"cache dtype must be float32, float16 or uint16 (bf16 bits), got {a.dtype}")


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data) if a is not None else ctypes.c_void_p(0)


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _desc(k_cache: np.ndarray, v_cache: np.ndarray, head_major: bool) -> _Cache:
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    assert k_cache.shape == v_cache.shape and k_cache.dtype == v_cache.dtype and k_cache.ndim == 4
    if head_major:
        NP, Hkv, P, d = k_cache.shape
        tok, head = d, P * d
    else:
        NP, P, Hkv, d = k_cache.shape
        tok, head = Hkv * d, d
    return _Cache(k_cache.ctypes.data, v_cache.ctypes.data, P * Hkv * d, tok, head,
                  NP, P, Hkv, d, _dtype_code(k_cache))


def _check(rc: int, what: str):
    if rc != 0:
        names = {-1: "bad argument", -2: "page id out of range", -3: "position beyond block table",
                 -4: "out of memory"}
        raise ValueError(f"{what}: {names.get(rc, rc)}")


def kv_append(k_cache, v_cache, k_new, v_new, seq_ids, positions, block_table, head_major=False):
    """Algorithm 1, Assign: scatter k_new/v_new ``[T, Hkv, d]`` into the pools IN PLACE."""
    lib = _load()
    c = _desc(k_cache, v_cache, head_major)
    k_new = np.ascontiguousarray(k_new)
    v_new = np.ascontiguousarray(v_new)
    assert k_new.dtype == k_cache.dtype and v_new.dtype == k_cache.dtype
    seq_ids, positions, bt = _i32(seq_ids), _i32(positions), _i32(block_table)
    T = int(seq_ids.shape[0])
    assert k_new.shape == (T, c.num_kv_heads, c.head_dim) and positions.shape == (T,)
    assert bt.ndim == 2
    rc = lib.oracle_kv_append(ctypes.byref(c), _ptr(k_new), _ptr(v_new), _ptr(seq_ids), _ptr(positions),
                              ctypes.c_int32(T), _ptr(bt), ctypes.c_int32(bt.shape[0]),
                              ctypes.c_int32(bt.shape[1]))
    _check(rc, "oracle_kv_append")


def kv_gather(k_cache, v_cache, block_table, seq_lens, head_major=False):
    """Algorithm 1, Gather: returns packed ``(K, V)`` of shape ``[sum(len), Hkv, d]``."""
    lib = _load()
    c = _desc(k_cache, v_cache, head_major)
    bt, lens = _i32(block_table), _i32(seq_lens)
    cu = np.zeros(lens.shape[0] + 1, dtype=np.int32)
    np.cumsum(lens, out=cu[1:])
    total = int(cu[-1])
    out_k = np.zeros((total, c.num_kv_heads, c.head_dim), dtype=k_cache.dtype)
    out_v = np.zeros_like(out_k)
    rc = lib.oracle_kv_gather(ctypes.byref(c), _ptr(out_k), _ptr(out_v), _ptr(bt), _ptr(lens), _ptr(cu),
                              ctypes.c_int32(lens.shape[0]), ctypes.c_int32(bt.shape[1]))
    _check(rc, "oracle_kv_gather")
    return out_k, out_v


class _Mods(ctypes.Structure):
    _fields_ = [("window", ctypes.c_int32), ("softcap", ctypes.c_double), ("alibi_slopes", ctypes.c_void_p),
                ("doc_ids", ctypes.c_void_p), ("doc_stride", ctypes.c_int64), ("prefix_lens", ctypes.c_void_p),
                ("prefix_bias", ctypes.c_double)]


def attention(k_cache, v_cache, q, block_table, seq_lens, scale, causal=False, cu_q_lens=None,
              head_major=False, return_weights=False, window=0, softcap=0.0, alibi_slopes=None, doc_ids=None,
              prefix_lens=None, prefix_bias=0.0):
    """Masked softmax attention over the paged cache by the direct definition, in fp64.

    q: ``[total_q, Hq, d]`` (same dtype as the cache).  ``cu_q_lens`` defaults to
    one query per sequence (decode).  Returns ``(out, lse)`` as float64 arrays
    ``[total_q, Hq, d]`` and ``[total_q, Hq]`` (+ weights ``[total_q, Hq, max_len]``).

    Modifications (FlexAttention's mask_mod / score_mod families): ``window`` > 0 keeps keys with
    |j - pos| < window; ``doc_ids`` int32 ``[batch, >= max len]`` keeps keys of the query's document;
    ``softcap`` > 0 replaces a score x by softcap * tanh(x / softcap); ``alibi_slopes`` ``[Hq]`` adds
    slope[h] * (j - pos); ``prefix_lens`` int32 ``[batch]`` is the prefix-LM family: keys j <= pos or
    j < prefix_lens[s] stay visible, and ``prefix_bias`` is added to the scores of the prefix keys.
    """
    lib = _load()
    c = _desc(k_cache, v_cache, head_major)
    q = np.ascontiguousarray(q)
    assert q.dtype == k_cache.dtype and q.ndim == 3 and q.shape[2] == c.head_dim
    bt, lens = _i32(block_table), _i32(seq_lens)
    B = int(lens.shape[0])
    if cu_q_lens is None:
        cu_q_lens = np.arange(B + 1, dtype=np.int32)
    cu = _i32(cu_q_lens)
    assert cu.shape == (B + 1,) and int(cu[-1]) == q.shape[0]
    total_q, Hq, d = q.shape
    out = np.zeros((total_q, Hq, d), dtype=np.float64)
    lse = np.zeros((total_q, Hq), dtype=np.float64)
    weights, wstride = None, 0
    if return_weights:
        wstride = int(lens.max()) if B else 0
        weights = np.zeros((total_q, Hq, max(wstride, 1)), dtype=np.float64)
        wstride = max(wstride, 1)
    slopes = None if alibi_slopes is None else np.ascontiguousarray(alibi_slopes, dtype=np.float64)
    docs = None if doc_ids is None else _i32(doc_ids)
    if slopes is not None:
        assert slopes.shape == (Hq,)
    if docs is not None:
        assert docs.ndim == 2 and docs.shape[0] == B and (B == 0 or docs.shape[1] >= int(lens.max()))
    prefix = None if prefix_lens is None else _i32(prefix_lens)
    if prefix is not None:
        assert prefix.shape == (B,)
    mods = _Mods(int(window), float(softcap), None if slopes is None else slopes.ctypes.data,
                 None if docs is None else docs.ctypes.data, 0 if docs is None else docs.shape[1],
                 None if prefix is None else prefix.ctypes.data, float(prefix_bias))
    rc = lib.oracle_attention_mod(ctypes.byref(c), _ptr(q), _ptr(out), _ptr(lse), _ptr(weights),
                                  ctypes.c_int64(wstride), _ptr(cu), _ptr(bt), _ptr(lens),
                                  ctypes.c_int32(B), ctypes.c_int32(Hq), ctypes.c_int32(bt.shape[1]),
                                  ctypes.c_double(float(scale)), ctypes.c_int32(1 if causal else 0),
                                  ctypes.byref(mods))
    _check(rc, "oracle_attention_mod")
    if return_weights:
        return out, lse, weights
    return out, lse


def merge_partials(o_parts, lse_parts):
    """Exact LSE merge of softmax partials over disjoint key sets.  o_parts ``[n, d]``, lse ``[n]``."""
    lib = _load()
    o_parts = np.ascontiguousarray(o_parts, dtype=np.float64)
    lse_parts = np.ascontiguousarray(lse_parts, dtype=np.float64)
    n, d = o_parts.shape
    out = np.zeros(d, dtype=np.float64)
    lse = ctypes.c_double(0.0)
    rc = lib.oracle_merge_partials(_ptr(o_parts), _ptr(lse_parts), ctypes.c_int32(n), ctypes.c_int32(d),
                                   _ptr(out), ctypes.byref(lse))
    _check(rc, "oracle_merge_partials")
    return out, lse.value


def widen(a: np.ndarray) -> np.ndarray:
    """The oracle's own exact widening of an input array (float32, float16, or uint16 bf16 bits) to float64."""
    a = np.ascontiguousarray(a)
    out = np.zeros(a.shape, dtype=np.float64)
    _check(_load().oracle_widen(_ptr(a), ctypes.c_int64(a.size), ctypes.c_int32(_dtype_code(a)), _ptr(out)),
           "oracle_widen")
    return out


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
