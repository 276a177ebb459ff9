"""ctypes binding of libpagedattn.so -- argument marshalling only.

Every function has the name and argument meaning of its C entry point in
``include/pagedattn.h``; torch tensors supply device pointers and the current
HIP stream, nothing else.  There is no CPU fallback: if the HIP library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "libpagedattn.so"
_lib = None

PA_DTYPE = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2}

EXPORTS = (
    "paged_kv_append", "paged_kv_gather", "paged_attention_workspace_bytes", "paged_attention_decode",
    "paged_attention_prefill", "paged_attention_decode_mod", "paged_attention_prefill_mod", "paged_decode_step",
    "paged_attention_decode_static", "pa_debug_check",
    "pa_status_string", "pa_set_option", "pa_stream_read", "pa_profile_enable", "pa_profile_reset",
    "pa_profile_read",
    "pa_pool_create", "pa_pool_destroy", "pa_pool_set_growth", "pa_pool_reserve", "pa_pool_release", "pa_pool_share_prefix",
    "pa_pool_make_writable", "pa_pool_num_free", "pa_pool_num_blocks", "pa_pool_get_row", "pa_pool_refcount",
)


class PagedAttnError(RuntimeError):
    pass


class _Desc(ctypes.Structure):
    _fields_ = [("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
                ("page_stride", ctypes.c_int64), ("token_stride", ctypes.c_int64),
                ("head_stride", ctypes.c_int64),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32)]


def library_path() -> str:
    return os.path.join(_HERE, _LIB_NAME)


def load_library():
    """Load the HIP library built in-tree (``python -m paper_2506_07311_amd.build``)."""
    global _lib
    if _lib is None:
        path = library_path()
        if not os.path.exists(path):
            raise PagedAttnError(
                f"{path} is missing: build the HIP library first (python -m paper_2506_07311_amd.build). "
                "There is no CPU fallback.")
        lib = ctypes.CDLL(path)
        lib.paged_attention_workspace_bytes.restype = ctypes.c_size_t
        lib.pa_status_string.restype = ctypes.c_char_p
        for name in EXPORTS:
            if name not in ("paged_attention_workspace_bytes", "pa_status_string"):
                getattr(lib, name).restype = ctypes.c_int
        _lib = lib
    return _lib


def _check(status: int, what: str):
    if status != 0:
        msg = load_library().pa_status_string(status).decode()
        raise PagedAttnError(f"{what}: {msg} (status {status})")


def _p(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _i32(t: torch.Tensor, what: str) -> torch.Tensor:
    if t.dtype != torch.int32 or not t.is_contiguous() or not t.is_cuda:
        raise PagedAttnError(f"{what} must be a contiguous int32 device tensor")
    return t


def cache_desc(k_cache: torch.Tensor, v_cache: torch.Tensor, head_major: bool = False) -> _Desc:
    """Descriptor of the pools.  Token-major ``[NP, P, Hkv, d]`` unless head_major (``[NP, Hkv, P, d]``).
    Either may be a strided view as long as head_dim is contiguous and K and V share strides."""
    if k_cache.dtype not in PA_DTYPE or v_cache.dtype != k_cache.dtype:
        raise PagedAttnError(f"unsupported cache dtype {k_cache.dtype}")
    if k_cache.dim() != 4 or k_cache.shape != v_cache.shape or k_cache.stride() != v_cache.stride():
        raise PagedAttnError("k_cache and v_cache must be 4-d with equal shapes and strides")
    if not (k_cache.is_cuda and v_cache.is_cuda) or k_cache.stride(3) != 1:
        raise PagedAttnError("caches must be device tensors with a contiguous head_dim")
    if head_major:
        NP, Hkv, P, d = k_cache.shape
        sp, sh, st, _ = k_cache.stride()
    else:
        NP, P, Hkv, d = k_cache.shape
        sp, st, sh, _ = k_cache.stride()
    return _Desc(k_cache.data_ptr(), v_cache.data_ptr(), sp, st, sh, NP, P, Hkv, d, PA_DTYPE[k_cache.dtype])


def _dense(t: torch.Tensor, what: str, dtype) -> torch.Tensor:
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise PagedAttnError(f"{what} must be a contiguous device tensor of dtype {dtype}")
    return t


class PreparedCall:
    """One entry point with its arguments already marshalled (pointers, sizes and the stream as of preparation).
    Calling it repeats exactly that call: for steady-state loops over the same buffers, where checking and
    converting the arguments again would cost more host time than the step takes on the GPU.  The tensors are kept
    alive by the object; their contents may change between calls, their addresses and shapes may not."""

    __slots__ = ("_fn", "_args", "_keep", "_what", "result")

    def __init__(self, fn, args, keep, what, result=None):
        self._fn, self._args, self._keep, self._what, self.result = fn, args, keep, what, result

    def __call__(self):
        st = self._fn(*self._args)
        if st:
            _check(st, self._what)
        return self.result


def prepare_kv_append(k_cache, v_cache, k_new, v_new, seq_ids, positions, block_table, *, head_major=False,
                      stream=None) -> PreparedCall:
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    T = int(seq_ids.shape[0])
    _dense(k_new, "k_new", k_cache.dtype), _dense(v_new, "v_new", k_cache.dtype)
    if tuple(k_new.shape) != (T, d.num_kv_heads, d.head_dim) or k_new.shape != v_new.shape:
        raise PagedAttnError("k_new/v_new must be [T, Hkv, d]")
    _i32(seq_ids, "seq_ids"), _i32(positions, "positions"), _i32(block_table, "block_table")
    args = (ctypes.byref(d), _p(k_new), _p(v_new), _p(seq_ids), _p(positions), ctypes.c_int32(T), _p(block_table),
            ctypes.c_int32(block_table.shape[0]), ctypes.c_int32(block_table.shape[1]), _stream(stream))
    return PreparedCall(lib.paged_kv_append, args, (d, k_cache, v_cache, k_new, v_new, seq_ids, positions, block_table),
                        "paged_kv_append")


def paged_kv_append(k_cache, v_cache, k_new, v_new, seq_ids, positions, block_table, *, head_major=False,
                    stream=None) -> None:
    prepare_kv_append(k_cache, v_cache, k_new, v_new, seq_ids, positions, block_table, head_major=head_major,
                      stream=stream)()


def paged_kv_gather(k_cache, v_cache, block_table, seq_lens, cu_seq_lens, total_tokens: int, max_seq_len: int, *,
                    head_major=False, stream=None) -> Tuple[torch.Tensor, torch.Tensor]:
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens"), _i32(cu_seq_lens, "cu_seq_lens")
    out_k = torch.empty((total_tokens, d.num_kv_heads, d.head_dim), dtype=k_cache.dtype, device=k_cache.device)
    out_v = torch.empty_like(out_k)
    st = lib.paged_kv_gather(ctypes.byref(d), _p(out_k), _p(out_v), _p(block_table), _p(seq_lens), _p(cu_seq_lens),
                             ctypes.c_int32(seq_lens.shape[0]), ctypes.c_int32(block_table.shape[1]),
                             ctypes.c_int32(max_seq_len), _stream(stream))
    _check(st, "paged_kv_gather")
    return out_k, out_v


def paged_attention_workspace_bytes(batch: int, num_q_heads: int, head_dim: int, total_q: int,
                                    max_seq_len: int) -> int:
    return int(load_library().paged_attention_workspace_bytes(
        ctypes.c_int32(batch), ctypes.c_int32(num_q_heads), ctypes.c_int32(head_dim), ctypes.c_int32(total_q),
        ctypes.c_int32(max_seq_len)))


def _workspace(workspace, nbytes, device):
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return workspace


def paged_attention_decode(k_cache, v_cache, q, block_table, seq_lens, max_seq_len: int, scale: float, *,
                           out=None, lse=None, workspace=None, head_major=False, stream=None):
    """Returns ``out`` ([B, Hq, d], dtype of q).  ``lse`` (float32 [B, Hq]) is filled when given."""
    return prepare_decode(k_cache, v_cache, q, block_table, seq_lens, max_seq_len, scale, out=out, lse=lse,
                          workspace=workspace, head_major=head_major, stream=stream)()


def prepare_decode(k_cache, v_cache, q, block_table, seq_lens, max_seq_len: int, scale: float, *,
                   out=None, lse=None, workspace=None, head_major=False, stream=None) -> PreparedCall:
    """paged_attention_decode with its arguments marshalled once; the call returns ``out``."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    B, Hq, hd = q.shape
    if hd != d.head_dim or seq_lens.shape[0] != B or block_table.shape[0] != B:
        raise PagedAttnError("q must be [B, Hq, d] with B matching seq_lens and block_table")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens")
    out = torch.empty_like(q) if out is None else _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    if workspace is None:   # (a workspace that is passed in is checked by the library itself)
        workspace = _workspace(None, paged_attention_workspace_bytes(B, Hq, hd, B, max_seq_len), q.device)
    args = (ctypes.byref(d), _p(q), _p(out), _p(lse), _p(block_table), _p(seq_lens), ctypes.c_int32(B),
            ctypes.c_int32(Hq), ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(max_seq_len),
            ctypes.c_float(scale), _p(workspace), ctypes.c_size_t(workspace.numel() * workspace.element_size()),
            _stream(stream))
    return PreparedCall(lib.paged_attention_decode, args,
                        (d, k_cache, v_cache, q, out, lse, block_table, seq_lens, workspace), "paged_attention_decode",
                        out)


def paged_attention_decode_static(k_cache, v_cache, q, block_table, seq_lens, max_seq_len: int, scale: float, *,
                                  out, lse=None, head_major=False, stream=None):
    """paged_attention_decode without a workspace: the split-KV partials go to the library's static scratch array.
    Nothing is allocated here either: ``out`` ([B, Hq, d], dtype of q) must be passed in and is returned."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    B, Hq, hd = q.shape
    if hd != d.head_dim or seq_lens.shape[0] != B or block_table.shape[0] != B:
        raise PagedAttnError("q must be [B, Hq, d] with B matching seq_lens and block_table")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens")
    _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    st = lib.paged_attention_decode_static(ctypes.byref(d), _p(q), _p(out), _p(lse), _p(block_table), _p(seq_lens),
                                           ctypes.c_int32(B), ctypes.c_int32(Hq), ctypes.c_int32(block_table.shape[1]),
                                           ctypes.c_int32(max_seq_len), ctypes.c_float(scale), _stream(stream))
    _check(st, "paged_attention_decode_static")
    return out


def paged_attention_prefill(k_cache, v_cache, q, cu_q_lens, max_q_len: int, block_table, seq_lens,
                            max_seq_len: int, scale: float, causal: bool, *, out=None, lse=None, workspace=None,
                            head_major=False, stream=None):
    """Returns ``out`` ([total_q, Hq, d], dtype of q).  ``lse`` (float32 [total_q, Hq]) is filled when given."""
    return prepare_prefill(k_cache, v_cache, q, cu_q_lens, max_q_len, block_table, seq_lens, max_seq_len, scale,
                           causal, out=out, lse=lse, workspace=workspace, head_major=head_major, stream=stream)()


def prepare_prefill(k_cache, v_cache, q, cu_q_lens, max_q_len: int, block_table, seq_lens, max_seq_len: int,
                    scale: float, causal: bool, *, out=None, lse=None, workspace=None, head_major=False,
                    stream=None) -> PreparedCall:
    """paged_attention_prefill with its arguments marshalled once; the call returns ``out``."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    total_q, Hq, hd = q.shape
    B = int(seq_lens.shape[0])
    if hd != d.head_dim or block_table.shape[0] != B or cu_q_lens.shape[0] != B + 1:
        raise PagedAttnError("q must be [total_q, Hq, d]; cu_q_lens int32[B+1]")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens"), _i32(cu_q_lens, "cu_q_lens")
    out = torch.empty_like(q) if out is None else _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    if workspace is None:
        workspace = _workspace(None, paged_attention_workspace_bytes(B, Hq, hd, total_q, max_seq_len), q.device)
    args = (ctypes.byref(d), _p(q), _p(out), _p(lse), _p(cu_q_lens), ctypes.c_int32(total_q),
            ctypes.c_int32(max_q_len), _p(block_table), _p(seq_lens), ctypes.c_int32(B), ctypes.c_int32(Hq),
            ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(max_seq_len), ctypes.c_float(scale),
            ctypes.c_int32(1 if causal else 0), _p(workspace),
            ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    return PreparedCall(lib.paged_attention_prefill, args,
                        (d, k_cache, v_cache, q, out, lse, cu_q_lens, block_table, seq_lens, workspace),
                        "paged_attention_prefill", out)


class _Mods(ctypes.Structure):
    _fields_ = [("window", ctypes.c_int32), ("softcap", ctypes.c_float), ("alibi_slopes", ctypes.c_void_p),
                ("doc_ids", ctypes.c_void_p), ("doc_stride", ctypes.c_int64), ("user_mod", ctypes.c_int32),
                ("user_data", ctypes.c_void_p)]


PA_MOD_PREFIX_LM = 1   # kId of pa_mod_prefix_lm in include/pagedattn_mods.h


def prefix_lm_data(prefix_len: torch.Tensor, prefix_bias: float = 0.0) -> torch.Tensor:
    """A pa_prefix_lm_data struct in device memory (pointer to int32[batch] prefix lengths, then the bias), to pass as
    ``user_data`` with ``user_mod=PA_MOD_PREFIX_LM``.  The caller keeps ``prefix_len`` alive while the struct is in use."""
    import struct
    _i32(prefix_len, "prefix_len")
    raw = struct.pack("<Qfi", prefix_len.data_ptr(), float(prefix_bias), 0)
    return torch.tensor(list(raw), dtype=torch.uint8).to(prefix_len.device)


def _mods(window, softcap, alibi_slopes, doc_ids, Hq, B, user_mod=0, user_data=None):
    if alibi_slopes is not None:
        _dense(alibi_slopes, "alibi_slopes", torch.float32)
        if tuple(alibi_slopes.shape) != (Hq,):
            raise PagedAttnError("alibi_slopes must be float32[Hq]")
    if doc_ids is not None:
        _i32(doc_ids, "doc_ids")
        if doc_ids.dim() != 2 or doc_ids.shape[0] != B:
            raise PagedAttnError("doc_ids must be int32[batch, doc_stride]")
    if user_mod and (user_data is None or not user_data.is_cuda):
        raise PagedAttnError("a user modification needs its user_data in device memory")
    return _Mods(int(window), float(softcap), None if alibi_slopes is None else alibi_slopes.data_ptr(),
                 None if doc_ids is None else doc_ids.data_ptr(), 0 if doc_ids is None else doc_ids.shape[1],
                 int(user_mod), None if user_data is None else user_data.data_ptr())


def paged_attention_decode_mod(k_cache, v_cache, q, block_table, seq_lens, max_seq_len: int, scale: float, *,
                               window: int = 0, softcap: float = 0.0, alibi_slopes=None, doc_ids=None,
                               user_mod: int = 0, user_data=None,
                               out=None, lse=None, workspace=None, head_major=False, stream=None):
    """paged_attention_decode with mask / score modifications (see pa_attn_mods in the header)."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    B, Hq, hd = q.shape
    if hd != d.head_dim or seq_lens.shape[0] != B or block_table.shape[0] != B:
        raise PagedAttnError("q must be [B, Hq, d] with B matching seq_lens and block_table")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens")
    out = torch.empty_like(q) if out is None else _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    mods = _mods(window, softcap, alibi_slopes, doc_ids, Hq, B, user_mod, user_data)
    workspace = _workspace(workspace, paged_attention_workspace_bytes(B, Hq, hd, B, max_seq_len), q.device)
    st = lib.paged_attention_decode_mod(ctypes.byref(d), _p(q), _p(out), _p(lse), _p(block_table), _p(seq_lens),
                                        ctypes.c_int32(B), ctypes.c_int32(Hq), ctypes.c_int32(block_table.shape[1]),
                                        ctypes.c_int32(max_seq_len), ctypes.c_float(scale), ctypes.byref(mods),
                                        _p(workspace),
                                        ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    _check(st, "paged_attention_decode_mod")
    return out


def prepare_decode_step(k_cache, v_cache, k_new, v_new, q, block_table, seq_lens, max_seq_len: int, scale: float, *,
                        window: int = 0, softcap: float = 0.0, alibi_slopes=None, doc_ids=None, user_mod: int = 0,
                        user_data=None, out=None, lse=None, workspace=None, head_major=False,
                        stream=None) -> PreparedCall:
    """paged_decode_step (append of one new token per sequence + decode, one call) with its arguments marshalled once;
    the call returns ``out``."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    B, Hq, hd = q.shape
    if hd != d.head_dim or seq_lens.shape[0] != B or block_table.shape[0] != B:
        raise PagedAttnError("q must be [B, Hq, d] with B matching seq_lens and block_table")
    _dense(k_new, "k_new", k_cache.dtype), _dense(v_new, "v_new", k_cache.dtype)
    if tuple(k_new.shape) != (B, d.num_kv_heads, hd) or tuple(v_new.shape) != (B, d.num_kv_heads, hd):
        raise PagedAttnError("k_new / v_new must be [B, Hkv, d]")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens")
    out = torch.empty_like(q) if out is None else _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    if workspace is None:
        workspace = _workspace(None, paged_attention_workspace_bytes(B, Hq, hd, B, max_seq_len), q.device)
    m = _mods(window, softcap, alibi_slopes, doc_ids, Hq, B, user_mod, user_data)
    args = (ctypes.byref(d), _p(k_new), _p(v_new), _p(q), _p(out), _p(lse), _p(block_table), _p(seq_lens),
            ctypes.c_int32(B), ctypes.c_int32(Hq), ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(max_seq_len),
            ctypes.c_float(scale), ctypes.byref(m), _p(workspace),
            ctypes.c_size_t(workspace.numel() * workspace.element_size()), _stream(stream))
    return PreparedCall(lib.paged_decode_step, args,
                        (d, m, k_cache, v_cache, k_new, v_new, q, out, lse, block_table, seq_lens, workspace,
                         alibi_slopes, doc_ids, user_data), "paged_decode_step", out)


def paged_decode_step(k_cache, v_cache, k_new, v_new, q, block_table, seq_lens, max_seq_len: int, scale: float,
                      **kw):
    """Appends token s of ``k_new`` / ``v_new`` ([B, Hkv, d]) at position seq_lens[s] - 1 and decodes, in one call.
    Returns ``out``; keyword arguments as for prepare_decode_step."""
    return prepare_decode_step(k_cache, v_cache, k_new, v_new, q, block_table, seq_lens, max_seq_len, scale, **kw)()


def paged_attention_prefill_mod(k_cache, v_cache, q, cu_q_lens, max_q_len: int, block_table, seq_lens,
                                max_seq_len: int, scale: float, causal: bool, *, window: int = 0,
                                softcap: float = 0.0, alibi_slopes=None, doc_ids=None, user_mod: int = 0,
                                user_data=None, out=None, lse=None, workspace=None, head_major=False, stream=None):
    """paged_attention_prefill with mask / score modifications (see pa_attn_mods in the header)."""
    lib = load_library()
    d = cache_desc(k_cache, v_cache, head_major)
    _dense(q, "q", k_cache.dtype)
    total_q, Hq, hd = q.shape
    B = int(seq_lens.shape[0])
    if hd != d.head_dim or block_table.shape[0] != B or cu_q_lens.shape[0] != B + 1:
        raise PagedAttnError("q must be [total_q, Hq, d]; cu_q_lens int32[B+1]")
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens"), _i32(cu_q_lens, "cu_q_lens")
    out = torch.empty_like(q) if out is None else _dense(out, "out", q.dtype)
    if lse is not None:
        _dense(lse, "lse", torch.float32)
    mods = _mods(window, softcap, alibi_slopes, doc_ids, Hq, B, user_mod, user_data)
    workspace = _workspace(workspace, paged_attention_workspace_bytes(B, Hq, hd, total_q, max_seq_len), q.device)
    st = lib.paged_attention_prefill_mod(ctypes.byref(d), _p(q), _p(out), _p(lse), _p(cu_q_lens),
                                         ctypes.c_int32(total_q), ctypes.c_int32(max_q_len), _p(block_table),
                                         _p(seq_lens), ctypes.c_int32(B), ctypes.c_int32(Hq),
                                         ctypes.c_int32(block_table.shape[1]), ctypes.c_int32(max_seq_len),
                                         ctypes.c_float(scale), ctypes.c_int32(1 if causal else 0),
                                         ctypes.byref(mods), _p(workspace),
                                         ctypes.c_size_t(workspace.numel() * workspace.element_size()),
                                         _stream(stream))
    _check(st, "paged_attention_prefill_mod")
    return out


def pa_debug_check(k_cache, v_cache, block_table, seq_lens, seq_ids=None, positions=None, *, head_major=False,
                   stream=None) -> Tuple[int, int, int]:
    """Counts of violated device-side preconditions: (page ids out of range, lengths out of range, appended tokens
    out of range).  Synchronises the stream."""
    d = cache_desc(k_cache, v_cache, head_major)
    _i32(block_table, "block_table"), _i32(seq_lens, "seq_lens")
    T = 0
    if seq_ids is not None:
        _i32(seq_ids, "seq_ids"), _i32(positions, "positions")
        T = int(seq_ids.shape[0])
    scratch = torch.empty(4, dtype=torch.int64, device=k_cache.device)
    counts = (ctypes.c_int64 * 3)()
    st = load_library().pa_debug_check(ctypes.byref(d), _p(block_table), _p(seq_lens),
                                       ctypes.c_int32(block_table.shape[0]), ctypes.c_int32(block_table.shape[1]),
                                       _p(seq_ids), _p(positions), ctypes.c_int32(T), _p(scratch), counts,
                                       _stream(stream))
    _check(st, "pa_debug_check")
    return int(counts[0]), int(counts[1]), int(counts[2])


def pa_set_option(name: str, value: int) -> None:
    _check(load_library().pa_set_option(name.encode(), ctypes.c_int64(value)), f"pa_set_option({name})")


def pa_stream_read(a: torch.Tensor, b: torch.Tensor, bytes_each: int, sink: torch.Tensor, *, stream=None) -> None:
    """Plain contiguous read of the first ``bytes_each`` bytes of two device tensors (bandwidth yardstick)."""
    if a.numel() * a.element_size() < bytes_each or b.numel() * b.element_size() < bytes_each:
        raise PagedAttnError("pa_stream_read: buffers shorter than bytes_each")
    _check(load_library().pa_stream_read(_p(a), _p(b), ctypes.c_size_t(bytes_each), _p(sink), _stream(stream)),
           "pa_stream_read")


def pa_profile_enable(on: bool) -> None:
    _check(load_library().pa_profile_enable(ctypes.c_int32(1 if on else 0)), "pa_profile_enable")


def pa_profile_reset() -> None:
    _check(load_library().pa_profile_reset(), "pa_profile_reset")


def pa_profile_read(kernel_prefix: str) -> Tuple[int, float]:
    n = ctypes.c_int32(0)
    ms = ctypes.c_double(0.0)
    _check(load_library().pa_profile_read(kernel_prefix.encode(), ctypes.byref(n), ctypes.byref(ms)),
           "pa_profile_read")
    return n.value, ms.value


# ---- KV page manager (host object; see the pa_pool_* block of include/pagedattn.h) ----------------------------

class PoolHandle(ctypes.c_void_p):
    """Opaque pa_pool*; remembers whether a device table is attached (then calls take the current stream)."""
    on_device = False


def pa_pool_create(num_pages: int, page_size: int, max_seqs: int, max_blocks: int,
                   device_table: Optional[torch.Tensor] = None) -> PoolHandle:
    """Returns the pool handle.  device_table: int32 [max_seqs, max_blocks] device tensor kept current by the pool,
    or None for a host-only pool (no GPU needed)."""
    if device_table is not None:
        _i32(device_table, "device_table")
        if tuple(device_table.shape) != (max_seqs, max_blocks):
            raise PagedAttnError("device_table must have shape [max_seqs, max_blocks]")
    handle = PoolHandle(0)
    handle.on_device = device_table is not None
    _check(load_library().pa_pool_create(ctypes.byref(handle), ctypes.c_int32(num_pages), ctypes.c_int32(page_size),
                                         ctypes.c_int32(max_seqs), ctypes.c_int32(max_blocks), _p(device_table)),
           "pa_pool_create")
    return handle


def pa_pool_destroy(pool) -> None:
    _check(load_library().pa_pool_destroy(pool), "pa_pool_destroy")


PA_GROW_EXACT, PA_GROW_POW2 = 0, 1


def pa_pool_set_growth(pool, policy: int) -> None:
    _check(load_library().pa_pool_set_growth(pool, ctypes.c_int32(policy)), "pa_pool_set_growth")


def _pool_stream(pool, stream) -> ctypes.c_void_p:
    return _stream(stream) if pool.on_device else ctypes.c_void_p(0)


def pa_pool_reserve(pool, seq: int, length: int, *, stream=None) -> None:
    _check(load_library().pa_pool_reserve(pool, ctypes.c_int32(seq), ctypes.c_int32(length),
                                          _pool_stream(pool, stream)), "pa_pool_reserve")


def pa_pool_release(pool, seq: int, *, stream=None) -> None:
    _check(load_library().pa_pool_release(pool, ctypes.c_int32(seq), _pool_stream(pool, stream)),
           "pa_pool_release")


def pa_pool_share_prefix(pool, dst_seq: int, src_seq: int, prefix_tokens: int, *, stream=None) -> None:
    _check(load_library().pa_pool_share_prefix(pool, ctypes.c_int32(dst_seq), ctypes.c_int32(src_seq),
                                               ctypes.c_int32(prefix_tokens), _pool_stream(pool, stream)),
           "pa_pool_share_prefix")


def pa_pool_make_writable(pool, k_cache, v_cache, seq: int, position: int, *, head_major=False, stream=None) -> None:
    desc = cache_desc(k_cache, v_cache, head_major)
    _check(load_library().pa_pool_make_writable(pool, ctypes.byref(desc), ctypes.c_int32(seq),
                                                ctypes.c_int32(position), _stream(stream)), "pa_pool_make_writable")


def pa_pool_num_free(pool) -> int:
    return load_library().pa_pool_num_free(pool)


def pa_pool_num_blocks(pool, seq: int) -> int:
    return load_library().pa_pool_num_blocks(pool, ctypes.c_int32(seq))


def pa_pool_get_row(pool, seq: int):
    """The sequence's mapped pages, in block order, as a list of ints."""
    n = pa_pool_num_blocks(pool, seq)
    if n < 0:
        raise PagedAttnError("pa_pool_get_row: invalid sequence")
    row = (ctypes.c_int32 * max(n, 1))()
    _check(load_library().pa_pool_get_row(pool, ctypes.c_int32(seq), row, ctypes.c_int32(n)), "pa_pool_get_row")
    return list(row[:n])


def pa_pool_refcount(pool, page: int) -> int:
    return load_library().pa_pool_refcount(pool, ctypes.c_int32(page))
