"""The decode entry point that brings its own scratch (paged_attention_decode_static) against
paged_attention_decode: same kernels, same plan, so the outputs must be bit-identical -- on two calls in a row, the
second with a smaller input, so that what the first call left in the static array is seen to be harmless."""
import ctypes

import pytest
import torch

from paper_2506_07311_amd import binding, workloads as W

pytestmark = pytest.mark.gpu

DEV = "cuda:0"


def _pair(w):
    """out / lse of the workspace entry point and of the static-scratch entry point on one workload."""
    ws = torch.full((binding.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.batch,
                                                             w.max_seq_len),), 0xFF, dtype=torch.uint8, device=DEV)
    lse_a = torch.full((w.batch, w.num_q_heads), float("nan"), dtype=torch.float32, device=DEV)
    lse_b = lse_a.clone()
    out_a = binding.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len,
                                           w.scale, lse=lse_a, workspace=ws)
    out_b = torch.full_like(w.q, float("nan"))
    binding.paged_attention_decode_static(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len,
                                          w.scale, out=out_b, lse=lse_b)
    torch.cuda.synchronize()
    return out_a, lse_a, out_b, lse_b


def test_static_scratch_decode_equals_the_workspace_entry_point_twice_in_a_row():
    binding.load_library()
    # first call: long enough for the tile stream to cut sequences across workgroups (partials + merge)
    big = W.make_workload("t", seq_lens=[9000, 4097, 12000, 777], num_q_heads=32, num_kv_heads=8, head_dim=128,
                          page_size=16, dtype=torch.bfloat16, seed=301, device=DEV)
    # second call: fewer and shorter sequences, still on the tile stream (3000 tokens is beyond the one-launch route)
    small = W.make_workload("t", seq_lens=[3000, 2500], num_q_heads=32, num_kv_heads=8, head_dim=128,
                            page_size=16, dtype=torch.bfloat16, seed=302, device=DEV)
    for w in (big, small):
        out_a, lse_a, out_b, lse_b = _pair(w)
        assert torch.isfinite(out_b.float()).all()
        assert torch.equal(out_a.view(torch.int16), out_b.view(torch.int16))
        assert torch.equal(lse_a, lse_b)


def test_static_scratch_rejects_a_call_beyond_the_array():
    """A forced grid of 2048 workgroups x 64 heads x 128 columns needs 67 MB of partials: refused, nothing launched."""
    lib = binding.load_library()
    w = W.make_workload("t", seq_lens=[70000], num_q_heads=64, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=303, device=DEV, poison=False)
    out = torch.zeros_like(w.q)
    binding.pa_set_option("decode_workgroups", 2048)
    try:
        with pytest.raises(binding.PagedAttnError, match="static scratch"):
            binding.paged_attention_decode_static(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens,
                                                  w.max_seq_len, w.scale, out=out)
    finally:
        binding.pa_set_option("decode_workgroups", 0)
    torch.cuda.synchronize()
    assert not bool(out.any().item())
