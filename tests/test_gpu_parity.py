"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element, on the same
seeded inputs.  Append / gather are bit-exact; attention is within the tolerances in tests/parity.py."""
import numpy as np
import pytest
import torch

from paper_2506_07311_amd import workloads as W
from tests import parity

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def pa():
    import paper_2506_07311_amd as pa_mod
    pa_mod.load_library()
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return pa_mod


def bits(a):
    return a.view(np.uint32) if a.dtype == np.float32 else a


@pytest.fixture(params=["stream", "one_launch"])
def decode_route(request, pa):
    """The two decode kernels on the matrix cores, each forced in turn: the tile stream with its merge kernel, and the
    one-launch kernel for short contexts (which the library would pick by itself only while the step is small)."""
    from paper_2506_07311_amd import binding
    binding.pa_set_option("decode_short", -1 if request.param == "stream" else 1)
    yield request.param
    binding.pa_set_option("decode_short", 0)


# ----------------------------------------------------------------------------- append / gather (bit-exact)
@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("P,Hkv,d", [(16, 8, 128), (1, 2, 64), (64, 8, 128), (4, 3, 32), (128, 1, 256)])
def test_append_and_gather_bit_exact(pa, oracle, dtype, P, Hkv, d):
    lens = [1, 37, 2 * P + 3, 5 * P, 129]
    w = W.make_workload("t", seq_lens=lens, q_lens=lens, num_q_heads=Hkv, num_kv_heads=Hkv, head_dim=d,
                        page_size=P, dtype=dtype, seed=21, device=DEV, poison=False)
    # sentinel pool: bytes no append writes must survive
    w.k_cache.fill_(-7.25)
    w.v_cache.fill_(3.5)
    k_ref, v_ref = W.to_numpy(w.k_cache).copy(), W.to_numpy(w.v_cache).copy()
    bt = W.to_numpy(w.block_table)
    oracle.kv_append(k_ref, v_ref, W.to_numpy(w.k_new), W.to_numpy(w.v_new), W.to_numpy(w.seq_ids),
                     W.to_numpy(w.positions), bt)
    pa.paged_kv_append(w.k_cache, w.v_cache, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
    torch.cuda.synchronize()
    assert np.array_equal(bits(W.to_numpy(w.k_cache)), bits(k_ref))
    assert np.array_equal(bits(W.to_numpy(w.v_cache)), bits(v_ref))
    # gather of the (oracle-written) pool
    gk_ref, gv_ref = oracle.kv_gather(k_ref, v_ref, bt, lens)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=DEV)
    gk, gv = pa.paged_kv_gather(w.k_cache, w.v_cache, w.block_table, w.seq_lens, cu, sum(lens), max(lens))
    torch.cuda.synchronize()
    assert np.array_equal(bits(W.to_numpy(gk)), bits(gk_ref))
    assert np.array_equal(bits(W.to_numpy(gv)), bits(gv_ref))
    assert np.array_equal(bits(W.to_numpy(gk)), bits(W.to_numpy(w.k_new)))   # gather o append = identity


def test_append_nothing_and_gather_empty(pa):
    w = W.make_workload("t", seq_lens=[0, 0], q_lens=[0, 0], num_q_heads=2, num_kv_heads=2, head_dim=64,
                        page_size=16, dtype=torch.float32, seed=1, device=DEV, num_pages=4, poison=False)
    before = w.k_cache.clone()
    pa.paged_kv_append(w.k_cache, w.v_cache, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
    cu = torch.zeros(3, dtype=torch.int32, device=DEV)
    gk, gv = pa.paged_kv_gather(w.k_cache, w.v_cache, w.block_table, w.seq_lens, cu, 0, 0)
    torch.cuda.synchronize()
    assert torch.equal(before, w.k_cache) and gk.numel() == 0


@pytest.mark.parametrize("d", [128, 64, 256])
def test_head_major_pool_through_strides(pa, oracle, d):
    """A [NP, Hkv, P, d] pool described by strides holds the same logical cache."""
    w = W.make_workload("t", seq_lens=[50, 17], num_q_heads=8, num_kv_heads=4, head_dim=d, page_size=16,
                        dtype=torch.bfloat16, seed=22, device=DEV)
    _, _, o_ref, _ = parity.oracle_step(oracle, w)
    kh = w.k_cache.permute(0, 2, 1, 3).contiguous()
    vh = w.v_cache.permute(0, 2, 1, 3).contiguous()
    pa.paged_kv_append(kh, vh, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table, head_major=True)
    out = pa.paged_attention_decode(kh, vh, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale, head_major=True)
    torch.cuda.synchronize()
    parity.assert_close(parity.to_f64(out), o_ref, w.dtype, "head-major decode")


# ----------------------------------------------------------------------------- the five workloads, small
def test_config1_fp32_single_sequence_decode(pa, oracle):
    parity.check_step(pa, oracle, W.config(1, device=DEV), "config 1")


@pytest.mark.parametrize("L", [128, 256, 512, 1024, 2048])
@pytest.mark.parametrize("step_call", [False, True], ids=["pair_of_calls", "step_call"])
def test_config2_bf16_gqa_decode(pa, oracle, L, step_call):
    """As the benchmark runs it: the library's own choice of kernels, through the pair of calls and through the single
    step call."""
    parity.check_step(pa, oracle, W.config(2, device=DEV, context=L), f"config 2 L={L}", step_call=step_call)


@pytest.mark.parametrize("S", [256, 333])
def test_config3_bf16_causal_prefill_small(pa, oracle, S):
    parity.check_step(pa, oracle, W.config(3, device=DEV, context=S), f"config 3 S={S}")


def test_config4_mixed_lengths_shared_prefix_small(pa, oracle):
    w = W.config(4, device=DEV, shrink=16)
    bt = W.to_numpy(w.block_table)
    assert (bt[1, :2] == bt[0, :2]).all()      # prefix pages really are aliased
    parity.check_step(pa, oracle, w, "config 4 / 16")


@pytest.mark.parametrize("P", [16, 64])
def test_config5_long_context_small(pa, oracle, P):
    parity.check_step(pa, oracle, W.config(5, device=DEV, shrink=32, page_size=P), f"config 5 / 32 P={P}")


# ----------------------------------------------------------------------------- edge cases and shape sweep
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.bfloat16, 64), (torch.float32, 64),
                                     (torch.float32, 128), (torch.bfloat16, 256)])
@pytest.mark.parametrize("P", [1, 2, 8, 16, 32, 128])
def test_decode_ragged_lengths_and_page_sizes(pa, oracle, dtype, d, P, decode_route):
    lens = [0, 1, 2, 15, 16, 17, 31, 33, 255, 257, 700, 1500]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=P, dtype=dtype,
                        seed=23 + P, device=DEV)
    parity.check_step(pa, oracle, w, f"ragged decode P={P} d={d} {dtype}")


@pytest.mark.parametrize("Hq,Hkv", [(1, 1), (8, 8), (16, 8), (32, 8), (64, 8), (16, 1), (24, 8), (40, 2), (32, 1),
                                    (71, 1), (96, 2)])
def test_decode_group_sizes(pa, oracle, Hq, Hkv, decode_route):
    w = W.make_workload("t", seq_lens=[300, 77, 1025], num_q_heads=Hq, num_kv_heads=Hkv, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, seed=31, device=DEV)
    parity.check_step(pa, oracle, w, f"decode Hq={Hq} Hkv={Hkv}")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8), (16, 1), (24, 8), (64, 4), (12, 4)])
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 64), (torch.bfloat16, 256), (torch.float16, 64),
                                     (torch.float16, 256)])
@pytest.mark.parametrize("wgs", [0, 7])
def test_decode_head_dims_on_the_matrix_cores(pa, oracle, Hq, Hkv, dtype, d, wgs):
    """head_dim 64 (half of each value product unused) and 256 (two column passes, 16-key tiles): every
    waves-per-workgroup variant, odd and maximal group sizes, default and forced cuts of the tile stream."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[300, 77, 1025, 16, 15, 0, 2049], num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d,
                        page_size=16, dtype=dtype, seed=35, device=DEV)
    binding.pa_set_option("decode_workgroups", wgs)
    try:
        parity.check_step(pa, oracle, w, f"decode d={d} Hq={Hq} Hkv={Hkv} {dtype} wgs={wgs}")
    finally:
        binding.pa_set_option("decode_workgroups", 0)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8), (16, 1), (24, 8), (64, 4), (12, 4)])
@pytest.mark.parametrize("dtype,d,P", [(torch.bfloat16, 64, 16), (torch.bfloat16, 256, 16), (torch.float16, 64, 4),
                                       (torch.float16, 256, 64), (torch.bfloat16, 128, 1), (torch.float16, 128, 128)])
def test_decode_in_one_launch(pa, oracle, Hq, Hkv, dtype, d, P):
    """The one-launch decode kernel forced on every head_dim: contexts shorter than the waves of a workgroup (waves
    without tiles), ragged tails, and contexts of many tiles per wave."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[300, 77, 1025, 16, 15, 2049, 1, 5000, 33], num_q_heads=Hq, num_kv_heads=Hkv,
                        head_dim=d, page_size=P, dtype=dtype, seed=36, device=DEV)
    binding.pa_set_option("decode_short", 1)
    binding.pa_profile_reset()
    binding.pa_profile_enable(True)
    try:
        parity.check_step(pa, oracle, w, f"one-launch decode d={d} Hq={Hq} Hkv={Hkv} {dtype} P={P}")
        torch.cuda.synchronize()
        assert binding.pa_profile_read("paged_decode_short_kernel")[0] == 1
        assert binding.pa_profile_read("paged_attention_merge_kernel")[0] == 0
    finally:
        binding.pa_profile_enable(False)
        binding.pa_profile_reset()
        binding.pa_set_option("decode_short", 0)


@pytest.mark.parametrize("splits", [2, 3, 7, 16])
@pytest.mark.parametrize("Hq,Hkv,dtype,d,P", [(32, 8, torch.bfloat16, 128, 16), (40, 2, torch.bfloat16, 128, 4),
                                              (8, 8, torch.float16, 64, 16), (24, 8, torch.bfloat16, 256, 64)])
@pytest.mark.parametrize("case", [None, dict(window=300), dict(docs=True, alibi=True, softcap=3.0)],
                         ids=["plain", "window", "hooks"])
def test_one_launch_decode_with_several_workgroups_per_sequence(pa, oracle, splits, Hq, Hkv, dtype, d, P, case):
    """The one-launch kernel with its context cut over several workgroups that merge through the workspace inside
    the launch: sequences shorter than the number of workgroups (workgroups without tiles),
    ragged tails, hooks; as the pair of calls and as the step call (the last workgroup's last wave appends)."""
    from paper_2506_07311_amd import binding
    lens = [300, 77, 1025, 16, 15, 2049, 1, 3000, 33]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=P, dtype=dtype,
                        seed=136, device=DEV)
    mods = build_mods(case, Hq, lens) if case else None
    binding.pa_set_option("decode_short", 1)
    binding.pa_set_option("decode_short_splits", splits)
    binding.pa_profile_reset()
    binding.pa_profile_enable(True)
    try:
        for step_call in (False, True):
            parity.check_step(pa, oracle, w, f"split one-launch decode x{splits} d={d} {case} step={step_call}",
                              mods=mods, step_call=step_call)
        torch.cuda.synchronize()
        assert binding.pa_profile_read("paged_decode_short_kernel")[0] == 2
        assert binding.pa_profile_read("paged_attention_merge_kernel")[0] == 0
        assert binding.pa_profile_read("paged_decode_mfma_kernel")[0] == 0
    finally:
        binding.pa_profile_enable(False)
        binding.pa_profile_reset()
        binding.pa_set_option("decode_short_splits", 0)
        binding.pa_set_option("decode_short", 0)


def test_split_one_launch_decode_is_stable_over_many_calls(pa):
    """300 calls in a row on the same inputs, the workspace poisoned between them: every call must give the bits of
    the first (the workgroup that merges changes from call to call; the merge order and the counters' state may
    not)."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[2048] * 8, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=137, device=DEV, poison=False)
    ws = torch.empty(pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.batch, w.max_seq_len),
                     dtype=torch.uint8, device=DEV)
    out = torch.empty_like(w.q)
    lse = torch.empty((w.batch, w.num_q_heads), dtype=torch.float32, device=DEV)
    first = None
    for it in range(300):
        ws.fill_(0xFF if it % 2 else 0x7F)
        out.zero_()
        pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale,
                                  out=out, lse=lse, workspace=ws)
        if first is None:
            torch.cuda.synchronize()
            first = (out.clone(), lse.clone())
        else:
            assert torch.equal(out, first[0]) and torch.equal(lse, first[1]), f"call {it} differs from the first"


@pytest.mark.parametrize("d", [64, 128, 256])
def test_decode_entry_with_an_empty_sequence(pa, decode_route, d):
    """seq_lens[s] == 0 through the decode entry point itself: zeros and lse = -inf for that sequence; the other
    sequences keep their values (bit for bit in the one-launch kernel, whose split of a sequence does not depend on
    the others; the tile stream cuts elsewhere, so there only up to rounding)."""
    w = W.make_workload("t", seq_lens=[300, 77, 5, 900], num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=16,
                        dtype=torch.bfloat16, seed=38, device=DEV)
    out0, lse0 = parity.gpu_step(pa, w, append=True)
    w.seq_lens[1] = 0
    out1, lse1 = parity.gpu_step(pa, w, append=False)
    keep = [0, 2, 3]
    if decode_route == "one_launch":
        assert torch.equal(out1[keep], out0[keep]) and torch.equal(lse1[keep], lse0[keep])
    else:
        parity.assert_close(parity.to_f64(out1[keep]), parity.to_f64(out0[keep]), torch.bfloat16, "other sequences")
        assert torch.allclose(lse1[keep], lse0[keep], atol=1e-4, rtol=0)
    assert (out1[1] == 0).all() and (lse1[1] == float("-inf")).all()


STEP_SHAPES = [
    # lens, Hq, Hkv, d, P, dtype
    ([300, 77, 1025, 16, 15, 33, 1, 64, 32], 32, 8, 128, 16, torch.bfloat16),
    ([300, 77, 1, 513, 32], 8, 8, 64, 16, torch.float16),
    ([300, 77, 1, 513, 16], 24, 8, 256, 64, torch.bfloat16),
    ([300, 77, 1, 513, 17], 40, 2, 128, 4, torch.bfloat16),      # 20 heads per KV head: two grid slices; P < 16
    ([5000, 77, 2049], 32, 8, 128, 16, torch.bfloat16),           # left to itself this takes the tile stream
    ([300, 77, 31], 8, 8, 64, 16, torch.float32),                 # portable kernel: append inside it, one launch
    ([5000, 77, 1], 8, 2, 64, 16, torch.float32),                 # portable kernel with a context split and a merge
    ([300, 77, 1025, 2], 12, 4, 96, 8, torch.bfloat16),           # head_dim 96: portable kernel, 16-bit rows
]


@pytest.mark.parametrize("shape", STEP_SHAPES, ids=lambda c: f"Hq{c[1]}-Hkv{c[2]}-d{c[3]}-P{c[4]}-n{len(c[0])}")
@pytest.mark.parametrize("route", [0, 1, -1])
@pytest.mark.parametrize("case", [None, dict(window=100), dict(docs=True, alibi=True, softcap=3.0)],
                         ids=["plain", "window", "hooks"])
def test_decode_step_is_the_append_followed_by_decode(pa, oracle, shape, route, case):
    """paged_decode_step against the pair of calls it stands for: pools and outputs bit-identical, whichever kernels
    the step runs on (route 0: the library's choice; 1: append inside the one-launch kernel; -1: append kernel, then
    tile stream and merge), and the pair itself is checked against the oracle."""
    from paper_2506_07311_amd import binding
    lens, Hq, Hkv, d, P, dtype = shape
    w = W.make_workload("t", seq_lens=lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=P, dtype=dtype,
                        seed=39, device=DEV)
    assert w.k_new.shape[0] == len(lens)                      # one new token per sequence, in sequence order
    mods = build_mods(case, Hq, lens) if case else None
    k0, v0 = w.k_cache.clone(), w.v_cache.clone()
    binding.pa_set_option("decode_short", route)
    try:
        res = parity.check_step(pa, oracle, w, f"pair {shape} {case}", mods=mods)
        out_pair, lse_pair = parity.gpu_step(pa, w, append=False, mods=mods)
        k_pair, v_pair = w.k_cache.clone(), w.v_cache.clone()
        w.k_cache.copy_(k0)
        w.v_cache.copy_(v0)
        kw = {}
        if mods:
            kw = dict(window=mods.get("window", 0), softcap=mods.get("softcap", 0.0))
            if mods.get("alibi_slopes") is not None:
                kw["alibi_slopes"] = torch.tensor(np.asarray(mods["alibi_slopes"]), dtype=torch.float32, device=DEV)
            if mods.get("doc_ids") is not None:
                kw["doc_ids"] = torch.tensor(np.asarray(mods["doc_ids"]), dtype=torch.int32, device=DEV)
        lse = torch.full((w.batch, Hq), float("nan"), dtype=torch.float32, device=DEV)
        binding.pa_profile_reset()
        binding.pa_profile_enable(True)
        out = pa.paged_decode_step(w.k_cache, w.v_cache, w.k_new, w.v_new, w.q, w.block_table, w.seq_lens,
                                   w.max_seq_len, w.scale, lse=lse, **kw)
        torch.cuda.synchronize()
        launches = sum(binding.pa_profile_read(n)[0] for n in ("paged_", ))
        binding.pa_profile_enable(False)
        view = torch.int32 if dtype == torch.float32 else torch.int16
        assert torch.equal(w.k_cache.view(view), k_pair.view(view)) and torch.equal(w.v_cache.view(view), v_pair.view(view))
        assert torch.equal(out.view(view), out_pair.view(view)), "out differs from the pair of calls"
        assert torch.equal(lse, lse_pair)
        # the append runs inside the decode kernel on every route: at most a merge follows
        assert launches <= 2
        if route == 1 and d in (64, 128, 256) and dtype != torch.float32:
            assert launches == 1, "the step on the one-launch kernel is a single launch"
    finally:
        binding.pa_profile_enable(False)
        binding.pa_profile_reset()
        binding.pa_set_option("decode_short", 0)


@pytest.mark.parametrize("own_kernel", [0, 1])
def test_decode_step_on_the_tile_stream_with_and_without_an_append_kernel(pa, own_kernel):
    """The tile stream performs the step's append inside the decode kernel (the wave that holds a sequence's last
    tile) or, with option step_append_kernel, in a kernel of its own: same pools, same outputs, bit for bit, as
    the pair of calls; 20 heads per KV head (two grid slices) and ragged tails included."""
    from paper_2506_07311_amd import binding
    for lens, Hq, Hkv, d, P in [([5000, 77, 2049, 1, 4096], 32, 8, 128, 16), ([3000, 31, 1500], 40, 2, 128, 4),
                                ([2500, 640], 16, 4, 256, 64), ([2500, 640, 7], 8, 8, 64, 16)]:
        w = W.make_workload("t", seq_lens=lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=P,
                            dtype=torch.bfloat16, seed=41, device=DEV)
        k0, v0 = w.k_cache.clone(), w.v_cache.clone()
        binding.pa_set_option("decode_short", -1)                 # both sides on the tile stream
        try:
            out_pair, lse_pair = parity.gpu_step(pa, w)
        finally:
            binding.pa_set_option("decode_short", 0)
        k_pair, v_pair = w.k_cache.clone(), w.v_cache.clone()
        w.k_cache.copy_(k0)
        w.v_cache.copy_(v0)
        binding.pa_set_option("step_append_kernel", own_kernel)
        binding.pa_set_option("decode_short", -1)
        binding.pa_profile_reset()
        binding.pa_profile_enable(True)
        try:
            out, lse = parity.gpu_step(pa, w, step_call=True)
            n_append = binding.pa_profile_read("paged_kv_append_last_kernel")[0]
        finally:
            binding.pa_profile_enable(False)
            binding.pa_profile_reset()
            binding.pa_set_option("step_append_kernel", 0)
            binding.pa_set_option("decode_short", 0)
        assert n_append == own_kernel
        assert torch.equal(w.k_cache.view(torch.int16), k_pair.view(torch.int16))
        assert torch.equal(w.v_cache.view(torch.int16), v_pair.view(torch.int16))
        assert torch.equal(out.view(torch.int16), out_pair.view(torch.int16)) and torch.equal(lse, lse_pair)


def test_decode_step_with_an_empty_sequence(pa):
    """A sequence of length 0 receives no token and gives zeros; the pools keep every byte outside the other
    sequences' slots."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[300, 77, 5, 900], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=40, device=DEV)
    w.seq_lens[1] = 0
    k0, v0 = w.k_cache.clone(), w.v_cache.clone()
    results = []
    for route in (1, -1):
        w.k_cache.copy_(k0)
        w.v_cache.copy_(v0)
        binding.pa_set_option("decode_short", route)
        try:
            lse = torch.full((4, 8), float("nan"), dtype=torch.float32, device=DEV)
            out = pa.paged_decode_step(w.k_cache, w.v_cache, w.k_new, w.v_new, w.q, w.block_table, w.seq_lens,
                                       w.max_seq_len, w.scale, lse=lse)
            torch.cuda.synchronize()
        finally:
            binding.pa_set_option("decode_short", 0)
        assert (out[1] == 0).all() and (lse[1] == float("-inf")).all()
        results.append((w.k_cache.clone().view(torch.int16), w.v_cache.clone().view(torch.int16), out.clone(), lse))
    assert torch.equal(results[0][0], results[1][0]) and torch.equal(results[0][1], results[1][1])
    # the slot the untouched sequence would have used (its former last position) still holds its poison
    changed = (results[0][0] != k0.view(torch.int16)).flatten(1).any(dim=1).sum().item()
    assert changed <= 3, "only the three live sequences' pages may change"
    parity.assert_close(parity.to_f64(results[0][2]), parity.to_f64(results[1][2]), torch.bfloat16, "routes agree")


def test_decode_route_follows_the_size_of_the_step(pa):
    """Left to itself the library takes the one-launch kernel while every wave would walk a few tiles only, and the
    tile stream (with its merge) beyond that or when the caller fixes the stream's workgroups."""
    from paper_2506_07311_amd import binding

    def kernels_of(L, batch=8, wgs=0):
        w = W.make_workload("t", seq_lens=[L] * batch, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                            dtype=torch.bfloat16, seed=37, device=DEV, poison=False)
        binding.pa_set_option("decode_workgroups", wgs)
        binding.pa_profile_reset()
        binding.pa_profile_enable(True)
        try:
            parity.gpu_step(pa, w, append=False)
            torch.cuda.synchronize()
            return (binding.pa_profile_read("paged_decode_short_kernel")[0],
                    binding.pa_profile_read("paged_decode_mfma_kernel")[0],
                    binding.pa_profile_read("paged_attention_merge_kernel")[0])
        finally:
            binding.pa_profile_enable(False)
            binding.pa_profile_reset()
            binding.pa_set_option("decode_workgroups", 0)

    assert kernels_of(128) == (1, 0, 0)
    assert kernels_of(1024) == (1, 0, 0)
    assert kernels_of(4096) == (1, 0, 0)                    # 64 (sequence, KV head) pairs: four workgroups each
    assert kernels_of(4097) == (0, 1, 1)
    assert kernels_of(1024, wgs=16) == (0, 1, 1)
    assert kernels_of(1025, batch=32) == (0, 1, 1)          # 256 pairs fill the machine: no split, 1024 tokens at most
    assert kernels_of(512, batch=64) == (1, 0, 0)
    assert kernels_of(512, batch=65) == (0, 1, 1)


@pytest.mark.parametrize("wgs", [1, 3, 7, 64, 256, 1000])
def test_decode_split_schedules(pa, oracle, wgs):
    """Every cut of the batch's key-tile stream merges to the same answer (the LSE merge is exact): one
    workgroup takes everything, boundaries inside and between sequences, more workgroups than tiles."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[2049, 64, 0, 31, 1000, 4096, 1], num_q_heads=32, num_kv_heads=8,
                        head_dim=128, page_size=16, dtype=torch.bfloat16, seed=32, device=DEV)
    binding.pa_set_option("decode_workgroups", wgs)
    try:
        parity.check_step(pa, oracle, w, f"decode workgroups={wgs}")
    finally:
        binding.pa_set_option("decode_workgroups", 0)


@pytest.mark.parametrize("chunk", [32, 256, 4096])
def test_portable_decode_chunk_schedules(pa, oracle, chunk):
    """The portable kernel's fixed-size chunk split, forced on a shape the MFMA kernel would take."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[2049, 64, 0, 31, 1000], num_q_heads=8, num_kv_heads=2, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, seed=33, device=DEV)
    binding.pa_set_option("decode_chunk_tokens", chunk)
    binding.pa_set_option("force_generic", 1)
    try:
        parity.check_step(pa, oracle, w, f"portable decode chunk={chunk}")
    finally:
        binding.pa_set_option("decode_chunk_tokens", 0)
        binding.pa_set_option("force_generic", 0)


@pytest.mark.parametrize("dtype,d,Hq,Hkv", [(torch.float32, 72, 3, 3), (torch.float32, 256, 5, 1),
                                            (torch.bfloat16, 200, 6, 2), (torch.float16, 64, 7, 7)])
@pytest.mark.parametrize("mode", ["decode", "prefill"])
def test_chunk_merge_shapes(pa, oracle, dtype, d, Hq, Hkv, mode):
    """The merge of fixed-size context chunks (eight (row, head) pairs per workgroup, four columns per lane): pair
    counts that do not fill the last workgroup, head_dims that leave lanes idle or need two passes, every output type,
    rows without keys in some chunks."""
    from paper_2506_07311_amd import binding
    lens = [1000, 3, 0, 257, 700]
    q_lens = None if mode == "decode" else [5, 3, 0, 1, 130]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=d, page_size=16,
                        dtype=dtype, causal=(mode == "prefill"), seed=34, device=DEV)
    binding.pa_set_option("decode_chunk_tokens", 128)
    binding.pa_set_option("prefill_chunk_tokens", 128)
    binding.pa_set_option("force_generic", 1)
    try:
        parity.check_step(pa, oracle, w, f"chunk merge {mode} {dtype} d={d} {Hq}/{Hkv}")
    finally:
        binding.pa_set_option("decode_chunk_tokens", 0)
        binding.pa_set_option("prefill_chunk_tokens", 0)
        binding.pa_set_option("force_generic", 0)


def test_many_sequences_decode(pa, oracle):
    """More sequences than lanes in a wave: the tile-stream schedule scans the lengths in blocks of 64."""
    rng = np.random.default_rng(5)
    lens = [int(x) for x in rng.integers(0, 200, size=300)]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=8, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=34, device=DEV)
    parity.check_step(pa, oracle, w, "300 sequences")


@pytest.mark.parametrize("dtype,d,P", [(torch.bfloat16, 128, 16), (torch.float32, 64, 16), (torch.bfloat16, 128, 64),
                                       (torch.bfloat16, 64, 4), (torch.bfloat16, 128, 2)])
@pytest.mark.parametrize("causal", [True, False])
def test_prefill_ragged(pa, oracle, dtype, d, P, causal):
    """Ragged packed queries, including chunked prefill (fewer queries than keys) and empty sequences."""
    lens = [130, 64, 1, 0, 257, 40]
    q_lens = [130, 10, 1, 0, 129, 40]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=8, num_kv_heads=2, head_dim=d,
                        page_size=P, dtype=dtype, causal=causal, seed=41, device=DEV)
    parity.check_step(pa, oracle, w, f"ragged prefill {dtype} d={d} P={P} causal={causal}")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (32, 8), (64, 8), (16, 1), (24, 8), (40, 2), (32, 1)])
def test_prefill_group_sizes(pa, oracle, Hq, Hkv):
    """Row tiles pack the query heads of a KV head (group sizes 1..16, and 3, 20, 32 which are not packed)."""
    w = W.make_workload("t", seq_lens=[300, 77, 513, 40], q_lens=[300, 1, 130, 7], num_q_heads=Hq,
                        num_kv_heads=Hkv, head_dim=128, page_size=16, dtype=torch.bfloat16, causal=True, seed=45,
                        device=DEV)
    parity.check_step(pa, oracle, w, f"prefill Hq={Hq} Hkv={Hkv}")


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8), (16, 1), (24, 8)])
@pytest.mark.parametrize("dtype,P", [(torch.bfloat16, 16), (torch.float16, 16), (torch.bfloat16, 4), (torch.bfloat16, 128)])
@pytest.mark.parametrize("causal,chunk", [(True, 0), (False, 0), (True, 256)])
def test_prefill_head_dim_64_on_the_matrix_cores(pa, oracle, Hq, Hkv, dtype, P, causal, chunk):
    """head_dim 64 runs the same kernel with half the steps of each product; few-query sequences of the batch take
    the decode kernel's head_dim 64 instantiation."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[300, 77, 513, 40, 0, 1300], q_lens=[300, 1, 130, 7, 0, 260], num_q_heads=Hq,
                        num_kv_heads=Hkv, head_dim=64, page_size=P, dtype=dtype, causal=causal, seed=47, device=DEV)
    binding.pa_set_option("prefill_chunk_tokens", chunk)
    try:
        parity.check_step(pa, oracle, w, f"prefill d=64 Hq={Hq} Hkv={Hkv} {dtype} P={P} causal={causal} chunk={chunk}")
    finally:
        binding.pa_set_option("prefill_chunk_tokens", 0)


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (32, 8), (16, 1), (24, 8)])
@pytest.mark.parametrize("dtype,P", [(torch.bfloat16, 16), (torch.float16, 64), (torch.bfloat16, 128), (torch.bfloat16, 4)])
@pytest.mark.parametrize("causal,chunk", [(True, 0), (False, 0), (True, 256)])
def test_prefill_head_dim_256_on_the_matrix_cores(pa, oracle, Hq, Hkv, dtype, P, causal, chunk):
    """head_dim 256: 512-byte LDS rows, 16 steps per score product, 8 column blocks of O, one workgroup per compute
    unit (page sizes below 16 take the portable kernel)."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[300, 77, 513, 40, 0, 1300], q_lens=[300, 1, 130, 7, 0, 260], num_q_heads=Hq,
                        num_kv_heads=Hkv, head_dim=256, page_size=P, dtype=dtype, causal=causal, seed=48, device=DEV)
    binding.pa_set_option("prefill_chunk_tokens", chunk)
    try:
        parity.check_step(pa, oracle, w, f"prefill d=256 Hq={Hq} Hkv={Hkv} {dtype} P={P} causal={causal} chunk={chunk}")
    finally:
        binding.pa_set_option("prefill_chunk_tokens", 0)


@pytest.mark.parametrize("chunk", [64, 256, 1024, 4096])
@pytest.mark.parametrize("P", [16, 128, 4])
def test_prefill_context_split_schedules(pa, oracle, chunk, P):
    """The matrix-core prefill kernel with its context cut into fixed chunks and merged, rows with and without
    keys in a chunk, chunks no row reaches, empty sequences."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[2049, 64, 0, 700, 4096, 1], q_lens=[5, 64, 0, 130, 1, 1], num_q_heads=8,
                        num_kv_heads=2, head_dim=128, page_size=P, dtype=torch.bfloat16, causal=True, seed=46,
                        device=DEV)
    binding.pa_set_option("prefill_chunk_tokens", chunk)
    try:
        parity.check_step(pa, oracle, w, f"prefill chunk={chunk} P={P}")
    finally:
        binding.pa_set_option("prefill_chunk_tokens", 0)


def test_prefill_chunk_of_a_long_prompt_is_split_by_default(pa, oracle):
    """Few query rows over a long context: the default plan cuts the context (no option set)."""
    w = W.make_workload("t", seq_lens=[20000], q_lens=[200], num_q_heads=32, num_kv_heads=8, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, causal=True, seed=47, device=DEV)
    parity.check_step(pa, oracle, w, "200 queries over 20000 keys")


def test_mixed_prefill_and_decode_rows_in_one_call(pa, oracle):
    """A jagged batch (Sec. III-B): decode rows over long contexts, a whole prompt, a chunk on top of cached
    context and an idle sequence in one call."""
    w = W.make_workload("t", seq_lens=[5000, 300, 1024, 77, 9000, 0, 2048], q_lens=[1, 300, 256, 1, 1, 0, 1],
                        num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16, dtype=torch.bfloat16, causal=True,
                        seed=48, device=DEV)
    parity.check_step(pa, oracle, w, "mixed prefill + decode")


@pytest.mark.parametrize("Hq,Hkv,q_small", [(32, 8, 4), (8, 8, 16), (16, 1, 1), (16, 8, 8), (24, 8, 5), (64, 8, 2)])
@pytest.mark.parametrize("causal", [True, False])
def test_few_query_sequences_take_the_decode_kernel(pa, oracle, Hq, Hkv, q_small, causal):
    """Sequences whose q_len * G rows fit 16 columns (decode rows, speculative tokens) are computed by the decode
    kernel inside a prefill call, each row with its own causal bound; longer ones by the prefill kernel.  Lengths
    straddle tile and segment boundaries so that some rows' bounds fall before a segment starts."""
    lens = [1000, 33, 64, 2048, 5, 300, 0, 4097, 96, 65]
    q_lens = [q_small, 1, q_small, 1, min(5, q_small), 300, 0, q_small, 40, q_small]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=Hq, num_kv_heads=Hkv, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, causal=causal, seed=50, device=DEV)
    parity.check_step(pa, oracle, w, f"few-query route Hq={Hq} Hkv={Hkv} q={q_small} causal={causal}")


@pytest.mark.parametrize("wgs", [1, 5, 64, 256])
def test_few_query_route_split_schedules(pa, oracle, wgs):
    from paper_2506_07311_amd import binding
    lens = [2049, 64, 0, 31, 1000, 4096, 1, 130]
    q_lens = [4, 3, 0, 2, 1, 4, 1, 130]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, causal=True, seed=51, device=DEV)
    binding.pa_set_option("decode_workgroups", wgs)
    try:
        parity.check_step(pa, oracle, w, f"few-query route on {wgs} workgroups")
    finally:
        binding.pa_set_option("decode_workgroups", 0)


def test_few_query_route_many_sequences_and_switch(pa, oracle):
    """More than 64 sequences, and the same call with the route switched off gives the same answer (two kernels)."""
    from paper_2506_07311_amd import binding
    rng = np.random.default_rng(9)
    lens = [int(x) for x in rng.integers(1, 400, size=150)]
    q_lens = [int(min(L, rng.choice([1, 1, 1, 2, 4, 60]))) for L in lens]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=16, num_kv_heads=4, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, causal=True, seed=52, device=DEV)
    parity.check_step(pa, oracle, w, "150 sequences, mixed")
    out_a, lse_a = parity.gpu_step(pa, w, append=False)
    binding.pa_set_option("no_small_q_route", 1)
    try:
        out_b, lse_b = parity.gpu_step(pa, w, append=False)
    finally:
        binding.pa_set_option("no_small_q_route", 0)
    parity.assert_close(parity.to_f64(out_a), parity.to_f64(out_b), w.dtype, "route on vs off")
    assert (lse_a - lse_b).abs().max().item() < 1e-3


@pytest.mark.parametrize("have", [0, 512, 1024, 3584])
def test_incremental_prefill_on_cached_context(pa, oracle, have):
    """Chat growth: 512 new tokens appended behind `have` cached ones and attended causally."""
    w = W.make_workload("t", seq_lens=[have + 512, have + 100], q_lens=[512, 100], num_q_heads=32, num_kv_heads=8,
                        head_dim=128, page_size=16, dtype=torch.bfloat16, causal=True, seed=49, device=DEV)
    parity.check_step(pa, oracle, w, f"chunk of 512 on {have} cached tokens")


def test_short_sequence_beside_long_ones(pa, oracle):
    """A 291-key sequence batched with several-thousand-key ones: the long sequences' small outputs pull the
    tensor-wide RMS (the floor of the max-rel measure) well below the short sequence's own scale, so the short
    sequence's rows must carry two-term weights although they see more than 256 keys."""
    w = W.make_workload("t", seq_lens=[2930, 4200, 291], q_lens=[436, 2100, 251], num_q_heads=16, num_kv_heads=4,
                        head_dim=128, page_size=64, dtype=torch.bfloat16, causal=True, seed=50, device=DEV)
    parity.check_step(pa, oracle, w, "short beside long")


@pytest.mark.parametrize("causal", [True, False])
def test_jagged_mixes_of_short_and_long_sequences(pa, oracle, causal):
    """Seeded jagged prefill batches whose sequences differ up to 40-fold in length, measured tensor-wide."""
    rng = np.random.default_rng(77)
    for it in range(6):
        B = int(rng.integers(2, 6))
        lens = [int(np.exp(rng.uniform(np.log(150), np.log(6000)))) for _ in range(B)]
        q_lens = [int(rng.integers(max(1, L // 8), L + 1)) for L in lens]
        w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=16, num_kv_heads=4, head_dim=128,
                            page_size=16, dtype=torch.bfloat16, causal=causal, seed=500 + it, device=DEV)
        a, r = parity.check_step(pa, oracle, w, f"jagged mix {it}: lens {lens} q_lens {q_lens}")
        print(f"jagged mix {it} causal={causal}: lens {lens} q_lens {q_lens} max-abs {a:.2e} max-rel {r:.2e}")


def test_prefill_row_equals_decode_at_that_length(pa):
    """Bottom-right causal alignment: row i of a causal prefill is the decode result at length i + 1."""
    S = 200
    w = W.make_workload("t", seq_lens=[S], q_lens=[S], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, causal=True, seed=42, device=DEV)
    out, _ = parity.gpu_step(pa, w)
    for i in [0, 15, 16, 100, S - 1]:
        lens = torch.tensor([i + 1], dtype=torch.int32, device=DEV)
        o = pa.paged_attention_decode(w.k_cache, w.v_cache, w.q[i:i + 1].contiguous(), w.block_table, lens, i + 1,
                                      w.scale)
        torch.cuda.synchronize()
        parity.assert_close(parity.to_f64(o[0]), parity.to_f64(out[i]), w.dtype, f"row {i}")


# ----------------------------------------------------------------------------- invariants on the GPU
def test_one_token_context_returns_v_exactly(pa):
    w = W.make_workload("t", seq_lens=[1] * 5, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=51, device=DEV)
    out, _ = parity.gpu_step(pa, w)
    v = w.v_new.repeat_interleave(4, dim=1)           # the single token's V per query head
    assert torch.equal(out, v)


def test_permuted_pages_equal_contiguous_layout_bitwise(pa, oracle):
    """Paging changes where bytes live, not what is computed: same logical cache, two physical layouts."""
    kw = dict(seq_lens=[513, 90, 2048], num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
              dtype=torch.bfloat16, device=DEV, poison=False)
    a = W.make_workload("perm", seed=52, **kw)
    out_a, _ = parity.gpu_step(pa, a)
    # re-house the same tokens contiguously: gather with the oracle, lay out in identity order
    k, v = W.to_numpy(a.k_cache), W.to_numpy(a.v_cache)
    gk, gv = oracle.kv_gather(k, v, W.to_numpy(a.block_table), a.seq_lens_host)
    b = W.make_workload("ident", seed=52, identity_pages=True, **kw)
    P = 16
    row = 0
    kb, vb = W.to_numpy(b.k_cache).copy(), W.to_numpy(b.v_cache).copy()
    btb = W.to_numpy(b.block_table)
    for s, L in enumerate(a.seq_lens_host):
        for blk in range((L + P - 1) // P):
            n = min(P, L - blk * P)
            kb[btb[s, blk], :n] = gk[row + blk * P: row + blk * P + n]
            vb[btb[s, blk], :n] = gv[row + blk * P: row + blk * P + n]
        row += L
    b.k_cache = torch.from_numpy(kb.view(np.int16)).view(torch.bfloat16).to(DEV)
    b.v_cache = torch.from_numpy(vb.view(np.int16)).view(torch.bfloat16).to(DEV)
    out_b = pa.paged_attention_decode(b.k_cache, b.v_cache, a.q, b.block_table, b.seq_lens, b.max_seq_len, a.scale)
    torch.cuda.synchronize()
    assert torch.equal(out_a, out_b)


def test_aliased_prefix_pages_equal_copied_pages_bitwise(pa):
    w = W.make_workload("t", seq_lens=[700, 300, 1100, 512], num_q_heads=32, num_kv_heads=8, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, seed=53, device=DEV, share_group=4,
                        share_prefix_tokens=256, pool_factor=3.0)
    out_alias, _ = parity.gpu_step(pa, w)
    # give every sequence private copies of the 16 shared prefix pages, in pages the pool left unused
    bt = W.to_numpy(w.block_table).copy()
    used = set(bt[bt >= 0].tolist())
    free = [p for p in range(w.num_pages) if p not in used]
    for s in range(1, 4):
        for b in range(16):
            dst = free.pop()
            w.k_cache[dst] = w.k_cache[int(bt[0, b])]
            w.v_cache[dst] = w.v_cache[int(bt[0, b])]
            bt[s, b] = dst
    out_copy = pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, torch.from_numpy(bt).to(DEV), w.seq_lens,
                                         w.max_seq_len, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(out_alias, out_copy)


# ----------------------------------------------------------------------------- full benchmark sizes
def test_config3_full_size_causal_prefill(pa, oracle):
    """All 4 x 2048 queries of the benchmark prefill, every row against the oracle."""
    parity.check_step(pa, oracle, W.config(3, device=DEV), "config 3 full")


def test_config4_full_size_mixed_decode(pa, oracle):
    """All 64 ragged sequences (lengths 64..32768, shared 1024-token prefixes), the launch bench.py times (one
    paged_decode_step call per step)."""
    parity.check_step(pa, oracle, W.config(4, device=DEV), "config 4 full", seqs=list(range(64)), step_call=True)


@pytest.mark.parametrize("P", [16, 64])
def test_config5_full_size_every_sequence(pa, oracle, P):
    """Batch 16 x 131072 context in the launch configuration bench.py times (P = 16: one paged_decode_step call
    per step, as the benchmark's default; P = 64: the pair of calls, its --step pair); all 16 sequences (all 64
    heads, full context) are recomputed by the oracle, four at a time."""
    w = W.config(5, device=DEV, page_size=P)
    a, r = parity.check_step_in_groups(pa, oracle, w, f"config 5 full P={P}", group=4, step_call=(P == 16))
    print(f"config 5 full P={P}: max-abs {a:.2e} max-rel {r:.2e}")
    del w
    torch.cuda.empty_cache()


@pytest.mark.parametrize("L", [128, 333, 2048])
@pytest.mark.parametrize("n", [9, 10], ids=["decode", "prefill"])
def test_paper_model_shape_full_size(pa, oracle, n, L):
    """The paper's own setting (Sec. IV): one LLaMA-7B layer -- 32 heads without grouping, head_dim 128, fp16 pools --
    with 64-token pages and a single sequence, at the ends of its 128 ... 2048-token prompt range (and one ragged
    length): a decode step at that context, and the prompt's causal prefill; every row against the oracle."""
    parity.check_step(pa, oracle, W.config(n, device=DEV, context=L), f"paper shape config {n} L={L}",
                      step_call=(n == 9))


# ----------------------------------------------------------------------------- HIP graph replay
@pytest.mark.parametrize("how", ["pair_of_calls", "step_call_one_launch", "step_call_tile_stream"])
def test_decode_step_replays_in_a_hip_graph(pa, oracle, how):
    """One step (append + decode + merge; or the single paged_decode_step call, as one launch or as append kernel +
    tile stream + merge) captured in a HIP graph: every replay, with eager work and synchronisations in between
    and fresh inputs written in place, must reproduce the eager result bitwise (the library records no memset
    node and allocates nothing, so the capture holds only its kernels)."""
    lens = [700, 64, 1000, 33] if how == "step_call_one_launch" else [700, 64, 2048, 33]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=32, num_kv_heads=8, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, seed=61, device=DEV)
    ws = torch.empty(pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.batch, w.max_seq_len),
                     dtype=torch.uint8, device=DEV)
    out = torch.empty_like(w.q)
    lse = torch.empty((w.batch, w.num_q_heads), dtype=torch.float32, device=DEV)

    def step():
        if how == "pair_of_calls":
            pa.paged_kv_append(w.k_cache, w.v_cache, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
            pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale,
                                      out=out, lse=lse, workspace=ws)
        else:
            pa.paged_decode_step(w.k_cache, w.v_cache, w.k_new, w.v_new, w.q, w.block_table, w.seq_lens,
                                 w.max_seq_len, w.scale, out=out, lse=lse, workspace=ws)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    gen = torch.Generator(device=DEV)
    gen.manual_seed(99)
    for it in range(4):
        # fresh inputs, written in place so the captured pointers stay valid
        w.q.copy_(torch.randn(w.q.shape, generator=gen, device=DEV).to(w.q.dtype))
        w.k_new.copy_(torch.randn(w.k_new.shape, generator=gen, device=DEV).to(w.q.dtype))
        w.v_new.copy_(torch.randn(w.v_new.shape, generator=gen, device=DEV).to(w.q.dtype))
        torch.cuda.synchronize()
        step()                                   # eager
        torch.cuda.synchronize()
        eager_out, eager_lse = out.clone(), lse.clone()
        out.zero_()
        lse.zero_()
        ws.fill_(0xFF)                           # the workspace need not survive between steps
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager_out), f"replay {it}: out differs from eager"
        assert torch.equal(lse, eager_lse), f"replay {it}: lse differs from eager"
    k_ref, v_ref, o_ref, _ = parity.oracle_step(oracle, w, append=False)   # pools already hold the last append
    parity.assert_close(parity.to_f64(out), o_ref, w.dtype, "graph replay vs oracle")


# ----------------------------------------------------------------------------- more shapes, paths and error handling
@pytest.mark.parametrize("scale", [4.0, 0.01, -0.2])
def test_extreme_and_negative_scales(pa, oracle, scale):
    """Large scales make the running max jump often (near one-hot softmax); a non-positive scale routes the
    prefill to the portable kernel.  Decode and prefill both.  At scale 4 the outputs are single V rows with
    |value| up to about 4.5, where the bf16 output format alone rounds by up to 2^-8 * 4.5 = 1.8e-2: the absolute
    bound is widened to that for this case only (the relative bound stays)."""
    tol = (2e-2, 2e-2) if scale == 4.0 else None
    w = W.make_workload("t", seq_lens=[300, 130, 64], q_lens=[300, 2, 64], num_q_heads=8, num_kv_heads=2,
                        head_dim=128, page_size=16, dtype=torch.bfloat16, causal=True, seed=71, device=DEV, scale=scale)
    parity.check_step(pa, oracle, w, f"prefill scale={scale}", tol=tol)
    w = W.make_workload("t", seq_lens=[300, 130, 2000], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=72, device=DEV, scale=scale)
    parity.check_step(pa, oracle, w, f"decode scale={scale}", tol=tol)


@pytest.mark.parametrize("d", [128, 64, 256])
def test_prefill_head_major_pool(pa, oracle, d):
    w = W.make_workload("t", seq_lens=[200, 77], q_lens=[200, 77], num_q_heads=8, num_kv_heads=4, head_dim=d,
                        page_size=16, dtype=torch.bfloat16, causal=True, seed=73, device=DEV)
    _, _, o_ref, _ = parity.oracle_step(oracle, w)
    kh = w.k_cache.permute(0, 2, 1, 3).contiguous()
    vh = w.v_cache.permute(0, 2, 1, 3).contiguous()
    pa.paged_kv_append(kh, vh, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table, head_major=True)
    out = pa.paged_attention_prefill(kh, vh, w.q, w.cu_q_lens, w.max_q_len, w.block_table, w.seq_lens, w.max_seq_len,
                                     w.scale, True, head_major=True)
    torch.cuda.synchronize()
    parity.assert_close(parity.to_f64(out), o_ref, w.dtype, "head-major prefill")


def test_mfma_kernels_agree_with_portable_kernels(pa):
    """Two independent GPU implementations of the same step (matrix-core kernels vs the portable VALU kernel)."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[513, 90, 1500], q_lens=[513, 1, 33], num_q_heads=16, num_kv_heads=4,
                        head_dim=128, page_size=16, dtype=torch.bfloat16, causal=True, seed=74, device=DEV)
    out_a, lse_a = parity.gpu_step(pa, w)
    binding.pa_set_option("force_generic", 1)
    try:
        out_b, lse_b = parity.gpu_step(pa, w)
    finally:
        binding.pa_set_option("force_generic", 0)
    parity.assert_close(parity.to_f64(out_a), parity.to_f64(out_b), w.dtype, "mfma vs portable")
    assert (lse_a - lse_b).abs().max().item() < 1e-3


def test_random_shapes_against_oracle(pa, oracle):
    """Seeded sweep over random batch / head / page / length combinations, decode and ragged prefill."""
    rng = np.random.default_rng(2025)
    for it in range(24):
        Hkv = int(rng.choice([1, 2, 3, 4, 8]))
        G = int(rng.choice([1, 2, 4, 5, 8, 16]))
        P = int(rng.choice([1, 4, 16, 32, 64]))
        d = int(rng.choice([128, 128, 64]))
        dtype = torch.bfloat16 if rng.random() < 0.8 else torch.float32
        B = int(rng.integers(1, 9))
        lens = [int(x) for x in rng.integers(0, 600, size=B)]
        prefill = rng.random() < 0.5
        if prefill:
            q_lens = [int(rng.integers(0, L + 1)) for L in lens]
            causal = bool(rng.random() < 0.7)
        else:
            q_lens, causal = None, False
        w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=Hkv * G, num_kv_heads=Hkv, head_dim=d,
                            page_size=P, dtype=dtype, causal=causal, seed=100 + it, device=DEV)
        if w.total_q == 0:
            continue
        parity.check_step(pa, oracle, w, f"random case {it}: B={B} Hkv={Hkv} G={G} P={P} d={d} {dtype} "
                                         f"prefill={prefill} causal={causal}", prefill=prefill)


def test_runtime_argument_errors(pa):
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[64, 64], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=75, device=DEV)
    small = torch.empty(256, dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.PagedAttnError, match="workspace"):
        pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, 64, w.scale, workspace=small)
    with pytest.raises(binding.PagedAttnError, match="invalid"):      # block table too short for max_seq_len
        pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, 10 ** 6, w.scale)
    with pytest.raises(binding.PagedAttnError):                        # q heads not a multiple of kv heads
        pa.paged_attention_decode(w.k_cache, w.v_cache, w.q[:, :7].contiguous(), w.block_table, w.seq_lens, 64, w.scale)
    torch.cuda.synchronize()


# ------------------------------------------------------------------------------------ fp16 pools
@pytest.mark.parametrize("d,P", [(128, 16), (128, 4), (64, 16), (256, 64)])
def test_fp16_append_gather_decode_and_prefill(pa, oracle, d, P):
    """fp16 pools (the paper's own precision): bit-exact data movement, attention on the matrix-core kernels
    (head_dim 128) and on the portable kernel (other head dims)."""
    lens = [300, 77, 1025, 0, 5]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=P,
                        dtype=torch.float16, seed=60, device=DEV)
    parity.check_step(pa, oracle, w, f"fp16 decode d={d} P={P}")
    w = W.make_workload("t", seq_lens=lens, q_lens=[300, 3, 130, 0, 5], num_q_heads=8, num_kv_heads=2, head_dim=d,
                        page_size=P, dtype=torch.float16, causal=True, seed=61, device=DEV)
    parity.check_step(pa, oracle, w, f"fp16 prefill d={d} P={P}")
    a = W.to_numpy(w.k_cache)
    ok, ov = oracle.kv_gather(a, W.to_numpy(w.v_cache), W.to_numpy(w.block_table), W.to_numpy(w.seq_lens))
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device=DEV)
    gk, gv = pa.paged_kv_gather(w.k_cache, w.v_cache, w.block_table, w.seq_lens, cu, sum(lens), max(lens))
    torch.cuda.synchronize()
    assert np.array_equal(W.to_numpy(gk).view(np.uint16), ok.view(np.uint16))
    assert np.array_equal(W.to_numpy(gv).view(np.uint16), ov.view(np.uint16))


def test_fp16_configs_small(pa, oracle):
    for n in (2, 3, 4, 5):
        w = W.config(n, device=DEV, shrink=16)
        for name in ("k_cache", "v_cache", "q", "k_new", "v_new"):
            setattr(w, name, getattr(w, name).to(torch.float16))
        w.dtype = torch.float16
        parity.check_step(pa, oracle, w, f"fp16 config {n} / 16")


def test_fp16_long_context_decode_sampled(pa, oracle):
    """Many small weights: 16 x 32768 tokens; two sequences against the oracle."""
    w = W.config(5, device=DEV, context=32768)
    for name in ("k_cache", "v_cache", "q", "k_new", "v_new"):
        setattr(w, name, getattr(w, name).to(torch.float16))
    w.dtype = torch.float16
    parity.check_step(pa, oracle, w, "fp16 16 x 32768", seqs=[3, 12])


# ------------------------------------------------------------------------------------ mask / score hooks
def alibi(Hq):
    return np.array([2.0 ** (-8.0 * (h + 1) / Hq) for h in range(Hq)])


def doc_ids(lens, seed, width=None):
    rng = np.random.default_rng(seed)
    width = width or max(lens) + 1
    ids = np.zeros((len(lens), width), dtype=np.int32)
    for s in range(len(lens)):
        cuts = np.sort(rng.integers(0, max(lens[s], 1), size=4))
        ids[s] = np.searchsorted(cuts, np.arange(width), side="right")
    return ids


MOD_CASES = [
    dict(window=100),
    dict(window=1),
    dict(window=33),
    dict(window=5000),
    dict(softcap=2.0),
    dict(alibi=True),
    dict(window=257, softcap=5.0, alibi=True),
    dict(docs=True),
    dict(docs=True, window=300, alibi=True, softcap=3.0),
]


def build_mods(case, Hq, lens):
    m = {}
    if "window" in case:
        m["window"] = case["window"]
    if "softcap" in case:
        m["softcap"] = case["softcap"]
    if case.get("alibi"):
        m["alibi_slopes"] = alibi(Hq)
    if case.get("docs"):
        m["doc_ids"] = doc_ids(lens, 7)
    return m


@pytest.mark.parametrize("case", MOD_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float16, 128), (torch.float32, 64),
                                     (torch.bfloat16, 64), (torch.float16, 256)])
def test_decode_with_mask_and_score_hooks(pa, oracle, case, dtype, d, decode_route):
    lens = [700, 64, 2049, 33, 1, 0, 300]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=16, dtype=dtype,
                        seed=70, device=DEV)
    parity.check_step(pa, oracle, w, f"decode hooks {case}", mods=build_mods(case, 8, lens))


@pytest.mark.parametrize("case", MOD_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_decode_hooks_with_a_group_larger_than_one_slice(pa, oracle, case, decode_route):
    """20 query heads per KV head: two grid slices of the decode kernel, the second with 4 live columns; the
    per-head slopes and the document ids must follow the slice's head offset."""
    lens = [700, 64, 1300, 33, 1]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=40, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=72, device=DEV)
    parity.check_step(pa, oracle, w, f"decode hooks G=20 {case}", mods=build_mods(case, 40, lens))


@pytest.mark.parametrize("case", MOD_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("d", [128, 64, 256])
def test_prefill_with_mask_and_score_hooks(pa, oracle, case, causal, d):
    lens = [400, 64, 700, 33, 0]
    q_lens = [400, 10, 130, 1, 0]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=16,
                        dtype=torch.bfloat16, causal=causal, seed=71, device=DEV)
    parity.check_step(pa, oracle, w, f"prefill hooks {case} causal={causal} d={d}", mods=build_mods(case, 8, lens))


@pytest.mark.parametrize("chunk,wgs", [(0, 0), (128, 5), (512, 64)])
@pytest.mark.parametrize("shuffled", [False, True])
@pytest.mark.parametrize("d", [128, 256])
def test_document_masks_with_context_splits_and_tile_skipping(pa, oracle, chunk, wgs, shuffled, d):
    """Document masks on the matrix-core kernels over many tiles: contiguous documents (waves skip the tiles of other
    documents) and ids in no order (nothing can be skipped, every tile is masked per key), with the context cut into
    chunks and the few-query sequences' stream cut between workgroups."""
    from paper_2506_07311_amd import binding
    lens = [1300, 700, 2049, 64, 300]
    q_lens = [1300, 3, 600, 1, 300]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=8, num_kv_heads=2, head_dim=d, page_size=16,
                        dtype=torch.bfloat16, causal=True, seed=74, device=DEV)
    ids = doc_ids(lens, 11)
    if shuffled:
        rng = np.random.default_rng(12)
        ids = rng.integers(0, 3, size=ids.shape).astype(np.int32)
    binding.pa_set_option("prefill_chunk_tokens", chunk)
    binding.pa_set_option("decode_workgroups", wgs)
    try:
        # rows that see one or two keys reach |out| >= 4, where a bf16 output rounds by 1.6e-2
        parity.check_step(pa, oracle, w, f"docs chunk={chunk} wgs={wgs} shuffled={shuffled} d={d}",
                          mods={"doc_ids": ids}, tol=(2e-2, 2e-2))
    finally:
        binding.pa_set_option("prefill_chunk_tokens", 0)
        binding.pa_set_option("decode_workgroups", 0)


@pytest.mark.parametrize("window", [64, 500, 1025])
@pytest.mark.parametrize("causal", [True, False])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_prefill_sliding_window_over_many_tiles(pa, oracle, window, causal, dtype):
    """The matrix-core prefill kernel with a window: workgroups start at their first row's window, waves skip the
    tiles before theirs, rows mask their own lower bound; with a soft cap and a position bias on top."""
    w = W.make_workload("t", seq_lens=[1500, 700, 130], q_lens=[1500, 300, 7], num_q_heads=8, num_kv_heads=2,
                        head_dim=128, page_size=16, dtype=dtype, causal=causal, seed=75, device=DEV)
    parity.check_step(pa, oracle, w, f"window {window} causal={causal} {dtype}", mods=dict(window=window))
    parity.check_step(pa, oracle, w, f"window {window} + cap + bias causal={causal} {dtype}",
                      mods=dict(window=window, softcap=4.0, alibi_slopes=alibi(8)))


@pytest.mark.parametrize("chunk", [256, 1024])
def test_prefill_window_with_context_split(pa, oracle, chunk):
    """Chunks that lie wholly before a row's window leave empty partials; the merge must ignore them."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[4096, 700], q_lens=[40, 130], num_q_heads=8, num_kv_heads=2, head_dim=128,
                        page_size=16, dtype=torch.bfloat16, causal=True, seed=76, device=DEV)
    binding.pa_set_option("prefill_chunk_tokens", chunk)
    try:
        parity.check_step(pa, oracle, w, f"window 600, chunk {chunk}", mods=dict(window=600))
        parity.check_step(pa, oracle, w, f"bias, chunk {chunk}", mods=dict(alibi_slopes=alibi(8)))
    finally:
        binding.pa_set_option("prefill_chunk_tokens", 0)


def test_prefill_window_without_causal_bound_and_context_split(pa, oracle):
    """Without a causal bound a window also ends a row's key range early: context chunks behind that end must
    leave empty partials (the merge counts chunks by the sequence length).  The workspace is filled with NaN first."""
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[2446, 651], q_lens=[2401, 123], num_q_heads=5, num_kv_heads=1, head_dim=128,
                        page_size=1, dtype=torch.bfloat16, causal=False, seed=77, device=DEV)
    k_ref, v_ref, o_ref, lse_ref = parity.oracle_step(oracle, w, mods=dict(window=64))
    pa.paged_kv_append(w.k_cache, w.v_cache, w.k_new, w.v_new, w.seq_ids, w.positions, w.block_table)
    for chunk in (0, 256):
        binding.pa_set_option("prefill_chunk_tokens", chunk)
        try:
            nbytes = pa.paged_attention_workspace_bytes(w.batch, w.num_q_heads, w.head_dim, w.total_q, w.max_seq_len)
            ws = torch.full((nbytes // 4,), float("nan"), dtype=torch.float32, device=DEV).view(torch.uint8)
            out = pa.paged_attention_prefill_mod(w.k_cache, w.v_cache, w.q, w.cu_q_lens, w.max_q_len, w.block_table,
                                                 w.seq_lens, w.max_seq_len, w.scale, False, window=64, workspace=ws)
            torch.cuda.synchronize()
        finally:
            binding.pa_set_option("prefill_chunk_tokens", 0)
        parity.assert_close(parity.to_f64(out), o_ref, w.dtype, f"non-causal window, chunk option {chunk}")


@pytest.mark.parametrize("wgs", [1, 7, 256])
def test_windowed_decode_split_schedules(pa, oracle, wgs):
    """The tile stream starts at the window: segments, merge and direct writes with a window in place."""
    from paper_2506_07311_amd import binding
    lens = [2049, 64, 0, 31, 1000, 4096, 1]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=32, num_kv_heads=8, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=72, device=DEV)
    binding.pa_set_option("decode_workgroups", wgs)
    try:
        parity.check_step(pa, oracle, w, f"window 700 on {wgs} workgroups",
                          mods=dict(window=700, alibi_slopes=alibi(32)))
    finally:
        binding.pa_set_option("decode_workgroups", 0)


# ----------------------------------------------------------------------------- user-defined modifications
@pytest.mark.parametrize("dtype,d,P", [(torch.bfloat16, 128, 16), (torch.float16, 64, 4), (torch.bfloat16, 256, 64),
                                       (torch.float32, 64, 16), (torch.bfloat16, 96, 16)])
@pytest.mark.parametrize("extra", [dict(), dict(window=700, softcap=3.0, alibi=True, docs=True)], ids=["alone", "with_built_ins"])
@pytest.mark.parametrize("bias", [0.0, 0.8])
def test_prefix_lm_user_modification_in_prefill(pa, oracle, dtype, d, P, extra, bias):
    """The prefix-LM pair of include/pagedattn_mods.h -- implemented only through the extension contract -- on every
    prefill kernel (matrix cores for head_dim 64 / 128 / 256, portable kernel for fp32 and head_dim 96): prefixes
    inside a sequence, empty, covering it, and past the queries' first position; ragged query counts."""
    lens = [700, 130, 1500, 64, 333]
    q_lens = [700, 100, 600, 64, 1]
    w = W.make_workload("t", seq_lens=lens, q_lens=q_lens, num_q_heads=16, num_kv_heads=4, head_dim=d, page_size=P,
                        dtype=dtype, causal=False, seed=180, device=DEV)
    mods = build_mods(extra, 16, lens) if extra else {}
    mods["prefix_lens"] = np.array([256, 0, 1200, 64, 100], dtype=np.int32)
    mods["prefix_bias"] = bias
    tol = (2e-2, 2e-2) if dtype == torch.bfloat16 else None   # rows concentrated on few keys: bf16 ulp at |out| >= 4
    parity.check_step(pa, oracle, w, f"prefix-LM prefill {dtype} d={d} {extra} bias={bias}", mods=mods, tol=tol)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float16, 64), (torch.bfloat16, 256), (torch.float32, 64)])
def test_prefix_lm_user_modification_in_decode(pa, oracle, dtype, d, decode_route):
    """The same pair through the decode entry points (tile stream, one launch with and without a split context,
    portable kernel) and the step call: every key is visible to the last position, the score hook still acts."""
    lens = [700, 130, 2500, 64, 333, 1]
    w = W.make_workload("t", seq_lens=lens, num_q_heads=16, num_kv_heads=4, head_dim=d, page_size=16, dtype=dtype,
                        seed=181, device=DEV)
    mods = dict(prefix_lens=np.array([256, 0, 1200, 64, 100, 1], dtype=np.int32), prefix_bias=-1.5)
    for step_call in (False, True):
        parity.check_step(pa, oracle, w, f"prefix-LM decode {dtype} d={d} step={step_call}", mods=mods,
                          step_call=step_call)


def test_unknown_user_modification_is_rejected(pa):
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[64, 64], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=182, device=DEV)
    data = torch.zeros(16, dtype=torch.uint8, device=DEV)
    with pytest.raises(binding.PagedAttnError, match="invalid argument"):
        pa.paged_attention_decode_mod(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale,
                                      user_mod=77, user_data=data)


def test_hooks_switched_off_equal_the_plain_entry_points(pa):
    w = W.make_workload("t", seq_lens=[700, 64, 300], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=73, device=DEV)
    a = pa.paged_attention_decode(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale)
    b = pa.paged_attention_decode_mod(w.k_cache, w.v_cache, w.q, w.block_table, w.seq_lens, w.max_seq_len, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_debug_check_counts_violated_preconditions(pa):
    from paper_2506_07311_amd import binding
    w = W.make_workload("t", seq_lens=[70, 33, 0, 16], num_q_heads=8, num_kv_heads=2, head_dim=128, page_size=16,
                        dtype=torch.bfloat16, seed=80, device=DEV)
    args = (w.k_cache, w.v_cache, w.block_table, w.seq_lens, w.seq_ids, w.positions)
    assert binding.pa_debug_check(*args) == (0, 0, 0)
    bt = w.block_table.clone()
    bt[0, 1] = w.num_pages              # dereferenced (70 tokens = 5 blocks): out of range
    bt[1, 2] = -7                       # dereferenced (33 tokens = 3 blocks)
    bt[3, 1] = 10 ** 6                  # NOT dereferenced (16 tokens = 1 block)
    assert binding.pa_debug_check(w.k_cache, w.v_cache, bt, w.seq_lens, w.seq_ids, w.positions) == (2, 0, 0)
    lens = w.seq_lens.clone()
    lens[2] = -1
    lens[3] = bt.shape[1] * 16 + 1
    assert binding.pa_debug_check(w.k_cache, w.v_cache, w.block_table, lens)[1] == 2
    pos = w.positions.clone()
    pos[0] = bt.shape[1] * 16
    ids = w.seq_ids.clone()
    ids[1] = 4
    assert binding.pa_debug_check(w.k_cache, w.v_cache, w.block_table, w.seq_lens, ids, pos) == (0, 0, 2)
