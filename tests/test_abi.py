"""CPU-side checks of the boundary: the library loads, exports every symbol the header declares, and
rejects host-checkable argument errors before touching the GPU (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2506_07311_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.library_path()):
        from paper_2506_07311_amd import build
        build.build()
    return binding.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pagedattn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(paged_\w+|pa_\w+)\s*\(", text)))


def test_header_declares_the_three_hot_path_calls():
    names = declared_functions()
    for n in ("paged_kv_append", "paged_attention_decode", "paged_attention_prefill", "paged_kv_gather",
              "paged_attention_workspace_bytes"):
        assert n in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_functions():
        assert hasattr(lib, name), f"{name} declared in pagedattn.h but not exported"
    assert set(binding.EXPORTS) == set(declared_functions())


def test_status_strings(lib):
    assert lib.pa_status_string(0) == b"ok"
    assert b"workspace" in lib.pa_status_string(3)


def _desc(**kw):
    d = dict(k_cache=0x1000, v_cache=0x2000, page_stride=16 * 8 * 128, token_stride=8 * 128, head_stride=128,
             num_pages=4, page_size=16, num_kv_heads=8, head_dim=128, dtype=1)
    d.update(kw)
    return binding._Desc(**d)


def test_prefill_workspace_covers_the_split_and_the_few_query_route(lib):
    """A call with few query rows over a long context is cut along the context: its workspace must hold the
    partials (total_q * Hq * nsplit * (d + 1) floats) on top of the few-query route's; a call with many rows is not
    cut and needs only the latter."""
    few = binding.paged_attention_workspace_bytes(1, 32, 128, 128, 131072)
    many = binding.paged_attention_workspace_bytes(4, 32, 128, 8192, 2048)
    route = binding.paged_attention_workspace_bytes(4, 32, 128, 8192, 64)
    assert many == route                                   # no split: same as a context too short to split
    assert few > binding.paged_attention_workspace_bytes(1, 32, 128, 128, 64) + 128 * 32 * 2 * 129 * 4


def test_workspace_bytes_is_positive_multiple_of_256(lib):
    for args in [(16, 64, 128, 16, 131072), (1, 8, 64, 1, 128), (4, 32, 128, 8192, 2048), (0, 8, 64, 0, 0)]:
        n = binding.paged_attention_workspace_bytes(*args)
        assert n > 0 and n % 256 == 0
    a = binding.paged_attention_workspace_bytes(16, 64, 128, 16, 131072)
    b = binding.paged_attention_workspace_bytes(16, 64, 128, 16, 1024)
    assert a >= b


def test_host_validation_rejects_before_launch(lib):
    null = ctypes.c_void_p(0)
    p = ctypes.c_void_p(0x4000)
    i32 = ctypes.c_int32
    # append: NULL descriptor, bad page size, T == 0 is a no-op
    assert lib.paged_kv_append(null, p, p, p, p, i32(1), p, i32(1), i32(1), null) == 1
    d = _desc(page_size=12)
    assert lib.paged_kv_append(ctypes.byref(d), p, p, p, p, i32(1), p, i32(1), i32(1), null) == 1
    d = _desc()
    assert lib.paged_kv_append(ctypes.byref(d), p, p, p, p, i32(0), p, i32(1), i32(1), null) == 0
    assert lib.paged_kv_append(ctypes.byref(d), null, p, p, p, i32(1), p, i32(1), i32(1), null) == 1
    d = _desc(head_dim=100)
    assert lib.paged_kv_append(ctypes.byref(d), p, p, p, p, i32(1), p, i32(1), i32(1), null) == 2
    d = _desc(dtype=7)
    assert lib.paged_kv_append(ctypes.byref(d), p, p, p, p, i32(1), p, i32(1), i32(1), null) == 2
    # decode: Hq not a multiple of Hkv, workspace too small, batch == 0 no-op, table too short
    d = _desc()
    f = ctypes.c_float(0.1)
    big = ctypes.c_size_t(1 << 40)
    ws = ctypes.c_void_p(0x10000)
    assert lib.paged_attention_decode(ctypes.byref(d), p, p, null, p, p, i32(2), i32(12), i32(4), i32(64), f, ws,
                                      big, null) == 1
    assert lib.paged_attention_decode(ctypes.byref(d), p, p, null, p, p, i32(2), i32(32), i32(4), i32(64), f, ws,
                                      ctypes.c_size_t(16), null) == 3
    assert lib.paged_attention_decode(ctypes.byref(d), p, p, null, p, p, i32(0), i32(32), i32(4), i32(64), f, ws,
                                      big, null) == 0
    assert lib.paged_attention_decode(ctypes.byref(d), p, p, null, p, p, i32(2), i32(32), i32(3), i32(64), f, ws,
                                      big, null) == 1
    # prefill: missing cu_q_lens
    assert lib.paged_attention_prefill(ctypes.byref(d), p, p, null, null, i32(8), i32(4), p, p, i32(2), i32(32),
                                       i32(4), i32(64), f, i32(1), ws, big, null) == 1
    # hooks: negative window, NaN cap, document ids narrower than the context
    m = binding._Mods(-1, 0.0, None, None, 0)
    assert lib.paged_attention_decode_mod(ctypes.byref(d), p, p, null, p, p, i32(2), i32(32), i32(4), i32(64), f,
                                          ctypes.byref(m), ws, big, null) == 1
    m = binding._Mods(0, float("nan"), None, None, 0)
    assert lib.paged_attention_decode_mod(ctypes.byref(d), p, p, null, p, p, i32(2), i32(32), i32(4), i32(64), f,
                                          ctypes.byref(m), ws, big, null) == 1
    m = binding._Mods(0, 0.0, None, 0x8000, 63)
    assert lib.paged_attention_prefill_mod(ctypes.byref(d), p, p, null, p, i32(8), i32(4), p, p, i32(2), i32(32),
                                           i32(4), i32(64), f, i32(1), ctypes.byref(m), ws, big, null) == 1
    # fp16 pools are accepted by the descriptor check (batch == 0: nothing is launched)
    d16 = _desc(dtype=2)
    assert lib.paged_attention_decode(ctypes.byref(d16), p, p, null, p, p, i32(0), i32(32), i32(4), i32(64), f, ws,
                                      big, null) == 0
    # step call: missing or misaligned new rows, the decode checks behind them, batch == 0 no-op
    step = lambda kn, vn, batch=2, hq=32, wsb=big, mods=null: lib.paged_decode_step(
        ctypes.byref(d), kn, vn, p, p, null, p, p, i32(batch), i32(hq), i32(4), i32(64), f, mods, ws, wsb, null)
    assert step(null, p) == 1 and step(p, null) == 1
    assert step(ctypes.c_void_p(0x4008), p) == 2
    assert step(p, p, hq=12) == 1
    assert step(p, p, wsb=ctypes.c_size_t(16)) == 3
    assert step(null, null, batch=0) == 0
    m = binding._Mods(-1, 0.0, None, None, 0)
    assert step(p, p, mods=ctypes.byref(m)) == 1
    # options
    for knob, bad in ((b"decode_short", 2), (b"decode_short", -2), (b"step_append_kernel", 2), (b"no_small_q_route", 3)):
        assert lib.pa_set_option(knob, ctypes.c_int64(bad)) == 1
    assert lib.pa_set_option(b"decode_short", ctypes.c_int64(-1)) == 0
    assert lib.pa_set_option(b"decode_short", ctypes.c_int64(0)) == 0
    assert lib.pa_set_option(b"no_such_knob", ctypes.c_int64(1)) == 1
    assert lib.pa_set_option(b"decode_chunk_tokens", ctypes.c_int64(0)) == 0


def test_options_are_kept_per_host_thread(lib):
    """A knob set on one thread shapes that thread's calls only: the workspace bound of another thread (and of the
    main thread) does not move when a worker forces a context split."""
    import threading
    args = (4, 32, 128, 8192, 2048)
    before = binding.paged_attention_workspace_bytes(*args)
    seen = {}

    def worker():
        assert lib.pa_set_option(b"prefill_chunk_tokens", ctypes.c_int64(256)) == 0
        seen["forced"] = binding.paged_attention_workspace_bytes(*args)

    t = threading.Thread(target=worker)
    t.start()
    t.join()
    assert seen["forced"] > before                       # the worker's bound grew with its forced split
    assert binding.paged_attention_workspace_bytes(*args) == before


def test_decode_workspace_bound_is_what_the_planner_can_use(lib):
    """The decode bound follows what the planners may choose -- the tile stream's largest grid (one workgroup per
    compute unit, 256 without a device: 9 MB of partials at 16 x 131072 with 64 heads) and the portable kernel's 64
    chunks per sequence (34 MB) -- not a fixed maximum of workgroups (it was 143 MB)."""
    n = binding.paged_attention_workspace_bytes(16, 64, 128, 16, 131072)
    assert 30_000_000 < n < 40_000_000


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_HERE", str(tmp_path))
    with pytest.raises(binding.PagedAttnError):
        binding.load_library()


def test_bench_refuses_more_than_one_gpu():
    """Every box of this build has one GPU: bench.py says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and not r.stdout.strip()


def test_product_sources_never_reach_for_the_oracle():
    """The oracle is test infrastructure: nothing under the package (binding, build, kernels) or include/ names it."""
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hits = []
    for top in ("paper_2506_07311_amd", "include"):
        for dirpath, _, files in os.walk(os.path.join(root, top)):
            if "_build" in dirpath or "__pycache__" in dirpath:
                continue
            for name in files:
                if not name.endswith((".py", ".h", ".hip", ".c", ".cpp")):
                    continue
                text = open(os.path.join(dirpath, name), errors="replace").read()
                if re.search(r"^\s*(import|from)\s+oracle\b|paged_oracle|libpaged_oracle", text, re.M):
                    hits.append(os.path.join(dirpath, name))
    assert not hits, hits
