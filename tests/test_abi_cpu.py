"""Host-only checks of the C ABI: the library loads, exports every symbol the
header declares, sizes workspaces and rejects bad arguments before any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def T():
    import paper_2502_02770_amd as T
    if not os.path.exists(T.binding.LIB_PATH):
        from paper_2502_02770_amd.build import build
        build(verbose=False)
    return T


def test_exports_every_declared_symbol(T):
    hdr = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include")))
                  if f.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(twilight_[a-z0-9_]+)\s*\(", hdr))
    assert {"twilight_kquant_append", "twilight_select_pages", "twilight_topp_prune",
            "twilight_sparse_decode"} <= names
    L = T.binding.lib()
    for n in names:
        assert hasattr(L, n), n
    assert L.twilight_abi_version() == 1
    assert L.twilight_strerror(0) == b"ok" and b"workspace" in L.twilight_strerror(-2)
    assert L.twilight_kernel_name(3) == b"int4_score"


def test_workspace_sizes(T):
    kv = T.make_kv(8, 32, 8, 2048, 16384, None, None)
    assert T.twilight_workspace_bytes(0, kv, 256, 0) == 8 * 32 * 2048 * 4
    assert T.twilight_workspace_bytes(1, kv, 256, 0) >= 8 * 32 * 256 * 16 * 4 + 8 * 32 * 4
    assert T.twilight_workspace_bytes(1, kv, 0, 0) >= 8 * 32 * 2048 * 16 * 4
    sparse = T.twilight_workspace_bytes(2, kv, 0, 16384)
    assert sparse >= 64 * (16384 // 64) * 4 * 130 * 4
    assert T.twilight_workspace_bytes(2, kv, 0, 0) > 0
    # one list per query head instead of one per KV head: same partials in total for the same stride
    per_head = T.twilight_workspace_bytes(3, kv, 0, 16384)
    assert per_head >= 8 * 32 * (16384 // 64) * 130 * 4 and T.twilight_workspace_bytes(3, kv, 0, 0) == 0
    bad = T.make_kv(8, 32, 5, 2048, 16384, None, None)           # 32 q heads over 5 kv heads
    assert T.twilight_workspace_bytes(0, bad, 256, 0) == 0


def test_bad_arguments_are_rejected_on_the_host(T):
    L = T.binding.lib()
    one = ctypes.c_void_p(4096)                                    # never dereferenced: checks fail first
    kv = T.make_kv(1, 32, 8, 16, 16, None, None)
    assert L.twilight_kquant_append(ctypes.byref(kv), one, None, one, one, one, 4, None) == -1   # NULL tables
    kv.page_table, kv.seq_lens = 4096, 4096
    kv.head_dim = 64
    assert L.twilight_select_pages(ctypes.byref(kv), one, one, one, one, 4, one, 1 << 20, None) == -1
    kv.head_dim = 128
    kv.kq_pool, kv.kq_meta, kv.page_minmax, kv.k_pool, kv.v_pool = 4096, 4096, 4096, 4096, 4096
    assert L.twilight_select_pages(ctypes.byref(kv), one, one, one, one, 4, one, 16, None) == -2  # workspace
    assert L.twilight_topp_prune(ctypes.byref(kv), one, one, one, 4, ctypes.c_float(1.5), one, None, 0, one, one,
                                 64, one, one, 1 << 20, None) == -1                                # p > 1
    assert L.twilight_topp_prune(ctypes.byref(kv), one, one, one, 4, ctypes.c_float(0.0), one, None, 0, one, one,
                                 64, one, one, 1 << 20, None) == -1                                # p = 0
    assert L.twilight_sparse_decode(ctypes.byref(kv), one, None, one, 64, one, None, one, 1 << 20, None) == -1
    assert L.twilight_sparse_decode(ctypes.byref(kv), one, one, one, 64, one, None, one, 8, None) == -2
    assert L.twilight_int4_score(ctypes.byref(kv), one, one, None, 4, one, None, None) == -1
    # append + select in one launch: needs the new rows and positions, the 4-bit copy, the select workspace
    assert L.twilight_append_select(ctypes.byref(kv), None, None, one, one, one, one, one, 4, one, 1 << 20, None) == -1
    assert L.twilight_append_select(ctypes.byref(kv), one, None, None, one, one, one, one, 4, one, 1 << 20, None) == -1
    assert L.twilight_append_select(ctypes.byref(kv), one, None, one, one, one, one, one, 4, one, 16, None) == -2
    # selector + pruner in one call: budgets, list outputs, p in (0, 1], its own workspace size
    f09 = ctypes.c_float(0.9)
    sp = lambda budget, p, ws_bytes, sel=one: L.twilight_select_prune(ctypes.byref(kv), None, None, None, one, budget, p, sel, one, 4,
                                                                      one, None, 0, one, one, 64, one, one, ws_bytes, None)
    assert sp(None, f09, 1 << 20) == -1
    assert sp(one, f09, 1 << 20, None) == -1
    assert sp(one, ctypes.c_float(1.5), 1 << 20) == -1
    assert sp(one, f09, 16) == -2
    assert T.twilight_workspace_bytes(T.TW_WS_SELECT_PRUNE, kv, 4, 0) == (T.twilight_workspace_bytes(T.TW_WS_SELECT, kv, 4, 0)
                                                                          + T.twilight_workspace_bytes(T.TW_WS_PRUNE, kv, 4, 0))
    assert T.twilight_workspace_bytes(T.TW_WS_SELECT_PRUNE, kv, 0, 0) == 0
    # per-head variant: no dense mode, needs counts, checks its own workspace size
    assert L.twilight_sparse_decode_per_head(ctypes.byref(kv), one, one, None, 64, one, None, one, 1 << 20, None) == -1
    assert L.twilight_sparse_decode_per_head(ctypes.byref(kv), one, None, one, 64, one, None, one, 1 << 20, None) == -1
    assert L.twilight_sparse_decode_per_head(ctypes.byref(kv), one, one, one, 64, one, None, one, 8, None) == -2
    # code width of the quantised K copy: 0 (= 4), 2, 4, 8 only
    kv.quant_bits = 3
    assert L.twilight_select_pages(ctypes.byref(kv), one, one, one, one, 4, one, 1 << 20, None) == -1
    assert T.twilight_workspace_bytes(0, kv, 4, 0) == 0
    kv.quant_bits = 8
    assert T.twilight_workspace_bytes(0, kv, 4, 0) > 0
    kv.quant_bits = 4
    # documented size limits: batch * query heads <= 65535, at most 2^22 candidates per head
    big = T.make_kv(4096, 32, 8, 16, 16, None, None)
    big.page_table, big.seq_lens = 4096, 4096
    big.kq_pool, big.kq_meta, big.page_minmax, big.k_pool, big.v_pool = 4096, 4096, 4096, 4096, 4096
    assert L.twilight_select_pages(ctypes.byref(big), one, one, one, one, 4, one, 1 << 40, None) == -1
    long_row = T.make_kv(1, 8, 8, 1 << 20, 1 << 20, None, None)
    long_row.page_table, long_row.seq_lens = 4096, 4096
    long_row.kq_pool, long_row.kq_meta, long_row.page_minmax, long_row.k_pool, long_row.v_pool = 4096, 4096, 4096, 4096, 4096
    assert L.twilight_topp_prune(ctypes.byref(long_row), one, None, None, 0, ctypes.c_float(0.9), one, None, 0, one, one,
                                 64, one, one, 1 << 40, None) == -1                                # 2^24 candidates
    # token-list candidates: row length a multiple of 16 and at most 8192, sequences of at most 196608 tokens
    assert L.twilight_topp_prune_tokens(ctypes.byref(kv), one, one, one, 100, f09, one, None, 0, one, one, 64, one, one, 1 << 30, None) == -1
    assert L.twilight_topp_prune_tokens(ctypes.byref(kv), one, one, one, 8208, f09, one, None, 0, one, one, 64, one, one, 1 << 30, None) == -1
    assert L.twilight_topp_prune_tokens(ctypes.byref(kv), one, None, one, 64, f09, one, None, 0, one, one, 64, one, one, 1 << 30, None) == -1
    assert L.twilight_topp_prune_tokens(ctypes.byref(kv), one, one, one, 64, f09, one, None, 0, one, one, 64, one, one, 8, None) == -2
    assert L.twilight_int4_score_tokens(ctypes.byref(kv), one, one, one, 24, one, None, None) == -1
    assert L.twilight_int4_score_tokens(ctypes.byref(long_row), one, one, one, 64, one, None, None) == -1
    assert T.twilight_workspace_bytes(T.TW_WS_PRUNE_TOKENS, kv, 64, 0) >= 32 * 64 * 4
    assert T.twilight_workspace_bytes(T.TW_WS_PRUNE_TOKENS, kv, 100, 0) == 0
    # pinned-pointer query: NULL arguments
    out = ctypes.c_void_p()
    assert L.twilight_pinned_device_pointer(None, ctypes.byref(out)) == -1
    assert L.twilight_pinned_device_pointer(one, None) == -1
    with pytest.raises(T.TwilightError):
        T.binding._check(-3)


def test_bench_reports_the_named_metric():
    """bench.py's JSON line carries the metric of the benchmark spec, spelled the same way."""
    import json
    src = open(os.path.join(ROOT, "bench.py"), encoding="utf-8").read()
    metric = re.search(r'"metric": "([^"]+)"', src).group(1).encode().decode("unicode_escape")
    assert metric == json.load(open(os.path.join(ROOT, "BASELINE.json"), encoding="utf-8"))["metric"]


def test_shipped_library_reads_no_environment(T):
    """Tuning switches exist only in -DTW_TUNING builds: the library as built by build() does not import getenv."""
    import subprocess
    syms = subprocess.run(["nm", "-D", "--undefined-only", T.binding.LIB_PATH], capture_output=True, text=True, check=True).stdout
    assert "getenv" not in syms
