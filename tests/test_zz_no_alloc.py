"""twilight_select_pages_static - the selector for callers that cannot allocate - against
twilight_select_pages, through the C ABI: two calls in a row, the second on a smaller input
(the fixed scratch array then still holds the first call's bound scores)."""
import ctypes

import pytest
import torch

from workloads import synth


def _both_selectors(T, w, max_sel):
    from tests.gpu_util import build_cache
    dev = "cuda:0"
    cache = build_cache(w, dev)
    q, budget = w.q.to(dev), w.budget.to(dev)
    i32 = dict(dtype=torch.int32, device=dev)
    ref_pages = torch.full((w.batch, w.num_q_heads, max_sel), -7, **i32)
    ref_count = torch.full((w.batch, w.num_q_heads), -7, **i32)
    ws = torch.empty(T.twilight_workspace_bytes(T.TW_WS_SELECT, cache.kv, max_sel), dtype=torch.uint8, device=dev)
    T.twilight_select_pages(cache.kv, q, budget, ref_pages, ref_count, max_sel, ws)
    got_pages = torch.full_like(ref_pages, -7)
    got_count = torch.full_like(ref_count, -7)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    T.twilight_select_pages_static(cache.kv, q, budget, got_pages, got_count, max_sel)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(got_count, ref_count)
    assert torch.equal(got_pages, ref_pages)            # page sets and the untouched tails: bit for bit
    assert int(ref_count.min()) > 0
    return cache


@pytest.mark.gpu
def test_static_selector_matches_twice_second_call_smaller():
    import paper_2502_02770_amd as T
    # 2 sequences x 6144 tokens (384 pages each, several workgroups and a ragged tail), then 1 x 1000 tokens
    big = synth.config(1, scale=3 / 16, seed=5, batch=2)
    _both_selectors(T, big, max_sel=int(-(-int(big.budget.max()) // 16)))
    small = synth.config(0, scale=1000 / 4096, seed=6)
    assert int(small.seq_lens.max()) < int(big.seq_lens.max())
    _both_selectors(T, small, max_sel=int(-(-int(small.budget.max()) // 16)))


def test_static_selector_rejects_sizes_beyond_its_scratch():
    import paper_2502_02770_amd as T
    L = T.binding.lib()
    one = ctypes.c_void_p(4096)                                    # never dereferenced: the size check fails first
    kv = T.make_kv(64, 32, 8, 4096, 1 << 16, None, None)           # 64 x 32 x 4096 x 4 B = 32 MiB of scores
    kv.page_table = kv.seq_lens = kv.page_minmax = 4096
    assert T.twilight_workspace_bytes(T.TW_WS_SELECT, kv, 512) > T.binding.TW_STATIC_SELECT_WS_BYTES
    assert L.twilight_select_pages_static(ctypes.byref(kv), one, one, one, one, 512, None) == -4
    assert b"scratch" in L.twilight_strerror(-4)
