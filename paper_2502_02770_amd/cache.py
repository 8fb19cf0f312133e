"""Device buffers for one layer's paged KV cache and for one decode step.

Plumbing only: torch allocates the memory, every computation is a call into
libtwilight.so through `binding`.
"""
import torch

from . import binding as B


class PagedKV:
    """The pools of include/twilight.h's twilight_kv_t, owned as torch tensors."""

    def __init__(self, num_q_heads, num_kv_heads, page_table, seq_lens, num_pool_pages, device="cuda",
                 need_v=True, quant_bits=4, offload_kv=False):
        dev = torch.device(device)
        self.Hq, self.Hkv = int(num_q_heads), int(num_kv_heads)
        self.page_table = page_table.to(dev, torch.int32).contiguous()
        self.seq_lens = seq_lens.to(dev, torch.int32).contiguous()
        self.batch, self.max_pages = self.page_table.shape
        self.num_pool_pages = int(num_pool_pages)
        P, H = self.num_pool_pages, self.Hkv
        # offload_kv: the bf16 K/V pools live in pinned host memory and are read over the host link
        kv_args = dict(dtype=torch.bfloat16, pin_memory=True) if offload_kv else dict(dtype=torch.bfloat16, device=dev)
        self.device = dev
        self.k_pool = torch.zeros(P, H, 16, 128, **kv_args)
        self.v_pool = torch.zeros(P, H, 16, 128, **kv_args) if need_v else None
        self.quant_bits = int(quant_bits)
        self.kq_pool = torch.zeros(P, H, 16, 16 * self.quant_bits, dtype=torch.uint8, device=dev)
        self.kq_meta = torch.zeros(P, H, 16, 4, 2, dtype=torch.float16, device=dev)
        self.page_minmax = torch.zeros(P, H, 2, 128, dtype=torch.bfloat16, device=dev)
        self.kv = B.make_kv(self.batch, self.Hq, self.Hkv, self.max_pages, P, self.page_table, self.seq_lens,
                            self.k_pool, self.v_pool, self.kq_pool, self.kq_meta, self.page_minmax,
                            quant_bits=self.quant_bits)

    def append(self, k_new, v_new, start_pos, n_new, new_offsets, max_new):
        """twilight_kquant_append; does not advance seq_lens."""
        B.twilight_kquant_append(self.kv, k_new, v_new, start_pos, n_new, new_offsets, max_new)

    def fill(self, k, v, seq_offsets):
        """Build the whole cache from logical K/V [total, Hkv, 128] (sequences concatenated)."""
        dev = self.device
        start = torch.zeros(self.batch, dtype=torch.int32, device=dev)
        offs = torch.tensor(seq_offsets[:-1], dtype=torch.int32, device=dev)
        self.append(k, v, start, self.seq_lens, offs, int(self.seq_lens.max().item()))


class DecodeStep:
    """Pre-allocated outputs and workspaces of one decode step; runs
    select -> prune -> attend through the C ABI."""

    def __init__(self, cache, max_sel=None, union_stride=None, with_kept_idx=False, with_lse=True):
        c, dev = cache, cache.device
        self.cache = c
        self.full = max_sel is None
        self.max_sel = 0 if self.full else int(max_sel)
        cand = (c.max_pages if self.full else self.max_sel) * 16
        G = c.Hq // c.Hkv
        self.union_stride = int(union_stride) if union_stride else min(G * cand, c.max_pages * 16)
        i32 = dict(dtype=torch.int32, device=dev)
        if not self.full:
            self.sel_pages = torch.zeros(c.batch, c.Hq, self.max_sel, **i32)
            self.sel_count = torch.zeros(c.batch, c.Hq, **i32)
            # one allocation for the selector's and the pruner's workspaces, laid out as twilight_select_prune wants
            # them; the separate calls get its two parts
            nsel = B.twilight_workspace_bytes(B.TW_WS_SELECT, c.kv, self.max_sel)
            self._ws_select_prune = torch.empty(B.twilight_workspace_bytes(B.TW_WS_SELECT_PRUNE, c.kv, self.max_sel),
                                                dtype=torch.uint8, device=dev)
            self.ws_select = self._ws_select_prune[:nsel]
            self.ws_prune = self._ws_select_prune[nsel:]
        else:
            self.sel_pages = self.sel_count = None
        self.kept_count = torch.zeros(c.batch, c.Hq, **i32)
        self.kept_stride = cand if with_kept_idx else 0
        self.kept_idx = torch.zeros(c.batch, c.Hq, cand, **i32) if with_kept_idx else None
        self.union_count = torch.zeros(c.batch * c.Hkv, **i32)
        self.union_idx = torch.zeros(c.batch * c.Hkv, self.union_stride, **i32)
        self.status = torch.zeros(1, **i32)
        if self.full:
            self.ws_prune = torch.empty(B.twilight_workspace_bytes(B.TW_WS_PRUNE, c.kv, self.max_sel), dtype=torch.uint8, device=dev)
        self.ws_decode = torch.empty(B.twilight_workspace_bytes(B.TW_WS_DECODE, c.kv, 0, self.union_stride), dtype=torch.uint8, device=dev)
        self.out = torch.zeros(c.batch, c.Hq, 128, dtype=torch.bfloat16, device=dev)
        self.lse = torch.zeros(c.batch, c.Hq, dtype=torch.float32, device=dev) if with_lse else None
        self._ws_dense = None
        self._ws_per_head = None

    def select(self, q, budget):
        B.twilight_select_pages(self.cache.kv, q, budget, self.sel_pages, self.sel_count, self.max_sel, self.ws_select)

    def append_select(self, k_new, v_new, new_pos, q, budget):
        """One new token per sequence appended and the pages selected in one launch."""
        B.twilight_append_select(self.cache.kv, k_new, v_new, new_pos, q, budget, self.sel_pages, self.sel_count,
                                 self.max_sel, self.ws_select)

    def select_prune(self, k_new, v_new, new_pos, q, budget, p):
        """Selector (with the step's new token appended when k_new is given) and pruner in two launches."""
        B.twilight_select_prune(self.cache.kv, k_new, v_new, new_pos, q, budget, p, self.sel_pages, self.sel_count,
                                self.max_sel, self.kept_count, self.kept_idx, self.kept_stride, self.union_count,
                                self.union_idx, self.union_stride, self.status, self._ws_select_prune)

    def prune(self, q, p):
        B.twilight_topp_prune(self.cache.kv, q, self.sel_pages, self.sel_count, self.max_sel, p, self.kept_count,
                              self.kept_idx, self.kept_stride, self.union_count, self.union_idx,
                              self.union_stride, self.status, self.ws_prune)

    def attend(self, q):
        B.twilight_sparse_decode(self.cache.kv, q, self.union_count, self.union_idx, self.union_stride, self.out,
                                 self.lse, self.ws_decode)

    def attend_per_head(self, q):
        """Every query head over its own kept set (needs with_kept_idx=True) instead of the group's union."""
        assert self.kept_idx is not None, "DecodeStep(with_kept_idx=True) keeps the per-head lists"
        if self._ws_per_head is None:
            self._ws_per_head = torch.empty(
                B.twilight_workspace_bytes(B.TW_WS_DECODE_PER_HEAD, self.cache.kv, 0, self.kept_stride),
                dtype=torch.uint8, device=self.out.device)
        B.twilight_sparse_decode_per_head(self.cache.kv, q, self.kept_count, self.kept_idx, self.kept_stride,
                                          self.out, self.lse, self._ws_per_head)

    def run(self, q, budget, p, separate=False):
        """Selector, pruner, attention.  With a page selector the first two are one call (twilight_select_prune);
        separate=True takes twilight_select_pages and twilight_topp_prune instead (same results bit for bit)."""
        if self.full:
            self.prune(q, p)
        elif separate:
            self.select(q, budget)
            self.prune(q, p)
        else:
            self.select_prune(None, None, None, q, budget, p)
        self.attend(q)
        return self.out

    def dense(self, q, out=None, lse=None):
        """Dense decode attention over all tokens through the same kernel (baseline)."""
        c = self.cache
        if self._ws_dense is None:
            self._ws_dense = torch.empty(B.twilight_workspace_bytes(B.TW_WS_DECODE, c.kv, 0, 0), dtype=torch.uint8,
                                         device=c.device)
        out = self.out if out is None else out
        B.twilight_sparse_decode(c.kv, q, None, None, 0, out, lse, self._ws_dense)
        return out
