"""Test-side helpers: data movement between the oracle's logical layout and
the library's paged layout (documented in include/twilight.h).  No method
arithmetic here."""
import numpy as np
import torch

from oracle import twilight_oracle as O
from workloads import synth


def build_cache(w, device="cuda", upto=None, bits=4):
    """PagedKV filled through twilight_kquant_append from a workload."""
    import paper_2502_02770_amd as T
    cache = T.PagedKV(w.num_q_heads, w.num_kv_heads, w.page_table, w.seq_lens, w.num_pool_pages, device,
                      need_v=w.v.numel() > 0, quant_bits=bits)
    k = w.k.to(device)
    v = w.v.to(device) if w.v.numel() else None
    cache.fill(k, v, w.seq_offsets)
    torch.cuda.synchronize()
    return cache


def gather_logical(pool, page_table_row, n):
    """pool [pages, Hkv, 16, ...] (cpu tensor) -> logical [n, Hkv, ...] of one sequence."""
    P = (n + 15) // 16
    pages = page_table_row[:P].long()
    x = pool[pages]                       # [P, Hkv, 16, ...]
    x = x.transpose(1, 2)
    x = x.reshape(P * 16, *x.shape[2:])
    return x[:n]


def unpack_codes(kq, bits=4):
    """u8 [..., 16*bits] packed as documented with twilight_kv_t -> codes u8 [..., 128]."""
    lead = kq.shape[:-1]
    a = np.asarray(kq)
    if bits == 4:      # word w, byte k: dim 8w+k low nibble, 8w+k+4 high nibble
        a = a.reshape(*lead, 16, 4)
        return np.concatenate([a & 0x0F, a >> 4], axis=-1).reshape(*lead, 128)
    if bits == 8:      # byte = code, in dim order
        return a.reshape(*lead, 128)
    # 2 bits: word w, byte i, bit pair k: dim 16w + 4k + i
    a = a.reshape(*lead, 8, 1, 4)
    k = np.arange(4, dtype=np.uint8).reshape(4, 1)
    return ((a >> (2 * k)) & 3).reshape(*lead, 128)


def u16(t):
    """bf16 / fp16 cpu tensor -> uint16 numpy bits."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def oracle_seq(w, b, **kw):
    """Run the oracle pipeline on sequence b of the workload."""
    return O.twilight_decode(synth.bits(w.q[b]), synth.bits(w.seq_k(b)),
                             synth.bits(w.seq_v(b)) if w.v.numel() else synth.bits(w.seq_k(b)),
                             int(w.budget[b]), w.p, full_selector=w.full_selector, **kw)
