"""Seeded synthetic decode workloads (inputs only - no method arithmetic).

Serves both the CPU oracle and the HIP path with the SAME bytes: tensors are
generated on the host with torch's CPU generator, rounded to bf16, and either
viewed as uint16 numpy arrays (oracle) or uploaded (GPU).

Shapes follow a LLaMA-3.1-8B-style attention layer (32 query heads, 8 KV
heads, head_dim 128) during decode, the model family the paper evaluates.
Its LongBench-derived prompts are not available here; these inputs stand in
for them: K, V, q ~ N(0,1) plus per-query-head "heavy hitter" tokens whose
keys are pushed along the query direction, K_t += alpha * q_hat * sqrt(128),
which adds alpha*|q| to the token's attention logit.
"""
from dataclasses import dataclass, field
import math
import numpy as np
import torch

HEAD_DIM = 128
PAGE = 16


@dataclass
class Workload:
    name: str
    q: torch.Tensor            # bf16 [b, Hq, 128]
    k: torch.Tensor            # bf16 [total_tokens, Hkv, 128]  logical, sequences concatenated
    v: torch.Tensor            # bf16 [total_tokens, Hkv, 128]  (may be empty for pruner-only)
    seq_lens: torch.Tensor     # int32 [b]
    seq_offsets: list          # python ints, len b+1, into k / v
    page_table: torch.Tensor   # int32 [b, max_pages_per_seq], -1 padded
    num_pool_pages: int
    budget: torch.Tensor       # int32 [b]  selector budget in tokens
    p: float
    num_q_heads: int
    num_kv_heads: int
    full_selector: bool = False
    alpha: torch.Tensor = None  # fp32 [b, Hq]
    info: dict = field(default_factory=dict)

    @property
    def batch(self):
        return int(self.seq_lens.numel())

    def seq_k(self, b):
        return self.k[self.seq_offsets[b]:self.seq_offsets[b + 1]]

    def seq_v(self, b):
        return self.v[self.seq_offsets[b]:self.seq_offsets[b + 1]]


def bits(t):
    """bf16 torch tensor -> uint16 numpy array of its bit patterns (no copy of values)."""
    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def _gen(seed, *key):
    g = torch.Generator(device="cpu")
    h = seed & 0xFFFFFFFF
    for x in key:
        h = (h * 1000003 + (hash(x) if not isinstance(x, int) else x)) & 0x7FFFFFFFFFFFFFFF
    g.manual_seed(h)
    return g


def _key_int(s):
    """Stable small integer for a string (python's hash() is salted per process)."""
    v = 0
    for ch in s:
        v = (v * 131 + ord(ch)) & 0x7FFFFFFF
    return v


def make_workload(name, seq_lens, num_q_heads=32, num_kv_heads=8, budget=None, p=0.95,
                  heavy_frac=0.01, alpha_range=(0.5, 3.0), alpha_cycle=None, spans=None,
                  shuffle_pool=False, extra_pool_pages=0, full_selector=False, need_v=True,
                  seed=0, heavy_frac_range=None):
    """Build one workload.

    seq_lens        list of context lengths
    budget          selector budget in tokens: int, list, or callable n -> int
    heavy_frac      fraction of tokens that are heavy hitters, per query head
    heavy_frac_range  (lo, hi): per-head fraction drawn uniformly instead
    alpha_range     alpha ~ U[lo, hi] per (sequence, query head)
    alpha_cycle     list: alpha of head h is alpha_cycle[h % len] instead
    spans           (count, length): heavy hitters are `count` contiguous spans
                    of `length` tokens per head instead of scattered tokens
    shuffle_pool    pages of all sequences randomly permuted in one shared pool
    """
    kname = _key_int(name)
    b = len(seq_lens)
    Hq, Hkv = num_q_heads, num_kv_heads
    G = Hq // Hkv
    offs = [0]
    for n in seq_lens:
        offs.append(offs[-1] + int(n))
    total = offs[-1]
    q = torch.randn(b, Hq, HEAD_DIM, generator=_gen(seed, kname, 1)).to(torch.bfloat16)
    if alpha_cycle is not None:
        alpha = torch.tensor([alpha_cycle[h % len(alpha_cycle)] for h in range(Hq)],
                             dtype=torch.float32).repeat(b, 1)
    else:
        alpha = torch.rand(b, Hq, generator=_gen(seed, kname, 2)) * (alpha_range[1] - alpha_range[0]) + alpha_range[0]
    k = torch.empty(total, Hkv, HEAD_DIM, dtype=torch.bfloat16)
    v = torch.empty(total if need_v else 0, Hkv, HEAD_DIM, dtype=torch.bfloat16)
    heavy_sets = {}
    for s in range(b):
        n = int(seq_lens[s])
        ks = torch.randn(n, Hkv, HEAD_DIM, generator=_gen(seed, kname, 3, s))
        qf = q[s].float()
        qhat = qf / qf.norm(dim=-1, keepdim=True).clamp_min(1e-20)
        gh = _gen(seed, kname, 4, s)
        for h in range(Hq):
            if heavy_frac_range is not None:
                frac = float(torch.rand(1, generator=gh)) * (heavy_frac_range[1] - heavy_frac_range[0]) + heavy_frac_range[0]
            else:
                frac = heavy_frac
            if spans is not None:
                cnt, ln = spans
                ln = min(ln, n)
                starts = torch.randint(0, n - ln + 1, (cnt,), generator=gh)
                idx = (starts[:, None] + torch.arange(ln)[None, :]).reshape(-1).unique()
            else:
                m = min(n, max(1, int(round(frac * n)))) if frac > 0 else 0
                idx = torch.randperm(n, generator=gh)[:m]
            if idx.numel() and float(alpha[s, h]) != 0.0:
                ks[idx, h // G, :] += float(alpha[s, h]) * math.sqrt(HEAD_DIM) * qhat[h]
            if n <= 1 << 17:
                heavy_sets[(s, h)] = np.sort(idx.numpy())
        k[offs[s]:offs[s + 1]] = ks.to(torch.bfloat16)
        del ks
        if need_v:
            v[offs[s]:offs[s + 1]] = torch.randn(n, Hkv, HEAD_DIM, generator=_gen(seed, kname, 5, s)).to(torch.bfloat16)
    pages_per_seq = [(int(n) + PAGE - 1) // PAGE for n in seq_lens]
    max_pages = max(pages_per_seq) if b else 0
    used = sum(pages_per_seq)
    num_pool_pages = used + int(extra_pool_pages)
    if shuffle_pool:
        perm = torch.randperm(num_pool_pages, generator=_gen(seed, kname, 6))[:used]
    else:
        perm = torch.arange(used)
    page_table = torch.full((b, max_pages), -1, dtype=torch.int32)
    c = 0
    for s in range(b):
        page_table[s, :pages_per_seq[s]] = perm[c:c + pages_per_seq[s]].to(torch.int32)
        c += pages_per_seq[s]
    if budget is None:
        bud = [int(n) for n in seq_lens]
    elif callable(budget):
        bud = [int(budget(int(n))) for n in seq_lens]
    elif isinstance(budget, (list, tuple)):
        bud = [int(x) for x in budget]
    else:
        bud = [int(budget)] * b
    return Workload(name=name, q=q, k=k, v=v,
                    seq_lens=torch.tensor([int(n) for n in seq_lens], dtype=torch.int32),
                    seq_offsets=offs, page_table=page_table, num_pool_pages=num_pool_pages,
                    budget=torch.tensor(bud, dtype=torch.int32), p=float(p),
                    num_q_heads=Hq, num_kv_heads=Hkv, full_selector=full_selector,
                    alpha=alpha, info=dict(heavy_sets=heavy_sets, seed=seed))


def ragged_lengths(count, lo, hi, seed=0):
    """`count` lengths log-uniform in [lo, hi]."""
    u = torch.rand(count, generator=_gen(seed, _key_int("ragged"), count))
    return [int(math.floor(math.exp(math.log(lo) + float(x) * (math.log(hi) - math.log(lo))))) for x in u]


# The five benchmark configurations C1..C5, and `scale`d
# variants: scale < 1 shrinks contexts and budgets by that factor for tests.
def config(idx, scale=1.0, seed=0, batch=None, kv_heads=None):
    def sc(x, lo=PAGE):
        return max(lo, int(round(x * scale)))
    if idx == 0:
        return make_workload("C1", [sc(4096)], budget=sc(1024), p=0.95, heavy_frac=0.01,
                             alpha_range=(0.5, 3.0), seed=seed)
    if idx == 1:
        b = 8 if batch is None else batch
        extra = {} if kv_heads is None else {"num_kv_heads": int(kv_heads)}   # 32 = the multi-head (G = 1) shape
        return make_workload("C2", [sc(32768)] * b, budget=sc(4096), p=0.9, heavy_frac=0.005,
                             alpha_range=(0.0, 4.0), shuffle_pool=True, seed=seed, **extra)
    if idx == 2:
        return make_workload("C3", [sc(131072)], budget=sc(8192), p=0.9, spans=(8, 64),
                             alpha_range=(1.0, 4.0), seed=seed)
    if idx == 3:
        b = 4 if batch is None else batch
        return make_workload("C4", [sc(262144)] * b, num_q_heads=64, num_kv_heads=8, p=0.95,
                             heavy_frac=0.005, alpha_cycle=[0.0, 0.5, 2.0, 6.0],
                             full_selector=True, need_v=False, seed=seed)
    if idx == 4:
        b = 64 if batch is None else batch
        lens = ragged_lengths(b, sc(2048), sc(65536), seed=seed)
        return make_workload("C5", lens, budget=lambda n: max(PAGE, n // 8), p=0.95,
                             heavy_frac_range=(0.001, 0.05), alpha_range=(0.0, 4.0),
                             shuffle_pool=True, seed=seed)
    raise ValueError("config index 0..4")


def calibrated_channels(w, r):
    """Channel sets for a channel-sparse token selector: per KV head the r of its 128 channels that an offline
    calibration pass would keep - stood in for here by the channels with the largest mean |K| x mean |q| over the
    workload's own tokens and heads.  Returns (lists [Hkv][r] ascending, bit masks uint32 [Hkv, 4] as int32 tensor)."""
    G = w.num_q_heads // w.num_kv_heads
    kmag = w.k.float().abs().mean(dim=0)                                  # [Hkv, 128]
    qmag = w.q.float().abs().mean(dim=0).reshape(w.num_kv_heads, G, HEAD_DIM).mean(dim=1)
    lists, masks = [], np.zeros((w.num_kv_heads, 4), dtype=np.uint32)
    for g in range(w.num_kv_heads):
        ch = np.sort(torch.argsort(-(kmag[g] * qmag[g]), stable=True)[:r].numpy())
        lists.append(ch)
        for d in ch:
            masks[g, d // 32] |= np.uint32(1) << np.uint32(d % 32)
    return lists, torch.from_numpy(masks.view(np.int32).copy())
