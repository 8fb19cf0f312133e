"""Plain CPU oracle of Twilight's decode-time hot path (numpy, slow, obvious).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the bench's
cpu_baseline leg.  It shares no code with the HIP path and imports nothing
from it.  Every function works on ONE sequence in its logical (un-paged)
layout; paging is pure data movement and is done by the callers.

What it follows (paper = "Twilight: Adaptive Attention Sparsity with
Hierarchical Top-p Pruning"):
  * sparse attention over an index set            - Definition 3.1 / Eq. (1)
  * the top-p index set                           - Definition 3.3, Algorithm 1
  * select-then-prune pipeline                    - Section 4.1, Figure 5
  * INT4 asymmetric K estimate, scale/zero fp16   - Section 4.2, Appendix B.1
  * per-group union for GQA                       - Appendix B.2
  * per-page (16 token) selector metadata         - Section 4 (challenge C1)

Where a result must be reproduced bit for bit by the GPU (INT4 codes, page
sets, integer dot products, fp32 estimated scores) the arithmetic is a fixed
sequence of individually rounded fp32 operations, written out below.  Where
the GPU is allowed a tolerance (softmax mass, attention output) the oracle
works in float64.

Parity pins: every function here is pinned by tests/test_oracle_*.py against
closed forms, brute force, library routines or invariants; none is unpinned.
(ds_scores / ds_select, the channel-sparse token selector, are pinned the
same way, but the paper gives no definition or value for that selector:
their reading is ours, "parity unpinned by paper values".)
The paper prints no worked numeric example for this path that can be
reproduced without model weights (its p=0.8 -> 97 tokens example is a real
attention head), so no pin uses a value printed by the paper except the cost
model of Section 4.3.
"""
import numpy as np

HEAD_DIM = 128      # d
PAGE = 16           # tokens per page (Section 4: pages of 16 tokens)
QGROUP = 32         # dims sharing one (scale, zero)
NGROUPS = HEAD_DIM // QGROUP

F32 = np.float32
_INV127 = F32(1.0 / 127.0)            # fp32 nearest to 1/127
_RSQRT_D = F32(1.0 / np.sqrt(128.0))  # fp32 nearest to 1/sqrt(128)


# --------------------------------------------------------------------------
# bf16 <-> fp32 (bf16 values are carried as their uint16 bit patterns)
# --------------------------------------------------------------------------
def bf16_to_f32(bits):
    """Exact widening: a bf16 is the top 16 bits of an fp32."""
    bits = np.asarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_bf16(x):
    """Round-to-nearest-even narrowing of finite fp32 values to bf16 bits."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    rounded = u + np.uint32(0x7FFF) + lsb
    return (rounded >> np.uint32(16)).astype(np.uint16)


# --------------------------------------------------------------------------
# Stage 4: INT4 asymmetric quantisation of K (Section 4.2; Appendix B.1,
# "Dequantization": dynamic, fp16 scale and zero).  Granularity: per token,
# per KV head, per group of 32 dims.
# --------------------------------------------------------------------------
def quantize_k(k_bits, bits=4):
    """k_bits uint16[n,128] -> (u uint8[n,128] in 0..L, scale f16[n,4], zero f16[n,4]), L = 2^bits - 1.

    Per group of 32: mn, mx; scale = fp16((mx-mn) * (1/L)); zero = fp16(mn);
    u = clamp(rint((x - zero) * (1/scale)), 0, L); scale == 0 -> u = 0.
    All fp32, each operation rounded on its own; rint is round-half-even.
    bits = 4 is the method's choice; 2 and 8 are the other widths of its
    bit-width study of the estimator (Section 4.2, Figure 6).
    """
    L = (1 << bits) - 1
    inv_l = F32(1.0 / L)                      # fp32 nearest to 1/L
    x = bf16_to_f32(k_bits).reshape(-1, NGROUPS, QGROUP)
    mn = x.min(axis=-1)
    mx = x.max(axis=-1)
    scale = ((mx - mn) * inv_l).astype(np.float16)
    zero = mn.astype(np.float16)
    sf = scale.astype(np.float32)
    zf = zero.astype(np.float32)
    ok = sf > 0
    inv = np.zeros_like(sf)
    inv[ok] = F32(1.0) / sf[ok]
    t = (x - zf[..., None]) * inv[..., None]
    u = np.clip(np.rint(t), 0, L).astype(np.uint8)
    u[~ok] = 0
    return u.reshape(-1, HEAD_DIM), scale, zero


def dequantize_k(u, scale, zero):
    """x_hat = u*scale + zero, in float64 (exact: at most 8-bit x 11-bit + 11-bit)."""
    u = np.asarray(u).reshape(-1, NGROUPS, QGROUP).astype(np.float64)
    s = np.asarray(scale).astype(np.float64)[..., None]
    z = np.asarray(zero).astype(np.float64)[..., None]
    return (u * s + z).reshape(-1, HEAD_DIM)


# --------------------------------------------------------------------------
# Stage 1: page selector.  The paper only says the base selector pools
# per 16-token page; the bound used is the element-wise upper bound of q.k
# over the page's [min, max] box.
# --------------------------------------------------------------------------
def page_minmax(k_bits):
    """k_bits uint16[n,128] -> (mn_bits, mx_bits) uint16[P,128], P = ceil(n/16).
    The last page covers its valid tokens only.  Exact (min/max of bf16)."""
    x = bf16_to_f32(k_bits)
    n = x.shape[0]
    P = (n + PAGE - 1) // PAGE
    mn = np.empty((P, HEAD_DIM), np.float32)
    mx = np.empty((P, HEAD_DIM), np.float32)
    full = n // PAGE
    if full:
        xf = x[: full * PAGE].reshape(full, PAGE, HEAD_DIM)
        mn[:full] = xf.min(axis=1)
        mx[:full] = xf.max(axis=1)
    if P > full:
        mn[full] = x[full * PAGE:].min(axis=0)
        mx[full] = x[full * PAGE:].max(axis=0)
    return f32_to_bf16(mn), f32_to_bf16(mx)


def page_upper_bounds(q_bits, mn_bits, mx_bits):
    """U[P] = sum_d max(q_d*mn[P,d], q_d*mx[P,d]) in fp32 with a FIXED order.

    Each product of two bf16 values is exact in fp32, so only the order of
    the 127 additions matters: 16 partial sums, partial l = left-to-right sum
    of dims 8l..8l+7, then a balanced pairwise tree over the 16 partials
    (l with l^1, then ^2, ^4, ^8).  A final +0.0 turns -0 into +0.
    """
    q = bf16_to_f32(q_bits).reshape(HEAD_DIM)
    mn = bf16_to_f32(mn_bits).reshape(-1, HEAD_DIM)
    mx = bf16_to_f32(mx_bits).reshape(-1, HEAD_DIM)
    t = np.maximum(q[None, :] * mn, q[None, :] * mx).reshape(-1, 16, 8)
    part = t[:, :, 0].copy()
    for j in range(1, 8):
        part = part + t[:, :, j]
    for step in (1, 2, 4, 8):
        lanes = np.arange(16)
        part = part + part[:, lanes ^ step]
    return (part[:, 0] + F32(0.0)).astype(np.float32)


def select_pages(U, budget_tokens, n):
    """Logical ids (ascending) of the Kp = min(ceil(B/16), P) pages with the
    largest bound; among equal bounds the lower page id wins."""
    P = (n + PAGE - 1) // PAGE
    assert U.shape[0] == P
    Kp = min((int(budget_tokens) + PAGE - 1) // PAGE, P)
    if Kp <= 0:
        return np.zeros(0, np.int32)
    order = np.lexsort((np.arange(P), -U.astype(np.float64)))  # by -U, then id
    return np.sort(order[:Kp]).astype(np.int32)


def candidate_tokens(pages, n):
    """Token indices (ascending) of the given logical pages, below n."""
    pages = np.asarray(pages, dtype=np.int64)
    t = (pages[:, None] * PAGE + np.arange(PAGE)[None, :]).reshape(-1)
    return t[t < n]


# --------------------------------------------------------------------------
# Stage 2a: estimated scores from INT4 K ("SpGEMV", Section 4.2, App. B.1).
# Integer formulation: q is quantised to int8 per head (symmetric), the
# group-of-32 dot products are exact integers, scale/zero are applied per
# group in fp32 in a fixed association.
# --------------------------------------------------------------------------
def quantize_q(q_bits):
    """q_bits uint16[128] -> (qi int8[128], sq fp32).  sq = amax*(1/127);
    qi = clamp(rint(q / sq), -127, 127); all zero when sq == 0."""
    q = bf16_to_f32(q_bits).reshape(HEAD_DIM)
    sq = F32(np.abs(q).max() * _INV127)
    if sq == 0:
        return np.zeros(HEAD_DIM, np.int8), sq
    qi = np.clip(np.rint(q / sq), -127, 127).astype(np.int8)
    return qi, sq


def int4_dots(qi, u):
    """I[t,j] = sum_{d in group j} qi_d * u[t,d]  (int32),  Qs[j] = sum qi_d."""
    qg = qi.astype(np.int32).reshape(NGROUPS, QGROUP)
    ug = np.asarray(u).astype(np.int32).reshape(-1, NGROUPS, QGROUP)
    I = (ug * qg[None]).sum(axis=-1, dtype=np.int32)
    Qs = qg.sum(axis=-1, dtype=np.int32)
    return I, Qs


def int4_scores(qi, sq, u, scale, zero):
    """s_hat[t] = ((T0+T1)+(T2+T3)) * (sq * 1/sqrt(128)),
    T_j = fl(scale_j*float(I_j)) + fl(zero_j*float(Qs_j)); every operation is
    a separately rounded fp32 operation (no fused multiply-add)."""
    I, Qs = int4_dots(qi, u)
    sf = np.asarray(scale).astype(np.float32)
    zf = np.asarray(zero).astype(np.float32)
    a = sf * I.astype(np.float32)
    b = zf * Qs.astype(np.float32)[None, :]
    T = a + b
    acc = (T[:, 0] + T[:, 1]) + (T[:, 2] + T[:, 3])
    c = F32(sq * _RSQRT_D)
    return (acc * c).astype(np.float32)


# --------------------------------------------------------------------------
# Another token selector in front of the pruner (Section 4.1: the base
# algorithm is a black box that hands over a token subset; Sections 4.3 and 5
# name a Double-Sparsity-style one, which ranks tokens by an estimate taken
# from a few channels of a 4-bit copy of K).  The paper defines it only by
# citation and prints no values for it: PARITY UNPINNED BY PAPER VALUES.
# Reading taken: a fixed set of channels per KV head (found offline; an input
# here), the estimate is the INT4 score above with the query's other channels
# set to zero, and the B tokens with the largest estimate are handed over.
# --------------------------------------------------------------------------
def ds_scores(qi, sq, u, scale, zero, channels):
    """Channel-sparse estimate: int4_scores with qi kept only on `channels`
    (dims 0..127 of the KV head's channel set); sq is the full query's."""
    keep = np.zeros(HEAD_DIM, bool)
    keep[np.asarray(channels, dtype=np.int64)] = True
    return int4_scores(np.where(keep, qi, 0).astype(np.int8), sq, u, scale, zero)


def ds_select(s_ds, budget_tokens, n):
    """Positions (ascending) of the min(B, n) tokens with the largest
    estimate; among equal estimates the lower position wins."""
    s_ds = np.asarray(s_ds, dtype=np.float32)
    assert s_ds.shape[0] == n
    K = min(int(budget_tokens), n)
    if K <= 0:
        return np.zeros(0, np.int32)
    order = np.lexsort((np.arange(n), -s_ds.astype(np.float64)))  # by -estimate, then position
    return np.sort(order[:K]).astype(np.int32)


# --------------------------------------------------------------------------
# Stage 2b/c: softmax over the candidates and the top-p set
# (Definition 3.3; Algorithm 1 returns the threshold set {W >= l}).
# --------------------------------------------------------------------------
def softmax_weights(s):
    """float64 softmax of the fp32 scores."""
    s = np.asarray(s, dtype=np.float64)
    e = np.exp(s - s.max())
    return e / e.sum()


def topp_set(s, p):
    """Boolean mask of the top-p threshold set over candidate scores s, and
    the threshold weight tau*.

    Sort the weights descending, k* = smallest prefix whose sum >= p,
    tau* = k*-th largest weight, keep every W >= tau* (all ties at the cut).
    p >= 1 keeps everything.  An empty candidate list gives an empty set.
    """
    s = np.asarray(s, dtype=np.float32)
    if s.size == 0:
        return np.zeros(0, bool), 0.0
    W = softmax_weights(s)
    if p >= 1.0:
        return np.ones(s.size, bool), float(W.min())
    Ws = np.sort(W)[::-1]
    csum = np.cumsum(Ws)
    hit = np.nonzero(csum >= float(p))[0]
    if hit.size == 0:          # rounding left the total a hair under p
        return np.ones(s.size, bool), float(W.min())
    tau = Ws[hit[0]]
    return W >= tau, float(tau)


def topp_binary_search(W, p, eps):
    """The threshold search of Algorithm 1 on one weight vector: bisect a
    weight threshold between 0 and the largest weight, keeping the lower end
    feasible (the weights at or above it sum to at least p) and the upper end
    infeasible, until all weights still undecided (above the lower end, at or
    below the upper one) lie within eps of each other; the result is the set
    of weights at or above the lower end.  With eps = 0 this is topp_set."""
    W = np.asarray(W, dtype=np.float64)
    l, r = 0.0, float(W.max())
    for _ in range(4096):
        m = 0.5 * (l + r)
        if W[W >= m].sum() >= p:
            l = m
        else:
            r = m
        und = W[(W > l) & (W <= r)]
        if und.size == 0 or und.max() - und.min() <= eps:
            break
    return W >= l


def group_union(index_sets):
    """Sorted unique union of the per-head kept sets of one query group
    (Appendix B.2)."""
    if len(index_sets) == 0:
        return np.zeros(0, np.int32)
    return np.unique(np.concatenate([np.asarray(s, np.int64) for s in index_sets])).astype(np.int32)


# --------------------------------------------------------------------------
# Stage 3: attention over an index set (Definition 3.1), weights
# renormalised over the attended set; float64.
# --------------------------------------------------------------------------
def attention(q_bits, k_bits, v_bits, idx=None):
    """q_bits uint16[128]; k_bits, v_bits uint16[n,128]; idx = token subset
    (None = all).  Returns (out float64[128], lse float64) with
    lse = log sum_t exp(q.k_t/sqrt(128)) over the attended set."""
    q = bf16_to_f32(q_bits).astype(np.float64).reshape(HEAD_DIM)
    K = bf16_to_f32(k_bits).astype(np.float64)
    V = bf16_to_f32(v_bits).astype(np.float64)
    if idx is not None:
        idx = np.asarray(idx, dtype=np.int64)
        K, V = K[idx], V[idx]
    if K.shape[0] == 0:
        return np.zeros(HEAD_DIM), -np.inf
    logits = (K @ q) / np.sqrt(float(HEAD_DIM))
    m = logits.max()
    e = np.exp(logits - m)
    Z = e.sum()
    return (e / Z) @ V, float(m + np.log(Z))


def true_mass(q_bits, k_bits, idx):
    """Exact softmax mass (over all n tokens) of the index set."""
    q = bf16_to_f32(q_bits).astype(np.float64).reshape(HEAD_DIM)
    K = bf16_to_f32(k_bits).astype(np.float64)
    logits = (K @ q) / np.sqrt(float(HEAD_DIM))
    e = np.exp(logits - logits.max())
    return float(e[np.asarray(idx, np.int64)].sum() / e.sum())


# --------------------------------------------------------------------------
# Whole pipeline for one sequence (Figure 5): select -> prune -> union ->
# attend.  GQA: query head h reads KV head h // G.
# --------------------------------------------------------------------------
def twilight_decode(q_bits, k_bits, v_bits, budget_tokens, p, full_selector=False, bits=4):
    """q_bits uint16[Hq,128]; k_bits, v_bits uint16[n,Hkv,128].

    Returns a dict with every intermediate, all in logical coordinates:
      u, scale, zero (per KV head), mn, mx, U[Hq,P], pages[h], cand[h],
      s_hat[h], kept[h], tau[h], union[g], out float64[Hq,128], lse[Hq],
      out_bf16 uint16[Hq,128].
    full_selector=True skips stage 1 (every token is a candidate).
    bits: width of the quantised K copy the estimate is taken from (4 = the method).
    """
    Hq = q_bits.shape[0]
    n, Hkv, _ = k_bits.shape
    G = Hq // Hkv
    r = dict(u=[], scale=[], zero=[], mn=[], mx=[], U=[], pages=[], cand=[],
             s_hat=[], kept=[], tau=[], union=[])
    for g in range(Hkv):
        u, sc, ze = quantize_k(k_bits[:, g], bits)
        mn, mx = page_minmax(k_bits[:, g])
        r["u"].append(u); r["scale"].append(sc); r["zero"].append(ze)
        r["mn"].append(mn); r["mx"].append(mx)
    P = (n + PAGE - 1) // PAGE
    for h in range(Hq):
        g = h // G
        if full_selector:
            U = None
            pages = np.arange(P, dtype=np.int32)
        else:
            U = page_upper_bounds(q_bits[h], r["mn"][g], r["mx"][g])
            pages = select_pages(U, budget_tokens, n)
        cand = candidate_tokens(pages, n)
        qi, sq = quantize_q(q_bits[h])
        s_hat = int4_scores(qi, sq, r["u"][g][cand], r["scale"][g][cand], r["zero"][g][cand])
        mask, tau = topp_set(s_hat, p)
        r["U"].append(U); r["pages"].append(pages); r["cand"].append(cand)
        r["s_hat"].append(s_hat); r["kept"].append(cand[mask].astype(np.int32)); r["tau"].append(tau)
    out = np.zeros((Hq, HEAD_DIM))
    lse = np.zeros(Hq)
    for g in range(Hkv):
        r["union"].append(group_union(r["kept"][g * G:(g + 1) * G]))
    for h in range(Hq):
        g = h // G
        out[h], lse[h] = attention(q_bits[h], k_bits[:, g], v_bits[:, g], r["union"][g])
    r["out"] = out
    r["lse"] = lse
    r["out_bf16"] = f32_to_bf16(out.astype(np.float32))
    return r


def dense_decode(q_bits, k_bits, v_bits):
    """Full attention o = softmax(q K^T / sqrt(d)) V for every query head."""
    Hq = q_bits.shape[0]
    G = Hq // k_bits.shape[1]
    out = np.zeros((Hq, HEAD_DIM))
    lse = np.zeros(Hq)
    for h in range(Hq):
        out[h], lse[h] = attention(q_bits[h], k_bits[:, h // G], v_bits[:, h // G], None)
    return out, lse


def cost_model_speedup(N, B0, B1):
    """Section 4.3: (N/16 + B0) / (N/16 + B0/4 + B1), in KV-token loads."""
    return (N / 16.0 + B0) / (N / 16.0 + B0 / 4.0 + B1)
