"""Pins of the CPU oracle against things other than itself: hand-derived
fixtures, closed forms, brute force on tiny inputs, library routines and
invariants.  No GPU, no HIP code."""
import itertools
import math
import os

import numpy as np
import pytest
import torch
from scipy.special import logsumexp
from scipy.stats import norm

from oracle import twilight_oracle as O
from workloads import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _lines(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.strip() for ln in f if ln.strip() and not ln.startswith("#")]


def _bf16_bits(x):
    return synth.bits(torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16))


# ------------------------------------------------------------------ bf16
def test_bf16_conversions_match_torch(rng):
    x = rng.standard_normal(20000).astype(np.float32) * np.exp(rng.uniform(-20, 20, 20000)).astype(np.float32)
    x = np.concatenate([x, np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.0e38, 1e-38])])
    tb = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(O.f32_to_bf16(x), synth.bits(tb))
    assert np.array_equal(O.bf16_to_f32(synth.bits(tb)), tb.float().numpy())


def test_bf16_ties_round_to_even():
    # 1 + 2^-8 is exactly half way between bf16 1.0 and 1+2^-7 -> even (1.0);
    # 1 + 3*2^-8 is half way between 1+2^-7 and 1+2^-6 -> even (1+2^-6).
    got = O.bf16_to_f32(O.f32_to_bf16(np.float32([1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8])))
    assert got.tolist() == [1.0, 1 + 2.0 ** -6]


# ------------------------------------------------------------------ INT4
def test_int4_codes_on_exact_grid_fixture():
    for ln in _lines("int4_grid.txt"):
        codes = np.array([int(t) for t in ln.split()], dtype=np.int64)
        assert codes.size == 32 and codes.min() == 0 and codes.max() == 15
        row = np.zeros(128, np.float32)
        for g in range(4):  # same group in every slot, rotated so slots differ
            row[32 * g:32 * g + 32] = -1.0 + 0.125 * np.roll(codes, g)
        u, s, z = O.quantize_k(_bf16_bits(row)[None, :])
        assert np.all(s == np.float16(0.125)) and np.all(z == np.float16(-1.0))
        for g in range(4):
            assert np.array_equal(u[0, 32 * g:32 * g + 32], np.roll(codes, g))
        assert np.array_equal(O.dequantize_k(u, s, z)[0], row.astype(np.float64))


def test_int4_round_trip_bound_and_invariants(rng):
    x = (rng.standard_normal((4000, 128)) * np.exp(rng.uniform(-3, 3, (4000, 1)))).astype(np.float32)
    x[7, 32:64] = 0.75          # constant group
    x[8, :] = 0.0
    kb = _bf16_bits(x)
    xb = O.bf16_to_f32(kb).astype(np.float64)
    u, s, z = O.quantize_k(kb)
    assert u.dtype == np.uint8 and u.max() <= 15
    xh = O.dequantize_k(u, s, z)
    sg = np.repeat(s.astype(np.float64), 32, axis=1)
    zg = np.repeat(z.astype(np.float64), 32, axis=1)
    g = xb.reshape(-1, 4, 32)
    mn = np.repeat(g.min(-1), 32, axis=1)
    # half a step, plus the fp16 rounding of zero and of scale (15 steps * 2^-11 relative)
    bound = 0.5 * sg + np.abs(mn) * 2.0 ** -11 + 15 * sg * 2.0 ** -11 + 1e-7
    assert np.all(np.abs(xb - xh) <= bound)
    # codes are the nearest grid level (up to fp32 rounding of the quotient)
    lv = zg[..., None] + sg[..., None] * np.arange(16)[None, None, :]
    best = np.abs(xb[..., None] - lv).min(-1)
    assert np.all(np.abs(xb - xh) <= best + 1e-6 * (np.abs(xb) + sg))
    # group minimum has code 0; when scale > 0 the maximum has code 15
    ug = u.reshape(-1, 4, 32)
    amin = g.argmin(-1)
    amax = g.argmax(-1)
    ii, jj = np.indices(amin.shape)
    assert np.all(ug[ii, jj, amin] == 0)
    pos = s.astype(np.float32) > 0
    assert np.all(ug[ii, jj, amax][pos] == 15)
    # constant groups: scale 0, all codes 0, exact
    assert s[7, 1] == 0 and np.all(ug[7, 1] == 0) and np.all(xh[7, 32:64] == 0.75)
    assert np.all(s[8] == 0) and np.all(u[8] == 0)
    # zero is the fp16 of the group minimum, scale the fp16 of range/15 (within 1 fp16 ulp)
    assert np.array_equal(z, g.min(-1).astype(np.float16))
    rng15 = (g.max(-1) - g.min(-1)) / 15.0
    assert np.all(np.abs(s.astype(np.float64) - rng15) <= rng15 * 2.0 ** -10 + 1e-8)


@pytest.mark.parametrize("bits", [2, 8])
def test_other_estimator_widths_grid_bound_and_levels(rng, bits):
    """The 2- and 8-bit copies of the bit-width study (Section 4.2, Figure 6) follow the 4-bit recipe with
    L = 2^bits - 1 levels: exact recovery on a power-of-two grid, half-a-step round trip, end points."""
    L = (1 << bits) - 1
    step = 2.0 ** -(bits - 1)                      # -1 + step*code is exact in bf16 for code <= 255
    codes = rng.integers(0, L + 1, (50, 4, 32))
    codes[:, :, 0] = 0
    codes[:, :, 1] = L
    row = (-1.0 + step * codes).astype(np.float32).reshape(50, 128)
    u, s, z = O.quantize_k(_bf16_bits(row), bits)
    assert np.all(s == np.float16(step)) and np.all(z == np.float16(-1.0))
    assert np.array_equal(u.reshape(50, 4, 32), codes)
    assert np.array_equal(O.dequantize_k(u, s, z), row.astype(np.float64))
    # random data: bound, nearest level, end points
    x = (rng.standard_normal((2000, 128)) * np.exp(rng.uniform(-3, 3, (2000, 1)))).astype(np.float32)
    kb = _bf16_bits(x)
    xb = O.bf16_to_f32(kb).astype(np.float64)
    u, s, z = O.quantize_k(kb, bits)
    assert u.max() <= L
    xh = O.dequantize_k(u, s, z)
    sg = np.repeat(s.astype(np.float64), 32, axis=1)
    zg = np.repeat(z.astype(np.float64), 32, axis=1)
    g = xb.reshape(-1, 4, 32)
    mn = np.repeat(g.min(-1), 32, axis=1)
    assert np.all(np.abs(xb - xh) <= 0.5 * sg + np.abs(mn) * 2.0 ** -11 + L * sg * 2.0 ** -11 + 1e-7)
    lv = zg[..., None] + sg[..., None] * np.arange(L + 1)[None, None, :]
    assert np.all(np.abs(xb - xh) <= np.abs(xb[..., None] - lv).min(-1) + 1e-6 * (np.abs(xb) + sg))
    ug = u.reshape(-1, 4, 32)
    ii, jj = np.indices(g.shape[:2])
    assert np.all(ug[ii, jj, g.argmin(-1)] == 0)
    # scale carries an fp16 rounding of up to 2^-11 relative, i.e. at most 255 * 2^-11 < 1/2 step at
    # the top: the maximum still lands on L
    pos = s.astype(np.float32) > 0
    assert np.all(ug[ii, jj, g.argmax(-1)][pos] == L)
    # coarser copies estimate worse: mean squared error falls with the width
    err = {b: np.mean((xb - O.dequantize_k(*O.quantize_k(kb, b))) ** 2) for b in (2, 4, 8)}
    assert err[2] > 10 * err[4] > 100 * err[8]


def test_int4_rint_is_half_even():
    # group 0: min 0, max 15 -> scale 1, zero 0; values k + 0.5 must round to even k
    row = np.zeros(128, np.float32)
    row[:32] = [0, 15, 0.5, 1.5, 2.5, 3.5, 4.5, 13.5, 14.5] + [7.0] * 23
    u, s, z = O.quantize_k(_bf16_bits(row)[None])
    assert s[0, 0] == 1 and z[0, 0] == 0
    assert u[0, :9].tolist() == [0, 15, 0, 2, 2, 4, 4, 14, 14]


# ------------------------------------------------------------------ selector
def test_page_minmax_against_loops(rng):
    for n in (1, 15, 16, 17, 100, 160):
        kb = _bf16_bits(rng.standard_normal((n, 128)))
        x = O.bf16_to_f32(kb)
        mn, mx = O.page_minmax(kb)
        P = (n + 15) // 16
        assert mn.shape == (P, 128)
        for pg in range(P):
            blk = x[pg * 16:min(n, pg * 16 + 16)]
            assert np.array_equal(O.bf16_to_f32(mn[pg]), blk.min(0))
            assert np.array_equal(O.bf16_to_f32(mx[pg]), blk.max(0))


def test_page_bound_fixed_order_fixture():
    one = _bf16_bits(np.ones(128))
    for ln in _lines("page_bound_order.txt"):
        exp, rest = ln.split("|")
        vals = np.zeros(128, np.float32)
        for tok in rest.split():
            d, v = tok.split(":")
            vals[int(d)] = float(v)
        vb = _bf16_bits(vals)
        assert np.array_equal(O.bf16_to_f32(vb), vals)  # fixture values are bf16-exact
        U = O.page_upper_bounds(one, vb[None], vb[None])
        assert U.dtype == np.float32 and U[0] == np.float32(float(exp)), ln


def test_page_bound_is_an_upper_bound_and_close_to_float64(rng):
    n = 16 * 40 + 5
    kb = _bf16_bits(rng.standard_normal((n, 128)) * 2)
    qb = _bf16_bits(rng.standard_normal(128))
    q = O.bf16_to_f32(qb).astype(np.float64)
    K = O.bf16_to_f32(kb).astype(np.float64)
    mn, mx = O.page_minmax(kb)
    U = O.page_upper_bounds(qb, mn, mx)
    ref = np.maximum(q * O.bf16_to_f32(mn).astype(np.float64), q * O.bf16_to_f32(mx).astype(np.float64)).sum(-1)
    assert np.allclose(U, ref, rtol=2e-6, atol=1e-4)
    dots = K @ q
    for pg in range(U.size):
        assert np.all(dots[pg * 16:pg * 16 + 16] <= U[pg] + 1e-3)
    # a negated query uses the other corner of the box
    Un = O.page_upper_bounds(_bf16_bits(-O.bf16_to_f32(qb)), mn, mx)
    refn = np.maximum(-q * O.bf16_to_f32(mn).astype(np.float64), -q * O.bf16_to_f32(mx).astype(np.float64)).sum(-1)
    assert np.allclose(Un, refn, rtol=2e-6, atol=1e-4)


def test_select_pages_brute_force_ties_and_full_budget(rng):
    for trial in range(200):
        P = int(rng.integers(1, 40))
        n = P * 16 - int(rng.integers(0, 16))
        U = rng.integers(-3, 4, P).astype(np.float32)   # many ties
        B = int(rng.integers(1, n + 40))
        Kp = min(-(-B // 16), P)
        ranked = sorted(range(P), key=lambda i: (-float(U[i]), i))
        exp = sorted(ranked[:Kp])
        got = O.select_pages(U, B, n)
        assert got.dtype == np.int32 and got.tolist() == exp
    assert O.select_pages(np.float32([1, 5, 3]), 48, 48).tolist() == [0, 1, 2]
    assert O.select_pages(np.float32([1, 5, 3]), 10_000, 40).tolist() == [0, 1, 2]
    assert O.select_pages(np.float32([1, 5, 3]), 17, 48).tolist() == [1, 2]
    assert O.select_pages(np.float32([5, 5, 5]), 16, 48).tolist() == [0]


def test_candidate_tokens():
    assert O.candidate_tokens([0, 2], 100).tolist() == list(range(16)) + list(range(32, 48))
    assert O.candidate_tokens([1, 6], 100).tolist() == list(range(16, 32)) + [96, 97, 98, 99]


# ------------------------------------------------------------------ INT4 scores
def test_quantize_q_properties(rng):
    for _ in range(50):
        qb = _bf16_bits(rng.standard_normal(128) * math.exp(rng.uniform(-4, 4)))
        q = O.bf16_to_f32(qb).astype(np.float64)
        qi, sq = O.quantize_q(qb)
        assert qi.dtype == np.int8 and np.abs(qi.astype(int)).max() == 127
        assert abs(float(sq) - np.abs(q).max() / 127) <= 1e-6 * float(sq)
        assert np.all(np.abs(q - float(sq) * qi) <= 0.5 * float(sq) * (1 + 1e-5))
        assert np.all(np.sign(qi[np.abs(q) > sq]) == np.sign(q[np.abs(q) > sq]))
    qi, sq = O.quantize_q(_bf16_bits(np.zeros(128)))
    assert sq == 0 and not qi.any()


def test_integer_dots_and_score_identity(rng):
    n = 700
    kb = _bf16_bits(rng.standard_normal((n, 128)) * 1.5 + 0.3)
    qb = _bf16_bits(rng.standard_normal(128))
    u, s, z = O.quantize_k(kb)
    qi, sq = O.quantize_q(qb)
    I, Qs = O.int4_dots(qi, u)
    assert I.dtype == np.int32 and Qs.dtype == np.int32
    # int64 matmul, arranged differently (library primitive)
    q64 = qi.astype(np.int64)
    for j in range(4):
        assert np.array_equal(I[:, j].astype(np.int64), u[:, 32 * j:32 * j + 32].astype(np.int64) @ q64[32 * j:32 * j + 32])
        assert Qs[j] == q64[32 * j:32 * j + 32].sum()
    # s_hat equals (sq*qi) . dequant(K) / sqrt(128) up to fp32 rounding
    s_hat = O.int4_scores(qi, sq, u, s, z)
    assert s_hat.dtype == np.float32
    ref = O.dequantize_k(u, s, z) @ (float(sq) * q64.astype(np.float64)) / math.sqrt(128.0)
    assert np.allclose(s_hat, ref, rtol=0, atol=2e-5 * np.abs(ref).max() + 1e-6)
    # and estimates the exact logit with INT4-sized noise (step/sqrt(12) per dim, |q|~sqrt(128))
    exact = O.bf16_to_f32(kb).astype(np.float64) @ O.bf16_to_f32(qb).astype(np.float64) / math.sqrt(128.0)
    err = s_hat - exact
    step = s.astype(np.float64).mean()
    assert abs(err.mean()) < 0.02 and err.std() < 1.5 * step / math.sqrt(12) * np.linalg.norm(O.bf16_to_f32(qb)) / math.sqrt(128) + 0.02


def test_score_association_is_the_stated_one():
    # scale=1, zero=0 in every group, q=127 at one dim per group: T_j = 127*u_j.  Choose codes so
    # that T = [A, 1, 1, -A]-like cancellation is impossible with codes >= 0; instead check linearity:
    row = np.zeros(128, np.float32)
    for j in range(4):
        row[32 * j] = 15.0           # max -> scale 1, zero 0
        row[32 * j + 1] = j + 1.0    # code j+1
    u, s, z = O.quantize_k(_bf16_bits(row)[None])
    assert np.all(s == 1) and np.all(z == 0)
    q = np.zeros(128, np.float32)
    q[[1, 33, 65, 97]] = 1.0
    qi, sq = O.quantize_q(_bf16_bits(q))
    assert qi[[1, 33, 65, 97]].tolist() == [127] * 4
    I, Qs = O.int4_dots(qi, u)
    assert I[0].tolist() == [127, 254, 381, 508] and Qs.tolist() == [127] * 4
    s_hat = O.int4_scores(qi, sq, u, s, z)
    # (1+2+3+4) * 127 * (1/127) / sqrt(128)
    assert abs(float(s_hat[0]) - 10.0 / math.sqrt(128.0)) < 1e-6


# ------------------------------------------------------------------ top-p
def _brute_topp(W, p):
    """Sort, accumulate, cut, then add ties at the cut - in pure Python."""
    order = sorted(range(len(W)), key=lambda i: -W[i])
    acc, k = 0.0, 0
    for k, i in enumerate(order, 1):
        acc += W[i]
        if acc >= p:
            break
    tau = W[order[k - 1]]
    return sorted(i for i in range(len(W)) if W[i] >= tau), k


def test_topp_matches_sort_brute_force_on_tiny_inputs(rng):
    for trial in range(300):
        m = int(rng.integers(1, 30))
        s = (rng.standard_normal(m) * rng.uniform(0.1, 4)).astype(np.float32)
        if trial % 3 == 0:
            s = np.round(s)  # ties
        p = float(rng.uniform(0.05, 0.999))
        mask, tau = O.topp_set(s, p)
        W = O.softmax_weights(s)
        exp, k = _brute_topp(list(W), p)
        assert np.nonzero(mask)[0].tolist() == exp
        assert mask.sum() >= k


def test_topp_is_the_minimum_set_by_subset_enumeration(rng):
    # Definition 3.3 by exhaustive search: the smallest subset with mass >= p has size k*,
    # and the oracle's set is the top-k* weights plus ties at the cut.
    for trial in range(25):
        m = int(rng.integers(2, 11))
        s = (rng.standard_normal(m) * 2).astype(np.float32)
        p = float(rng.uniform(0.2, 0.98))
        W = O.softmax_weights(s)
        kmin = None
        for k in range(1, m + 1):
            if any(sum(W[list(c)]) >= p for c in itertools.combinations(range(m), k)):
                kmin = k
                break
        mask, tau = O.topp_set(s, p)
        kept = np.nonzero(mask)[0]
        assert len(kept) >= kmin
        assert np.sort(W)[::-1][kmin - 1] == tau
        assert len(kept) == (W >= tau).sum()
        if len(np.unique(W)) == m:
            assert len(kept) == kmin


def test_topp_closed_forms():
    m = 64
    mask, _ = O.topp_set(np.zeros(m, np.float32), 0.3)      # uniform: every weight ties at the cut
    assert mask.all()
    s = np.full(m, -50.0, np.float32)
    s[17] = 30.0
    mask, _ = O.topp_set(s, 0.99)                           # one-hot
    assert np.nonzero(mask)[0].tolist() == [17]
    # geometric weights W_i ~ r^i: k* = ceil(ln(1 - p(1-r^m)) / ln r)
    for r, p in ((0.5, 0.9), (0.8, 0.95), (0.9, 0.5), (0.97, 0.8)):
        s = (np.arange(m) * math.log(r)).astype(np.float32)
        W = O.softmax_weights(s)
        rr = W[1] / W[0]
        k = math.ceil(math.log(1 - p * (1 - rr ** m)) / math.log(rr) - 1e-9)
        mask, _ = O.topp_set(s, p)
        assert np.nonzero(mask)[0].tolist() == list(range(k)), (r, p)
    mask, _ = O.topp_set(np.float32([0.3, -1.0, 2.0]), 1.0)  # p = 1 keeps everything
    assert mask.all()
    mask, _ = O.topp_set(np.zeros(0, np.float32), 0.9)
    assert mask.size == 0


def test_topp_invariants(rng):
    for trial in range(100):
        m = int(rng.integers(5, 3000))
        s = (rng.standard_normal(m) * rng.uniform(0.2, 5)).astype(np.float32)
        p = float(rng.uniform(0.3, 0.995))
        mask, tau = O.topp_set(s, p)
        W = O.softmax_weights(s)
        assert mask.any() and mask[np.argmax(s)]
        assert W[mask].sum() >= p - 1e-12
        assert W[mask].min() >= W[~mask].max() if (~mask).any() else True   # threshold set
        lowest = W[mask].min()
        assert W[mask & (W > lowest)].sum() < p                             # minimal
    # monotone in p
    s = (rng.standard_normal(500) * 2).astype(np.float32)
    sizes = [O.topp_set(s, p)[0].sum() for p in (0.1, 0.5, 0.8, 0.9, 0.95, 0.99, 1.0)]
    assert sizes == sorted(sizes) and sizes[-1] == 500


def test_algorithm1_bisection_agrees_with_sorted_definition(rng):
    for trial in range(100):
        m = int(rng.integers(2, 400))
        s = (rng.standard_normal(m) * rng.uniform(0.3, 4)).astype(np.float32)
        p = float(rng.uniform(0.2, 0.99))
        W = O.softmax_weights(s)
        mask, tau = O.topp_set(s, p)
        # skip the measure-zero case where a prefix sum lands within rounding of p
        cs = np.cumsum(np.sort(W)[::-1])
        if np.abs(cs - p).min() < 1e-12:
            continue
        got = O.topp_binary_search(W, p, eps=0.0)
        assert np.array_equal(got, mask)
    # a coarse eps may only ADD tokens (l stops below tau*), never drop any
    W = O.softmax_weights((rng.standard_normal(300) * 2).astype(np.float32))
    exact = O.topp_set(np.log(W).astype(np.float32), 0.9)[0]
    coarse = O.topp_binary_search(W, 0.9, eps=1e-3)
    assert coarse.sum() >= (W >= np.sort(W)[::-1][np.nonzero(np.cumsum(np.sort(W)[::-1]) >= 0.9)[0][0]]).sum()
    assert exact.sum() > 0


def test_topp_gaussian_closed_form_at_scale(rng):
    # logits ~ N(0, sigma^2): kept fraction -> Phi(Phi^-1(p) - sigma)
    n = 200_000
    for sigma, p in ((1.0, 0.95), (1.0, 0.9), (2.0, 0.9), (0.5, 0.8)):
        s = (rng.standard_normal(n) * sigma).astype(np.float32)
        frac = O.topp_set(s, p)[0].mean()
        assert abs(frac - norm.cdf(norm.ppf(p) - sigma)) < 0.01, (sigma, p, frac)


# ------------------------------------------------------------------ attention
def test_attention_matches_library_sdpa(rng):
    n = 333
    qb = _bf16_bits(rng.standard_normal((4, 128)))
    kb = _bf16_bits(rng.standard_normal((n, 128)))
    vb = _bf16_bits(rng.standard_normal((n, 128)))
    q = torch.from_numpy(O.bf16_to_f32(qb)).double()
    K = torch.from_numpy(O.bf16_to_f32(kb)).double()
    V = torch.from_numpy(O.bf16_to_f32(vb)).double()
    ref = torch.nn.functional.scaled_dot_product_attention(q[None, :, None, :], K[None, None].expand(1, 4, n, 128),
                                                           V[None, None].expand(1, 4, n, 128))[0, :, 0].numpy()
    idx = np.sort(rng.choice(n, 57, replace=False))
    refs = torch.nn.functional.scaled_dot_product_attention(q[None, :, None, :], K[idx][None, None].expand(1, 4, 57, 128),
                                                            V[idx][None, None].expand(1, 4, 57, 128))[0, :, 0].numpy()
    for h in range(4):
        out, lse = O.attention(qb[h], kb, vb)
        assert np.allclose(out, ref[h], rtol=1e-10, atol=1e-12)
        assert abs(lse - logsumexp((K @ q[h]).numpy() / math.sqrt(128))) < 1e-10
        outs, _ = O.attention(qb[h], kb, vb, idx)
        assert np.allclose(outs, refs[h], rtol=1e-10, atol=1e-12)


def test_attention_special_cases_and_split_invariance(rng):
    n = 200
    qb = _bf16_bits(rng.standard_normal(128))
    kb = _bf16_bits(rng.standard_normal((n, 128)))
    vb = _bf16_bits(rng.standard_normal((n, 128)))
    out, _ = O.attention(qb, kb, vb, [42])
    assert np.array_equal(out, O.bf16_to_f32(vb[42]).astype(np.float64))
    out, lse = O.attention(qb, kb, vb, [])
    assert not out.any() and lse == -np.inf
    # log-sum-exp combine of two halves equals the whole
    idx = np.arange(n)
    oa, la = O.attention(qb, kb, vb, idx[:77])
    ob, lb = O.attention(qb, kb, vb, idx[77:])
    ow, lw = O.attention(qb, kb, vb, idx)
    l = np.logaddexp(la, lb)
    assert np.allclose(oa * np.exp(la - l) + ob * np.exp(lb - l), ow, atol=1e-12) and abs(l - lw) < 1e-12
    # duplicates in the set are NOT expected (union is unique); permutation of the set is irrelevant
    perm = rng.permutation(n)
    op, _ = O.attention(qb, kb, vb, perm)
    assert np.allclose(op, ow, atol=1e-12)


def test_sparse_attention_error_bound(rng):
    # Eq. (2) adapted to weights renormalised over the set:
    # |o - o_hat| <= 2 (1 - M) max_t |V_t|, M = true mass of the set.
    n = 600
    qb = _bf16_bits(rng.standard_normal(128) * 3)
    kb = _bf16_bits(rng.standard_normal((n, 128)))
    vb = _bf16_bits(rng.standard_normal((n, 128)))
    dense, _ = O.attention(qb, kb, vb)
    vmax = np.linalg.norm(O.bf16_to_f32(vb).astype(np.float64), axis=1).max()
    logits = O.bf16_to_f32(kb).astype(np.float64) @ O.bf16_to_f32(qb).astype(np.float64) / math.sqrt(128)
    for p in (0.5, 0.8, 0.95, 0.999):
        mask, _ = O.topp_set(logits.astype(np.float32), p)
        idx = np.nonzero(mask)[0]
        M = O.true_mass(qb, kb, idx)
        assert M >= p - 1e-6
        sp, _ = O.attention(qb, kb, vb, idx)
        assert np.linalg.norm(dense - sp) <= 2 * (1 - M) * vmax + 1e-12


# ------------------------------------------------------------------ pipeline
def test_pipeline_p1_full_budget_is_dense_attention():
    w = synth.make_workload("pin_dense", [300], num_q_heads=8, num_kv_heads=2, budget=300, p=1.0, seed=3)
    qb, kb, vb = synth.bits(w.q[0]), synth.bits(w.seq_k(0)), synth.bits(w.seq_v(0))
    r = O.twilight_decode(qb, kb, vb, 300, 1.0)
    dense, lse = O.dense_decode(qb, kb, vb)
    assert np.array_equal(r["out"], dense) and np.array_equal(r["lse"], lse)
    assert all(u.tolist() == list(range(300)) for u in r["union"])
    r2 = O.twilight_decode(qb, kb, vb, 10 ** 6, 1.0, full_selector=True)
    assert np.array_equal(r2["out"], dense)


def test_pipeline_structure_and_heavy_hitters():
    w = synth.config(0, scale=0.5, seed=1)      # 2048 tokens, budget 512
    qb, kb, vb = synth.bits(w.q[0]), synth.bits(w.seq_k(0)), synth.bits(w.seq_v(0))
    n = kb.shape[0]
    r = O.twilight_decode(qb, kb, vb, int(w.budget[0]), w.p)
    G = w.num_q_heads // w.num_kv_heads
    for h in range(w.num_q_heads):
        g = h // G
        assert len(r["pages"][h]) == min(-(-int(w.budget[0]) // 16), -(-n // 16))
        assert np.all(np.diff(r["pages"][h]) > 0) and np.all(np.diff(r["kept"][h]) > 0)
        assert set(r["kept"][h]) <= set(r["cand"][h]) and set(r["kept"][h]) <= set(r["union"][g])
        # estimated mass >= p by construction; the TRUE mass (exact logits, over the candidates) is close
        W = O.softmax_weights(r["s_hat"][h])
        assert W[np.isin(r["cand"][h], r["kept"][h])].sum() >= w.p - 1e-12
        # the box bound ranks this head's heavy-hitter pages (logit boost alpha*|q|) above the average page
        heavy = w.info["heavy_sets"][(0, h)]
        if float(w.alpha[0, h]) >= 1.0:
            assert r["U"][h][np.unique(heavy // 16)].mean() > r["U"][h].mean() + 10
        # INT4 estimate is good: the kept set's EXACT mass within the candidates is close to p
        cand = r["cand"][h]
        ex = O.bf16_to_f32(kb[cand, g]).astype(np.float64) @ O.bf16_to_f32(qb[h]).astype(np.float64) / math.sqrt(128)
        We = np.exp(ex - ex.max())
        We /= We.sum()
        assert We[np.isin(cand, r["kept"][h])].sum() > w.p - 0.05
    for g in range(w.num_kv_heads):
        un = r["union"][g]
        assert np.all(np.diff(un) > 0)
        assert set(un) == set().union(*[set(r["kept"][h]) for h in range(g * G, g * G + G)])
    # error bound of the final output against dense attention
    dense, _ = O.dense_decode(qb, kb, vb)
    for h in range(w.num_q_heads):
        g = h // G
        M = O.true_mass(qb[h], kb[:, g], r["union"][g])
        vmax = np.linalg.norm(O.bf16_to_f32(vb[:, g]).astype(np.float64), axis=1).max()
        assert np.linalg.norm(dense[h] - r["out"][h]) <= 2 * (1 - M) * vmax + 1e-9


def test_cost_model_fixture():
    for ln in _lines("cost_model.txt"):
        N, B0, B1, exp = ln.split()
        got = O.cost_model_speedup(float(N), float(B0), float(B1))
        assert abs(got - float(exp)) < 1e-12
    assert 1.9 < O.cost_model_speedup(1 << 16, 1 << 14, 1 << 10) < 2.3   # "approximately 2x"


def test_workload_generator_is_deterministic_and_shaped():
    a = synth.config(1, scale=1 / 64, seed=0, batch=2)
    b = synth.config(1, scale=1 / 64, seed=0, batch=2)
    assert torch.equal(a.k.view(torch.int16), b.k.view(torch.int16)) and torch.equal(a.page_table, b.page_table)
    assert a.k.shape == (2 * 512, 8, 128) and a.q.shape == (2, 32, 128) and a.page_table.shape == (2, 32)
    used = a.page_table[a.page_table >= 0]
    assert used.unique().numel() == used.numel() == 64 and int(used.max()) < a.num_pool_pages
    c = synth.config(1, scale=1 / 64, seed=1, batch=2)
    assert not torch.equal(a.k.view(torch.int16), c.k.view(torch.int16))
    r = synth.config(4, scale=1 / 32, batch=5)
    assert r.batch == 5 and all(64 <= int(n) <= 2048 for n in r.seq_lens)
    assert [int(x) for x in r.budget] == [max(16, int(n) // 8) for n in r.seq_lens]


def test_attention_tolerance_rule_accepts_only_rounding_ties():
    """The GPU parity tests compare attention outputs with the oracle's result rounded to bf16; an element
    whose exact value sits on the midpoint of two bf16 neighbours (within fp32 error) may round either way.
    The helper accepts exactly that, and still rejects a one-ulp error anywhere else."""
    from tests.gpu_util import assert_attention, bf16_round
    rng = np.random.default_rng(0)
    x = rng.normal(size=128) * 0.01
    assert_attention(bf16_round(x), x)
    x[3] = 0.583984218                          # 1.6e-7 below the midpoint of 0.58203125 and 0.5859375
    g = bf16_round(x)
    assert g[3] == 0.58203125
    g[3] = 0.5859375                            # the other neighbour: 0.4 % of the dominant element
    assert_attention(g, x)
    x[3] = 0.5825                               # well inside the lower half: the same output is now wrong
    with pytest.raises(AssertionError):
        assert_attention(g, x)


def test_scale_ties_round_to_even_in_the_fp16_subnormal_range():
    """Appendix B.1 keeps scale and zero in fp16.  A group spanning [-33, 34.5] * 2^-24 has
    (max - min) * fl(1/15) = 4.5 * 2^-24 exactly in fp32 (67.5 * 0.0666666701 = 4.50000023, below the fp32 midpoint
    4.50000024), a tie between the fp16 subnormals 4 and 5 steps: round to nearest EVEN gives 0x0004.  (The GPU's
    own conversion instruction returns 5 here, which is how this case was found.)"""
    x = np.full(128, -33 * 2.0 ** -24, dtype=np.float32)
    x[1::2] = 34.5 * 2.0 ** -24
    bits = O.f32_to_bf16(x)
    assert np.array_equal(O.bf16_to_f32(bits), x)                 # both values are bf16-exact
    r = np.float32(x.max() - x.min()) * np.float32(1.0 / 15.0)
    assert float(r) * 2.0 ** 24 == 4.5
    u, s, z = O.quantize_k(bits[None, :])
    assert s.view(np.uint16).tolist() == [[4, 4, 4, 4]]
    assert z.view(np.uint16).tolist() == [[0x8021] * 4]          # -33 steps
    # codes follow from the rounded scale: (34.5 + 33) / 4 = 16.875 -> clamped to 15; the minimum maps to 0
    assert set(u[0].tolist()) == {0, 15}


def test_set_check_accepts_a_mass_on_the_threshold_only_within_1e6():
    """The parity tests accept a GPU set that differs from the oracle's by a token far from tau* only when the
    cumulative mass itself sits on p (within 1e-6): the set must lie between the oracle's sets for p -/+ 1e-6."""
    from tests.test_gpu_parity import check_topp
    # four weights 0.5 + 1e-9, 0.3, 0.15, 0.05 - 1e-9 (as logits): at p = 0.5 the first token alone just suffices
    W = np.array([0.5 + 1e-9, 0.3, 0.15, 0.05 - 1e-9])
    s = np.log(W).astype(np.float64)
    cand = np.arange(4)
    mask, _ = O.topp_set(s, 0.5)
    assert mask.tolist() == [True, False, False, False]
    check_topp(np.array([0]), s, cand, 0.5)
    check_topp(np.array([0, 1]), s, cand, 0.5)            # one more token: the mass was 1e-9 over p
    with pytest.raises(AssertionError):
        check_topp(np.array([0, 1, 2]), s, cand, 0.5)     # two more: not explained by the mass arithmetic
    W2 = np.array([0.5 + 1e-4, 0.3, 0.15, 0.05 - 1e-4])    # mass clearly over p: the extra token is an error
    with pytest.raises(AssertionError):
        check_topp(np.array([0, 1]), np.log(W2), cand, 0.5)


# ------------------------------------------------------------------ channel-sparse token selector
def test_ds_scores_full_channel_set_is_the_int4_score_and_masking_hits_the_right_dims(rng):
    """All 128 channels: the estimate IS the INT4 score (bit for bit).  A subset: it equals, in float64, the dot
    product of the quantised query with the dequantised keys over exactly those channels."""
    k = _bf16_bits(rng.standard_normal((300, 128)))
    u, sc, ze = O.quantize_k(k)
    qi, sq = O.quantize_q(_bf16_bits(rng.standard_normal(128)))
    assert np.array_equal(O.ds_scores(qi, sq, u, sc, ze, np.arange(128)), O.int4_scores(qi, sq, u, sc, ze))
    for r in (1, 8, 16, 40):
        ch = np.sort(rng.choice(128, size=r, replace=False))
        got = O.ds_scores(qi, sq, u, sc, ze, ch).astype(np.float64)
        xhat = O.dequantize_k(u, sc, ze).astype(np.float64)
        want = (xhat[:, ch] * qi[ch].astype(np.float64)).sum(1) * float(sq) / math.sqrt(128.0)
        assert np.allclose(got, want, rtol=1e-5, atol=1e-6 * np.abs(want).max())
        other = np.setdiff1d(np.arange(128), ch)                 # the two halves add up to the full score
        rest = O.ds_scores(qi, sq, u, sc, ze, other).astype(np.float64)
        assert np.allclose(got + rest, O.int4_scores(qi, sq, u, sc, ze), rtol=1e-5, atol=1e-5)


def test_ds_scores_hand_example():
    """One channel (dim 5), codes 0..15 over 16 tokens, scale 0.5 and zero -1 in group 0: with q = 127 on that
    channel (sq = 1) the estimate of token t is (0.5 * 127 t - 127) / sqrt(128)."""
    u = np.zeros((16, 128), np.uint8)
    u[:, 5] = np.arange(16)
    sc = np.zeros((16, 4), np.float16); sc[:, 0] = 0.5
    ze = np.zeros((16, 4), np.float16); ze[:, 0] = -1.0
    qi = np.zeros(128, np.int8); qi[5] = 127; qi[70] = -50
    got = O.ds_scores(qi, np.float32(1.0), u, sc, ze, [5])
    want = (0.5 * 127.0 * np.arange(16) - 127.0) / math.sqrt(128.0)
    assert np.allclose(got, want, rtol=1e-6)
    assert np.all(O.ds_scores(qi, np.float32(1.0), u, sc, ze, []) == 0)      # no channels: every estimate is zero


def test_ds_select_brute_force_ties_and_budgets(rng):
    for n, B in ((1, 1), (7, 3), (50, 50), (50, 80), (200, 37), (64, 0)):
        s = rng.integers(0, 6, n).astype(np.float32)             # few distinct values: many ties
        got = O.ds_select(s, B, n)
        order = sorted(range(n), key=lambda i: (-float(s[i]), i))        # pure-Python sort, ties to the lower position
        want = sorted(order[:min(B, n)])
        assert got.tolist() == want
    s = np.zeros(40, np.float32)
    assert O.ds_select(s, 12, 40).tolist() == list(range(12))            # all equal: the first B positions
    # a heavy token is found from the channels its key was pushed along
    k = rng.standard_normal((500, 128)).astype(np.float32)
    q = rng.standard_normal(128).astype(np.float32)
    ch = np.argsort(-np.abs(q))[:16]
    k[123, ch] += 8.0 * np.sign(q[ch])
    u, sc, ze = O.quantize_k(_bf16_bits(k))
    qi, sq = O.quantize_q(_bf16_bits(q))
    assert 123 in O.ds_select(O.ds_scores(qi, sq, u, sc, ze, ch), 5, 500).tolist()
