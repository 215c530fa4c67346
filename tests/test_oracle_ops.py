"""Pins of the CPU oracle's single operators against what the paper and the mathematics fix:
hand-worked examples, brute force on tiny inputs, closed forms and invariants.
(CPU only; nothing here touches the GPU library.)"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- token / channel budget
def test_budget_is_integer_ceiling():
    # Appendix "Budgeted token selection": b = ceil(kappa * K_t), clamped; exact rational ceil.
    for num, den in [(1, 10), (3, 10), (1, 8), (1, 4), (1, 2), (1, 1), (7, 13), (1, 16)]:
        for n in list(range(1, 70)) + [1023, 1024, 8191, 8192]:
            want = max(1, min(n, math.ceil(Fraction(num, den) * n)))
            assert oracle.budget(num, den, n) == want
    assert oracle.budget(1, 10, 30) == 3          # 0.1*30 is 3.0000000000000004 in binary fp
    assert oracle.budget(3, 4, 1024) == 768 and oracle.budget(1, 4, 14336) == 3584


# ---------------------------------------------------------------- fake quantiser
def _golden_rows():
    rows = []
    with open(os.path.join(GOLDEN, "fake_quant_worked.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            b, z, c, zh = [p.strip() for p in line.split("|")]
            rows.append((int(b), np.array(z.split(), np.float32), np.array(c.split(), np.int32),
                         np.array(zh.split(), np.float32)))
    return rows


@pytest.mark.parametrize("bits,z,codes,zhat", _golden_rows())
def test_fake_quant_worked_examples(bits, z, codes, zhat):
    out, c, _ = oracle.fake_quant(z, bits)
    assert np.array_equal(c, codes)
    assert np.array_equal(out, zhat)


@pytest.mark.parametrize("bits", [4, 5, 6, 8, 12, 15])
def test_fake_quant_invariants(bits):
    rng = np.random.default_rng(bits)
    qmax = 2 ** (bits - 1) - 1
    for n in (1, 7, 64, 1000):
        z = rng.standard_normal(n).astype(np.float32) * 3
        out, codes, s = oracle.fake_quant(z, bits)
        a = np.abs(z).max()
        assert np.float32(s) == np.float32(a) / np.float32(qmax)
        assert codes.min() >= -qmax and codes.max() <= qmax
        assert abs(codes[np.argmax(np.abs(z))]) == qmax             # arg-absmax maps to +-q_max
        assert np.all(np.abs(out.astype(np.float64) - z) <= 0.5 * s * (1 + 1e-6))
        assert len(np.unique(out)) <= 2 * qmax + 1
        assert np.array_equal(np.sign(codes) * np.sign(z) >= 0, np.ones(n, bool))
        # idempotent on codes (values may move by an ulp of the scale, codes may not)
        out2, codes2, _ = oracle.fake_quant(out, bits)
        assert np.array_equal(codes2, codes)
        assert np.allclose(out2, out, rtol=3e-7, atol=0)
        # exact scale equivariance under powers of two
        out4, codes4, s4 = oracle.fake_quant(z * np.float32(4), bits)
        assert np.array_equal(codes4, codes) and np.array_equal(out4, out * np.float32(4))
        # monotone: a larger input never gets a smaller code
        order = np.argsort(z, kind="stable")
        assert np.all(np.diff(codes[order]) >= 0)


def test_fake_quant_bypass_and_zero_row():
    z = np.array([0.3, -2.0, 1e-3], np.float32)
    for bits in (16, 17, 32):
        out, codes, _ = oracle.fake_quant(z, bits)
        assert np.array_equal(out, z)
    out, codes, s = oracle.fake_quant(np.zeros(5, np.float32), 4)
    assert np.array_equal(out, np.zeros(5, np.float32)) and not codes.any() and s == 0.0


# ---------------------------------------------------------------- magnitude top-m mask
def _brute_rank_mask(key, m):
    """keep[c] iff fewer than m entries beat c (larger key, or equal key and lower index)."""
    n = len(key)
    keep = np.zeros(n, np.uint8)
    for c in range(n):
        beat = sum(1 for e in range(n) if key[e] > key[c] or (key[e] == key[c] and e < c))
        keep[c] = beat < m
    return keep


def test_topm_mask_brute_force_with_ties():
    rng = np.random.default_rng(0)
    for n in (1, 2, 5, 16, 33):
        for trial in range(6):
            a = rng.integers(-4, 5, n).astype(np.float32) if trial % 2 else rng.standard_normal(n).astype(np.float32)
            for m in range(0, n + 2):
                got = oracle.topm_mask(a, m)
                want = _brute_rank_mask(np.abs(a), min(m, n))
                assert np.array_equal(got, want), (n, m, a)


def test_topm_mask_properties():
    rng = np.random.default_rng(1)
    a = rng.standard_normal(1024).astype(np.float32)
    prev = np.zeros(1024, np.uint8)
    for m in (1, 256, 512, 768, 1024):
        k = oracle.topm_mask(a, m)
        assert k.sum() == m
        if m < 1024:
            assert np.abs(a[k == 1]).min() >= np.abs(a[k == 0]).max()
        assert np.all(k >= prev)                                     # nested in m
        prev = k
    # sign plays no role
    assert np.array_equal(oracle.topm_mask(a, 300), oracle.topm_mask(-a, 300))


# ---------------------------------------------------------------- key selection, one key per page
def test_select_keys_matches_stable_sort():
    rng = np.random.default_rng(2)
    for n in (1, 2, 3, 8, 16):
        for trial in range(8):
            s = rng.integers(-3, 4, n).astype(np.float32) if trial % 2 else rng.standard_normal(n).astype(np.float32)
            for b in range(1, n + 1):
                got = oracle.select_keys(s, b)
                top = sorted(range(n), key=lambda j: (-s[j], j))[:b]
                want = np.zeros(n, np.uint8)
                want[top] = 1
                assert np.array_equal(got, want), (n, b, s)
                assert got.sum() == b


def test_select_keys_nested_and_ordered():
    rng = np.random.default_rng(3)
    s = rng.standard_normal(257).astype(np.float32)
    prev = np.zeros(257, np.uint8)
    for num, den in [(1, 16), (1, 8), (1, 4), (1, 2), (1, 1)]:
        b = oracle.budget(num, den, 257)
        k = oracle.select_keys(s, b)
        assert k.sum() == b == math.ceil(257 * num / den)
        if b < 257:
            assert s[k == 1].min() >= s[k == 0].max()
        assert np.all(k >= prev)
        prev = k


def test_select_keys_sink_and_window_inside_budget():
    s = np.array([-9, -9, 5, 4, 3, 2, 1, 0, -9, -9], np.float32)
    # 2 sinks + 2 window keys are forced and count inside the budget: 6 kept = 4 forced + best 2
    k = oracle.select_keys(s, 6, n_sink=2, n_window=2)
    assert k.tolist() == [1, 1, 1, 1, 0, 0, 0, 0, 1, 1]
    # budget below the forced count: the forced keys alone are kept
    k = oracle.select_keys(s, 2, n_sink=2, n_window=2)
    assert k.tolist() == [1, 1, 0, 0, 0, 0, 0, 0, 1, 1]
    # forced sets may overlap on short rows
    k = oracle.select_keys(np.array([1, 2, 3], np.float32), 1, n_sink=2, n_window=2)
    assert k.tolist() == [1, 1, 1]


# ---------------------------------------------------------------- Quest page bound
def test_page_bound_is_upper_bound_and_exact_at_page_size_one():
    rng = np.random.default_rng(4)
    dh, n = 16, 37
    q = rng.standard_normal(dh).astype(np.float32)
    K = rng.standard_normal((n, dh)).astype(np.float32)
    dots = (K.astype(np.float64) @ q.astype(np.float64))
    for S in (1, 4, 8, 16):
        _, ps = oracle.select_pages(q, K, b=n, S=S)
        for u in range(len(ps)):
            best = dots[u * S:min(n, u * S + S)].max()
            assert ps[u] >= best - 1e-5
            if S == 1:
                assert abs(ps[u] - best) < 1e-5          # q+.k + q-.(-k) collapses to q.k
    # brute closed form of the bound for one page
    S = 4
    _, ps = oracle.select_pages(q, K, b=n, S=S)
    page = K[4:8].astype(np.float64)
    qq = q.astype(np.float64)
    want = np.sum(np.where(qq >= 0, qq * page.max(0), qq * page.min(0)))
    assert abs(ps[1] - want) < 1e-5


def test_select_pages_keeps_top_pages_and_equals_keys_at_s1():
    rng = np.random.default_rng(5)
    dh, n = 8, 23
    q = rng.standard_normal(dh).astype(np.float32)
    K = rng.standard_normal((n, dh)).astype(np.float32)
    score = (K.astype(np.float64) @ q.astype(np.float64)).astype(np.float32)
    for b in (1, 5, 12, 22):
        k1, _ = oracle.select_pages(q, K, b=b, S=1)
        assert np.array_equal(k1, oracle.select_keys(score, b))
    for S in (4, 8):
        for b in (1, 4, 9, 17):
            keep, ps = oracle.select_pages(q, K, b=b, S=S)
            n_pages = math.ceil(b / S)
            top = sorted(range(len(ps)), key=lambda u: (-ps[u], u))[:n_pages]
            want = np.zeros(n, np.uint8)
            for u in top:
                want[u * S:min(n, u * S + S)] = 1
            assert np.array_equal(keep, want)
    keep, _ = oracle.select_pages(q, K, b=4, S=4, n_sink=4, n_window=2)
    assert keep[:4].all() and keep[-2:].all()


# ---------------------------------------------------------------- softmax over kept keys, times V
def test_softmax_v_closed_forms():
    rng = np.random.default_rng(6)
    n, dh = 19, 8
    s = rng.standard_normal(n).astype(np.float32)
    V = rng.standard_normal((n, dh)).astype(np.float32)
    keep = (rng.random(n) < 0.5).astype(np.uint8)
    keep[3] = 1
    o, p = oracle.softmax_v(s, keep, V)
    assert abs(p.sum() - 1) < 1e-6 and np.all(p[keep == 0] == 0)
    # additive -inf mask formulation through the tensor library
    bias = torch.where(torch.from_numpy(keep.astype(bool)), 0.0, -math.inf).double()
    pw = torch.softmax(torch.from_numpy(s).double() + bias, 0)
    assert np.allclose(p, pw.numpy(), atol=1e-7)
    assert np.allclose(o, (pw @ torch.from_numpy(V).double()).numpy(), atol=1e-6)
    # constant V => constant output; a dominant kept score => that row of V
    o2, _ = oracle.softmax_v(s, keep, np.full((n, dh), 2.5, np.float32))
    assert np.allclose(o2, 2.5, atol=1e-6)
    s3 = s.copy()
    s3[3] = 200.0
    o3, _ = oracle.softmax_v(s3, keep, V)
    assert np.allclose(o3, V[3], atol=1e-6)
    # a dropped key has no influence, however large its score
    s4 = s.copy()
    s4[np.argmin(keep)] = 1e4
    o4, _ = oracle.softmax_v(s4, keep, V)
    assert np.array_equal(o4, o)


# ---------------------------------------------------------------- NLL
def test_nll_row_closed_forms():
    rng = np.random.default_rng(7)
    d, V = 16, 50
    hf = rng.standard_normal(d).astype(np.float32)
    W = rng.standard_normal((V, d)).astype(np.float32)
    assert abs(oracle.nll_row(hf, np.zeros((V, d), np.float32), 3) - math.log(V)) < 1e-6
    logits = torch.from_numpy(W).double() @ torch.from_numpy(hf).double()
    lsm = torch.log_softmax(logits, 0)
    tot = 0.0
    for y in range(V):
        v = oracle.nll_row(hf, W, y)
        assert abs(v + lsm[y].item()) < 1e-5
        tot += math.exp(-v)
    assert abs(tot - 1) < 1e-5


def test_rmsnorm_and_bf16_rounding():
    rng = np.random.default_rng(8)
    x = rng.standard_normal(64).astype(np.float32) * 3
    w = rng.standard_normal(64).astype(np.float32)
    got = oracle.rmsnorm(x, w, 1e-5)
    xt = torch.from_numpy(x).double()
    want = xt * torch.rsqrt(xt.pow(2).mean() + 1e-5) * torch.from_numpy(w).double()
    assert np.allclose(got, want.numpy(), rtol=1e-6, atol=1e-7)
    # unit gain => unit mean square
    g1 = oracle.rmsnorm(x, np.ones(64, np.float32), 0.0)
    assert abs(np.mean(g1.astype(np.float64) ** 2) - 1) < 1e-6
    vals = np.concatenate([rng.standard_normal(200).astype(np.float32) * 10,
                           np.array([1.00390625, 1.01171875, 0.0, -0.0, 3.3895314e38], np.float32)])
    want = torch.from_numpy(vals).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.round_bf16(vals), want)
