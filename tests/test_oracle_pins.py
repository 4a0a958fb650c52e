"""Pins for the CPU oracle: every check compares it with something other than itself --
exact integer brute force, closed forms, invariants and library routines -- chosen so that a
dropped term, a wrong sign or index, or a transposed operand fails at least one of them.
The Mosaic paper prints no worked numeric example for this path (it has no tables or
equations for it), so no paper-quoted values exist to pin against."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch
from scipy.special import logsumexp, softmax

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def bits(a):
    """fp32/64 array -> bf16 bit patterns (values must be exactly representable, checked)."""
    t = torch.as_tensor(np.asarray(a, dtype=np.float32))
    b = t.to(torch.bfloat16)
    assert torch.equal(b.float(), t), "test value not representable in bf16"
    return b.view(torch.uint16).numpy()


def rand_bf16(shape, std, seed):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(shape, generator=g) * std).to(torch.bfloat16)


# ---------------------------------------------------------------- selection (a1's definition)
@pytest.mark.parametrize("T", [0, 1, 2, 63, 64, 65, 255, 256, 257, 1000, 4097])
def test_mask_select_bruteforce(T):
    rng = np.random.default_rng(T)
    mask = (rng.random(T) < 0.37).astype(np.uint8) * rng.integers(1, 256, T).astype(np.uint8)
    want = [t for t in range(T) if mask[t] != 0]
    got = oracle.mask_select(mask)
    assert got.dtype == np.int32 and got.tolist() == want


def test_mask_select_invariants():
    T = 5000
    assert oracle.mask_select(np.ones(T, np.uint8)).tolist() == list(range(T))
    assert oracle.mask_select(np.zeros(T, np.uint8)).size == 0
    m = np.zeros(T, np.uint8)
    m[[0, 255, 256, 4095, 4096, T - 1]] = [1, 2, 128, 255, 7, 1]   # any nonzero byte counts
    assert oracle.mask_select(m).tolist() == [0, 255, 256, 4095, 4096, T - 1]
    rng = np.random.default_rng(1)
    m = (rng.random(T) < 0.5).astype(np.uint8)
    idx = oracle.mask_select(m)
    assert np.all(np.diff(idx) > 0) and idx.size == int(m.sum()) and np.all(m[idx] != 0)


# ---------------------------------------------------------------- logits: exact integer brute force
def test_logits_exact_integers_bruteforce():
    """Small-integer bf16 inputs give integer logits exactly; pure-Python rational arithmetic is the
    definition.  Asymmetric shapes and values: a transposed operand, a wrong stride or a dropped k
    changes the result."""
    rng = np.random.default_rng(7)
    T, d, V = 5, 12, 9
    H = rng.integers(-6, 7, (T, d)).astype(np.float32)
    W = rng.integers(-5, 6, (V, d)).astype(np.float32) * 0.5      # halves are exact in bf16 too
    Hb, Wb = bits(H), bits(W)
    for t in range(T):
        x = oracle.row_logits(Hb[t], Wb)
        for v in range(V):
            want = sum(Fraction(float(H[t, k])) * Fraction(float(W[v, k])) for k in range(d))
            assert Fraction(float(x[v])) == want, (t, v)
    res, logits = oracle.positions(Hb, Wb, np.arange(T), return_logits=True)
    for t in range(T):
        row = [sum(Fraction(float(H[t, k])) * Fraction(float(W[v, k])) for k in range(d)) for v in range(V)]
        mx = max(row)
        assert res.tok[t] == row.index(mx)                       # lowest id among maxima
        assert Fraction(float(res.rowmax[t])) == mx
        others = [r for i, r in enumerate(row) if i != row.index(mx)]
        assert Fraction(float(res.gap[t])) == mx - max(others)
        s = sum(math.exp(float(r - mx)) for r in row)
        assert res.lse[t] == pytest.approx(float(mx) + math.log(s), abs=1e-6)
        assert res.conf[t] == pytest.approx(1.0 / s, rel=1e-6)


def test_logits_fp64_accumulation_not_fp32():
    """A sum that fp32 accumulation gets wrong in every order but fp64 gets right:
    256 + 1/256 + ... : each product is exact, the total needs > 24 bits."""
    d = 16
    h = np.ones(d, np.float32)
    w = np.array([[256.0] + [2.0 ** -18] * (d - 1)], np.float32)
    x = oracle.row_logits(bits(h), bits(w))
    exact = 256.0 + (d - 1) * 2.0 ** -18          # = 256.0000572...
    assert x[0] == np.float32(exact)              # correctly rounded once
    assert x[0] != np.float32(256.0)              # what step-by-step fp32 adds would give


def test_sequential_fp32_mode_shows_what_accumulation_order_costs():
    """The auxiliary fp32-sequential logits: wrong exactly where the fp64 reference is right (the planted sum),
    identical on integer inputs, and within ~1e-5 of the reference on benchmark-like rows (d = 4096) -- three
    orders below the parity tolerances, which is why a GPU's own accumulation order is acceptable."""
    d = 16
    h = np.ones(d, np.float32)
    w = np.array([[256.0] + [2.0 ** -18] * (d - 1)], np.float32)
    assert oracle.row_logits_f32seq(bits(h), bits(w))[0] == np.float32(256.0)      # every small addend is lost
    rng = np.random.default_rng(9)
    hi = rng.integers(-4, 5, 96).astype(np.float32)
    wi = rng.integers(-3, 4, (40, 96)).astype(np.float32)
    assert np.array_equal(oracle.row_logits_f32seq(bits(hi), bits(wi)), oracle.row_logits(bits(hi), bits(wi)))
    H = rand_bf16((1, 4096), 1.0, 5)
    W = rand_bf16((2048, 4096), 4096 ** -0.5, 6)
    hb, wb = H.view(torch.uint16).numpy()[0], W.view(torch.uint16).numpy()
    diff = np.abs(oracle.row_logits_f32seq(hb, wb).astype(np.float64) - oracle.row_logits(hb, wb))
    assert 0 < diff.max() < 2e-5


# ---------------------------------------------------------------- library special cases
def test_logits_vs_torch_fp64_matmul():
    H = rand_bf16((7, 320), 1.0, 1)
    W = rand_bf16((513, 320), 320 ** -0.5, 2)
    want = (H.double() @ W.double().T).numpy()
    _, logits = oracle.positions(H.view(torch.uint16).numpy(), W.view(torch.uint16).numpy(), np.arange(7),
                                 return_logits=True)
    assert np.array_equal(logits, want.astype(np.float32))       # fp64 sum rounded once: same bits


def test_reduce_vs_scipy():
    rng = np.random.default_rng(3)
    for V, scale in [(1, 1.0), (2, 1.0), (777, 1.0), (8192, 3.0), (5000, 30.0)]:
        x = (rng.standard_normal(V) * scale).astype(np.float32)
        tok, conf, lse, gap, mx = oracle.row_reduce(x)
        xd = x.astype(np.float64)
        assert tok == int(np.argmax(xd))
        assert lse == pytest.approx(float(logsumexp(xd)), abs=1e-6 * max(1.0, abs(float(logsumexp(xd)))))
        assert conf == pytest.approx(float(softmax(xd).max()), rel=2e-6)
        assert mx == x.max()
        if V > 1:
            srt = np.sort(xd)
            assert gap == pytest.approx(float(srt[-1] - srt[-2]), abs=1e-6)
        else:
            assert math.isinf(gap)


# ---------------------------------------------------------------- closed forms
def golden_lnV():
    out = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#") and not line.startswith("philox"):
            v, l = line.split()
            out[int(v)] = float(l)
    return out


@pytest.mark.parametrize("V", [8192, 126464, 152064])
def test_constant_row_gives_lnV(V):
    lnV = golden_lnV()[V]
    x = np.zeros(V, np.float32)
    tok, conf, lse, gap, mx = oracle.row_reduce(x)
    assert tok == 0 and gap == 0.0 and mx == 0.0
    assert lse == pytest.approx(lnV, abs=2e-6) and conf == pytest.approx(1.0 / V, rel=1e-6)
    tok, conf, lse, gap, mx = oracle.row_reduce(x + np.float32(-3.25))
    assert tok == 0 and lse == pytest.approx(-3.25 + lnV, abs=2e-6) and conf == pytest.approx(1.0 / V, rel=1e-6)


def test_zero_hidden_row_and_identical_w_rows():
    V, d = 8192, 64
    W = rand_bf16((V, d), 0.125, 5).view(torch.uint16).numpy()
    H = np.zeros((1, d), np.uint16)
    r = oracle.positions(H, W, [0])
    assert r.tok[0] == 0 and r.lse[0] == pytest.approx(golden_lnV()[V], abs=2e-6)
    w_row = rand_bf16((1, d), 0.125, 6)
    h = rand_bf16((1, d), 1.0, 7)
    c = float((h.double() @ w_row.double().T).item())
    Wsame = w_row.repeat(V, 1).view(torch.uint16).numpy()
    r = oracle.positions(h.view(torch.uint16).numpy(), Wsame, [0])
    assert r.tok[0] == 0 and r.gap[0] == 0.0
    assert r.lse[0] == pytest.approx(c + golden_lnV()[V], abs=2e-6 * max(1, abs(c)))
    assert r.conf[0] == pytest.approx(1.0 / V, rel=1e-6)


@pytest.mark.parametrize("vstar", [0, 1, 255, 256, 4095, 8191])
@pytest.mark.parametrize("a", [2.0, 9.0, 20.0])
def test_planted_dominant_logit(vstar, a):
    V, d = 8192, 8
    H = np.zeros((1, d), np.float32); H[0, 3] = 1.0
    W = np.zeros((V, d), np.float32); W[vstar, 3] = a
    W[:, 5] = 7.0                                                 # multiplies a zero of h: must not leak in
    r = oracle.positions(bits(H), bits(W), [0])
    s = math.exp(a) + V - 1
    assert r.tok[0] == vstar and r.rowmax[0] == a and r.gap[0] == pytest.approx(a)
    assert r.lse[0] == pytest.approx(math.log(s), abs=2e-6)
    assert r.conf[0] == pytest.approx(math.exp(a) / s, rel=1e-6)


@pytest.mark.parametrize("gap", [0.0, 0.0078125, 0.03125])
def test_two_valued_rows_gap_and_tie(gap):
    """Top value at ids 5 and (if gap==0) also 3: lowest id must win, gap must be exact."""
    V = 1000
    x = np.full(V, -1.0, np.float32)
    x[5] = 1.0
    x[3] = 1.0 - gap
    tok, conf, lse, g, mx = oracle.row_reduce(x)
    assert tok == (3 if gap == 0.0 else 5)
    assert g == np.float32(gap)
    s = 1.0 + math.exp(-gap) + (V - 2) * math.exp(-2.0)
    assert lse == pytest.approx(1.0 + math.log(s), abs=2e-6) and conf == pytest.approx(1.0 / s, rel=1e-6)


# ---------------------------------------------------------------- exact invariances
def test_power_of_two_scaling_and_row_permutation():
    H = rand_bf16((3, 128), 1.0, 11)
    W = rand_bf16((700, 128), 128 ** -0.5, 12)
    Hb, Wb = H.view(torch.uint16).numpy(), W.view(torch.uint16).numpy()
    r1, l1 = oracle.positions(Hb, Wb, [0, 1, 2], return_logits=True)
    r2, l2 = oracle.positions((H * 4).view(torch.uint16).numpy(), Wb, [0, 1, 2], return_logits=True)
    assert np.array_equal(l2, l1 * 4) and np.array_equal(r1.tok, r2.tok)
    perm = np.random.default_rng(0).permutation(700)
    r3, l3 = oracle.positions(Hb, Wb[perm], [0, 1, 2], return_logits=True)
    assert np.array_equal(l3, l1[:, perm])
    assert np.array_equal(perm[r3.tok], r1.tok)
    assert np.allclose(r3.lse, r1.lse, atol=1e-6) and np.allclose(r3.conf, r1.conf, rtol=1e-6)


def test_full_then_select_is_restriction_and_independent_of_other_rows():
    H = rand_bf16((40, 64), 1.0, 21)
    W = rand_bf16((300, 64), 0.125, 22)
    Hb, Wb = H.view(torch.uint16).numpy(), W.view(torch.uint16).numpy()
    rng = np.random.default_rng(2)
    mask = (rng.random(40) < 0.4).astype(np.uint8)
    idx, sel = oracle.full_then_select(Hb, Wb, mask)
    assert idx.tolist() == [t for t in range(40) if mask[t]]
    allr = oracle.positions(Hb, Wb, np.arange(40))
    for name in ("tok", "conf", "lse", "gap", "rowmax"):
        assert np.array_equal(getattr(sel, name), getattr(allr, name)[idx]), name
    # every selected row equals the direct definition on that row alone (numpy fp64, library matmul)
    x = (H.double() @ W.double().T).numpy().astype(np.float32).astype(np.float64)
    assert np.array_equal(sel.tok, x.argmax(1)[idx])
    assert np.allclose(sel.lse, logsumexp(x, axis=1)[idx], atol=1e-6)
    # changing unmasked rows changes nothing
    H2 = H.clone(); H2[torch.from_numpy(mask == 0)] = 0
    idx2, sel2 = oracle.full_then_select(H2.view(torch.uint16).numpy(), Wb, mask)
    assert np.array_equal(idx2, idx) and np.array_equal(sel2.lse, sel.lse) and np.array_equal(sel2.tok, sel.tok)
    # empty and full masks
    idx0, sel0 = oracle.full_then_select(Hb, Wb, np.zeros(40, np.uint8))
    assert idx0.size == 0 and sel0.tok.size == 0
    idx1, sel1 = oracle.full_then_select(Hb, Wb, np.ones(40, np.uint8))
    assert np.array_equal(idx1, np.arange(40)) and np.array_equal(sel1.lse, allr.lse)


def test_statistics_of_gaussian_logits():
    """Not parity: a sanity check that the tiny workload's logits look like N(0,1) rows, so that
    E[lse] ~ ln V + 1/2 and the row maximum sits near sqrt(2 ln V)."""
    from paper_2601_06562_amd import workloads
    wl = workloads.make("tiny")
    r = oracle.positions(workloads.bf16_bits(wl.hidden), workloads.bf16_bits(wl.w), np.arange(0, 512, 8))
    assert abs(float(r.lse.mean()) - (math.log(8192) + 0.5)) < 0.15
    assert 3.2 < float(r.rowmax.mean()) < 4.6


# ---------------------------------------------------------------- sampling tail (next row of the path)
def test_unmask_topn_against_sorting_and_invariants():
    """Pin: a stable sort by (-confidence, position) per sequence is the same selection; the rest of the
    state must be untouched; duplicates of the confidence exercise the tie rule."""
    rng = np.random.default_rng(4)
    T, B = 300, 3
    seq_starts = np.array([0, 100, 180, 300], np.int32)
    mask = (rng.random(T) < 0.4).astype(np.uint8)
    idx = np.nonzero(mask)[0].astype(np.int32)
    conf = rng.choice(np.array([0.1, 0.25, 0.5, 0.75, 0.9], np.float32), idx.size)     # many ties
    tok = rng.integers(0, 1000, idx.size).astype(np.int32)
    tokens = np.full(T, -1, np.int32)
    n_per_seq = np.array([5, 0, 1000], np.int32)                                        # some, none, all
    new_tokens, new_mask, n = oracle.unmask_topn(conf, tok, idx, seq_starts, n_per_seq, tokens, mask)
    want_tokens, want_mask, total = tokens.copy(), mask.copy(), 0
    for b in range(B):
        rows = [j for j in range(idx.size) if seq_starts[b] <= idx[j] < seq_starts[b + 1]]
        rows.sort(key=lambda j: (-float(conf[j]), int(idx[j])))
        for j in rows[:n_per_seq[b]]:
            want_tokens[idx[j]] = tok[j]
            want_mask[idx[j]] = 0
            total += 1
    assert n == total and np.array_equal(new_tokens, want_tokens) and np.array_equal(new_mask, want_mask)
    assert np.array_equal(new_mask[100:180], mask[100:180])            # n = 0: sequence untouched
    assert new_mask[180:].sum() == 0                                   # n >= m: everything unmasked
    assert np.array_equal(tokens, np.full(T, -1, np.int32))            # inputs were not modified
    # hand case: confidences 0.5 at positions 2 and 7, 0.9 at 5 -> n = 2 takes 5 then 2 (lower position on the tie)
    t, m, _ = oracle.unmask_topn([0.5, 0.9, 0.5], [11, 22, 33], [2, 5, 7], [0, 10], [2], np.zeros(10, np.int32),
                                 np.array([0, 0, 1, 0, 0, 1, 0, 1, 0, 0], np.uint8))
    assert t.tolist() == [0, 0, 11, 0, 0, 22, 0, 0, 0, 0] and m.tolist() == [0, 0, 0, 0, 0, 0, 0, 1, 0, 0]


def test_shift_indices_definition():
    idx = np.array([0, 1, 5, 9, 10, 11, 19], np.int32)
    got = oracle.shift_indices(idx, np.array([0, 10, 20], np.int32))
    assert got.tolist() == [0, 0, 4, 8, 10, 10, 18]                   # sequence starts 0 and 10 keep their own row
    assert oracle.shift_indices(np.array([], np.int32), np.array([0, 4], np.int32)).size == 0


# ---------------------------------------------------------------- sampling with temperature
def test_philox_known_answers():
    n = 0
    for line in open(GOLDEN):
        if line.startswith("philox"):
            w = [int(x, 16) for x in line.split()[1:]]
            assert oracle.philox4x32_10(w[0:4], w[4:6]).tolist() == w[6:10]
            n += 1
    assert n == 3


def test_uniform_and_gumbel_statistics():
    u = np.array([oracle.uniform(12345, t, v) for t in range(40) for v in range(500)])
    assert u.min() > 0 and u.max() < 1
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.003
    g = -np.log(-np.log(u))
    assert abs(g.mean() - 0.5772156649) < 0.03 and abs(g.var() - math.pi ** 2 / 6) < 0.08
    assert oracle.gumbel(12345, 3, 77) == pytest.approx(-math.log(-math.log(oracle.uniform(12345, 3, 77))), abs=1e-12)
    # a pure function of (seed, position, id); the three really are distinct axes
    assert oracle.uniform(1, 2, 3) == oracle.uniform(1, 2, 3)
    assert len({oracle.uniform(1, 2, 3), oracle.uniform(2, 2, 3), oracle.uniform(1, 3, 3), oracle.uniform(1, 2, 4)}) == 4


def test_uniform_counter_layout_and_gumbel_inverse_cdf():
    """The uniform is word v % 4 of the (separately pinned) Philox block at counter (v / 4, position, 0, 0) under the
    key (seed low, seed high), reduced to 23 bits plus one half; the Gumbel variate is the one whose distribution
    function exp(-exp(-g)) gives that uniform back."""
    seed = 0x0123456789ABCDEF
    for position, v in ((0, 0), (5, 3), (5, 4), (77, 126463), (2 ** 31 - 1, 6), (131071, 152063)):
        words = oracle.philox4x32_10([v // 4, position, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])
        u = oracle.uniform(seed, position, v)
        k = u * 2 ** 23 - 0.5
        assert k == int(k) and 0 <= k < 2 ** 23                   # 23 bits, never 0 or 1
        assert int(k) == int(words[v % 4]) >> 9
        g = oracle.gumbel(seed, position, v)
        assert math.exp(-math.exp(-g)) == pytest.approx(u, rel=1e-12)
    # the four ids of one counter block take the four words in order, the next id starts a new block
    block = oracle.philox4x32_10([10, 9, 0, 0], [1, 0])
    assert [int(oracle.uniform(1, 9, 40 + j) * 2 ** 23 - 0.5) for j in range(4)] == [int(w) >> 9 for w in block]
    assert int(oracle.uniform(1, 9, 44) * 2 ** 23 - 0.5) == int(oracle.philox4x32_10([11, 9, 0, 0], [1, 0])[0]) >> 9


def test_sampling_reduces_to_greedy_and_follows_softmax():
    rng = np.random.default_rng(8)
    x = rng.standard_normal(300).astype(np.float32)
    tok0, conf0, lse0, _, _ = oracle.row_reduce(x)
    tok, conf, lse, gap = oracle.row_sample(x, 0.0, 99, 5)
    assert (tok, conf, lse) == (tok0, conf0, lse0)                       # tau = 0 is the greedy rule
    # Gumbel-max with noise scaled by tau draws from softmax(x / tau): frequencies over many positions
    x4 = np.array([1.0, 0.0, -1.0, 0.5], np.float32)
    for tau in (1.0, 2.0):
        p = np.exp(x4 / tau) / np.exp(x4 / tau).sum()
        picks = np.array([oracle.row_sample(x4, tau, 7, t)[0] for t in range(6000)])
        freq = np.bincount(picks, minlength=4) / picks.size
        assert np.abs(freq - p).max() < 0.025, (tau, freq, p)
    # confidence is the soft-max probability of the token actually picked, lse is unperturbed
    tok, conf, lse, _ = oracle.row_sample(x4, 1.0, 7, 11)
    assert lse == pytest.approx(float(logsumexp(x4.astype(np.float64))), abs=1e-6)
    assert conf == pytest.approx(float(np.exp(x4[tok] - logsumexp(x4.astype(np.float64)))), rel=1e-6)
    # brute force of the definition on one row
    y = [float(x4[v]) + 1.0 * oracle.gumbel(7, 11, v) for v in range(4)]
    assert tok == int(np.argmax(y))
