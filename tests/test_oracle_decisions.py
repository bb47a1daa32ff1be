"""Pins for the oracle's decision stage (accept test, local expansion, residual
resampling, up-sampling, uniforms) against what the paper and the mathematics
fix.  CPU only."""
import itertools
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import scipy.stats

from oracle import accept as A
from oracle import local as LOC
from oracle import philox as PH
from oracle import resample as RS
from oracle import step as ST
from oracle import upsample as UP


# ------------------------------------------------------------------ uniforms
def test_philox_is_philox4x32_10_by_its_published_known_answers():
    """The generator's identity: the three known-answer vectors published with the reference implementation of
    Salmon et al. (SC'11) for philox4x32 with 10 rounds (tests/golden/philox4x32_10_known_answers.txt).  A wrong
    multiplier, Weyl constant, round count or output-word order fails all 12 words."""
    import os
    path = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_known_answers.txt")
    rows = [[int(x, 16) for x in line.split()] for line in open(path) if line.strip() and not line.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        out = PH.philox4x32(r[0], r[1], r[2], r[3], r[4], r[5])
        assert [int(o) for o in out] == r[6:10]
    # the vectorised path gives the same words as the scalar one
    c = np.array([r[:4] for r in rows], dtype=np.uint64)
    for i, r in enumerate(rows):
        out = PH.philox4x32(c[:, 0], c[:, 1], c[:, 2], c[:, 3], r[4], r[5])
        assert [int(o[i]) for o in out] == r[6:10]


def test_philox_zero_rounds_is_identity_and_rounds_matter():
    c = [np.arange(5), np.arange(5) + 7, 3, 9]
    out0 = PH.philox4x32(*c, 11, 22, rounds=0)
    assert [o.tolist() for o in out0] == [list(range(5)), list(range(7, 12)), [3] * 5, [9] * 5]
    o9 = PH.philox4x32(*c, 11, 22, rounds=9)
    o10 = PH.philox4x32(*c, 11, 22, rounds=10)
    assert not np.array_equal(o9[0], o10[0])


def test_philox_uniformity_and_moments():
    w = PH.step_words(seed=0, rng_counter=0, stream=0, B=4, L=1 << 18).ravel()
    # chi-square over the top 8 bits
    counts = np.bincount(w >> 24, minlength=256)
    chi2 = ((counts - w.size / 256) ** 2 / (w.size / 256)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 255)
    # and over the bottom 8 bits
    counts = np.bincount(w & 0xFF, minlength=256)
    chi2 = ((counts - w.size / 256) ** 2 / (w.size / 256)).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, 255)
    u = PH.uniform24(w).astype(np.float64)
    assert abs(u.mean() - 0.5) < 5 / np.sqrt(12 * w.size)
    assert abs(u.var() - 1 / 12) < 1e-3
    assert u.min() >= 0.0 and u.max() <= 1 - 2.0 ** -24
    # serial correlation between neighbouring counters
    assert abs(np.corrcoef(u[:-1], u[1:])[0, 1]) < 5 / np.sqrt(w.size)


def test_philox_avalanche_and_stream_separation():
    base = PH.philox4x32(np.arange(4096), 0, 5, 0, 1, 2)[0]
    for word, bit in [(0, 12), (1, 0), (2, 31), (3, 24)]:
        c = [np.arange(4096), 0, 5, 0]
        c[word] = np.asarray(c[word]) ^ (1 << bit)
        flipped = PH.philox4x32(*c, 1, 2)[0]
        frac = np.unpackbits((base ^ flipped).view(np.uint8)).mean()
        assert 0.48 < frac < 0.52
    a = PH.step_words(3, 9, PH.STREAM_ACCEPT, 2, 4096)
    s = PH.step_words(3, 9, PH.STREAM_SAMPLE, 2, 4096)
    assert (a == s).mean() < 0.01
    assert not np.array_equal(a, PH.step_words(3, 10, PH.STREAM_ACCEPT, 2, 4096))
    assert not np.array_equal(a, PH.step_words(4, 9, PH.STREAM_ACCEPT, 2, 4096))


def test_philox_counter_independence():
    full = PH.step_words(7, 1 << 33, 1, 3, 100)
    # the word of (b, t) does not depend on which other positions are generated
    sub = PH.step_words(7, 1 << 33, 1, 2, 40)
    assert np.array_equal(full[:2, :40], sub)
    c3 = (1 << 24) | 2
    one = PH.philox4x32(17, 2, 0, c3, 7, 0)[0]
    assert one == full[2, 17]


def test_uniform24_exact_values():
    assert PH.uniform24(np.uint32(0)) == 0.0
    assert PH.uniform24(np.uint32(0xFFFFFFFF)) == np.float32(1 - 2.0 ** -24)
    assert PH.uniform24(np.uint32(0x80000000)) == 0.5
    assert PH.uniform24(np.uint32(0x000000FF)) == 0.0        # low 8 bits are dropped


# --------------------------------------------------------------- up-sampling
def test_upsample_rows_sum_to_one_and_children_equal_parent():
    rng = np.random.default_rng(0)
    B, h, w, r, V = 2, 3, 5, 2, 37
    logits = rng.normal(0, 2, (B, h * w, V)).astype(np.float32)
    toks = rng.integers(0, V, (B, h * w))
    x_hi, q_lo, q_row, q_hi = UP.upsample_draft(logits, toks, h, w, r, materialise=True)
    assert np.abs(q_lo.astype(np.float64).sum(-1) - 1).max() < 1e-6
    assert np.abs(UP.softmax_rows(logits).sum(-1) - 1).max() < 1e-12
    H, W = r * h, r * w
    # brute-force parent map, written with loops
    for i in range(H):
        for j in range(W):
            u = i * W + j
            par = (i // r) * w + (j // r)
            assert q_row[u] == par
            assert np.array_equal(q_hi[:, u], q_lo[:, par])
            assert np.array_equal(x_hi[:, u], toks[:, par])
    # r x r children are constant
    g = x_hi.reshape(B, h, r, w, r)
    assert (g == g[:, :, :1, :, :1]).all()
    assert x_hi.shape == (B, H * W) and q_hi.shape == (B, H * W, V)


def test_upsample_softmax_matches_library_and_closed_forms():
    rng = np.random.default_rng(1)
    z = rng.normal(0, 3, (4, 9, 64))
    _, q_lo, _, _ = UP.upsample_draft(z, np.zeros((4, 9), int), 3, 3, 2)
    assert np.abs(q_lo - scipy.special.softmax(z, axis=-1)).max() < 1e-7
    # constant logits -> uniform; a shift of the logits changes nothing; huge logits do not overflow
    _, q_c, _, _ = UP.upsample_draft(np.full((1, 1, 10), 3.5), [[0]], 1, 1, 2)
    assert np.allclose(q_c, 0.1, atol=1e-8)
    _, q_s, _, _ = UP.upsample_draft(z + 1000.0, np.zeros((4, 9), int), 3, 3, 2)
    assert np.abs(q_s - q_lo).max() < 1e-6
    # two-entry softmax is the logistic function
    _, q2, _, _ = UP.upsample_draft([[[0.0, 1.5]]], [[0]], 1, 1, 1)
    assert abs(q2[0, 0, 1] - 1 / (1 + np.exp(-1.5))) < 1e-7


def test_upsample_r1_is_identity_and_probs_are_copied():
    rng = np.random.default_rng(2)
    probs = rng.dirichlet(np.ones(8), (2, 6)).astype(np.float32)
    toks = rng.integers(0, 8, (2, 6))
    x_hi, q_lo, q_row, q_hi = UP.upsample_draft(probs, toks, 2, 3, 1, input_is_probs=True,
                                                materialise=True)
    assert np.array_equal(x_hi, toks) and np.array_equal(q_row, np.arange(6))
    assert np.array_equal(q_lo, probs) and np.array_equal(q_hi, probs)


# --------------------------------------------------------------- accept test
def test_q_equal_p_accepts_everything():
    rng = np.random.default_rng(3)
    logits = rng.normal(0, 2, (3, 64, 50)).astype(np.float32)
    p = A.target_probs(logits)
    toks = rng.integers(0, 50, (3, 64))
    out = ST.decide(logits, p, None, toks, W=8, n0=0, radius=1, seed=5, rng_counter=2)
    assert out["accept"].all() and not out["mask"].any()
    assert (out["t0"] == 64).all() and np.array_equal(out["tokens_out"], toks)
    # also for the largest uniform the generator can emit
    assert A.accept_test(p[0, 0], p[0, 0], np.float32(1 - 2.0 ** -24)).all()


def test_accept_probability_is_min_one_p_over_q_by_exact_count():
    # all 2^24 uniforms the generator can emit: the accepted count is exactly the closed form
    u = (np.arange(1 << 24, dtype=np.uint32).astype(np.float32) * np.float32(2.0 ** -24))
    for pv, qv in [(0.25, 0.5), (0.3, 0.1), (0.1, 0.7), (1e-5, 3e-3), (0.2, 0.2), (0.0, 0.3), (0.3, 0.0)]:
        pv32, qv32 = np.float32(pv), np.float32(qv)
        n = int(A.accept_test(pv32, qv32, u).sum())
        want = 1.0 if qv == 0 and pv > 0 else (0.0 if pv == 0 else min(1.0, float(pv32) / float(qv32)))
        assert abs(n / 2 ** 24 - want) <= 2.0 ** -23, (pv, qv, n)
    # monotone in u
    acc = A.accept_test(np.float32(0.25), np.float32(0.5), u)
    assert not np.any(np.diff(acc.astype(np.int8)) > 0)


def test_pooling_k1_equals_unpooled_and_full_pool_is_one():
    rng = np.random.default_rng(4)
    V = 32
    p = A.target_probs(rng.normal(0, 2, (10, V)))
    toks = rng.integers(0, V, 10)
    ident = np.arange(V, dtype=np.int32)[:, None]
    assert np.array_equal(A.pooled_mass(p, toks, None), A.pooled_mass(p, toks, ident))
    assert np.array_equal(A.pooled_mass(p, toks, None), p[np.arange(10), toks])
    full = np.stack([np.roll(np.arange(V), -x) for x in range(V)]).astype(np.int32)  # nbr[x,0]=x
    assert np.allclose(A.pooled_mass(p, toks, full), 1.0, atol=1e-6)
    # a hand-checked pooled sum
    nbr = np.array([[0, 2], [1, 0], [2, 1]], dtype=np.int32)
    pp = np.array([[0.5, 0.125, 0.375]], dtype=np.float32)
    assert A.pooled_mass(pp, [2], nbr)[0] == np.float32(0.5)       # p[2] + p[1]
    # pooling can only raise acceptance
    k4 = np.stack([np.roll(np.arange(V), -x)[:4] for x in range(V)]).astype(np.int32)
    assert (A.pooled_mass(p, toks, k4) >= A.pooled_mass(p, toks, None)).all()


# ------------------------------------------------- exactness of Eq. 1 + Eq. 2
def _sampler_law(Wi):
    """Exact law of oracle.resample.draw over all 2^32 words, as Fractions, from
    the closed form #words{T(word) < c} = ceil(c 2^32 / tot)."""
    cdf = np.cumsum(Wi, dtype=np.uint64)
    tot = int(cdf[-1])
    below = lambda c: -((-c * (1 << 32)) // tot)
    law, lo = [], 0
    for x in range(len(Wi)):
        hi = int(cdf[x])
        law.append(Fraction(below(hi) - below(lo), 1 << 32))
        lo = hi
    return law, tot


@pytest.mark.parametrize("V,seed", [(2, 0), (3, 1), (5, 2), (8, 3), (8, 4)])
def test_accept_plus_residual_reproduces_target_law(V, seed):
    """Sec. 3.1: accepting with min(1, p/q) and re-drawing rejections from
    norm(max(0, p - q)) samples exactly from p.  Enumerate the draft token."""
    rng = np.random.default_rng(seed)
    p = A.target_probs(rng.normal(0, 1.5, V))
    q = A.target_probs(rng.normal(0, 1.5, V))
    # acceptance probability of each draft token through the oracle's own rule, counted on a u grid
    u = (np.arange(1 << 20, dtype=np.uint32).astype(np.float32) * np.float32(2.0 ** -20))
    acc = np.array([A.accept_test(p[x], q[x], u).mean() for x in range(V)])
    law, _ = _sampler_law(RS.residual_weights(p, q))
    res = np.array([float(f) for f in law])
    out = q.astype(np.float64) * acc + (1 - (q.astype(np.float64) * acc).sum()) * res
    assert np.abs(out - p).max() < 3e-6
    # the residual itself against its definition evaluated in exact rationals
    pf = [Fraction(float(v)) for v in p]
    qf = [Fraction(float(v)) for v in q]
    r = [max(Fraction(0), a - b) for a, b in zip(pf, qf)]
    tot = sum(r)
    assert max(abs(float(ri / tot) - res[i]) for i, ri in enumerate(r)) < 1e-6


def test_draw_boundaries_closed_form_and_word_count():
    rng = np.random.default_rng(6)
    p = A.target_probs(rng.normal(0, 2, 8))
    q = A.target_probs(rng.normal(0, 2, 8))
    Wi = RS.residual_weights(p, q)
    law, tot = _sampler_law(Wi)
    assert sum(law) == 1
    cdf = np.cumsum(Wi, dtype=np.uint64)
    # share of words within +-1 word of W/tot
    for x in range(8):
        assert abs(law[x] * (1 << 32) - Fraction(int(Wi[x]) * (1 << 32), tot)) <= 1
    # first word of every non-empty cell maps to that cell, the word before to an earlier cell
    lo = 0
    for x in range(8):
        hi = int(cdf[x])
        if Wi[x] > 0:
            first = -((-lo * (1 << 32)) // tot)
            if first < (1 << 32):
                assert RS.draw(Wi, first) == x
                if first > 0:
                    assert RS.draw(Wi, first - 1) < x
        lo = hi
    assert RS.draw(Wi, 0) == int(np.flatnonzero(Wi)[0])
    assert RS.draw(Wi, 0xFFFFFFFF) == int(np.flatnonzero(Wi)[-1])
    # zero-weight tokens are never drawn
    words = PH.step_words(0, 0, 1, 1, 4096)[0]
    drawn = {RS.draw(Wi, w) for w in words}
    assert all(Wi[x] > 0 for x in drawn)


def test_sampler_chi_square_against_residual():
    rng = np.random.default_rng(7)
    p = A.target_probs(rng.normal(0, 1, 8))
    q = A.target_probs(rng.normal(0, 1, 8))
    Wi = RS.residual_weights(p, q)
    words = PH.step_words(11, 3, PH.STREAM_SAMPLE, 8, 125000).ravel()           # 10^6 draws
    cdf = np.cumsum(Wi, dtype=np.uint64)
    tot = int(cdf[-1])
    draws = np.array([RS.threshold(w, tot) for w in words[:20000]], dtype=np.uint64)
    # vectorised route for the rest: T = word*th + ((word*tl) >> 32) is the same integer
    th, tl = tot >> 32, tot & 0xFFFFFFFF
    Tv = words.astype(np.uint64) * np.uint64(th) + ((words.astype(np.uint64) * np.uint64(tl)) >> np.uint64(32))
    assert np.array_equal(Tv[:20000], draws)
    x = np.searchsorted(cdf, Tv, side="right")
    assert np.array_equal(x[:200], [RS.draw(Wi, w) for w in words[:200]])
    counts = np.bincount(x, minlength=8).astype(np.float64)
    expect = Wi.astype(np.float64) / tot * words.size
    keep = expect > 0
    assert counts[~keep].sum() == 0
    chi2 = ((counts[keep] - expect[keep]) ** 2 / expect[keep]).sum()
    assert chi2 < scipy.stats.chi2.ppf(1 - 1e-6, keep.sum() - 1)


def test_residual_special_cases():
    p = np.array([0.5, 0.25, 0.25], dtype=np.float32)
    # hand example: p - q = (0.25, -0.25, 0) -> all residual mass on token 0
    q = np.array([0.25, 0.5, 0.25], dtype=np.float32)
    Wi = RS.residual_weights(p, q)
    assert Wi.tolist() == [1 << 38, 0, 0]
    assert all(RS.draw(Wi, w) == 0 for w in (0, 1, 0x7FFFFFFF, 0xFFFFFFFF))
    # q == p: residual is empty -> falls back to p; the split of the words is p itself
    Wi = RS.residual_weights(p, p)
    assert Wi.tolist() == [1 << 39, 1 << 38, 1 << 38]
    assert RS.draw(Wi, 0x7FFFFFFF) == 0 and RS.draw(Wi, 0x80000000) == 1
    assert RS.draw(Wi, 0xBFFFFFFF) == 1 and RS.draw(Wi, 0xC0000000) == 2
    # integer weights are exact scalings
    assert RS.integer_weights(np.float32(2.0 ** -40)) == 1
    assert RS.integer_weights(np.float32(2.0 ** -41)) == 0
    assert RS.integer_weights(np.float32(1.0)) == 1 << 40
    # unmarked positions keep the draft token; marked ones are re-drawn
    out = RS.resample_block(np.stack([p, p]), np.stack([q, q]), [0, 1], [2, 2], [0, 1], [1, 0],
                            np.array([5, 5], dtype=np.uint32))
    assert out.tolist() == [2, 0]
    # mode 1: an accepted-but-marked position draws from p, not from the residual
    words = PH.step_words(0, 0, 1, 1, 2000)[0]
    outs = {int(RS.resample_block(p[None], q[None], [0], [2], [1], [1], np.array([w]), mode=1)[0])
            for w in words}
    assert outs == {0, 1, 2}
    outs0 = {int(RS.resample_block(p[None], q[None], [0], [2], [1], [1], np.array([w]), mode=0)[0])
             for w in words[:200]}
    assert outs0 == {0}


# -------------------------------------------------------- local expansion
def _brute_RX(accept, H, W, n0, L, l):
    """Eq. 6-7 by constructing every neighbourhood cell by cell."""
    rej = [t for t in range(L) if not accept[t]]
    if not rej:
        return set(), L
    t0 = rej[0]
    RX = set()
    for t in rej:
        it, jt = divmod(n0 + t, W)
        for di in range(-l, l + 1):
            for dj in range(-l, l + 1):
                i, j = it + di, jt + dj
                if 0 <= i < H and 0 <= j < W:
                    u = i * W + j - n0
                    if 0 <= u < L and u >= t0:
                        RX.add(u)
    return RX, t0


def test_local_mask_exhaustive_small_grids():
    for H, W in [(2, 2), (3, 4), (4, 3), (2, 6)]:
        L = H * W
        for bits in range(1 << L):
            acc = np.array([(bits >> t) & 1 for t in range(L)], dtype=np.uint8)
            for l in (0, 1, 2):
                mask, t0 = LOC.local_mask(acc, W, 0, l)
                RX, bt0 = _brute_RX(acc, H, W, 0, L, l)
                assert t0 == bt0
                assert set(np.flatnonzero(mask)) == RX


def test_local_mask_random_blocks_and_properties():
    rng = np.random.default_rng(8)
    H = W = 16
    for trial in range(60):
        rows = int(rng.choice([2, 4, 8, 16]))
        L = rows * W
        n0 = int(rng.integers(0, (H - rows) // rows + 1)) * rows * W if rows < H else 0
        acc = (rng.random(L) < rng.choice([0.5, 0.9, 0.98])).astype(np.uint8)
        prev = None
        for l in (0, 1, 2, 3):
            mask, t0 = LOC.local_mask(acc, W, n0, l)
            RX, bt0 = _brute_RX(acc, H, W, n0, L, l)
            assert t0 == bt0 and set(np.flatnonzero(mask)) == RX
            rej = np.flatnonzero(acc == 0)
            assert mask[rej].all()                                  # R_T is inside R_X
            assert not mask[:t0].any()                              # nothing before t0
            if l == 0:
                assert np.array_equal(mask, (acc == 0).astype(np.uint8))   # naive local verification
            if prev is not None:
                assert (mask >= prev).all()                         # monotone in the radius
            prev = mask
        # dilating e times by l equals once by e*l
        m21, _ = LOC.local_mask(acc, W, n0, 1, expand=2)
        m12, _ = LOC.local_mask(acc, W, n0, 2, expand=1)
        assert np.array_equal(m21, m12)
        # a radius that covers the grid is the raster-scan rule, and so is radius -1
        big, t0 = LOC.local_mask(acc, W, n0, 64)
        ras, _ = LOC.local_mask(acc, W, n0, -1)
        assert np.array_equal(big, ras)
        assert np.array_equal(ras, (np.arange(L) >= t0).astype(np.uint8))
        # monotone in R_T
        acc2 = acc.copy()
        acc2[rng.integers(0, L)] = 0
        m_a, _ = LOC.local_mask(acc, W, n0, 1)
        m_b, t0b = LOC.local_mask(acc2, W, n0, 1)
        assert (m_b[max(t0, 0):] >= m_a[max(t0, 0):]).all()


def test_local_mask_no_column_wrap_and_hand_example():
    # 4x4 grid, one rejection at the end of row 1 (index 7): radius 1 must not
    # wrap onto column 0 of rows 1-2 (indices 8 stays out, 4 is before t0)
    acc = np.ones(16, dtype=np.uint8)
    acc[7] = 0
    mask, t0 = LOC.local_mask(acc, 4, 0, 1)
    assert t0 == 7
    assert set(np.flatnonzero(mask)) == {7, 10, 11}
    # all accepted
    mask, t0 = LOC.local_mask(np.ones(16, dtype=np.uint8), 4, 0, 1)
    assert t0 == 16 and not mask.any()
    # block offset: second block of two rows in a 4x4 grid, rejection at block position 1
    acc = np.ones(8, dtype=np.uint8)
    acc[1] = 0
    mask, t0 = LOC.local_mask(acc, 4, 8, 1)
    assert set(np.flatnonzero(mask)) == {1, 2, 4, 5, 6}


# --------------------------------------------------------------- whole decision stage
def test_decide_consistency_and_stats():
    rng = np.random.default_rng(9)
    B, H, W, V = 2, 8, 8, 64
    L = H * W
    zp = rng.normal(0, 1.3, (B, L, V)).astype(np.float32)
    zq = zp + rng.normal(0, 1.0, (B, L, V)).astype(np.float32)
    q = A.target_probs(zq)
    toks = np.stack([[rng.choice(V, p=q[b, t].astype(np.float64) / q[b, t].sum(dtype=np.float64))
                      for t in range(L)] for b in range(B)])
    out = ST.decide(zp, q, None, toks, W=W, n0=0, radius=1, seed=1, rng_counter=4)
    acc, mask = out["accept"].astype(bool), out["mask"].astype(bool)
    assert 0.3 < acc.mean() < 0.9
    assert np.array_equal(out["stats"][:, 0], acc.sum(1))
    assert np.array_equal(out["stats"][:, 0] + out["stats"][:, 1], [L, L])
    assert np.array_equal(out["stats"][:, 2], mask.sum(1))
    assert np.array_equal(out["tokens_out"][~mask], toks[~mask])
    for b in range(B):
        rej = np.flatnonzero(~acc[b])
        assert out["t0"][b] == (rej[0] if rej.size else L)
        # a re-drawn token of a rejected position has positive residual weight
        for u_ in np.flatnonzero(mask[b]):
            x = out["tokens_out"][b, u_]
            assert out["p"][b, u_, x] > q[b, u_, x] or (out["p"][b, u_] <= q[b, u_]).all()
    # different rng counter -> different decisions; same counter -> identical
    again = ST.decide(zp, q, None, toks, W=W, n0=0, radius=1, seed=1, rng_counter=4)
    other = ST.decide(zp, q, None, toks, W=W, n0=0, radius=1, seed=1, rng_counter=5)
    assert np.array_equal(again["tokens_out"], out["tokens_out"])
    assert not np.array_equal(other["accept"], out["accept"])


def test_acceptance_rate_closed_form_large_vocab():
    """For i.i.d. target logits and q = softmax(z_p + sigma*eps) with x~ ~ q the
    expected acceptance is 1 - TV(p, q) ~ 2 Phi(-sigma/2) for a large codebook."""
    rng = np.random.default_rng(10)
    V, n = 4096, 400
    for sigma in (0.5, 1.0, 2.0):
        zp = rng.normal(0, 1.28, (1, n, V)).astype(np.float32)
        zq = zp + sigma * rng.normal(0, 1, (1, n, V)).astype(np.float32)
        q = A.target_probs(zq)
        cdf = np.cumsum(q[0].astype(np.float64), axis=1)
        toks = (cdf / cdf[:, -1:] > rng.random((n, 1))).argmax(axis=1)[None]
        out = ST.decide(zp, q, None, toks, W=20, n0=0, radius=0, seed=2, rng_counter=0)
        want = 2 * scipy.stats.norm.cdf(-sigma / 2)
        tv = 0.5 * np.abs(out["p"][0].astype(np.float64) - q[0]).sum(-1).mean()
        assert abs((1 - tv) - want) < 0.03
        assert abs(out["accept"].mean() - (1 - tv)) < 4 * np.sqrt(0.25 / n)


# ------------------------------------------------------------------ threshold rule (Eq. 5)
def test_tau_rule_hand_example_and_the_tie_is_accepted():
    # two-entry codebook, logits (0, ln 3): p = (1/4, 3/4) exactly representable
    z = np.array([[[0.0, np.log(3.0)], [0.0, np.log(3.0)], [0.0, 0.0], [0.0, 0.0]]], np.float32)
    toks = np.array([[0, 1, 0, 1]])
    out = ST.decide(z, None, None, toks, W=4, n0=0, radius=0, accept_mode=1, tau=0.3, mode=2)
    assert np.allclose(out["pbar"][0], [0.25, 0.75, 0.5, 0.5], atol=1e-7)
    assert out["accept"][0].tolist() == [0, 1, 1, 1]
    # Eq. 5 reads ">=": a pooled mass of exactly tau is accepted (a ">" would reject rows 2 and 3)
    out = ST.decide(z, None, None, toks, W=4, n0=0, radius=0, accept_mode=1, tau=0.5, mode=2)
    assert out["pbar"][0, 2] == np.float32(0.5) and out["accept"][0].tolist() == [0, 1, 1, 1]
    # pooling over both entries (k = V): mass 1 everywhere, everything accepted at any tau <= 1
    nbr = np.array([[0, 1], [1, 0]])
    out = ST.decide(z, None, None, toks, W=4, n0=0, radius=0, accept_mode=1, tau=0.99, mode=2, nbr=nbr)
    assert out["accept"].all() and (out["tokens_out"] == toks).all() and (out["t0"] == 4).all()


def test_tau_rule_limits_monotone_and_deterministic():
    rng = np.random.default_rng(21)
    B, H, W, V = 2, 6, 6, 96
    L = H * W
    z = rng.normal(0, 2.0, (B, L, V)).astype(np.float32)
    toks = rng.integers(0, V, (B, L))
    kw = dict(W=W, n0=0, radius=1, accept_mode=1, mode=2, seed=3)
    assert ST.decide(z, None, None, toks, tau=0.0, **kw)["accept"].all()          # pbar >= 0 always
    assert not ST.decide(z, None, None, toks, tau=1.5, **kw)["accept"].any()      # a probability never reaches 1.5
    prev = None
    for tau in (1e-4, 1e-3, 1e-2, 1e-1, 0.5):
        acc = ST.decide(z, None, None, toks, tau=tau, **kw)["accept"].astype(bool)
        if prev is not None:
            assert not (acc & ~prev).any()      # raising tau only removes accepted positions
        prev = acc
    # accepted set = {pbar >= tau} for the float64 softmax evaluated independently (scipy)
    p_ref = scipy.special.softmax(z.astype(np.float64), axis=-1)
    pt = np.take_along_axis(p_ref, toks[..., None], -1)[..., 0]
    out = ST.decide(z, None, None, toks, tau=1e-2, **kw)
    clear = np.abs(pt - 1e-2) > 1e-6
    assert np.array_equal(out["accept"].astype(bool)[clear], (pt >= 1e-2)[clear])
    # no random number enters the accept decision: it does not move with the counter ...
    a = ST.decide(z, None, None, toks, tau=1e-2, rng_counter=1, **kw)
    b = ST.decide(z, None, None, toks, tau=1e-2, rng_counter=2, **kw)
    assert np.array_equal(a["accept"], b["accept"]) and np.array_equal(a["mask"], b["mask"])
    # ... while the re-drawn tokens do
    assert not np.array_equal(a["tokens_out"], b["tokens_out"])


def test_tau_rule_marked_positions_are_drawn_from_the_target_distribution():
    # Step 6 of Alg. 1: a marked position gets a sample of p (mode 2), by the integer inverse CDF
    rng = np.random.default_rng(5)
    V, L = 40, 64
    z = rng.normal(0, 1.5, (1, L, V)).astype(np.float32)
    toks = rng.integers(0, V, (1, L))
    out = ST.decide(z, None, None, toks, W=8, n0=0, radius=0, accept_mode=1, tau=0.01, mode=2, seed=11, rng_counter=7)
    mask = out["mask"][0].astype(bool)
    assert mask.any() and not mask.all()
    for u_ in np.flatnonzero(mask):
        Wi = RS.integer_weights(out["p"][0, u_])
        assert out["tokens_out"][0, u_] == RS.draw(Wi, out["words"][0, u_])
    assert np.array_equal(out["tokens_out"][0][~mask], toks[0][~mask])
    # law of the draw: over many words the frequencies follow p (chi-square against p itself)
    p = out["p"][0, 0].astype(np.float64)
    Wi = RS.integer_weights(out["p"][0, 0])
    words = PH.step_words(123, 0, PH.STREAM_SAMPLE, 1, 20000)[0]
    cnt = np.bincount([RS.draw(Wi, w) for w in words], minlength=V)
    keep = p * len(words) > 5
    chi = ((cnt[keep] - p[keep] * len(words)) ** 2 / (p[keep] * len(words))).sum()
    assert chi < scipy.stats.chi2.ppf(0.9999, keep.sum() - 1)


def test_tau_rule_pooled_mass_with_neighbour_table():
    # pooled mass over k neighbours is the plain sum of those probabilities (Eq. 5 with B_k)
    rng = np.random.default_rng(8)
    V, L, k = 32, 16, 5
    z = rng.normal(0, 1.0, (1, L, V)).astype(np.float32)
    toks = rng.integers(0, V, (1, L))
    nbr = np.stack([np.concatenate([[x], rng.choice(np.delete(np.arange(V), x), k - 1, replace=False)]) for x in range(V)])
    out = ST.decide(z, None, None, toks, W=4, n0=0, radius=1, accept_mode=1, tau=0.2, mode=2, nbr=nbr)
    p_ref = scipy.special.softmax(z[0].astype(np.float64), axis=-1)
    for t in range(L):
        want = sum(p_ref[t, x] for x in nbr[toks[0, t]])
        assert abs(out["pbar"][0, t] - want) < 1e-6
        if abs(want - 0.2) > 1e-5:
            assert bool(out["accept"][0, t]) == (want >= 0.2)
    one = ST.decide(z, None, None, toks, W=4, n0=0, radius=1, accept_mode=1, tau=0.2, mode=2)
    assert (out["accept"] >= one["accept"]).all()      # pooling can only add mass


# ------------------------------------------------------------------ classifier-free guidance
def test_guidance_special_scales_closed_form_and_effect_on_decisions():
    rng = np.random.default_rng(17)
    B, L, V = 1, 16, 12
    zc = rng.normal(0, 1.5, (B, L, V)).astype(np.float32)
    zu = rng.normal(0, 1.5, (B, L, V)).astype(np.float32)
    toks = rng.integers(0, V, (B, L))
    kw = dict(W=4, n0=0, radius=1, accept_mode=1, tau=0.05, mode=2, seed=2)
    base_c = ST.decide(zc, None, None, toks, **kw)
    base_u = ST.decide(zu, None, None, toks, **kw)
    s1 = ST.decide(zc, None, None, toks, logits_uncond=zu, cfg_scale=1.0, **kw)
    s0 = ST.decide(zc, None, None, toks, logits_uncond=zu, cfg_scale=0.0, **kw)
    assert np.array_equal(s1["p"], base_c["p"]) and np.array_equal(s1["tokens_out"], base_c["tokens_out"])   # s = 1: conditional
    assert np.array_equal(s0["p"], base_u["p"]) and np.array_equal(s0["accept"], base_u["accept"])           # s = 0: unconditional
    same = ST.decide(zc, None, None, toks, logits_uncond=zc, cfg_scale=4.0, **kw)                            # z_c = z_u: no effect at any scale
    assert np.allclose(same["p"], base_c["p"], atol=1e-7)
    # closed form: guided p is proportional to p_c^s p_u^(1-s)
    g = ST.decide(zc, None, None, toks, logits_uncond=zu, cfg_scale=4.0, **kw)
    pc = scipy.special.softmax(zc.astype(np.float64), -1); pu = scipy.special.softmax(zu.astype(np.float64), -1)
    ref = pc ** 4.0 * pu ** -3.0
    ref /= ref.sum(-1, keepdims=True)
    assert np.abs(g["p"] - ref).max() < 1e-6
    # a two-entry hand example: z_c = (0, ln 3), z_u = (0, 0), s = 2 -> z = (0, 2 ln 3) -> p = (1/10, 9/10)
    h = ST.decide(np.array([[[0.0, np.log(3.0)]]], np.float32), None, None, np.array([[1]]), W=1, n0=0, radius=0,
                  accept_mode=1, tau=0.5, mode=2, logits_uncond=np.zeros((1, 1, 2), np.float32), cfg_scale=2.0)
    assert np.allclose(h["p"][0, 0], [0.1, 0.9], atol=1e-6) and h["accept"][0, 0] == 1
    assert not np.array_equal(g["accept"], base_c["accept"]) or not np.array_equal(g["tokens_out"], base_c["tokens_out"])


# ------------------------------------------------------------------ rejection islands (Eq. 8)
def test_rejection_islands_match_library_labelling_and_partition_the_marked_set():
    import scipy.ndimage
    rng = np.random.default_rng(3)
    eight = np.ones((3, 3), int)
    for H, W, row0, rows, dens in [(8, 8, 0, 8, 0.3), (16, 16, 4, 8, 0.2), (12, 7, 3, 5, 0.5), (64, 64, 48, 16, 0.12), (5, 9, 0, 5, 0.9)]:
        L, n0 = rows * W, row0 * W
        mask = rng.random(L) < dens
        island, rank, n, largest = LOC.rejection_islands(mask, W, n0)
        lab, n_ref = scipy.ndimage.label(mask.reshape(rows, W), structure=eight)
        lab = lab.reshape(-1)
        assert n == n_ref
        assert ((island > 0) == mask).all() and ((rank >= 0) == mask).all()
        # same partition: a bijection between the two labellings on the marked set
        pairs = set(zip(island[mask].tolist(), lab[mask].tolist()))
        assert len(pairs) == n and len({a for a, _ in pairs}) == n and len({b for _, b in pairs}) == n
        # canonical label = 1 + first member; ranks count the members before a position
        for lbl in np.unique(island[mask]):
            mem = np.flatnonzero(island == lbl)
            assert lbl == mem[0] + 1 and np.array_equal(rank[mem], np.arange(mem.size))
        assert largest == (np.bincount(lab[mask]).max() if mask.any() else 0)


def test_rejection_islands_hand_examples():
    # diagonal neighbours join (8-connectivity; a 4-connected labelling would report three islands)
    m = np.array([1, 0, 0,
                  0, 1, 0,
                  0, 0, 1], bool)
    island, rank, n, largest = LOC.rejection_islands(m, 3, 0)
    assert n == 1 and largest == 3 and island.tolist() == [1, 0, 0, 0, 1, 0, 0, 0, 1] and rank[[0, 4, 8]].tolist() == [0, 1, 2]
    # the last column of a row and the first column of the next are NOT neighbours (no wrap) ...
    m = np.array([0, 0, 1,
                  1, 0, 0], bool)
    assert LOC.rejection_islands(m, 3, 0)[2] == 2
    # ... and a block that starts in the middle of the grid uses the true coordinates
    assert LOC.rejection_islands(m, 3, 9)[2] == 2
    m = np.array([0, 1, 1, 0,
                  0, 0, 0, 0,
                  1, 0, 0, 1], bool)
    island, rank, n, largest = LOC.rejection_islands(m, 4, 8)
    assert n == 3 and largest == 2 and island.tolist() == [0, 2, 2, 0, 0, 0, 0, 0, 9, 0, 0, 12]
    assert LOC.rejection_islands(np.zeros(6, bool), 3, 0)[2:] == (0, 0)
