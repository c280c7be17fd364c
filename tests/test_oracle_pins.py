"""Pins of the CPU oracle against what the paper and the mathematics fix.

Nothing here touches the HIP library.  Each test names the passage of the paper
(arXiv 2102.08374) that fixes the checked fact.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle
from tests import pyref

F32 = np.float32


# ----------------------------------------------------------------------------- P1
def test_philox_known_answers(golden_dir):
    """Generator = Philox4x32-10: the published known-answer values."""
    rows = []
    with open(golden_dir + "/philox4x32_10_kat.txt") as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            v = [int(tok, 16) for tok in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(oracle.philox4x32_10(ctr, key)) == want
        assert pyref.philox4x32_10(ctr, key) == want


def test_philox_matches_bigint_version():
    rng = np.random.default_rng(1)
    for _ in range(10000):
        ctr = rng.integers(0, 2**32, 4, dtype=np.uint64)
        key = rng.integers(0, 2**32, 2, dtype=np.uint64)
        assert list(oracle.philox4x32_10(ctr, key)) == pyref.philox4x32_10(ctr, key)


def test_random_word_indexing():
    """Counter = (lo32(j/4), hi32(j/4), worker, step), key = (lo32 seed, hi32 seed),
    word j mod 4 -- including indices and seeds beyond 32 bits."""
    cases = [(0, 0, 0, 0), (0x123456789ABCDEF0, 7, 3, 5), (1, 2, 15, (1 << 34) + 3),
             (2**64 - 1, 2**32 - 1, 2**32 - 1, 2**40 + 2)]
    for seed, step, worker, j in cases:
        assert oracle.random_word(seed, step, worker, j) == pyref.random_word(seed, step, worker, j)
    # the four coordinates of one quad share a Philox call
    out = pyref.philox4x32_10([5, 0, 2, 9], [11, 0])
    assert [oracle.random_word(11, 9, 2, 20 + c) for c in range(4)] == out


# ----------------------------------------------------------------------------- P2/P3
@pytest.mark.parametrize("t", [0.25, 0.75, -0.25, 3.1415927, -7.6, 1e-3, 0.5, 123456.7,
                               1.0 - 2.0**-24, 2.0**-30, -(2.0**-30)])
def test_round_up_threshold_is_exact(t):
    """Section 2: P(Int(t) = [t]+1) = t-[t].  With u on the 2^-24 grid the number of
    grid points that round up must be ceil(p 2^24): check both sides of the
    threshold and a random sample of the grid (the decision is monotone in u)."""
    t = F32(t)
    fl = math.floor(Fraction(float(t)))
    p = Fraction(float(F32(t) - F32(fl)))
    m_star = math.ceil(p * (1 << 24))            # first grid index that does NOT round up
    if m_star > 0:
        assert oracle.int_random(t, ((m_star - 1) << 8) | 0xFF) == fl + 1
        assert oracle.int_random(t, 0) == fl + 1
    if m_star < (1 << 24):
        assert oracle.int_random(t, m_star << 8) == fl
        assert oracle.int_random(t, 0xFFFFFFFF) == fl
    rng = np.random.default_rng(7)
    for w in rng.integers(0, 2**32, 4000, dtype=np.uint64):
        w = int(w)
        assert oracle.int_random(t, w) == fl + (1 if (w >> 8) < m_star else 0)
        # the low 8 bits of the word are unused
        assert oracle.int_random(t, w) == oracle.int_random(t, w & 0xFFFFFF00)


def test_integers_pass_through_unchanged():
    for t in [0.0, -0.0, 1.0, -1.0, 17.0, -2.0**23, 2.0**24, -2.0**30]:
        for w in (0, 0xFFFFFFFF, 0x80000000):
            assert oracle.int_random(t, w) == t
        assert oracle.int_nearest(t) == t


def test_unbiased_and_variance_lemma1():
    """Lemma 1: E[Int(alpha x)]/alpha = x and E|Int(alpha x) - alpha x|^2 = p(1-p) <= 1/4;
    sup-norm bound |y - Int(y)| < 1 from its proof."""
    alpha = F32(37.5)
    x = np.array([0.013, -0.2, 0.5, 0.0266666, -1.0 / 3.0, 0.9], F32)
    t = np.array([pyref.scale(alpha, v) for v in x], F32)
    m = 20000
    acc = np.zeros(x.size)
    acc2 = np.zeros(x.size)
    for seed in range(m):
        q, cnt = oracle.compress(x, alpha, rounding=1, L=2**31 - 1, seed=seed, step=3, worker=1)
        assert cnt == 0
        err = q.astype(np.float64) - t.astype(np.float64)
        assert np.all(np.abs(err) < 1.0)
        acc += q
        acc2 += err * err
    mean = acc / m
    p = t.astype(np.float64) - np.floor(t.astype(np.float64))
    assert np.all(np.abs(mean - t) <= 4.0 * 0.5 / math.sqrt(m))
    var = acc2 / m
    assert np.all(var <= 0.25 + 1e-12)
    assert np.allclose(var, p * (1 - p), atol=4.0 * 0.25 / math.sqrt(m))
    # decoded: (1/alpha) E Int(alpha x) = x up to the fp32 rounding of alpha*x
    assert np.allclose(mean / float(alpha), x, atol=4.0 * 0.5 / math.sqrt(m) / float(alpha) + 1e-7)


# ----------------------------------------------------------------------------- P4
def test_nearest_even_ties_and_error_bound():
    """Section 5.1 (deterministic rounding = torch.round): ties to even, error <= 1/2."""
    ties = {0.5: 0, -0.5: 0, 1.5: 2, -1.5: -2, 2.5: 2, -2.5: -2, 3.5: 4, 1e6 + 0.5: 1e6}
    for t, want in ties.items():
        assert oracle.int_nearest(t) == want
    rng = np.random.default_rng(3)
    g = rng.normal(0, 1, 5000).astype(F32)
    for alpha in (F32(0.37), F32(11.3), F32(1234.5)):
        q, cnt = oracle.compress(g, alpha, rounding=0, L=2**31 - 1)
        assert cnt == 0
        t32 = (alpha * g).astype(np.float64)
        assert np.all(np.abs(q - t32) <= 0.5)
        exact = float(alpha) * g.astype(np.float64)
        # against the real product the bound holds up to the fp32 rounding of alpha*g
        assert np.all(np.abs(q / float(alpha) - g.astype(np.float64))
                      <= (0.5 + np.abs(exact) * 2.0**-24) / float(alpha))
        for k in range(0, g.size, 97):
            assert q[k] == pyref.int_nearest_exact(pyref.scale(alpha, g[k]))


# ----------------------------------------------------------------------------- P5
def test_saturation_rules():
    """Section 5.1: local values are clipped so the aggregate fits the wire type.
    The clip bound need not be an fp32 number."""
    L = (2**31 - 1) // 4                         # 536870911, not representable in fp32
    assert oracle.saturate(F32(536870912.0), L) == (L, 1)
    assert oracle.saturate(F32(536870880.0), L) == (536870880, 0)
    assert oracle.saturate(F32(-536870912.0), L) == (-L, 1)
    assert oracle.saturate(F32(2.0**31), 2**31 - 1) == (2**31 - 1, 1)
    assert oracle.saturate(F32(-2.0**31), 2**31 - 1) == (-(2**31 - 1), 1)
    assert oracle.saturate(F32(np.inf), 127) == (127, 1)
    assert oracle.saturate(F32(-np.inf), 127) == (-127, 1)
    assert oracle.saturate(F32(np.nan), 127) == (0, 1)
    assert oracle.saturate(F32(127.0), 127) == (127, 0)
    assert oracle.saturate(F32(-127.0), 127) == (-127, 0)
    assert oracle.saturate(F32(128.0), 127) == (127, 1)
    assert oracle.saturate(F32(-0.0), 127) == (0, 0)


def test_sum_is_exact_and_bounded():
    rng = np.random.default_rng(5)
    n, d, L = 5, 300, 127
    g = rng.standard_t(3, (n, d)).astype(F32) * F32(40.0)
    qs, cnts = [], []
    for i in range(n):
        q, c = oracle.compress(g[i], F32(1.7), rounding=1, L=L, seed=9, step=2, worker=i)
        # clip count by brute force on exact integers
        want_c = 0
        for j in range(d):
            r = pyref.int_random_exact(pyref.scale(1.7, g[i, j]), pyref.random_word(9, 2, i, j))
            v, c1 = pyref.clip(r, L)
            want_c += c1
            assert q[j] == v
        assert c == want_c and c > 0
        qs.append(q)
        cnts.append(c)
    S, ovf = oracle.int_sum(qs)
    assert ovf == 0
    want = [sum(int(q[j]) for q in qs) for j in range(d)]
    assert S.tolist() == want
    assert np.all(np.abs(S) <= n * L)
    # an aggregate that does not fit int32 is reported
    big = [np.full(4, 2**31 - 1, np.int32), np.full(4, 1, np.int32)]
    assert oracle.int_sum(big)[1] == 4


# ----------------------------------------------------------------------------- P6
def test_decode_identity_in_rationals():
    """Section 2.2: (1/(n alpha)) sum_i Int(alpha g_i) = (1/n) sum_i Q(g_i); the oracle's
    fp32 outputs are the correctly rounded rational values (up to fp64 slack)."""
    rng = np.random.default_rng(11)
    n, d = 3, 16
    alpha = F32(913.37)
    eta = 0.1
    g = rng.normal(0, 0.01, (n, d)).astype(F32)
    x = rng.normal(0, 1, d).astype(F32)
    qs = [oracle.compress(g[i], alpha, rounding=1, L=(2**31 - 1) // n, seed=4, step=1, worker=i)[0]
          for i in range(n)]
    S, _ = oracle.int_sum(qs)
    xn, gt = oracle.decode_update(S, alpha, x, n=n, eta=eta, want_gtilde=True)
    a = Fraction(float(alpha))
    for j in range(d):
        lhs = Fraction(int(S[j])) / (n * a)
        rhs = sum(Fraction(int(q[j])) / a for q in qs) / n      # (1/n) sum_i Q(g_i)_j
        assert lhs == rhs
        assert abs(Fraction(float(gt[j])) - lhs) <= Fraction(pyref.ulp32(lhs)) * Fraction(501, 1000)
        X = Fraction(float(x[j])) - Fraction(eta) * lhs
        assert abs(Fraction(float(xn[j])) - X) <= Fraction(pyref.ulp32(X)) * Fraction(501, 1000)


def test_power_of_two_scaling_is_plain_sgd():
    """alpha = 2^m and gradients on the 2^-m grid: rounding is the identity, so the
    step must equal full-precision averaged SGD (Algorithm 1 with exact messages)."""
    rng = np.random.default_rng(13)
    n, d, m = 4, 1000, 10
    g = (rng.integers(-5000, 5000, (n, d)) / 2.0**m).astype(F32)
    x = rng.normal(0, 1, d).astype(F32)
    eta = 0.25
    for rounding in (0, 1):
        out = oracle.step(list(g), F32(2.0**m), x, rounding=rounding, L=(2**31 - 1) // n, eta=eta,
                          seed=1, step=1)
        assert out["sat_count"].sum() == 0 and out["overflow"] == 0
        assert np.array_equal(out["S"], (g.astype(np.float64).sum(0) * 2**m).astype(np.int64))
        want = (x.astype(np.float64) - eta * g.astype(np.float64).mean(0)).astype(F32)
        assert np.array_equal(out["x_new"], want)
        nrm = float(((want.astype(np.float64) - x.astype(np.float64)) ** 2).sum())
        assert math.isclose(out["normsq"][0], nrm, rel_tol=1e-13)


# ----------------------------------------------------------------------------- P7
def test_alpha_recurrence_closed_form():
    """Proposition 2 and its proof: eta^2 d / alpha_k^2 = eta^2 eps^2 + 2 n r_k with
    r_k = (1-beta) sum_t beta^t ||x^{k-t} - x^{k-t-1}||^2 (so r_0 = 0)."""
    d, n, beta, eps, eta = 1000, 7, Fraction(9, 10), Fraction(1, 10**8), Fraction(1, 10)
    norms = [Fraction(3, 1000), Fraction(1, 500), Fraction(7, 10000), Fraction(1, 3), Fraction(0)]
    r = np.zeros(1)
    for k in range(1, len(norms) + 1):
        r, ad, af, bad = oracle.next_alpha([float(norms[k - 1])], r, d=d, n=n, beta=float(beta),
                                           eps=float(eps), eta=float(eta))
        assert bad == 0
        r_closed = (1 - beta) * sum(beta**t * norms[k - 1 - t] for t in range(k))
        assert math.isclose(r[0], float(r_closed), rel_tol=1e-13)
        lhs = float(eta) ** 2 * d / ad[0] ** 2
        rhs = float(eta**2 * eps**2 + 2 * n * r_closed)
        assert math.isclose(lhs, rhs, rel_tol=1e-12)
        assert af[0] == F32(ad[0])


def test_alpha_beta0_eps0_is_proposition3():
    """Proposition 3: beta = 0, eps = 0 gives alpha = eta sqrt(d) / (sqrt(2n) ||dx||)."""
    d, n, eta, nrm = 4096, 5, 0.05, 0.0123
    r, ad, af, bad = oracle.next_alpha([nrm * nrm], [123.0], d=d, n=n, beta=0.0, eps=0.0, eta=eta)
    assert bad == 0 and r[0] == nrm * nrm
    assert math.isclose(ad[0], eta * math.sqrt(d) / (math.sqrt(2 * n) * nrm), rel_tol=1e-14)
    # zero update and no safeguard: the rule divides by zero and says so
    assert oracle.next_alpha([0.0], [0.0], d=d, n=n, beta=0.0, eps=0.0, eta=eta)[3] == 1


def test_block_alpha_algorithm2():
    """Algorithm 2 / Proposition 4: sum_l d_l eta^2/alpha_l^2 = 2n sum_l r_l + eta^2 eps^2,
    beta = 0 = eps gives alpha_l = eta sqrt(d_l)/(sqrt(2n) ||dx_l||), and B = 1 is Algorithm 1."""
    offsets = np.array([0, 10, 250, 251, 1000], np.uint64)
    d, n, eta, beta, eps = 1000, 3, 0.1, 0.9, 1e-3
    normsq = np.array([1e-4, 3e-2, 5e-7, 0.2])
    r0 = np.array([1e-5, 0.0, 2e-6, 0.5])
    r, ad, af, bad = oracle.next_alpha(normsq, r0, d=d, n=n, beta=beta, eps=eps, eta=eta,
                                       offsets=offsets)
    assert bad == 0
    dl = np.diff(offsets.astype(np.int64))
    assert np.allclose(r, beta * r0 + (1 - beta) * normsq, rtol=1e-14)
    lhs = float((dl * eta**2 / ad**2).sum())
    assert math.isclose(lhs, 2 * n * float(r.sum()) + eta**2 * eps**2, rel_tol=1e-12)
    r2, ad2, _, _ = oracle.next_alpha(normsq, r0, d=d, n=n, beta=0.0, eps=0.0, eta=eta,
                                      offsets=offsets)
    assert np.allclose(ad2, eta * np.sqrt(dl) / (math.sqrt(2 * n) * np.sqrt(normsq)), rtol=1e-14)
    # one block: Algorithm 2's formula (evaluated here by hand) equals Algorithm 1's
    _, a1, _, _ = oracle.next_alpha([0.03], [0.01], d=d, n=n, beta=beta, eps=eps, eta=eta)
    rr = beta * 0.01 + (1 - beta) * 0.03
    alg2 = eta * math.sqrt(d) / math.sqrt(2 * n * rr + eta**2 * (d / d) * eps**2)
    assert math.isclose(a1[0], alg2, rel_tol=1e-14)


# ----------------------------------------------------------------------------- P8
def test_range_bound_section_4_2():
    """Section 4.2: with beta = eps = 0 and ||x^k - x^{k-1}|| = ||eta g||, the scaled
    gradient obeys ||alpha g||_inf <= sqrt(d)/sqrt(2n); the printed example needs < 14 bits."""
    rng = np.random.default_rng(17)
    d, n, eta = 20000, 8, 0.1
    g = rng.normal(0, 1e-3, d).astype(F32)
    nrm2 = float((eta * g.astype(np.float64)) @ (eta * g.astype(np.float64)))
    _, ad, af, _ = oracle.next_alpha([nrm2], [0.0], d=d, n=n, beta=0.0, eps=0.0, eta=eta)
    q, cnt = oracle.compress(g, af, rounding=0, L=2**31 - 1)
    assert cnt == 0
    assert np.abs(q).max() <= math.ceil(math.sqrt(d) / math.sqrt(2 * n))
    assert 1 + math.log2(math.sqrt(5e7)) < 14


# ----------------------------------------------------------------------------- P9
ADVERSARIAL = [0.0, -0.0, 1e-45, -1e-45, 0.5, -0.5, 1.5, 2.5, -2.5, 126.5, 127.49, 127.5, -127.5,
               128.0, 1e9, -1e9, 16777216.0, 16777217.0, 2147483648.0, -2147483648.0, 4e9,
               float("inf"), float("-inf"), float("nan"), 0.99999994, -0.99999994]


@pytest.mark.parametrize("rounding", [0, 1])
@pytest.mark.parametrize("L,n", [(127, 3), ((2**31 - 1) // 3, 3), (2**31 - 1, 1), (1, 2)])
def test_whole_step_brute_force_small(rounding, L, n):
    """Every stage of Algorithm 1 / Algorithm 2 recomputed with Python integers and
    rationals on d <= 16, random and adversarial inputs, one and two blocks."""
    rng = np.random.default_rng(100 * rounding + n + L % 7)
    for trial in range(6):
        d = int(rng.integers(1, 17))
        if trial % 2 == 0 or d < 2:
            offsets, B = None, 1
            alpha = np.array([rng.choice([1.0, 0.37, 113.7, 3e4])], F32)
        else:
            cut = int(rng.integers(1, d))
            offsets, B = np.array([0, cut, d], np.uint64), 2
            alpha = np.array([0.37, 113.7], F32)
        g = rng.normal(0, 1.0, (n, d)).astype(F32)
        adv = rng.choice(np.array(ADVERSARIAL, F32), (n, d))
        mask = rng.random((n, d)) < 0.4
        g = np.where(mask, adv, g).astype(F32)
        x = rng.normal(0, 1, d).astype(F32)
        eta, seed, step, j0 = 0.1, 0xDEADBEEF12345, 4, 0
        out = oracle.step(list(g), alpha, x, rounding=rounding, L=L, eta=eta, seed=seed, step=step,
                          j0=j0, offsets=offsets)
        blk = lambda j: 0 if B == 1 else int(j >= offsets[1])
        S = [0] * d
        sat = [0] * n
        for i in range(n):
            for j in range(d):
                t = pyref.scale(alpha[blk(j)], g[i, j])
                if np.isnan(t):
                    v, c = 0, 1
                elif np.isinf(t):
                    v, c = (L if t > 0 else -L), 1
                else:
                    if rounding == 1:
                        lo = math.floor(Fraction(float(t)))
                        r = pyref.int_random_exact(t, pyref.random_word(seed, step, i, j))
                        assert r in (lo, lo + 1)
                    else:
                        r = pyref.int_nearest_exact(t)
                    v, c = pyref.clip(r, L)
                S[j] += v
                sat[i] += c
        assert out["S"].tolist() == S
        assert out["sat_count"].tolist() == sat
        assert out["overflow"] == 0
        nrm = [Fraction(0)] * B
        for j in range(d):
            a = Fraction(float(alpha[blk(j)]))
            X = Fraction(float(x[j])) - Fraction(eta) * Fraction(S[j]) / (n * a)
            got = Fraction(float(out["x_new"][j]))
            assert abs(got - X) <= Fraction(pyref.ulp32(X)) * Fraction(501, 1000)
            nrm[blk(j)] += (got - Fraction(float(x[j]))) ** 2
        for l in range(B):
            assert math.isclose(out["normsq"][l], float(nrm[l]), rel_tol=1e-13, abs_tol=1e-300)


def test_slices_compose():
    """A step on [0,d) equals the steps on its slices (global indexing of the random
    stream and of the blocks)."""
    rng = np.random.default_rng(23)
    n, d = 3, 103
    offsets = np.array([0, 5, 50, 103], np.uint64)
    alpha = np.array([10.0, 200.0, 3000.0], F32)
    g = rng.normal(0, 0.01, (n, d)).astype(F32)
    x = rng.normal(0, 1, d).astype(F32)
    kw = dict(rounding=1, L=1000, eta=0.1, seed=77, step=9, offsets=offsets)
    full = oracle.step(list(g), alpha, x, **kw)
    ns = np.zeros(3)
    xs, Ss, sat = [], [], np.zeros(n, np.uint64)
    for a, b in [(0, 7), (7, 64), (64, 103)]:
        part = oracle.step([gi[a:b] for gi in g], alpha, x[a:b], j0=a, normsq=ns, **kw)
        xs.append(part["x_new"]); Ss.append(part["S"]); sat += part["sat_count"]
    assert np.array_equal(np.concatenate(xs), full["x_new"])
    assert np.array_equal(np.concatenate(Ss), full["S"])
    assert np.array_equal(sat, full["sat_count"])
    assert np.allclose(ns, full["normsq"], rtol=1e-14)


# ----------------------------------------------------------------------------- P10
def test_steady_state_alpha_fixed_point():
    """Algorithm 1 run on iid N(0, sigma^2) gradients: the recurrence settles where
    alpha^2 sigma^2 = 1/2 - q, q = mean squared rounding error per worker-coordinate
    (from the alpha rule and the update line; loose sanity, not a parity claim)."""
    rng = np.random.default_rng(29)
    n, d, eta, sigma, beta, eps = 4, 1 << 15, 0.1, 1e-3, 0.9, 1e-8
    x = rng.normal(0, 1, d).astype(F32)
    r = np.zeros(1)
    nrm = eta**2 * d * sigma**2 / n
    alphas = []
    for k in range(1, 80):
        r, ad, af, _ = oracle.next_alpha([nrm], r, d=d, n=n, beta=beta, eps=eps, eta=eta)
        g = rng.normal(0, sigma, (n, d)).astype(F32)
        out = oracle.step(list(g), af, x, rounding=1, L=(2**31 - 1) // n, eta=eta, seed=0, step=k)
        x, nrm = out["x_new"], float(out["normsq"][0])
        alphas.append(float(ad[0]))
    a = np.mean(alphas[-10:])
    t = a * g.astype(np.float64)
    p = t - np.floor(t)
    q = float((p * (1 - p)).mean())
    assert math.isclose((a * sigma) ** 2, 0.5 - q, rel_tol=0.08)


# ----------------------------------------------------------------------------- momentum form
def test_momentum_update_in_rationals_and_special_cases():
    """Momentum / weight-decay update (the optimizer of Section 5's experiments): each stored
    value is the correctly rounded rational result of its own line; mu = wd = 0 stores the
    decoded gradient in m and takes the plain SGD step with it."""
    rng = np.random.default_rng(31)
    n, d = 3, 16
    alpha = F32(713.25)
    S = rng.integers(-40, 40, d).astype(np.int32)
    x = rng.normal(0, 1, d).astype(F32)
    m = rng.normal(0, 0.01, d).astype(F32)
    eta, mu, wd = 0.1, 0.9, 1e-4
    xn, mn = oracle.decode_update_momentum(S, alpha, x, m, n=n, eta=eta, mu=mu, wd=wd)
    a = Fraction(float(alpha))
    half = Fraction(501, 1000)
    for j in range(d):
        gt = Fraction(int(S[j])) / (n * a)
        M = Fraction(mu) * Fraction(float(m[j])) + gt + Fraction(wd) * Fraction(float(x[j]))
        assert abs(Fraction(float(mn[j])) - M) <= Fraction(pyref.ulp32(M)) * half
        X = Fraction(float(x[j])) - Fraction(eta) * Fraction(float(mn[j]))    # uses the STORED m'
        assert abs(Fraction(float(xn[j])) - X) <= Fraction(pyref.ulp32(X)) * half
    xn0, mn0 = oracle.decode_update_momentum(S, alpha, x, m, n=n, eta=eta, mu=0.0, wd=0.0)
    _, gt32 = oracle.decode_update(S, alpha, x, n=n, eta=eta, want_gtilde=True)
    assert np.all(np.abs(mn0.astype(np.float64) - gt32.astype(np.float64))
                  <= np.spacing(np.abs(gt32)).astype(np.float64))
    want = (x.astype(np.float64) - eta * mn0.astype(np.float64)).astype(F32)
    assert np.array_equal(xn0, want)


def test_momentum_matches_torch_sgd():
    """Several steps against torch.optim.SGD(momentum, weight_decay) run in float64 on the
    decoded gradients: same recursion, so agreement to fp32 rounding of the stored state."""
    import torch
    rng = np.random.default_rng(37)
    n, d, alpha = 4, 500, F32(256.0)           # power of two: decoded gradient exact in fp32
    eta, mu, wd = 0.05, 0.9, 1e-4
    x = rng.normal(0, 1, d).astype(F32)
    m = np.zeros(d, F32)
    p = torch.tensor(x.astype(np.float64), requires_grad=True)
    opt = torch.optim.SGD([p], lr=eta, momentum=mu, weight_decay=wd)
    for k in range(12):
        S = rng.integers(-30, 30, d).astype(np.int32)
        x, m = oracle.decode_update_momentum(S, alpha, x, m, n=n, eta=eta, mu=mu, wd=wd)
        p.grad = torch.tensor(S.astype(np.float64) / (n * float(alpha)))
        opt.step()
        ref = p.detach().numpy()
        assert np.all(np.abs(x - ref) <= (k + 1) * 4 * np.spacing(np.abs(ref).astype(F32)) + 1e-7)
    buf = opt.state[p]["momentum_buffer"].numpy()
    assert np.allclose(m, buf, rtol=1e-4, atol=1e-6)


def test_momentum_geometric_closed_form():
    """Constant decoded gradient, no decay: m_K = g (1 - mu^K)/(1 - mu)."""
    n, alpha, eta, mu = 2, F32(64.0), 0.1, 0.5
    S = np.array([8, -24, 0, 128], np.int32)
    g = S / (n * 64.0)
    x = np.zeros(4, F32)
    m = np.zeros(4, F32)
    K = 10
    for _ in range(K):
        x, m = oracle.decode_update_momentum(S, alpha, x, m, n=n, eta=eta, mu=mu, wd=0.0)
    assert np.allclose(m, g * (1 - mu**K) / (1 - mu), rtol=1e-6)
    total = sum(g * (1 - mu**k) / (1 - mu) for k in range(1, K + 1))
    assert np.allclose(x, -eta * total, rtol=1e-5)


def test_step_momentum_composes():
    rng = np.random.default_rng(41)
    n, d = 3, 64
    g = rng.normal(0, 0.01, (n, d)).astype(F32)
    x = rng.normal(0, 1, d).astype(F32)
    m = rng.normal(0, 0.01, d).astype(F32)
    kw = dict(rounding=1, L=1000, eta=0.1, seed=5, step=2)
    plain = oracle.step(list(g), F32(300.0), x, **kw)
    mom = oracle.step_momentum(list(g), F32(300.0), x, m, mu=0.9, wd=1e-4, **kw)
    assert np.array_equal(plain["S"], mom["S"]) and np.array_equal(plain["sat_count"], mom["sat_count"])
    xn, mn = oracle.decode_update_momentum(mom["S"], F32(300.0), x, m, n=n, eta=0.1, mu=0.9, wd=1e-4)
    assert np.array_equal(xn, mom["x_new"]) and np.array_equal(mn, mom["m_new"])
    nrm = float(((xn.astype(np.float64) - x.astype(np.float64)) ** 2).sum())
    assert math.isclose(mom["normsq"][0], nrm, rel_tol=1e-13)


# ----------------------------------------------------------------------------- IntDIANA (Algorithm 3)
def test_diana_lines_in_rationals():
    """Every stored value of one IntDIANA step is the correctly rounded rational value of
    its line of Algorithm 3; zero shifts reproduce IntSGD's integers and (to 1 ulp) its x."""
    rng = np.random.default_rng(43)
    n, d = 3, 16
    alpha = F32(411.75)
    eta = 0.1
    g = rng.normal(0, 0.02, (n, d)).astype(F32)
    hl = rng.normal(0, 0.02, (n, d)).astype(F32)
    x = rng.normal(0, 1, d).astype(F32)
    h = hl.astype(np.float64).mean(0).astype(F32)
    kw = dict(rounding=1, L=10**6, seed=21, step=6)
    out = oracle.diana_step(list(g), list(hl), alpha, x, h, eta=eta, **kw)
    a = Fraction(float(alpha))
    half = Fraction(501, 1000)
    S = [0] * d
    for i in range(n):
        for j in range(d):
            delta = F32(g[i, j]) - F32(hl[i, j])
            t = pyref.scale(alpha, delta)
            q = pyref.int_random_exact(t, pyref.random_word(21, 6, i, j))
            S[j] += q
            H = Fraction(float(hl[i, j])) + Fraction(q) / a
            got = Fraction(float(out["h_local_new"][i][j]))
            assert abs(got - H) <= Fraction(pyref.ulp32(H)) * half + Fraction(1, 10**12)
    assert out["S"].tolist() == S
    for j in range(d):
        G = Fraction(float(h[j])) + Fraction(S[j]) / (n * a)
        assert abs(Fraction(float(out["h_new"][j])) - G) <= Fraction(pyref.ulp32(G)) * half
        X = Fraction(float(x[j])) - Fraction(eta) * G
        assert abs(Fraction(float(out["x_new"][j])) - X) <= Fraction(pyref.ulp32(X)) * half
    zero = [np.zeros(d, F32)] * n
    o0 = oracle.diana_step(list(g), zero, alpha, x, np.zeros(d, F32), eta=eta, **kw)
    p0 = oracle.step(list(g), alpha, x, eta=eta, **kw)
    assert np.array_equal(o0["S"], p0["S"])
    assert np.all(np.abs(o0["x_new"].astype(np.float64) - p0["x_new"].astype(np.float64))
                  <= np.spacing(np.abs(p0["x_new"])).astype(np.float64))


def test_diana_global_shift_is_mean_of_local_shifts():
    """Algorithm 3 keeps h = (1/n) sum_i h_i (both start at 0 and move by the same decoded
    messages); in fp32 storage the identity holds to rounding over many steps."""
    rng = np.random.default_rng(47)
    n, d, eta = 4, 200, 0.2
    b = rng.normal(0, 1, (n, d))
    x = rng.normal(0, 1, d).astype(F32)
    hl = [np.zeros(d, F32) for _ in range(n)]
    h = np.zeros(d, F32)
    alpha = F32(50.0)
    for k in range(1, 40):
        g = [(x.astype(np.float64) - b[i]).astype(F32) for i in range(n)]
        out = oracle.diana_step(g, hl, alpha, x, h, rounding=1, L=10**6, eta=eta, seed=1, step=k)
        x, h, hl = out["x_new"], out["h_new"], out["h_local_new"]
        mean = np.mean([v.astype(np.float64) for v in hl], axis=0)
        scale = np.max(np.abs(np.array(hl + [h])), axis=0).astype(F32)      # rounding happens at |h_i|
        assert np.all(np.abs(h - mean) <= 40 * np.spacing(scale + F32(1e-3)))


def test_diana_keeps_integers_small_where_intsgd_does_not():
    """Appendix A.2: with heterogeneous workers and exact gradients, IntSGD's integers grow
    like |grad f_i(x*)| / ||x^k - x^{k-1}|| while IntDIANA's stay bounded, and IntDIANA's
    iterates converge linearly.  f_i(x) = 0.5 ||x - b_i||^2, adaptive alpha with beta = 0."""
    rng = np.random.default_rng(53)
    n, d, eta = 4, 64, 0.25
    b = rng.normal(0, 1, (n, d))
    xstar = b.mean(0)
    def run(diana):
        x = np.zeros(d, F32)
        hl = [np.zeros(d, F32) for _ in range(n)]
        h = np.zeros(d, F32)
        nrm = float(eta**2 * ((x - xstar) ** 2).sum())       # exact first step
        x = (x.astype(np.float64) - eta * (x - xstar)).astype(F32)
        maxint, dist = [], []
        for k in range(1, 45):
            _, ad, af, bad = oracle.next_alpha([nrm], [0.0], d=d, n=n, beta=0.0, eps=1e-12, eta=eta)
            g = [(x.astype(np.float64) - b[i]).astype(F32) for i in range(n)]
            kw = dict(rounding=1, L=2**31 - 1 >> 2, seed=3, step=k)
            if diana:
                sent = [oracle.diana_compress(g[i], hl[i], af, worker=i, **kw)[0] for i in range(n)]
                out = oracle.diana_step(g, hl, af, x, h, eta=eta, **kw)
                h, hl = out["h_new"], out["h_local_new"]
            else:
                sent = [oracle.compress(g[i], af, worker=i, **kw)[0] for i in range(n)]
                out = oracle.step(g, af, x, eta=eta, **kw)
            assert np.array_equal(np.sum(sent, axis=0), out["S"])
            maxint.append(int(np.abs(np.array(sent)).max()))    # largest integer a worker transmits
            x, nrm = out["x_new"], max(float(out["normsq"][0]), 1e-300)
            dist.append(float(np.linalg.norm(x - xstar)))
        return maxint, dist
    mi_sgd, _ = run(False)
    mi_dia, dist = run(True)
    assert max(mi_dia[10:]) <= 64                      # a few bits per coordinate
    assert max(mi_sgd[25:]) > 50 * max(mi_dia[25:])    # IntSGD's messages blow up
    assert dist[30] < 1e-3 * dist[0]                   # linear convergence of IntDIANA


# ----------------------------------------------------------------------------- Heuristic IntSGD
def test_heuristic_scaling_rule():
    """Section 5.2: alpha = (2^nb - 1)/(n 2^max_exp) with 2^max_exp >= max|g|: hand-picked
    values, exact rationals, power-of-two scale invariance, and the no-overflow property
    |alpha g| <= (2^nb - 1)/n that the paper credits the rule with."""
    n = 8
    cases = {0.75: 0, 1.0: 0, 1.0000001: 1, 0.5: -1, 0.50000006: 0, 3.0: 2, 1e-3: -9, 1e-45: -149,
             3e-45: -147, 2.0**-126: -126, 3.0e38: 128}
    for m, e in cases.items():
        for nb in (7, 31):
            ad, af = oracle.heuristic_alpha([m], n=n, nb=nb)
            want = Fraction(2**nb - 1, n) / Fraction(2) ** e
            if want > Fraction(float(np.finfo(F32).max)):
                want = Fraction(float(np.finfo(F32).max))
            assert Fraction(float(ad[0])) == want, (m, nb)
            assert af[0] == F32(float(want))
    assert oracle.heuristic_alpha([0.0], n=n, nb=7)[1][0] == 1.0
    rng = np.random.default_rng(59)
    g = rng.normal(0, 1e-3, (n, 5000)).astype(F32)
    g[2, 17] = np.inf
    g[3, 99] = np.nan
    offsets = np.array([0, 100, 4000, 5000], np.uint64)
    m = np.zeros(3, F32)
    for i in range(n):
        oracle.max_abs(g[i, :3000], offsets=offsets, B=3, out=m)
        oracle.max_abs(g[i, 3000:], j0=3000, offsets=offsets, B=3, out=m)
    fin = np.where(np.isfinite(g), np.abs(g), 0)
    want = [fin[:, 0:100].max(), fin[:, 100:4000].max(), fin[:, 4000:].max()]
    assert m.tolist() == [float(v) for v in want]
    for nb in (7, 31):
        ad, af = oracle.heuristic_alpha(m, n=n, nb=nb)
        for l, (a, b) in enumerate([(0, 100), (100, 4000), (4000, 5000)]):
            assert float(ad[l]) * float(want[l]) <= (2**nb - 1) / n
            assert float(ad[l]) * float(want[l]) > (2**nb - 1) / n / 2      # and not more than 2x slack
        ad2, _ = oracle.heuristic_alpha(m * F32(1024.0), n=n, nb=nb)
        assert np.array_equal(ad2 * 1024.0, ad)
        # the integers it produces fit: nearest rounding of |alpha g| <= (2^nb - 1)/n
        q, cnt = oracle.compress(np.where(np.isfinite(g[0]), g[0], 0).astype(F32), af, rounding=0,
                                 L=2**nb - 1, offsets=offsets)
        assert cnt == 0 and np.abs(q).max() <= math.ceil((2**nb - 1) / n)


# ----------------------------------------------------------------------------- largest integer
def test_largest_integer_in_the_aggregate():
    """Appendix A.2 reports the max integer in the aggregated vector: planted extremes per
    block, slices that combine, both ends of int32, a closed form (equal gradients: S = n
    round(alpha c)), the bound n L with the value attained when every worker clips, and brute
    force over random aggregates in pure Python."""
    offsets = np.array([0, 3, 10, 11, 40], np.uint64)
    S = np.zeros(40, np.int32)
    S[1], S[2] = 5, -7            # block 0: the negative one wins
    S[9] = 3                      # block 1: last coordinate of the block
    S[10] = -1                    # block 2: one coordinate
    S[11], S[39] = -2**31, 2**31 - 1   # block 3: both ends of the type
    assert oracle.max_abs_sum(S, offsets=offsets, B=4).tolist() == [7, 3, 1, 2**31]
    assert oracle.max_abs_sum(S).tolist() == [2**31]
    assert oracle.max_abs_sum(np.zeros(0, np.int32)).tolist() == [0]
    # slices in any order give the same running maximum
    m = np.zeros(4, np.uint32)
    for a, b in ((25, 40), (0, 2), (2, 25)):
        oracle.max_abs_sum(S[a:b], j0=a, offsets=offsets, B=4, out=m)
    assert m.tolist() == [7, 3, 1, 2**31]
    # equal gradients: S_j = n * round(alpha c)
    n, c, alpha = 6, F32(0.3), np.array([41.0], F32)
    g = [np.full(17, c, F32) for _ in range(n)]
    out = oracle.step(g, alpha, np.zeros(17, F32), rounding=0, L=10**6, eta=0.1)
    assert oracle.max_abs_sum(out["S"]).tolist() == [n * 12]          # 41 * 0.3 = 12.3 -> 12
    # every worker clips with the same sign: the bound n L is attained, and never exceeded
    L = 127
    g = [np.full(9, F32(-50.0), F32) for _ in range(n)]
    out = oracle.step(g, np.array([1000.0], F32), np.zeros(9, F32), rounding=1, L=L, eta=0.1, seed=3)
    assert oracle.max_abs_sum(out["S"]).tolist() == [n * L]
    rng = np.random.default_rng(101)
    for trial in range(20):
        d = int(rng.integers(1, 60))
        B = int(rng.integers(1, min(d, 5) + 1))
        cuts = np.sort(rng.choice(np.arange(1, d), B - 1, replace=False)) if B > 1 else []
        off = np.array([0, *cuts, d], np.uint64)
        S = rng.integers(-1000, 1000, d).astype(np.int32)
        want = [max(abs(int(v)) for v in S[int(off[l]):int(off[l + 1])]) for l in range(B)]
        assert oracle.max_abs_sum(S, offsets=off, B=B).tolist() == want
