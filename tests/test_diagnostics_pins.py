"""Pins of the diagnostics oracle (oracle/diagnostics.py) against what Section 3 of the paper and the
mathematics fix: closed forms, invariants, brute force, special cases.  No GPU."""
import numpy as np

from oracle import diagnostics as dg


# ---- k3 estimate (Section 3.1, KL Divergence Estimation)
def test_k3_is_zero_for_identical_policies_and_closed_form_for_a_constant_ratio():
    lp = np.log(np.random.default_rng(0).uniform(0.01, 1.0, 1000)).astype(np.float32)
    assert dg.k3_kl(lp, lp) == 0.0
    for c in (0.5, 0.9, 1.25, 3.0):
        shift = np.float32(np.log(c))
        lt = (lp.astype(np.float64) + np.float64(shift)).astype(np.float32)
        d = lt.astype(np.float64) - lp.astype(np.float64)             # what float32 storage kept of log c
        want = np.mean(np.exp(d) - 1 - d)
        assert abs(dg.k3_kl(lt, lp) - want) <= 1e-15
        assert abs(dg.k3_kl(lt, lp) - (c - 1 - np.log(c))) <= 2e-6 * max(1.0, c)   # r - 1 - log r at r = c


def test_k3_is_nonnegative_and_is_not_symmetric():
    rng = np.random.default_rng(1)
    a = rng.normal(-2, 1, 5000).astype(np.float32)
    b = (a + rng.normal(0, 0.3, 5000)).astype(np.float32)
    assert dg.k3_kl(a, b) > 0 and dg.k3_kl(b, a) > 0
    assert abs(dg.k3_kl(a, b) - dg.k3_kl(b, a)) > 1e-6             # e^d - 1 - d is not even in d


def test_k3_estimates_the_kl_divergence_of_a_small_categorical_pair():
    """E_{x~q}[r - 1 - log r], r = p/q, equals KL(q || p) exactly; with samples drawn from q the mean of the
    estimate converges to it (the estimator's defining property in the cited note)."""
    rng = np.random.default_rng(2)
    p = np.array([0.5, 0.3, 0.2])
    q = np.array([0.4, 0.4, 0.2])
    kl_qp = float(np.sum(q * np.log(q / p)))
    exact = float(np.sum(q * (p / q - 1 - np.log(p / q))))
    assert abs(exact - kl_qp) < 1e-15
    x = rng.choice(3, 400000, p=q)
    est = dg.k3_kl(np.log(p[x]).astype(np.float32), np.log(q[x]).astype(np.float32))
    assert abs(est - kl_qp) < 3e-4


# ---- extreme token fraction (Section 3.1, F(tau))
def test_extreme_fraction_counts_ratios_in_either_direction():
    lt = np.log(np.array([0.5, 0.5, 0.5, 0.5, 0.5], np.float32))
    li = np.log(np.array([0.5, 0.2, 0.9, 0.25, 0.1], np.float32))      # ratios 1, 2.5, 1/1.8, 2, 5
    f = dg.extreme_fraction(lt, li, [1.0, 1.5, 1.9, 2.2, 4.0, 6.0])
    assert f == [4 / 5, 4 / 5, 3 / 5, 2 / 5, 1 / 5, 0.0]
    assert dg.extreme_fraction(li, lt, [1.9]) == [3 / 5]                # symmetric in the two policies


def test_extreme_fraction_is_monotone_and_is_the_ratio_count_of_the_definition():
    rng = np.random.default_rng(3)
    a = rng.normal(-3, 1, 20000).astype(np.float32)
    b = (a + rng.standard_t(3, 20000) * 0.2).astype(np.float32)
    taus = [1.0, 1.1, 1.5, 2.0, 3.0, 10.0, 100.0]
    f = dg.extreme_fraction(a, b, taus)
    assert all(x >= y for x, y in zip(f, f[1:]))
    # the definition itself, on probability ratios: max(r, 1/r) > tau (tokens within 1e-12 of a threshold
    # may fall either way between the two forms)
    r = np.exp(a.astype(np.float64) - b.astype(np.float64))
    m = np.maximum(r, 1.0 / r)
    for tau, got in zip(taus, f):
        near = np.count_nonzero(np.abs(m - tau) <= 1e-12 * tau)
        assert abs(round(got * m.size) - np.count_nonzero(m > tau)) <= near
    assert f[0] == np.count_nonzero(a != b) / a.size            # tau = 1: every token whose two values differ


# ---- routing differences (Section 3.2)
def _records(L, T, K, E, seed, flip=0.2):
    rng = np.random.default_rng(seed)
    a = np.stack([np.stack([np.sort(rng.choice(E, K, replace=False)) for _ in range(T)]) for _ in range(L)])
    b = a.copy()
    for l in range(L):
        for t in range(T):
            if rng.random() < flip:
                b[l, t] = np.sort(rng.choice(E, K, replace=False))
    return a, b


def test_identical_and_disjoint_records():
    a, _ = _records(3, 17, 4, 32, 0)
    hist, tc, tr, sm = dg.routing_diff(a, a, [0, 5, 17])
    assert hist.tolist() == [3 * 17, 0, 0, 0, 0] and not tc.any() and not tr.any() and sm.tolist() == [0.0, 0.0]
    lo = np.stack([np.arange(4)] * 17)[None].repeat(3, 0)           # ids 0..3 against ids 28..31
    hi = lo + 28
    hist, tc, tr, sm = dg.routing_diff(lo, hi, [0, 17])
    assert hist.tolist() == [0, 0, 0, 0, 3 * 17] and (tc == 12).all() and (tr == 3).all() and sm.tolist() == [3.0]


def test_counts_are_consistent_with_each_other_and_order_free():
    a, b = _records(5, 40, 8, 128, 1)
    hist, tc, tr, sm = dg.routing_diff(a, b, [0, 10, 10, 40])
    L, T, K = a.shape
    assert hist.sum() == L * T
    assert (hist * np.arange(K + 1)).sum() == tc.sum()               # router level and token level agree
    assert (L * T - hist[0]) == tr.sum()
    assert sm[1] == 0.0 and abs(sm[0] * 10 + sm[2] * 30 - tr.sum()) < 1e-9
    assert ((tr == 0) == (tc == 0)).all() and (tc >= tr).all() and (tc <= K * tr).all()
    # a set has no order: shuffling the K ids of every router changes nothing; swapping the records neither
    rng = np.random.default_rng(5)
    bs = rng.permuted(b, axis=2)
    h2, tc2, tr2, _ = dg.routing_diff(a, bs)
    assert (h2 == hist).all() and (tc2 == tc).all() and (tr2 == tr).all()
    h3, tc3, tr3, _ = dg.routing_diff(b, a)
    assert (h3 == hist).all() and (tc3 == tc).all() and (tr3 == tr).all()


def test_single_changed_expert_counts_one():
    a, _ = _records(2, 6, 8, 128, 2)
    b = a.copy()
    free = [e for e in range(128) if e not in set(a[1, 3])][0]
    b[1, 3, 5] = free
    hist, tc, tr, _ = dg.routing_diff(a, b)
    assert hist.tolist() == [11, 1, 0, 0, 0, 0, 0, 0, 0] and tc.tolist() == [0, 0, 0, 1, 0, 0] and tr[3] == 1


def test_membership_version_equals_the_set_version():
    a, b = _records(4, 60, 8, 128, 3, flip=0.5)
    off = [0, 7, 7, 33, 60]
    want = dg.routing_diff(a, b, off)
    got = dg.routing_diff_fast(a, b, 128, off)
    for w, g in zip(want, got):
        assert np.array_equal(np.asarray(w), np.asarray(g))
