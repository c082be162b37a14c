"""Pins for the float64 oracle: what the paper and the mathematics fix, computed here without
calling the oracle for the expected value (closed forms, brute force, library routines,
theorems).  A plausible slip anywhere in the oracle (dropped term, swapped p/q, wrong sign,
wrong tie-break, union counted twice) fails at least one of these.
"""
import math
import os

import numpy as np
import pytest
import scipy.special

from oracle import obrs_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _softmax64(l):
    l = np.asarray(l, dtype=np.float64)
    return scipy.special.softmax(l)


def _rand_logits(rng, V, sigma=2.0):
    return rng.normal(0.0, sigma, V)


def _rows_from(outs):
    arr = np.zeros(len(outs), dtype=orc.ROW_DTYPE)
    for i, o in enumerate(outs):
        for name in orc.ROW_DTYPE.names:
            arr[name][i] = getattr(o, name)
    return arr


# ---- P10: a worked two-token example (derived by hand from Eq. obrs_accept / obrs_dist and
# the weight of Alg. 1 step 3; values stored in tests/golden/two_token_example.txt) -------------

def _read_golden(name):
    vals = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            k, v = line.split("=")
            vals[k.strip()] = [float(t) for t in v.split(",")]
    return vals


def test_two_token_hand_example():
    g = _read_golden("two_token_example.txt")
    q, p, lam = np.array(g["q"]), np.array(g["p"]), g["lambda"][0]
    lq, lp = np.log(q), np.log(p) + 3.25          # logits are defined up to a shift
    for x in (0, 1):
        out, kq, kp = orc.row(lq, lp, x, 0.0, lam, 2)
        assert out.accept == pytest.approx(g["accept"][x], rel=1e-14)
        assert out.z_exact == pytest.approx(g["Z"][0], rel=1e-14)
        assert out.z_approx == pytest.approx(g["Z"][0], rel=1e-14)
        assert out.logratio == pytest.approx(math.log(p[x] / q[x]), abs=1e-14)
        b, w, rho = orc.batch(_rows_from([out]), [1], lam, 1e9, 1e9)
        # kappa rescales Z; the un-corrected weight is w / kappa = Z * max(lambda, p/q)
        assert w[0] / b.kappa == pytest.approx(g["w"][x], rel=1e-13)
    qt, z = orc.post_rejection(lq, lp, lam)
    np.testing.assert_allclose(qt, g["q_tilde"], rtol=1e-14)
    assert list(kq) == [0, 1]          # q ties -> lowest id first
    assert list(kp) == [0, 1]


# ---- P12: log-sum-exp / log-softmax against library routines --------------------------------

@pytest.mark.parametrize("V,sigma", [(1, 1.0), (7, 3.0), (1024, 2.0), (5000, 30.0)])
def test_logsumexp_matches_scipy(V, sigma):
    rng = np.random.default_rng(V)
    l = _rand_logits(rng, V, sigma)
    assert orc.logsumexp(l) == pytest.approx(scipy.special.logsumexp(l), rel=1e-14, abs=1e-14)
    out, _, _ = orc.row(l, l + 1.0, V // 2, 0.5, 1.0, 1)
    assert out.logq_x == pytest.approx(scipy.special.log_softmax(l)[V // 2], abs=1e-12)


def test_logsumexp_large_offset_and_minus_inf():
    l = np.array([1000.0, 1000.0, -np.inf, 999.0])
    assert orc.logsumexp(l) == pytest.approx(1000.0 + math.log(2.0 + math.exp(-1.0)), rel=1e-15)
    l = np.array([-1000.0, -1001.0])
    assert orc.logsumexp(l) == pytest.approx(-1000.0 + math.log1p(math.exp(-1.0)), rel=1e-15)


# ---- top-k: order (value desc, id asc) against a stable library sort and an O(V^2) rank count --

@pytest.mark.parametrize("V,k", [(16, 5), (300, 300), (1024, 32), (4096, 256)])
def test_topk_matches_stable_argsort(V, k):
    rng = np.random.default_rng(V + k)
    l = np.round(rng.normal(0, 1, V) * 4) / 4          # coarse grid -> many exact ties
    want = np.argsort(-l, kind="stable")[:k]
    np.testing.assert_array_equal(orc.topk(l, k), want)


def test_topk_rank_count_bruteforce():
    rng = np.random.default_rng(5)
    for V in (3, 8, 16):
        l = rng.integers(-2, 3, V).astype(np.float64)
        for k in range(1, V + 1):
            got = orc.topk(l, k)
            rank = [sum((l[j] > l[i]) or (l[j] == l[i] and j < i) for j in range(V)) for i in range(V)]
            want = sorted(range(V), key=lambda i: rank[i])[:k]
            assert list(got) == want


# ---- P11: constant rows pin tie-break and the set union ---------------------------------------

@pytest.mark.parametrize("lam", [0.5, 1.0, 4.0])
def test_constant_logits(lam):
    V, k = 96, 10
    out, kq, kp = orc.row(np.full(V, 1.5), np.full(V, -0.25), 17, 0.3, lam, k)
    assert list(kq) == list(range(k)) and list(kp) == list(range(k))
    assert out.union_size == k
    assert out.z_exact == pytest.approx(min(1.0, 1.0 / lam), rel=1e-13)
    assert out.z_approx == pytest.approx(k / V * min(1.0, 1.0 / lam), rel=1e-13)


def test_union_is_a_set_and_bounds():
    # q peaks on ids 0..3, p on ids 2..5 -> union of top-4 lists has 6 members
    lq = np.array([9., 8., 7., 6., 0., 0., 0., 0.])
    lp = np.array([0., 0., 7., 9., 8., 6., 0., 0.])
    out, kq, kp = orc.row(lq, lp, 0, 0.5, 1.0, 4)
    assert list(kq) == [0, 1, 2, 3] and list(kp) == [3, 4, 2, 5]
    assert out.union_size == 6
    q, p = _softmax64(lq), _softmax64(lp)
    assert out.z_approx == pytest.approx(np.minimum(q, p)[:6].sum(), rel=1e-13)


# ---- P1, P2, P7: normaliser identities --------------------------------------------------------

@pytest.mark.parametrize("lam", [0.3, 1.0, 2.5])
def test_normaliser_identities(lam):
    rng = np.random.default_rng(11)
    V = 257
    lq, lp = _rand_logits(rng, V), _rand_logits(rng, V)
    q, p = _softmax64(lq), _softmax64(lp)
    qt, z = orc.post_rejection(lq, lp, lam)
    assert qt.sum() == pytest.approx(1.0, abs=1e-13)                       # P1
    a = np.minimum(1.0, p / (lam * q))
    assert z == pytest.approx((q * a).sum(), rel=1e-13)                    # P2: Z = E_q[a]
    A = p / q > lam                                                        # P7: partition form
    assert z == pytest.approx(q[A].sum() + p[~A].sum() / lam, rel=1e-13)
    assert z <= min(1.0, 1.0 / lam) + 1e-15
    out, _, _ = orc.row(lq, lp, 3, 0.5, lam, 8)
    assert out.z_exact == pytest.approx(z, rel=1e-14)
    assert out.accept == pytest.approx(a[3], rel=1e-13)


# ---- P3: matched distributions ------------------------------------------------------------------

@pytest.mark.parametrize("lam", [0.25, 1.0, 3.0])
def test_matched_distributions(lam):
    rng = np.random.default_rng(3)
    V = 200
    l = _rand_logits(rng, V)
    for x in (0, 57, V - 1):
        out, _, _ = orc.row(l, l - 7.0, x, 0.999, lam, V)      # a shift of the logits changes nothing
        assert out.logratio == pytest.approx(0.0, abs=1e-13)
        assert out.accept == pytest.approx(min(1.0, 1.0 / lam), rel=1e-13)
        assert out.z_exact == pytest.approx(min(1.0, 1.0 / lam), rel=1e-13)
        b, w, _ = orc.batch(_rows_from([out]), [1], lam, 1e9, 1e9)
        assert w[0] / b.kappa == pytest.approx(1.0, rel=1e-12)     # p / q~ = 1


# ---- strict "<" of the Bernoulli draw (Alg. 2) ----------------------------------------------

def test_mask_is_strict_less_than():
    l = np.array([0.0, 1.0, 2.0])
    out, _, _ = orc.row(l, l, 1, 0.5, 2.0, 1)           # a = 1/2 exactly
    assert out.accept == 0.5 and out.mask == 0
    out, _, _ = orc.row(l, l, 1, np.nextafter(0.5, 0.0), 2.0, 1)
    assert out.mask == 1
    out, _, _ = orc.row(l, l, 1, 0.0, 1.0, 1)
    assert out.mask == 1


# ---- P4, P5: the top-k estimate --------------------------------------------------------------

def test_topk_estimate_monotone_and_exact_at_full_k():
    rng = np.random.default_rng(21)
    V = 512
    lq = _rand_logits(rng, V, 3.0)
    lp = lq + rng.normal(0, 1.5, V)
    prev = 0.0
    for k in (1, 2, 5, 20, 100, 400, V):
        out, _, _ = orc.row(lq, lp, 0, 0.5, 1.3, k)
        assert out.z_approx <= out.z_exact + 1e-15
        assert out.z_approx >= prev - 1e-15
        assert k <= out.union_size <= min(2 * k, V)
        prev = out.z_approx
    assert out.z_approx == out.z_exact                  # k = V: identical sums, bit for bit
    assert out.union_size == V


def test_topk_estimate_against_numpy():
    rng = np.random.default_rng(22)
    V, k, lam = 1000, 20, 0.8
    lq = _rand_logits(rng, V, 3.0)
    lp = lq + rng.normal(0, 2.0, V)
    q, p = _softmax64(lq), _softmax64(lp)
    U = set(np.argsort(-lq, kind="stable")[:k]) | set(np.argsort(-lp, kind="stable")[:k])
    want = sum(min(q[v], p[v] / lam) for v in sorted(U))
    out, _, _ = orc.row(lq, lp, 5, 0.5, lam, k)
    assert out.union_size == len(U)
    assert out.z_approx == pytest.approx(want, rel=1e-12)


# ---- P6: Sec. 3.3 theorem, App. A proposition and corollary ------------------------------------

def _kl(p, r):
    m = p > 0
    return float((p[m] * (np.log(p[m]) - np.log(r[m]))).sum())


def test_kl_contraction_and_monotonicity():
    rng = np.random.default_rng(31)
    for V in (5, 64, 700):
        lq, lp = _rand_logits(rng, V), _rand_logits(rng, V)
        q, p = _softmax64(lq), _softmax64(lp)
        ratio = p / q
        kl_pq = _kl(p, q)
        prev = None
        for lam in (ratio.min() * 0.5, 0.2, 0.7, 1.0, 1.9, 6.0, ratio.max() * 1.01):
            out, _, _ = orc.row(lq, lp, 0, 0.5, lam, 1)
            assert out.kl_p_q == pytest.approx(kl_pq, rel=1e-11, abs=1e-13)
            qt, _ = orc.post_rejection(lq, lp, lam)
            assert out.kl_p_qtilde == pytest.approx(_kl(p, qt), rel=1e-9, abs=1e-12)
            assert out.kl_p_qtilde <= kl_pq + 1e-12
        for lam in sorted([ratio.min() * 0.5, 0.2, 0.7, 1.0, 1.9, 6.0, ratio.max() * 1.01]):
            out, _, _ = orc.row(lq, lp, 0, 0.5, lam, 1)
            if prev is not None:
                assert out.kl_p_qtilde <= prev + 1e-12      # non-increasing in lambda
            prev = out.kl_p_qtilde
        qt, z = orc.post_rejection(lq, lp, ratio.max() * 1.01)   # classical rejection sampling
        np.testing.assert_allclose(qt, p, rtol=1e-12)
        assert z == pytest.approx(1.0 / (ratio.max() * 1.01), rel=1e-12)
        qt, z = orc.post_rejection(lq, lp, ratio.min() * 0.5)    # everything accepted
        np.testing.assert_allclose(qt, q, rtol=1e-12)
        assert z == pytest.approx(1.0, rel=1e-12)


# ---- Sec. 3.2 (numerical simulation): Dirichlet pairs at growing distance ----------------------
# The paper's own noise model is not printed, so nothing numeric is taken from its figure; what the
# mathematics fixes on such pairs is: at lambda = 1 the normaliser (= acceptance rate) is one minus
# the total variation distance, hence at least 1 - sqrt(KL(p || q) / 2) (Pinsker), and the
# post-rejection distribution is never farther from p than q was.

@pytest.mark.parametrize("noise", [0.05, 0.3, 1.0, 2.5])
def test_dirichlet_pairs_acceptance_is_one_minus_total_variation(noise):
    rng = np.random.default_rng(int(noise * 100) + 5)
    V = 500
    for _ in range(6):
        q = rng.dirichlet(np.full(V, 0.3)) + 1e-300
        lq = np.log(q)
        lp = lq + rng.normal(0.0, noise, V)
        p = _softmax64(lp)
        q = _softmax64(lq)
        out, _, _ = orc.row(lq, lp, 0, 0.5, 1.0, 16)
        tv = 0.5 * np.abs(p - q).sum()
        assert out.z_exact == pytest.approx(1.0 - tv, rel=1e-12)
        assert out.z_exact >= 1.0 - math.sqrt(_kl(p, q) / 2.0) - 1e-12
        assert out.kl_p_qtilde <= out.kl_p_q + 1e-12
        qt, z = orc.post_rejection(lq, lp, 1.0)
        np.testing.assert_allclose(qt, np.minimum(q, p) / (1.0 - tv), rtol=1e-12)


# ---- P8: w = p / q~ -------------------------------------------------------------------------

def test_weight_is_ratio_to_post_rejection_distribution():
    rng = np.random.default_rng(41)
    V, lam = 50, 1.2
    lq, lp = _rand_logits(rng, V), _rand_logits(rng, V)
    p = _softmax64(lp)
    qt, _ = orc.post_rejection(lq, lp, lam)
    for x in range(0, V, 7):
        out, _, _ = orc.row(lq, lp, x, 0.5, lam, V)
        b, w, _ = orc.batch(_rows_from([out]), [1], lam, 1e9, 1e9)
        assert (w[0] / b.kappa) * qt[x] == pytest.approx(p[x], rel=1e-12)


# ---- P9: exhaustive brute force on tiny vocabularies ---------------------------------------------

def test_bruteforce_tiny_vocab():
    rng = np.random.default_rng(51)
    for V in (2, 3, 5, 9, 16):
        for lam in (0.5, 1.0, 2.0):
            lq = np.round(rng.normal(0, 1.5, V) * 2) / 2
            lp = np.round(rng.normal(0, 1.5, V) * 2) / 2
            eq, ep = np.exp(lq), np.exp(lp)
            q, p = eq / eq.sum(), ep / ep.sum()
            kept = np.array([q[x] * min(1.0, p[x] / (lam * q[x])) for x in range(V)])
            Z = kept.sum()
            for k in (1, max(1, V // 2), V):
                def rank(l, i):
                    return sum((l[j] > l[i]) or (l[j] == l[i] and j < i) for j in range(V))
                bits = 0
                for i in range(V):
                    if rank(lq, i) < k:
                        bits |= 1 << i
                    if rank(lp, i) < k:
                        bits |= 1 << i
                members = [i for i in range(V) if bits >> i & 1]
                for x in range(V):
                    out, kq, kp = orc.row(lq, lp, x, 0.5, lam, k)
                    assert out.accept * q[x] == pytest.approx(kept[x], rel=1e-12)   # P(x kept)
                    assert out.z_exact == pytest.approx(Z, rel=1e-12)
                    assert out.union_size == len(members)
                    assert sorted(set(kq) | set(kp)) == members
                    assert out.z_approx == pytest.approx(kept[members].sum(), rel=1e-12)


def test_budget_optimality_against_random_rules():
    # App. A.2: among acceptance rules with the same budget sum_v q_v alpha_v = Z, none gives a
    # smaller KL(p || kept) than the OBRS rule.
    rng = np.random.default_rng(61)
    V, lam = 8, 0.9
    lq, lp = _rand_logits(rng, V, 1.0), _rand_logits(rng, V, 1.0)
    q, p = _softmax64(lq), _softmax64(lp)
    out, _, _ = orc.row(lq, lp, 0, 0.5, lam, 1)
    a_star = np.minimum(1.0, p / (lam * q))
    budget = (q * a_star).sum()
    for _ in range(300):
        a = a_star.copy()
        for _ in range(6):                       # budget-preserving pairwise moves inside [0,1]^V
            i, j = rng.choice(V, 2, replace=False)
            hi = min((1 - a[i]) * q[i], a[j] * q[j])
            d = rng.uniform(0, hi) * 0.9
            a[i] += d / q[i]
            a[j] -= d / q[j]
        assert (q * a).sum() == pytest.approx(budget, rel=1e-12)
        kept = q * a / budget
        assert _kl(p, kept) >= out.kl_p_qtilde - 1e-12


# ---- P12b: Monte-Carlo run of the sampling loop of Alg. 2 ---------------------------------------

def test_monte_carlo_sampler_matches_post_rejection_distribution():
    rng = np.random.default_rng(71)
    V, lam, N = 6, 1.4, 400_000
    lq, lp = _rand_logits(rng, V, 1.0), _rand_logits(rng, V, 1.0)
    q, p = _softmax64(lq), _softmax64(lp)
    xs = rng.choice(V, size=N, p=q)
    us = rng.random(N)
    acc = us < np.minimum(1.0, p[xs] / (lam * q[xs]))
    qt, z = orc.post_rejection(lq, lp, lam)
    rate = acc.mean()
    assert abs(rate - z) < 4 * math.sqrt(z * (1 - z) / N)
    hist = np.bincount(xs[acc], minlength=V) / acc.sum()
    assert np.all(np.abs(hist - qt) < 4 * np.sqrt(qt * (1 - qt) / acc.sum()) + 1e-9)


# ---- batch stage: bias correction (Sec. 4.4.2) -------------------------------------------------

def test_kappa_closed_forms_and_padding():
    l = np.array([0.0, 1.0, 2.0, 3.0])
    outs = [orc.row(l, l, t % 4, 0.5, 1.0, 1)[0] for t in range(8)]     # Z_approx = q(3) each
    outs.append(orc.row(l, l, -1, 0.5, 1.0, 1)[0])                       # padding row
    rows = _rows_from(outs)
    q3 = float(_softmax64(l)[3])
    mask = [1, 1, 1, 0, 1, 1, 0, 1, 1]                                   # 6 of 8 valid accepted
    b, w, rho = orc.batch(rows, mask, 1.0, 0.7, 1e9)
    assert (b.n_valid, b.n_accept) == (8, 6)
    assert b.alpha_hat == pytest.approx(0.75)
    assert b.mean_z_approx == pytest.approx(q3, rel=1e-14)
    assert b.kappa == pytest.approx(0.75 / q3, rel=1e-14)
    np.testing.assert_allclose(w[:8], 0.75, rtol=1e-13)                  # kappa Z max(1, 1) = alpha
    np.testing.assert_allclose(rho[:8], 0.7, rtol=1e-13)                 # clipped by c1
    assert w[8] == 0.0 and rho[8] == 0.0
    b2, _, _ = orc.batch(rows, mask, 1.0, 0.7, 1e9, use_expected_alpha=True)
    assert b2.kappa == pytest.approx(1.0 / q3, rel=1e-14)                # mean a = 1


def test_rho_reference_factor():
    rng = np.random.default_rng(81)
    lq, lp = _rand_logits(rng, 30), _rand_logits(rng, 30)
    out, _, _ = orc.row(lq, lp, 4, 0.1, 1.0, 30)
    rows = _rows_from([out])
    _, w, rho0 = orc.batch(rows, [1], 1.0, 1e9, 3.0)
    for fac, c2, want in ((2.0, 3.0, 2.0), (5.0, 3.0, 3.0), (0.25, 3.0, 0.25)):
        ref = np.array([out.logp_x + math.log(fac)])
        _, w2, rho = orc.batch(rows, [1], 1.0, 1e9, c2, ref_logprob=ref)
        assert w2[0] == w[0]
        assert rho[0] == pytest.approx(rho0[0] * want, rel=1e-13)


def test_bias_correction_recovers_true_normaliser():
    # Z equals the expected acceptance rate, so kappa * Z_approx estimates Z without bias:
    # many draws x ~ q at one position, Bernoulli(a(x)) masks, small k.
    rng = np.random.default_rng(91)
    V, lam, k, B = 40, 1.0, 2, 60_000
    lq = _rand_logits(rng, V, 1.0)
    lp = lq + rng.normal(0, 1.0, V)
    q = _softmax64(lq)
    per_x = [orc.row(lq, lp, x, 0.0, lam, k)[0] for x in range(V)]
    xs = rng.choice(V, size=B, p=q)
    us = rng.random(B)
    rows = _rows_from([per_x[x] for x in xs])
    mask = (us < rows["accept"]).astype(np.int32)
    b, _, _ = orc.batch(rows, mask, lam, 1e9, 1e9)
    z = per_x[0].z_exact
    assert per_x[0].z_approx < 0.9 * z                       # the raw estimate is biased low
    assert abs(b.kappa * per_x[0].z_approx - z) < 4 * math.sqrt(z * (1 - z) / B)


# ---- multi-row driver equals the single-row routine, for every storage dtype ---------------------

def test_rows_driver_matches_single_rows_and_widens_exactly():
    rng = np.random.default_rng(101)
    T, V, k = 9, 333, 7
    a32 = rng.normal(0, 2, (T, V)).astype(np.float32)
    p32 = (a32 + rng.normal(0, 1, (T, V))).astype(np.float32)
    x = rng.integers(0, V, T).astype(np.int32)
    x[4] = -1
    u = rng.random(T).astype(np.float32)
    bits_a = (a32.view(np.uint32) >> 16).astype(np.uint16)        # truncation: any bf16 pattern will do
    bits_p = (p32.view(np.uint32) >> 16).astype(np.uint16)
    for A, P in ((a32, p32), (bits_a, bits_p)):
        if A.dtype == np.uint16:
            A64 = (A.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
            P64 = (P.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        else:
            A64, P64 = A.astype(np.float64), P.astype(np.float64)
        R = orc.rows(A, P, x, u, 1.1, k, n_threads=3)
        for t in range(T):
            out, kq, kp = orc.row(A64[t], P64[t], x[t], float(u[t]), 1.1, k)
            for name in ("logq_x", "logp_x", "accept", "z_approx", "z_exact", "mask", "valid"):
                assert R.out[name][t] == getattr(out, name)
            if x[t] >= 0:
                np.testing.assert_array_equal(R.topk_q[t], kq)
                np.testing.assert_array_equal(R.topk_p[t], kp)


# ---- distillation term (Sec. 4.2 (3), Eq. distill_loss): KL(p || q) per token, batch mean ---------

def test_distillation_kl_against_scipy_rel_entr_and_batch_mean():
    rng = np.random.default_rng(111)
    V = 300
    outs, want = [], []
    for sigma in (0.0, 0.3, 1.0, 2.5):
        lq = _rand_logits(rng, V)
        lp = lq + rng.normal(0, sigma, V) if sigma > 0 else lq.copy()
        q, p = _softmax64(lq), _softmax64(lp)
        out, _, _ = orc.row(lq, lp, 0, 0.5, 1.0, 4)
        kl = float(scipy.special.rel_entr(p, q).sum())
        assert out.kl_p_q == pytest.approx(kl, rel=1e-10, abs=1e-14)
        assert out.kl_p_q >= -1e-15                      # Gibbs' inequality
        outs.append(out)
        want.append(kl)
    assert outs[0].kl_p_q == pytest.approx(0.0, abs=1e-15)      # p == q
    outs.append(orc.row(lq, lp, -1, 0.5, 1.0, 4)[0])             # padding row is not averaged
    b, _, _ = orc.batch(_rows_from(outs), [1] * 5, 1.0, 3.0, 3.0)
    assert b.mean_kl_p_q == pytest.approx(sum(want) / 4, rel=1e-12)
    # KL is not symmetric: swapping the roles of the two rows changes the value
    out_sw, _, _ = orc.row(lp, lq, 0, 0.5, 1.0, 4)
    assert abs(out_sw.kl_p_q - outs[3].kl_p_q) > 1e-3


# ---- gradient of the distillation term w.r.t. the actor logits: q - p ------------------------------

def test_distillation_gradient_against_finite_differences():
    rng = np.random.default_rng(222)
    V = 40
    lq = _rand_logits(rng, V)
    lp = lq + rng.normal(0, 1.0, V)
    p = _softmax64(lp)

    def kl_of(lq_):                                   # scipy only: no oracle call in the expected value
        return float(scipy.special.rel_entr(p, _softmax64(lq_)).sum())

    g = orc.distill_grad_row(lq, lp, 1.0)
    h = 1e-5
    for v in range(V):
        e = np.zeros(V)
        e[v] = h
        fd = (kl_of(lq + e) - kl_of(lq - e)) / (2 * h)
        assert g[v] == pytest.approx(fd, abs=2e-9)
    assert abs(g.sum()) < 1e-14                       # softmax gradients sum to zero
    np.testing.assert_allclose(orc.distill_grad_row(lq, lp, -2.5), -2.5 * g, rtol=1e-14, atol=0)
    np.testing.assert_array_equal(orc.distill_grad_row(lq, lq, 1.0), np.zeros(V))   # p == q
    # two tokens, closed form: q = (s(a), 1 - s(a)), p = (s(b), 1 - s(b)) with the logistic function s
    a, b = 0.7, -1.1
    g2 = orc.distill_grad_row([a, 0.0], [b, 0.0], 1.0)
    s = lambda z: 1.0 / (1.0 + math.exp(-z))
    assert g2[0] == pytest.approx(s(a) - s(b), rel=1e-14)
    assert g2[1] == pytest.approx(s(b) - s(a), rel=1e-14)


def test_distillation_gradient_batch_driver():
    rng = np.random.default_rng(223)
    T, V = 5, 33
    a32 = rng.normal(0, 2, (T, V)).astype(np.float32)
    p32 = (a32 + rng.normal(0, 1, (T, V))).astype(np.float32)
    x = np.array([3, -1, 0, V, 7], dtype=np.int32)    # row 1 padding, row 3 id out of range
    rs = np.array([1.0, 2.0, 0.5, 1.0, -1.5], dtype=np.float32)
    G = orc.distill_grad(a32, p32, x, rs, scale=0.25)
    for t in range(T):
        if x[t] < 0 or x[t] >= V:
            np.testing.assert_array_equal(G[t], np.zeros(V))
        else:
            want = 0.25 * float(rs[t]) * (_softmax64(a32[t]) - _softmax64(p32[t]))
            np.testing.assert_allclose(G[t], want, rtol=1e-12, atol=1e-16)
    # bf16 storage is widened exactly
    abits = (a32.view(np.uint32) >> 16).astype(np.uint16)
    pbits = (p32.view(np.uint32) >> 16).astype(np.uint16)
    Gb = orc.distill_grad(abits, pbits, x)
    a_w = (abits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    p_w = (pbits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    np.testing.assert_allclose(Gb[0], _softmax64(a_w[0]) - _softmax64(p_w[0]), rtol=1e-12, atol=1e-16)


# ---- stored-actor form (Alg. 1: Phase 1 keeps TopK_inf log-probabilities and p_inf(a_t)) ------------

def _stable_topk(l, k):
    return np.argsort(-np.asarray(l), kind="stable")[:k]


def _z_stored_numpy(lp, ids_q, logq_ids, lam, k, rule):
    """Z_approx of the stored form written out with numpy sets (no oracle call)."""
    V = lp.size
    p = _softmax64(lp)
    q_of = {}
    for v, lq in zip(ids_q, logq_ids):
        if 0 <= v < V and v not in q_of:
            q_of[int(v)] = math.exp(lq)
    n = len(q_of)
    kth = min(q_of.values()) if n else 1.0
    if rule == 0 or n == V:
        qhat = 0.0
    elif rule == 1:
        qhat = kth
    else:
        qhat = min(kth, max(0.0, 1.0 - sum(q_of.values())) / (V - n))
    z = sum(min(qv, p[v] / lam) for v, qv in q_of.items())
    extra = [int(v) for v in _stable_topk(lp, k) if int(v) not in q_of]
    z += sum(min(qhat, p[v] / lam) for v in extra)
    return z, n + len(extra)


@pytest.mark.parametrize("rule", [0, 1, 2])
def test_stored_actor_form_against_numpy_sets(rule):
    rng = np.random.default_rng(333 + rule)
    for V, k, lam in ((50, 5, 1.0), (200, 16, 0.6), (64, 64, 2.0), (300, 20, 1.3)):
        lq = _rand_logits(rng, V)
        lp = lq + rng.normal(0, 1.0, V)
        logq = lq - scipy.special.logsumexp(lq)
        ids_q = _stable_topk(lq, k)
        x = int(rng.integers(V))
        u = float(rng.random())
        out, kp = orc.row_stored(lp, ids_q, logq[ids_q], logq[x], x, u, lam, k, rule)
        z, usize = _z_stored_numpy(lp, ids_q, logq[ids_q], lam, k, rule)
        assert out.z_approx == pytest.approx(z, rel=1e-12)
        assert out.union_size == usize
        np.testing.assert_array_equal(kp, _stable_topk(lp, k))
        logp = lp - scipy.special.logsumexp(lp)
        assert out.logratio == pytest.approx(logp[x] - logq[x], abs=1e-12)
        assert out.accept == pytest.approx(min(1.0, math.exp(logp[x] - logq[x]) / lam), rel=1e-12)
        assert out.mask == (1 if u < out.accept else 0)
        assert math.isnan(out.z_exact)


def test_stored_actor_form_brackets_and_reduces_to_the_full_form():
    rng = np.random.default_rng(337)
    V, k, lam = 400, 24, 1.1
    lq = _rand_logits(rng, V)
    lp = lq + rng.normal(0, 1.5, V)
    logq = lq - scipy.special.logsumexp(lq)
    ids_q = _stable_topk(lq, k)
    full, kq_full, _ = orc.row(lq, lp, 7, 0.5, lam, k)
    np.testing.assert_array_equal(kq_full, ids_q)
    z = [orc.row_stored(lp, ids_q, logq[ids_q], logq[7], 7, 0.5, lam, k, r)[0].z_approx for r in (0, 1, 2)]
    # dropping the unknown terms under-estimates, the k-th-value bound over-estimates the estimate
    # made with the true q; the even share of the remaining mass lies between the two
    assert z[0] <= full.z_approx + 1e-15 <= z[1] + 2e-15
    assert z[0] <= z[2] <= z[1]
    assert z[0] < z[1]                                         # the lists differ for this seed
    assert full.union_size == orc.row_stored(lp, ids_q, logq[ids_q], logq[7], 7, 0.5, lam, k, 1)[0].union_size
    # with the whole vocabulary stored nothing is unknown: every rule gives the full form's value
    allv = np.arange(V)
    fullV, _, _ = orc.row(lq, lp, 7, 0.5, lam, V)
    for r in (0, 1, 2):
        o, _ = orc.row_stored(lp, allv, logq, logq[7], 7, 0.5, lam, V, r)
        assert o.z_approx == pytest.approx(fullV.z_approx, rel=1e-13)
        assert o.z_approx == pytest.approx(fullV.z_exact, rel=1e-13)
    # p == q and lambda <= 1: acceptance 1; the estimate is the stored mass (+ nothing new in TopK_new)
    o, _ = orc.row_stored(lq, ids_q, logq[ids_q], logq[7], 7, 0.99, 1.0, k, 1)
    assert o.accept == 1.0 and o.mask == 1
    assert o.z_approx == pytest.approx(np.exp(logq[ids_q]).sum(), rel=1e-13)
    assert o.union_size == k


def test_stored_actor_form_unused_slots_duplicates_and_batch_driver():
    rng = np.random.default_rng(339)
    T, V, k = 6, 120, 8
    pol = rng.normal(0, 2, (T, V)).astype(np.float32)
    act = (pol + rng.normal(0, 1, (T, V))).astype(np.float64)
    logq = act - scipy.special.logsumexp(act, axis=1, keepdims=True)
    ids = np.stack([_stable_topk(act[t], k) for t in range(T)]).astype(np.int32)
    lq_ids = np.take_along_axis(logq, ids, axis=1).astype(np.float32)
    ids[1, 3] = -1                                            # an unused slot
    ids[3, 5] = ids[3, 0]                                     # a repeated id counts once
    x = np.array([3, 5, -1, 9, 0, 11], dtype=np.int32)         # row 2 is padding
    lqx = logq[np.arange(T), np.maximum(x, 0)].astype(np.float32)
    u = rng.random(T).astype(np.float32)
    R = orc.rows_stored(pol, ids, lq_ids, lqx, x, u, 1.2, k, orc.TAIL_REST)
    for t in range(T):
        if x[t] < 0:
            assert R.out["valid"][t] == 0 and R.out["z_approx"][t] == 0.0
            continue
        z, usize = _z_stored_numpy(pol[t].astype(np.float64), ids[t], lq_ids[t].astype(np.float64), 1.2, k, 2)
        assert R.out["z_approx"][t] == pytest.approx(z, rel=1e-12)
        assert R.out["union_size"][t] == usize
        o, kp = orc.row_stored(pol[t], ids[t], lq_ids[t], lqx[t], x[t], u[t], 1.2, k, 2)
        assert o.z_approx == R.out["z_approx"][t] and o.mask == R.out["mask"][t]
        np.testing.assert_array_equal(kp, R.topk_p[t])


# ---- adjustment functions F (Sec. 2) and the third distribution's token log-probability -----------

def test_adjustment_functions_closed_forms():
    assert orc.adjust(0.7, orc.F_TRUNCATE, 3.0) == 0.7 and orc.adjust(5.0, orc.F_TRUNCATE, 3.0) == 3.0
    assert orc.adjust(5.0, orc.F_IDENTITY, 3.0) == 5.0
    for w, want in ((0.4, 0.0), (0.5, 0.5), (1.3, 1.3), (2.0, 2.0), (2.01, 0.0)):
        assert orc.adjust(w, orc.F_BAND, 3.0, 0.5, 2.0) == want
    # in the batch stage: w = kappa Z max(lambda, p/q); rho = F(w) min(p_ref/p, c2)
    rows = np.zeros(3, dtype=orc.ROW_DTYPE)
    rows["valid"] = 1
    rows["z_approx"] = [0.5, 0.25, 0.75]
    rows["accept"] = [1.0, 0.5, 0.25]
    rows["logratio"] = np.log([4.0, 0.5, 1.0])
    rows["logp_x"] = np.log([0.2, 0.1, 0.3])
    mask = [1, 1, 0]
    ref = np.log([0.1, 0.4, 0.3])
    kappa = (2 / 3) / 0.5
    w_want = kappa * np.array([0.5 * 4.0, 0.25 * 1.0, 0.75 * 1.0])       # lambda = 1
    second = np.minimum(np.array([0.5, 4.0, 1.0]), 3.0)
    for mode, F in ((orc.F_TRUNCATE, lambda w: np.minimum(w, 1.5)), (orc.F_IDENTITY, lambda w: w),
                    (orc.F_BAND, lambda w: np.where((w >= 0.5) & (w <= 2.0), w, 0.0))):
        b, w, rho = orc.batch_f(rows, mask, 1.0, mode, 1.5, 0.5, 2.0, 3.0, ref)
        assert b.kappa == pytest.approx(kappa, rel=1e-14)
        np.testing.assert_allclose(w, w_want, rtol=1e-14)
        np.testing.assert_allclose(rho, F(w_want) * second, rtol=1e-14)
    b0, w0, rho0 = orc.batch(rows, mask, 1.0, 1.5, 3.0, ref)             # the default is the truncation
    b1, w1, rho1 = orc.batch_f(rows, mask, 1.0, orc.F_TRUNCATE, 1.5, 9.0, 9.0, 3.0, ref)
    np.testing.assert_array_equal(rho0, rho1)


def test_token_logprob_against_scipy_log_softmax():
    rng = np.random.default_rng(444)
    T, V = 7, 123
    l32 = rng.normal(0, 3, (T, V)).astype(np.float32)
    x = np.array([0, 5, -1, 122, V, 60, 7], dtype=np.int32)
    got = orc.token_logprob(l32, x)
    ls = scipy.special.log_softmax(l32.astype(np.float64), axis=1)
    for t in range(T):
        if x[t] < 0:
            assert got[t] == 0.0
        elif x[t] >= V:
            assert math.isnan(got[t])
        else:
            assert got[t] == pytest.approx(ls[t, x[t]], abs=1e-13)
    bits = (l32.view(np.uint32) >> 16).astype(np.uint16)
    wide = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    gb = orc.token_logprob(bits, np.full(T, 3, np.int32))
    np.testing.assert_allclose(gb, scipy.special.log_softmax(wide, axis=1)[:, 3], atol=1e-13)


# ---- the scaling factor for an acceptance budget (Sec. 3.3, Theorem 2) ------------------------------

def _z_of_lambda(q, p, lam):
    return float(np.minimum(q, p / lam).sum())


def test_lambda_for_budget_against_bisection_and_closed_forms():
    rng = np.random.default_rng(555)
    V = 200
    lq = _rand_logits(rng, V)
    lp = lq + rng.normal(0, 1.2, V)
    q, p = _softmax64(lq), _softmax64(lp)
    prev = None
    for abar in (0.999, 0.9, 0.5, 0.2, 0.05, 0.001):
        lam = orc.lambda_for_budget(lq, lp, abar)
        assert _z_of_lambda(q, p, lam) == pytest.approx(abar, rel=1e-12)        # the budget is met exactly
        lo, hi = 1e-12, 1e12                                                     # plain bisection on Z
        for _ in range(200):
            mid = math.sqrt(lo * hi)
            lo, hi = (mid, hi) if _z_of_lambda(q, p, mid) > abar else (lo, mid)
        assert lam == pytest.approx(math.sqrt(lo * hi), rel=1e-9)
        qt, z = orc.post_rejection(lq, lp, lam)                                  # and through Eq. obrs_dist
        assert z == pytest.approx(abar, rel=1e-12)
        assert prev is None or lam > prev                                        # smaller budget, larger lambda
        prev = lam
    # budget 1: the largest lambda that still accepts everything is min_v p/q
    assert orc.lambda_for_budget(lq, lp, 1.0) == pytest.approx(float((p / q).min()), rel=1e-12)
    # p == q: Z(lambda) = min(1, 1/lambda)
    assert orc.lambda_for_budget(lq, lq, 0.25) == pytest.approx(4.0, rel=1e-12)
    assert orc.lambda_for_budget(lq, lq, 1.0) == pytest.approx(1.0, rel=1e-12)
    # beyond the largest ratio Z = 1/lambda
    tiny = 0.5 / float((p / q).max())
    assert orc.lambda_for_budget(lq, lp, tiny) == pytest.approx(1.0 / tiny, rel=1e-12)
    # two tokens by hand: q = (.5, .5), p = (.8, .2): Z = .5 + .2/lambda on [0.4, 1.6] -> abar = .7 at lambda = 1
    l2q, l2p = np.log([0.5, 0.5]), np.log([0.8, 0.2])
    assert orc.lambda_for_budget(l2q, l2p, 0.7) == pytest.approx(1.0, rel=1e-13)
    assert orc.lambda_for_budget(l2q, l2p, 0.5) == pytest.approx(2.0, rel=1e-13)   # Z = 1/lambda beyond 1.6
    assert orc.lambda_for_budget(l2q, l2p, 0.9) == pytest.approx(0.5, rel=1e-13)   # .5 + .2/.5
    for bad in (0.0, -0.1, 1.0001, float("nan")):
        assert math.isnan(orc.lambda_for_budget(lq, lp, bad))
    # masked entries take no part
    lq2, lp2 = lq.copy(), lp.copy()
    lq2[:50] = -np.inf
    lp2[100:120] = -np.inf
    q2, p2 = _softmax64(lq2), _softmax64(lp2)
    lam = orc.lambda_for_budget(lq2, lp2, 0.3)
    with np.errstate(divide="ignore", invalid="ignore"):
        assert _z_of_lambda(q2, p2, lam) == pytest.approx(0.3, rel=1e-12)


def test_lambda_for_budget_rows_driver():
    rng = np.random.default_rng(556)
    T, V = 5, 77
    a = rng.normal(0, 2, (T, V)).astype(np.float32)
    p = (a + rng.normal(0, 1, (T, V))).astype(np.float32)
    x = np.array([1, -1, 3, 4, 5], dtype=np.int32)
    rt = np.array([0.9, 0.5, 0.5, 0.1, 1.0], dtype=np.float32)
    got = orc.lambda_for_budget_rows(a, p, x, 0.5, rt)
    got_scalar = orc.lambda_for_budget_rows(a, p, x, 0.5)
    for t in range(T):
        if x[t] < 0:
            assert got[t] == 0.0
            continue
        assert got[t] == orc.lambda_for_budget(a[t], p[t], float(rt[t]))
        assert _z_of_lambda(_softmax64(a[t]), _softmax64(p[t]), got_scalar[t]) == pytest.approx(0.5, rel=1e-12)


def test_lambda_for_budget_batch_against_bisection_on_the_mean():
    rng = np.random.default_rng(557)
    T, V = 9, 64
    a = rng.normal(0, 2, (T, V)).astype(np.float32)
    p = (a + rng.normal(0, 1, (T, V)) * rng.uniform(0.1, 2.0, (T, 1))).astype(np.float32)
    x = np.array([1, 2, -1, 3, 4, 5, -1, 6, 7], dtype=np.int32)
    valid = x >= 0
    Q = scipy.special.softmax(a[valid].astype(np.float64), axis=1)
    P = scipy.special.softmax(p[valid].astype(np.float64), axis=1)

    def zbar(lam):
        return float(np.minimum(Q, P / lam).sum(axis=1).mean())

    prev = None
    for abar in (0.95, 0.6, 0.3, 0.02):
        lam = orc.lambda_for_budget_batch(a, p, x, abar)
        assert zbar(lam) == pytest.approx(abar, rel=1e-12)
        lo, hi = 1e-12, 1e12
        for _ in range(200):
            mid = math.sqrt(lo * hi)
            lo, hi = (mid, hi) if zbar(mid) > abar else (lo, mid)
        assert lam == pytest.approx(math.sqrt(lo * hi), rel=1e-9)
        assert prev is None or lam > prev
        prev = lam
    assert orc.lambda_for_budget_batch(a, p, x, 1.0) == pytest.approx(float((P / Q).min()), rel=1e-12)
    # one valid row: the per-row solver's answer
    x1 = np.full(T, -1, np.int32); x1[4] = 0
    assert orc.lambda_for_budget_batch(a, p, x1, 0.4) == pytest.approx(orc.lambda_for_budget(a[4], p[4], 0.4), rel=1e-13)
    assert math.isnan(orc.lambda_for_budget_batch(a, p, np.full(T, -1, np.int32), 0.5))
    assert math.isnan(orc.lambda_for_budget_batch(a, p, x, 0.0))


# ---- logits of the fused lm_head form: exact products of the stored bf16 values ------------------
# (not an operation of the paper; the workload defines the logits as hidden states [n, d] times the
# vocabulary projection [d, V], both bf16, with nothing rounded before the OBRS computation)

def _bf16_as_fraction(bits):
    """The value of one bfloat16 bit pattern as an exact rational: 1 sign, 8 exponent, 7 fraction bits."""
    from fractions import Fraction
    sign = -1 if (bits >> 15) & 1 else 1
    e = (bits >> 7) & 0xff
    m = bits & 0x7f
    assert e != 0xff
    if e == 0:
        return sign * Fraction(m, 1 << 7) * Fraction(1, 1 << 126)
    two_e = Fraction(1 << (e - 127)) if e >= 127 else Fraction(1, 1 << (127 - e))
    return sign * Fraction((1 << 7) | m, 1 << 7) * two_e


def _bf16_bits(rng, shape, e_lo=121, e_hi=131):
    """Random bf16 bit patterns with biased exponents in [e_lo, e_hi] (values between 2^-6 and 2^5)."""
    s = rng.integers(0, 2, shape).astype(np.uint16)
    e = rng.integers(e_lo, e_hi + 1, shape).astype(np.uint16)
    m = rng.integers(0, 128, shape).astype(np.uint16)
    return (s << 15) | (e << 7) | m


@pytest.mark.parametrize("n,d,V", [(3, 5, 7), (4, 4, 4), (1, 9, 2), (2, 1, 6)])
def test_lm_head_logits_are_the_exact_products_of_the_bf16_values(n, d, V):
    rng = np.random.default_rng(500 + 31 * n + 7 * d + V)
    H, W = _bf16_bits(rng, (n, d)), _bf16_bits(rng, (d, V))
    H[0, 0] = 0x0000                     # +0
    W[-1, -1] = 0x8000                   # -0
    if d > 1:
        H[-1, 1] = 0x3f80                # 1.0
        W[1, 0] = 0xc000                 # -2.0
    got = orc.lm_head_logits(H, W)
    assert got.shape == (n, V) and got.dtype == np.float64
    for i in range(n):
        for v in range(V):
            exact = sum(_bf16_as_fraction(int(H[i, j])) * _bf16_as_fraction(int(W[j, v])) for j in range(d))
            # 16-bit products with exponents 22 apart at most: every partial sum is exact in float64
            assert got[i, v] == float(exact), (i, v)
            assert float(exact) == exact


def test_lm_head_logits_known_values_and_float_inputs():
    # H = [[1, 2, 0.5]], W rows (1, -1), (0.25, 3), (-4, 8): logits (1 + 0.5 - 2, -1 + 6 + 4) = (-0.5, 9)
    H = np.array([[0x3f80, 0x4000, 0x3f00]], dtype=np.uint16)
    W = np.array([[0x3f80, 0xbf80], [0x3e80, 0x4040], [0xc080, 0x4100]], dtype=np.uint16)
    np.testing.assert_array_equal(orc.lm_head_logits(H, W), [[-0.5, 9.0]])
    # the same through float inputs (values taken as they are)
    Hf = np.array([[1.0, 2.0, 0.5]], dtype=np.float32)
    Wf = np.array([[1.0, -1.0], [0.25, 3.0], [-4.0, 8.0]])
    np.testing.assert_array_equal(orc.lm_head_logits(Hf, Wf), [[-0.5, 9.0]])
    # a bit pattern is not its integer value: 0x3f80 is 1.0, not 16256
    assert orc.lm_head_logits(np.array([[0x3f80]], dtype=np.uint16), np.array([[0x3f80]], dtype=np.uint16))[0, 0] == 1.0


def test_row_with_a_sampled_id_outside_the_vocabulary_is_left_out():
    rng = np.random.default_rng(77)
    V = 12
    lq, lp = _rand_logits(rng, V), _rand_logits(rng, V)
    bad, _, _ = orc.row(lq, lp, V, 0.3, 1.0, 3)
    assert bad.valid == 0 and math.isnan(bad.accept) and math.isnan(bad.z_approx)
    good, kq, _ = orc.row(lq, lp, V - 1, 0.3, 1.0, 3)
    assert good.valid == 1
    b, w, rho = orc.batch(_rows_from([good, bad]), [good.mask, 0], 1.0, 3.0, 3.0)
    assert b.n_valid == 1 and b.mean_z_approx == good.z_approx and w[1] == 0.0 and rho[1] == 0.0
    sb, _ = orc.row_stored(lp, kq, lq[kq] - scipy.special.logsumexp(lq), -1.0, V + 5, 0.3, 1.0, 3, 1)
    assert sb.valid == 0 and math.isnan(sb.z_approx)
