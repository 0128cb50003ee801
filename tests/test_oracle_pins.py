"""Pins for the float64 CPU oracle: each test checks the oracle against something
the paper or the mathematics fixes, not against itself.  All CPU."""
import math
import os

import numpy as np
import pytest
import scipy.optimize
import scipy.special
import scipy.stats

from oracle import wildcat_oracle as wo

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _gold(name):
    vals = {}
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                k, *rest = line.split()
                vals[k] = [float(x) for x in rest]
    return vals


def _kernel(X, Y, b):
    return np.exp(b * (X @ Y.T))


# ---------------------------------------------------------------- eq. (1)
def test_exact_attention_brute_force():
    """eq. (1) written as three nested loops."""
    rng = np.random.default_rng(1)
    m, n, d, dv, beta = 5, 7, 3, 4, 0.7
    Q, K, V = rng.standard_normal((m, d)), rng.standard_normal((n, d)), rng.standard_normal((n, dv))
    ref = np.zeros((m, dv))
    for i in range(m):
        den = 0.0
        for l in range(n):
            a = math.exp(beta * sum(Q[i, t] * K[l, t] for t in range(d)))
            den += a
            for j in range(dv):
                ref[i, j] += a * V[l, j]
        ref[i] /= den
    np.testing.assert_allclose(wo.exact_attention(Q, K, V, beta, chunk=2), ref, rtol=1e-13, atol=1e-15)


def test_exact_attention_rows_are_convex_combinations():
    rng = np.random.default_rng(2)
    Q, K, V = rng.standard_normal((9, 4)) * 3, rng.standard_normal((33, 4)) * 3, rng.standard_normal((33, 5))
    O = wo.exact_attention(Q, K, V, 0.5)
    assert np.all(O <= V.max(axis=0) + 1e-12) and np.all(O >= V.min(axis=0) - 1e-12)
    # one dominant key: softmax collapses onto it
    K2 = K.copy(); K2[7] = 50 * Q[0] / np.linalg.norm(Q[0])
    O2 = wo.exact_attention(Q[:1], K2, V, 5.0)
    np.testing.assert_allclose(O2[0], V[7], atol=1e-9)


# ---------------------------------------------------------------- Lambert W, temperature
@pytest.mark.parametrize("z", [1e-12, 1e-6, 0.01, 0.2, 2 / math.e ** 2, 1.0, math.e, 10.0, 1e3, 1e12, 1e200])
def test_lambert_w0_defining_equation_and_scipy(z):
    w = wo.lambert_w0(z)
    assert w > 0
    # w + log w = log z is the defining equation w e^w = z in logarithms
    assert abs(w + math.log(w) - math.log(z)) <= 8e-16 * max(1.0, abs(math.log(z)), w)
    assert w == pytest.approx(scipy.special.lambertw(z).real, rel=1e-13)


def test_lambert_w0_special_values_and_bounds():
    gold = _gold("paper_constants.txt")
    assert wo.lambert_w0(0.0) == 0.0
    assert wo.lambert_w0(math.e) == pytest.approx(1.0, rel=1e-15)
    assert wo.lambert_w0(2 * math.e ** 2) == pytest.approx(2.0, rel=1e-15)
    c = gold["lambert_lower_coeff"][0]
    for z in np.logspace(-8, 8, 50):
        assert wo.lambert_w0(z) >= c * math.log1p(z)          # Lemma "Lambert W lower bound"
    # Theorem "Fast Lambert W calculation": the stated iteration from the stated start stays within the
    # printed error bound.  (The iterates approach W0 from below, i.e. the printed sign of the gap is
    # reversed; the magnitude bound is what is pinned.)
    a, b = gold["lambert_iter_base_a"][0], gold["lambert_iter_base_b"][0]
    for z in [0.05, 0.5, 2.0, 3.0, 30.0, 1e4, 1e9]:
        lz = math.log(z)
        bn = lz - math.log(lz) if z > math.e else math.exp(lz - 1.0)
        for it in range(1, 7):
            bn = bn / (1 + bn) * (1 + lz - math.log(bn))
            gap = bn - wo.lambert_w0(z)
            assert gap <= 1e-14 and -gap < max(a ** (2 ** it), b ** (2 ** it) / 3) + 1e-14


def test_rho0_matches_paper_and_minimises_l0():
    gold = _gold("paper_constants.txt")
    val, tol = gold["rho0"]
    assert abs(wo.RHO0 - val) <= tol
    assert 2.0 / (wo.RHO0 ** 2 + 1.0) <= gold["two_over_rho0sq_plus1_max"][0]

    def l_b(rho, b):
        q = (rho * rho + b * rho + 1.0) / math.e
        return q / (rho * scipy.special.lambertw(q).real)

    res = scipy.optimize.minimize_scalar(lambda x: l_b(x, 0.0), bounds=(1.5, 10.0), method="bounded",
                                         options={"xatol": 1e-12})
    assert res.x == pytest.approx(wo.RHO0, rel=1e-6)


@pytest.mark.parametrize("beta,RQ,RK,n", [(0.125, 10.5, 1.3, 1024), (1 / math.sqrt(128), 14.0, 14.0, 32768),
                                          (0.125, 3.0, 40.0, 100), (1.0, 0.1, 0.1, 7)])
def test_temperature_closed_form_and_bounds(beta, RQ, RK, n):
    tau, rho, b0 = wo.temperature(beta, RQ, RK, n)
    assert b0 == pytest.approx(math.log(n) / (beta * RQ * RK) + 2.0, rel=1e-15)
    # rho solves the simplified ODE of Corollary "Bounds on optimal rho":  rho = rho_0 exp(W0(b/(2 rho_0)))
    # (x(t) = x_0 exp(W(t/x_0)), Lemma "Lambert W derivative") -- a second closed form of the same number
    w = scipy.special.lambertw(b0 / (2 * wo.RHO0)).real
    assert rho == pytest.approx(wo.RHO0 * math.exp(w), rel=1e-12)
    assert tau == pytest.approx(math.sqrt(rho * RK / RQ), rel=1e-15)
    # the corollary: max(rho_0, 4/5 rho) <= rho_b <= rho for the true minimiser rho_b of l_b

    def l_b(x):
        q = (x * x + b0 * x + 1.0) / math.e
        return q / (x * scipy.special.lambertw(q).real)

    rho_b = scipy.optimize.minimize_scalar(l_b, bounds=(1.5, 200.0), method="bounded", options={"xatol": 1e-10}).x
    assert max(wo.RHO0, 0.8 * rho) - 1e-6 <= rho_b <= rho + 1e-6


def test_temperature_worked_values():
    """eq. (kernel-temperature) on two inputs worked outside the oracle (tests/golden/temperature_worked_values.txt):
    catches a dropped "+2", a swapped radius or a misplaced factor that a restated formula would repeat."""
    with open(os.path.join(GOLD, "temperature_worked_values.txt")) as f:
        rows = [[float(x) for x in line.split()] for line in f if line.strip() and not line.startswith("#")]
    assert len(rows) == 2
    for beta, RQ, RK, n, b0_ref, rho_ref, tau_ref in rows:
        tau, rho, b0 = wo.temperature(beta, RQ, RK, int(n))
        assert b0 == pytest.approx(b0_ref, rel=2e-5)
        assert rho == pytest.approx(rho_ref, rel=2e-5)
        assert tau == pytest.approx(tau_ref, rel=2e-5)


def test_temperature_special_cases_and_scaling_laws():
    """Facts eq. (kernel-temperature) fixes without evaluating it the way the oracle does."""
    # n = 1: log n = 0, so b_0 = 2 whatever beta and the radii are, and rho = 1 / W0(1 / rho_0).
    tau, rho, b0 = wo.temperature(0.37, 2.5, 0.75, 1)
    assert b0 == 2.0
    assert rho * scipy.special.lambertw(1.0 / wo.RHO0).real == pytest.approx(1.0, rel=1e-12)
    # W0(e) = 1: inputs with b_0 = 2 e rho_0 give rho = e rho_0 (= rho_0 exp(1)) and tau^2 = e rho_0 R_K / R_Q.
    RQ, RK, n = 3.0, 0.5, 4096
    beta = math.log(n) / ((2.0 * math.e * wo.RHO0 - 2.0) * RQ * RK)
    tau, rho, b0 = wo.temperature(beta, RQ, RK, n)
    assert rho == pytest.approx(math.e * wo.RHO0, rel=1e-12)
    assert tau * tau == pytest.approx(math.e * wo.RHO0 * RK / RQ, rel=1e-12)
    # b_0 and rho depend on the radii through the product R_Q R_K only; tau carries the ratio: moving a factor c
    # from the keys to the queries (R_Q c, R_K / c) divides tau by c -- the asymmetric roles of Sec. 2.4.  A
    # temperature with the radii swapped would multiply by c instead.
    t1, r1, b1 = wo.temperature(0.2, 4.0, 6.0, 500)
    t2, r2, b2 = wo.temperature(0.2, 4.0 * 3.0, 6.0 / 3.0, 500)
    assert b2 == pytest.approx(b1, rel=1e-14) and r2 == pytest.approx(r1, rel=1e-13)
    assert t2 == pytest.approx(t1 / 3.0, rel=1e-13)
    # rho >= rho_0 always (Corollary "Bounds on optimal rho"), with equality approached as log n / (beta R_Q R_K) -> 0
    # only up to the "+2": at b_0 = 2 the value is 1 / W0(1 / rho_0) > rho_0.
    assert wo.temperature(1.0, 50.0, 50.0, 2)[1] >= wo.RHO0
    # rescaled radii: the product of the rescaled radii tau R_Q and R_K / tau is unchanged, their ratio is rho
    tau, rho, _ = wo.temperature(0.11, 7.0, 2.0, 10000)
    assert (tau * 7.0) * (2.0 / tau) == pytest.approx(14.0, rel=1e-14)
    assert (tau * 7.0) / (2.0 / tau) == pytest.approx(rho, rel=1e-12)


def test_temperature_rescaling_leaves_attention_matrix_unchanged():
    """(Q, K) -> (tau Q, K / tau) leaves A, hence eq. (1), unchanged (Sec. 2.4)."""
    rng = np.random.default_rng(3)
    Q, K, V = rng.standard_normal((6, 4)), rng.standard_normal((11, 4)), rng.standard_normal((11, 3))
    tau, _, _ = wo.temperature(0.5, 2.0, 2.5, 11)
    np.testing.assert_allclose(wo.exact_attention(tau * Q, K / tau, V, 0.5), wo.exact_attention(Q, K, V, 0.5),
                               rtol=1e-12)


# ---------------------------------------------------------------- uniforms
def test_splitmix_matches_published_vectors():
    with open(os.path.join(GOLD, "splitmix64_vectors.txt")) as f:
        rows = [list(map(int, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for seed, *outs in rows:
        u = wo.splitmix_uniforms(seed, len(outs))
        for got, z in zip(u, outs):
            assert got == (z >> 11) / 2.0 ** 53
    u = wo.splitmix_uniforms(7, 20000)
    assert 0.0 <= u.min() and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 0.01 and abs(u.var() - 1 / 12) < 0.005
    np.testing.assert_array_equal(wo.splitmix_uniforms(7, 5, offset=3), u[3:8])


# ---------------------------------------------------------------- Alg. 1 invariants
def _setup(n=48, d=3, seed=0, scale=1.0):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((n, d)) * scale
    return K - K.mean(axis=0), rng


@pytest.mark.parametrize("r", [1, 2, 5, 17])
def test_rpnys_invariants_against_direct_solve(r):
    """M H_SS = I, W = solve(H_SS, H_S), W[:,S] = I, p = diag(H - H_:S H_SS^-1 H_S:), p >= 0, p_S = 0,
    and every prefix of the run satisfies the same (Prop. "Recursive update of kernel inverse")."""
    Kc, rng = _setup()
    bt = 0.4
    H = _kernel(Kc, Kc, bt)
    u = rng.random(r)
    res = wo.rpnys(Kc, bt, r, u, rank_tol=0.0, keep_p_trace=True)
    S = res.S
    assert len(S) == r and len(set(S.tolist())) == r
    HSS = H[np.ix_(S, S)]
    np.testing.assert_allclose(res.M @ HSS, np.eye(r), atol=1e-8)
    Wd = np.linalg.solve(HSS, H[S])
    np.testing.assert_allclose(res.W, Wd, atol=1e-8)
    np.testing.assert_allclose(res.W[:, S], np.eye(r), atol=1e-8)
    np.testing.assert_allclose(res.R, H[S], rtol=1e-13)
    pd = np.diag(H - H[:, S] @ Wd)
    np.testing.assert_allclose(res.p, np.maximum(pd, 0), atol=1e-9)
    assert np.all(res.p >= 0) and np.all(res.p[S] == 0)
    for i in range(r):                                   # state before draw i = residual of the first i pivots
        Si = S[:i]
        pdi = np.diag(H) - (np.einsum("ls,sl->l", H[:, Si], np.linalg.solve(H[np.ix_(Si, Si)], H[Si])) if i else 0)
        np.testing.assert_allclose(res.p_trace[i], np.maximum(pdi, 0), atol=1e-9)
        assert res.T[i] == pytest.approx(pdi.sum(), rel=1e-8)


def test_rpnys_sampling_rule_is_inverse_cdf_with_strict_inequality():
    """Forces chosen pivots through u and checks min{l : c_l > u T}; zero-mass indices are never returned."""
    Kc, _ = _setup(n=10, d=2)
    bt = 0.3
    p0 = np.exp(bt * (Kc * Kc).sum(1))
    c = np.cumsum(p0)
    for s in range(10):
        lo = c[s - 1] if s else 0.0
        for frac in (0.0, 0.5, 0.999999):
            u = (lo + frac * (c[s] - lo)) / c[-1]
            got = wo.rpnys(Kc, bt, 1, np.array([u])).S[0]
            # u*T may round across an edge only when frac == 0 sits exactly on it
            assert got == s or (frac == 0.0 and got in (s - 1, s))
    # second draw can never return the first pivot, whatever u is
    for u2 in np.linspace(0, 0.999999999, 57):
        S = wo.rpnys(Kc, bt, 2, np.array([0.35, u2])).S
        assert S[0] != S[1]
    # u = 0 lands exactly on the edge c_0 = 0 left by the first pivot: the strict rule skips the zero-mass index
    np.testing.assert_array_equal(wo.rpnys(Kc, bt, 3, np.zeros(3)).S, [0, 1, 2])
    # u just below 1: clamps to the last index of positive mass
    S = wo.rpnys(Kc, bt, 2, np.array([1 - 2.0 ** -53, 1 - 2.0 ** -53])).S
    assert S[0] == 9 and S[1] == 8


def test_rpnys_one_step_expectation_identity():
    """E[H_res^{i+1}] = H_res^i - (H_res^i)^2 / tr(H_res^i), enumerating every possible next pivot
    (proof of Thm. 1); checked for the first and the second draw.  Pins pmf, update and weights at once."""
    n, bt = 7, 0.5
    Kc, _ = _setup(n=n, d=2, seed=5)
    H = _kernel(Kc, Kc, bt)

    def residual(res):
        return H - H[:, res.S] @ res.W

    def u_for(pvec, s):                      # a uniform in the middle of cell s of the cdf of pvec
        c = np.cumsum(pvec)
        return ((c[s - 1] if s else 0.0) + 0.5 * pvec[s]) / c[-1]

    p0 = np.diag(H)
    exp1 = sum(p0[s] / p0.sum() * residual(wo.rpnys(Kc, bt, 1, np.array([u_for(p0, s)]))) for s in range(n))
    np.testing.assert_allclose(exp1, H - H @ H / np.trace(H), atol=1e-12)
    # second draw, after a fixed first pivot s1
    s1 = 3
    u1 = u_for(p0, s1)
    r1 = wo.rpnys(Kc, bt, 1, np.array([u1]))
    assert r1.S[0] == s1
    H1 = residual(r1)
    p1 = r1.p
    np.testing.assert_allclose(p1, np.maximum(np.diag(H1), 0), atol=1e-12)
    exp2 = np.zeros_like(H)
    for s2 in range(n):
        if s2 == s1:
            continue
        r2 = wo.rpnys(Kc, bt, 2, np.array([u1, u_for(p1, s2)]))
        assert list(r2.S) == [s1, s2]
        exp2 += p1[s2] / p1.sum() * residual(r2)
    np.testing.assert_allclose(exp2, H1 - H1 @ H1 / np.trace(H1), atol=1e-11)


def test_rpnys_pivot_frequencies_follow_residual_diagonal():
    n, bt = 8, 0.6
    Kc, rng = _setup(n=n, d=2, seed=6, scale=1.5)
    p0 = np.exp(bt * (Kc * Kc).sum(1))
    N = 20000
    us = rng.random(N)
    counts = np.bincount([wo.rpnys(Kc, bt, 1, us[t:t + 1]).S[0] for t in range(N)], minlength=n)
    chi2, pval = scipy.stats.chisquare(counts, N * p0 / p0.sum())
    assert pval > 1e-4


def test_rpnys_residual_decreases_monotonically():
    """sum p strictly decreases and ||H - H-hat^i||_op does not grow with i (Loewner order of residuals)."""
    Kc, rng = _setup(n=96, d=4, seed=7)
    bt = 0.35
    H = _kernel(Kc, Kc, bt)
    u = rng.random(40)
    full = wo.rpnys(Kc, bt, 40, u)
    assert np.all(np.diff(full.T) < 0)
    prev = np.inf
    for i in (1, 2, 4, 8, 16, 32, 40):
        res = wo.rpnys(Kc, bt, i, u[:i])
        np.testing.assert_array_equal(res.S, full.S[:i])         # prefix property of the sequential draw
        E = H - H[:, res.S] @ res.W
        E = 0.5 * (E + E.T)
        ev = np.linalg.eigvalsh(E)
        assert ev[0] > -1e-9                                      # residual stays p.s.d.
        assert ev[-1] <= prev + 1e-9
        prev = ev[-1]


def test_nystrom_exact_at_full_rank_and_at_kernel_rank():
    rng = np.random.default_rng(8)
    n, d, beta = 16, 6, 0.5                      # d large enough that H is well conditioned at r = n
    Q, K, V = rng.standard_normal((10, d)), rng.standard_normal((n, d)), rng.standard_normal((n, 5))
    O = wo.exact_attention(Q, K, V, beta)
    out, cs, _ = wo.wildcat(Q, K, V, beta, n, rng.random(n), rank_tol=0.0, return_coreset=True)
    assert sorted(cs.idx.tolist()) == list(range(n))
    Wperm = np.zeros((n, n)); Wperm[np.arange(n), cs.idx] = 1.0
    np.testing.assert_allclose(cs.rp.W, Wperm, atol=1e-6)
    np.testing.assert_allclose(out, O, atol=1e-7)
    # keys drawn from q distinct vectors: rank(H) = q; r = q recovers O exactly; r > q stops at q
    q = 5
    proto = rng.standard_normal((q, d))
    lab = np.concatenate([np.arange(q), rng.integers(0, q, n - q)])
    rng.shuffle(lab)
    Kd = proto[lab]
    Od = wo.exact_attention(Q, Kd, V, beta)
    for r in (q, q + 4):
        out, cs, _ = wo.wildcat(Q, Kd, V, beta, r, rng.random(r), return_coreset=True)
        assert cs.r_eff == q
        assert sorted(lab[cs.idx[:q]].tolist()) == list(range(q))
        assert np.all(cs.idx[q:] == -1) and np.all(cs.w[q:] == 0) and np.all(cs.V_S[q:] == 0)
        assert np.all(cs.rp.p == 0)
        np.testing.assert_allclose(out, Od, atol=1e-9)
        # weights of a group of duplicates add up to the group size
        np.testing.assert_allclose(cs.w[:q], np.bincount(lab, minlength=q)[lab[cs.idx[:q]]], rtol=1e-9)


# ---------------------------------------------------------------- Alg. 2-4
def test_compress_kv_shift_invariance_and_definitions():
    rng = np.random.default_rng(9)
    n, d, r, beta = 64, 4, 12, 0.5
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, 3))
    Q = rng.standard_normal((20, d))
    u = rng.random(r)
    RQ = float(np.linalg.norm(Q, axis=1).max())
    a = wo.compress_kv(K, V, RQ, beta, r, u)
    shift = rng.standard_normal(d) * 3
    b = wo.compress_kv(K + shift, V, RQ, beta, r, u)
    np.testing.assert_array_equal(a.idx, b.idx)
    assert a.tau == pytest.approx(b.tau, rel=1e-12)
    np.testing.assert_allclose(a.w, b.w, rtol=1e-9)
    np.testing.assert_allclose(a.V_S, b.V_S, rtol=1e-8, atol=1e-10)
    np.testing.assert_allclose(b.K_S, a.K_S + shift, rtol=1e-13)
    # definitions of Alg. 2 from scratch
    kbar = K.mean(0); Kc = K - kbar
    RK = np.linalg.norm(Kc, axis=1).max()
    assert a.R_K == pytest.approx(RK, rel=1e-14)
    assert a.tau == pytest.approx(wo.temperature(beta, RQ, RK, n)[0], rel=1e-15)
    Ht = _kernel(Kc, Kc, beta / a.tau ** 2)
    S = a.idx
    W = np.linalg.solve(Ht[np.ix_(S, S)], Ht[S])
    np.testing.assert_allclose(a.V_S, W @ V, atol=1e-8)
    np.testing.assert_allclose(a.w, W.sum(1), atol=1e-8)
    np.testing.assert_array_equal(a.K_S, K[S])
    # outputs of the whole pipeline are shift invariant too
    va, vb = V.min(0), V.max(0)
    oa = wo.wtd_attn(Q, a.K_S, a.V_S, a.w, va, vb, beta)
    ob = wo.wtd_attn(Q, b.K_S, b.V_S, b.w, va, vb, beta)
    np.testing.assert_allclose(oa, ob, atol=1e-8)


def test_identical_keys_collapse_to_one_pivot_and_the_value_mean():
    """R_K = 0: the kernel matrix is all ones (rank 1), one pivot carries weight n and WildCat returns the
    mean value row, which is what eq. (1) gives for identical keys."""
    rng = np.random.default_rng(14)
    K = np.tile(rng.standard_normal((1, 5)).astype(np.float32).astype(np.float64), (40, 1))   # mean is exact
    V, Q = rng.standard_normal((40, 3)), rng.standard_normal((6, 5))
    out, cs, _ = wo.wildcat(Q, K, V, 0.4, 4, rng.random(4), return_coreset=True)
    assert cs.r_eff == 1 and math.isinf(cs.tau) and cs.beta_tau == 0.0
    assert cs.w[0] == pytest.approx(40.0, rel=1e-12)
    np.testing.assert_allclose(out, np.tile(V.mean(0), (6, 1)), rtol=1e-12)
    np.testing.assert_allclose(out, wo.exact_attention(Q, K, V, 0.4), rtol=1e-12)


def test_wtd_attn_all_keys_unit_weights_is_exact_attention():
    rng = np.random.default_rng(10)
    Q, K, V = rng.standard_normal((13, 5)), rng.standard_normal((29, 5)), rng.standard_normal((29, 4))
    O = wo.exact_attention(Q, K, V, 0.45)
    got = wo.wtd_attn(Q, K, V, np.ones(29), V.min(0), V.max(0), 0.45, chunk=4)
    np.testing.assert_allclose(got, O, rtol=1e-12, atol=1e-14)


def test_wtd_attn_definition_guard_and_clip():
    rng = np.random.default_rng(11)
    m, r, d, dv, beta = 6, 4, 3, 2, 0.8
    Q, KS, VS = rng.standard_normal((m, d)), rng.standard_normal((r, d)), rng.standard_normal((r, dv)) * 5
    w = np.array([1.0, -0.2, 0.5, 2.0])
    vmin, vmax = np.array([-1.0, 0.5]), np.array([1.0, 2.0])
    got = wo.wtd_attn(Q, KS, VS, w, vmin, vmax, beta)
    for i in range(m):                                     # Alg. 3 entry by entry, no max shift
        a = [math.exp(beta * float(Q[i] @ KS[s])) for s in range(r)]
        den = sum(a[s] * w[s] for s in range(r))
        for j in range(dv):
            o = sum(a[s] * VS[s, j] for s in range(r)) / den if den > 0 else 0.0
            assert got[i, j] == pytest.approx(min(max(o, vmin[j]), vmax[j]), rel=1e-12)
    # non-positive normaliser: 0, then clipped into the value range (here column 1 has v_min > 0)
    wneg = -np.abs(w)
    got = wo.wtd_attn(Q, KS, VS, wneg, vmin, vmax, beta)
    np.testing.assert_array_equal(got, np.tile(np.clip(0.0, vmin, vmax), (m, 1)))
    assert np.all(got[:, 1] == 0.5)
    # mixed: only chosen rows have non-positive normalisers
    wmix = np.array([1.0, 1.0, 1.0, -1e6])
    A = np.exp(beta * Q @ KS.T)
    bad = (A @ wmix) <= 0
    got = wo.wtd_attn(Q, KS, VS, wmix, vmin, vmax, beta)
    assert bad.any()
    np.testing.assert_array_equal(got[bad], np.tile(np.clip(0.0, vmin, vmax), (bad.sum(), 1)))
    assert np.all(got >= vmin) and np.all(got <= vmax)


def test_wildcat_composition_and_gqa_radius():
    rng = np.random.default_rng(12)
    n, d, r, beta = 80, 4, 10, 0.5
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, 4))
    Q = rng.standard_normal((3, n, d)) * np.array([1.0, 2.0, 0.5])[:, None, None]
    u = rng.random(r)
    out, cs, (vmin, vmax, RQ) = wo.wildcat(Q, K, V, beta, r, u, return_coreset=True)
    assert RQ == pytest.approx(np.linalg.norm(Q.reshape(-1, d), axis=1).max(), rel=1e-15)
    np.testing.assert_array_equal(vmin, V.min(0)); np.testing.assert_array_equal(vmax, V.max(0))
    ref = wo.compress_kv(K, V, RQ, beta, r, u)
    np.testing.assert_array_equal(cs.idx, ref.idx)
    for h in range(3):
        np.testing.assert_array_equal(out[h], wo.wtd_attn(Q[h], ref.K_S, ref.V_S, ref.w, vmin, vmax, beta))
    # single-head call equals the stacked call with one head
    o1 = wo.wildcat(Q[1], K, V, beta, r, u)
    o1s = wo.wildcat(Q[1:2], K, V, beta, r, u)
    np.testing.assert_array_equal(o1, o1s[0])


# ---------------------------------------------------------------- error bounds of the paper
@pytest.mark.parametrize("seed,n,d,r,beta,scale", [(20, 128, 3, 10, 0.5, 1.0), (21, 256, 4, 24, 0.5, 0.7),
                                                   (22, 64, 2, 6, 1.0, 1.0), (23, 200, 8, 40, 0.35, 0.5)])
def test_lemma1_lemma2_and_value_range_bounds(seed, n, d, r, beta, scale):
    rng = np.random.default_rng(seed)
    K = rng.standard_normal((n, d)) * scale
    Q = rng.standard_normal((n, d)) * scale
    V = rng.standard_normal((n, 3))
    u = rng.random(r)
    out, cs, (vmin, vmax, RQ) = wo.wildcat(Q, K, V, beta, r, u, return_coreset=True)
    O = wo.exact_attention(Q, K, V, beta)
    err = np.abs(O - out).max()
    assert err <= (vmax - vmin).max() + 1e-12                       # proof of Lemma 1, first display
    Kc = K - K.mean(0)
    S = cs.idx
    A = _kernel(Q, Kc, beta)
    Ahat = _kernel(Q, Kc[S], beta) @ cs.rp.W
    rowerr = np.sqrt(((A - Ahat) ** 2).sum(1)).max()
    lemma1 = np.abs(V).max() * min(3 / math.sqrt(n) * rowerr / A.min(), 2.0)
    assert err <= lemma1 * (1 + 1e-9)
    Ht = _kernel(Kc, Kc, cs.beta_tau)
    Hres = Ht - Ht[:, S] @ cs.rp.W
    op = np.linalg.norm(0.5 * (Hres + Hres.T), 2)
    lemma2 = math.exp(cs.tau ** 2 * beta * RQ ** 2 / 2) * math.sqrt(op)   # tau-form, App. "Choosing a Rescaling..."
    assert rowerr <= lemma2 * (1 + 1e-9)


def test_theorem1_monte_carlo():
    """E||H - H-hat^r||_op <= eps once r >= rank(T) log(||H||/eps) + tr(H - T)(1/eps - 1/||H||), with T the
    best rank-q eigen-truncation of H (T <= H in Loewner order)."""
    Kc, rng = _setup(n=64, d=2, seed=30, scale=0.8)
    bt = 0.5
    H = _kernel(Kc, Kc, bt)
    ev = np.sort(np.linalg.eigvalsh(H))[::-1]
    Hn = ev[0]
    eps = 0.02 * Hn
    need = min(q * math.log(Hn / eps) + ev[q:].sum() * (1 / eps - 1 / Hn) for q in range(1, 30))
    r = int(math.ceil(need))
    assert r < 64
    errs = []
    for t in range(300):
        res = wo.rpnys(Kc, bt, r, rng.random(r))
        E = H - H[:, res.S] @ res.W
        errs.append(np.linalg.norm(0.5 * (E + E.T), 2))
    assert np.mean(errs) <= eps


# ---------------------------------------------------------------- Alg. 2 with bins (Sec. 2.5)
def _equal_mean_bins(rng, B, nb, d, scale=0.6):
    """Keys whose B contiguous bins all have the same row mean c (so the global mean of Alg. 2 is every bin's own)."""
    c = rng.standard_normal(d) * 0.3
    blocks = []
    for _ in range(B):
        X = rng.standard_normal((nb, d)) * scale * rng.uniform(0.5, 1.5)
        blocks.append(X - X.mean(axis=0) + c)
    return np.concatenate(blocks)


def test_binned_compress_equals_separate_one_bin_runs_when_bins_share_their_mean():
    """If every bin has the global mean, the bin loop of Alg. 2 is B independent one-bin CompressKV calls on
    (K^b, V^b) with r/B pivots each, fed the matching slice of the uniforms, and the results are concatenated with
    the pivot indices offset by b n/B.  Catches wrong slicing of keys, values or uniforms, a wrong index offset and
    a temperature computed from the wrong length."""
    rng = np.random.default_rng(21)
    B, nb, d, dv, rb, beta, RQ = 4, 60, 5, 3, 6, 0.45, 2.2
    K = _equal_mean_bins(rng, B, nb, d)
    V = rng.standard_normal((B * nb, dv))
    u = rng.uniform(size=B * rb)
    cs = wo.compress_kv(K, V, RQ, beta, B * rb, u, bins=B)
    assert cs.r_eff == B * rb and list(cs.r_effs) == [rb] * B
    for b in range(B):
        one = wo.compress_kv(K[b * nb:(b + 1) * nb], V[b * nb:(b + 1) * nb], RQ, beta, rb, u[b * rb:(b + 1) * rb])
        sl = slice(b * rb, (b + 1) * rb)
        np.testing.assert_array_equal(cs.idx[sl], one.idx + b * nb)
        np.testing.assert_allclose(cs.taus[b], one.tau, rtol=1e-12)
        np.testing.assert_allclose(cs.K_S[sl], one.K_S, rtol=0, atol=0)
        np.testing.assert_allclose(cs.V_S[sl], one.V_S, rtol=1e-7, atol=1e-9)
        np.testing.assert_allclose(cs.w[sl], one.w, rtol=1e-7, atol=1e-9)
    # bins really differ (different radii -> different temperatures), so a shared tau would have been caught
    assert np.ptp(cs.taus) > 1e-3


def test_binned_weights_are_the_block_diagonal_nystrom_solve():
    """W = diag(W^1..W^B) with W^b = h_tau_b(S_b, S_b)^-1 h_tau_b(S_b, K^b) on the globally recentred keys: V_S and w
    recomputed with a dense r x n matrix W assembled from library solves."""
    rng = np.random.default_rng(22)
    B, nb, d, dv, rb, beta, RQ = 3, 50, 4, 6, 5, 0.5, 1.7
    n, r = B * nb, B * rb
    K = rng.standard_normal((n, d)) * 0.7 + rng.standard_normal(d)      # bins do NOT share their mean here
    V = rng.standard_normal((n, dv))
    u = rng.uniform(size=r)
    cs = wo.compress_kv(K, V, RQ, beta, r, u, bins=B)
    Kc = K - K.mean(axis=0)
    W = np.zeros((r, n))
    for b in range(B):
        rows = np.arange(b * nb, (b + 1) * nb)
        S = cs.idx[b * rb:(b + 1) * rb]
        assert np.all((S >= b * nb) & (S < (b + 1) * nb)) and len(set(S)) == rb
        RK = np.sqrt((Kc[rows] ** 2).sum(1).max())
        tau = wo.temperature(beta, RQ, RK, nb)[0]
        np.testing.assert_allclose(cs.taus[b], tau, rtol=1e-13)
        bt = beta / tau ** 2
        W[b * rb:(b + 1) * rb, rows] = np.linalg.solve(_kernel(Kc[S], Kc[S], bt), _kernel(Kc[S], Kc[rows], bt))
    np.testing.assert_allclose(cs.V_S, W @ V, rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(cs.w, W.sum(axis=1), rtol=1e-6, atol=1e-8)
    np.testing.assert_array_equal(cs.K_S, K[cs.idx])


def test_binned_wildcat_is_exact_when_every_bin_has_low_kernel_rank():
    """Each bin's keys take only q <= r/B distinct values: Nystrom is exact within each bin whatever the
    temperature, hence A-hat = A column by column and Alg. 4 returns exact attention over all n keys.  Fails if the
    bins' weights were mixed up, normalised jointly, or if slots of one bin picked up values of another."""
    rng = np.random.default_rng(23)
    B, nb, d, dv, q, rb, beta = 4, 40, 6, 5, 3, 4, 0.4
    n = B * nb
    K = np.concatenate([rng.standard_normal((q, d))[rng.integers(0, q, nb)] for _ in range(B)])
    V = rng.standard_normal((n, dv))
    Q = rng.standard_normal((17, d))
    out, cs, _ = wo.wildcat(Q, K, V, beta, B * rb, rng.uniform(size=B * rb), return_coreset=True, bins=B)
    assert np.all(cs.r_effs <= q) and cs.r_eff == cs.r_effs.sum() and np.all(cs.r_effs >= 1)
    for b in range(B):                                  # exhausted bins leave empty slots behind their pivots
        k = cs.r_effs[b]
        assert np.all(cs.idx[b * rb + k:(b + 1) * rb] == -1) and np.all(cs.w[b * rb + k:(b + 1) * rb] == 0)
    np.testing.assert_allclose(out, wo.exact_attention(Q, K, V, beta), rtol=1e-6, atol=1e-8)


def test_binned_all_keys_selected_gives_identity_weights():
    """r/B = n/B: every key of every bin is a pivot, W is a permutation matrix and w = 1."""
    rng = np.random.default_rng(24)
    B, nb, d = 3, 7, 4
    n = B * nb
    K, V = rng.standard_normal((n, d)), rng.standard_normal((n, 2))
    cs = wo.compress_kv(K, V, 1.5, 0.5, n, rng.uniform(size=n), bins=B)
    assert sorted(cs.idx) == list(range(n))
    np.testing.assert_allclose(cs.w, 1.0, rtol=1e-6)
    np.testing.assert_allclose(cs.V_S, V[cs.idx], rtol=1e-5, atol=1e-7)


def test_binned_temperature_length_switch_and_argument_checks():
    rng = np.random.default_rng(25)
    B, nb, d, rb, beta, RQ = 2, 64, 4, 3, 0.5, 2.0
    K, V = rng.standard_normal((B * nb, d)), rng.standard_normal((B * nb, 2))
    u = rng.uniform(size=B * rb)
    Kc = K - K.mean(axis=0)
    full = wo.compress_kv(K, V, RQ, beta, B * rb, u, bins=B, temperature_n="full")
    binl = wo.compress_kv(K, V, RQ, beta, B * rb, u, bins=B)
    for b in range(B):
        RK = np.sqrt((Kc[b * nb:(b + 1) * nb] ** 2).sum(1).max())
        np.testing.assert_allclose(full.taus[b], wo.temperature(beta, RQ, RK, B * nb)[0], rtol=1e-13)
        np.testing.assert_allclose(binl.taus[b], wo.temperature(beta, RQ, RK, nb)[0], rtol=1e-13)
        assert full.taus[b] > binl.taus[b]                 # tau grows with log n
    with pytest.raises(ValueError):
        wo.compress_kv(K, V, RQ, beta, 7, u, bins=2)        # B does not divide r
    with pytest.raises(ValueError):
        wo.compress_kv(K[:-1], V[:-1], RQ, beta, 6, u, bins=2)   # B does not divide n
    one = wo.compress_kv(K, V, RQ, beta, 6, u)              # B = 1 is the default and reports per-bin arrays too
    assert one.taus.shape == (1,) and one.taus[0] == one.tau and one.r_effs[0] == one.r_eff
