"""Float64 CPU oracle for the WildCat hot path (CompressKV -> WtdAttn).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP library is checked against.  Nothing in the product path may import it;
only the tests, the smoke check and the CPU-baseline leg of the benchmark do.
It shares no code, constants or helpers with the HIP sources and imports
nothing from the package that wraps them.

Everything is NumPy float64.  Inputs that live in a narrower storage type
(fp32, bf16) are widened exactly by the caller before they get here.

What each function follows (paper = "WildCat: Near-Linear Attention in Theory
and Practice"):

  exact_attention   eq. (1), Sec. 2           softmax attention by definition
  lambert_w0        App. "Properties of the Lambert W Function" (definition
                    w e^w = z, principal branch)
  RHO0, temperature eq. (kernel-temperature), Sec. 2.4; rho_0 from the Lemma
                    "Optimal choice of rho"
  rpnys             Alg. 1 (RPNys), Sec. 2.3, with the inverse update of the
                    Proposition "Recursive update of kernel inverse"
  compress_kv       Alg. 2 (CompressKV), any number of bins B (Sec. 2.5)
  wtd_attn          Alg. 3 (WtdAttn)
  wildcat           Alg. 4 (WildCat)
  splitmix_uniforms the counter-based uniform generator that stands in for the
                    paper's unspecified sampler (Alg. 1 only says "s ~ p/sum p")

Readings taken where the paper is silent or garbled are marked "Reading:" at
the place they apply.

Pins (tests/test_oracle_*.py, all CPU): brute-force attention on tiny inputs;
WtdAttn over all keys with unit weights equals exact attention; Nystrom
exactness at full rank and at the kernel rank; per-step invariants of Alg. 1
(M H_SS = I, W[:,S] = I, p = from-scratch residual diagonal, W = solve(H_SS,
H_S)); monotone residual; exact one-step expectation identity; chi-square of
pivot frequencies; shift invariance and prefix property; rho_0 ~ 3.19 and the
constants the paper prints; Lemma 1, Lemma 2 and the trivial value-range bound;
Theorem 1 by Monte Carlo; guard/clip behaviour; binning: bins with a common
mean equal separate one-bin runs, W is the block-diagonal solve, per-bin
low-rank keys reproduce exact attention, temperature length switch.
Parity unpinned: absolute values of O-hat, S or W on any of the paper's own
workloads (the paper prints none).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "exact_attention", "lambert_w0", "RHO0", "temperature", "rpnys",
    "compress_kv", "wtd_attn", "wildcat", "splitmix_uniforms",
    "RpnysResult", "Coreset",
]


# ----------------------------------------------------------------------------
# eq. (1): exact softmax attention
# ----------------------------------------------------------------------------
def exact_attention(Q, K, V, beta, chunk=2048):
    """O = D^{-1} A V with A_il = exp(beta <q_i, k_l>), D = diag(A 1)  (eq. (1)).

    Rows are processed in chunks only to bound memory; each row is shifted by
    its own maximum exponent before exp(), a positive per-row factor that
    cancels between numerator and denominator.
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    out = np.empty((Q.shape[0], V.shape[1]), dtype=np.float64)
    for a in range(0, Q.shape[0], chunk):
        Z = beta * (Q[a:a + chunk] @ K.T)
        Z -= Z.max(axis=1, keepdims=True)
        A = np.exp(Z)
        out[a:a + chunk] = (A @ V) / A.sum(axis=1, keepdims=True)
    return out


# ----------------------------------------------------------------------------
# Lambert W (principal branch) and the temperature of Sec. 2.4
# ----------------------------------------------------------------------------
def lambert_w0(z):
    """Principal-branch W_0(z) for z >= 0: the w >= 0 with w e^w = z.

    Newton's method on f(w) = w + log(w) - log(z) (the logarithm of the
    defining equation, well scaled for every z > 0), started from log(1+z),
    and stopped when the defining equation holds to a few ulp.
    """
    z = float(z)
    if z < 0.0:
        raise ValueError("lambert_w0: z must be >= 0")
    if z == 0.0:
        return 0.0
    lz = math.log(z)
    w = math.log1p(z)              # >= W_0(z); f is concave, so Newton then
    for _ in range(100):           # approaches the root from the left
        f = w + math.log(w) - lz
        step = f / (1.0 + 1.0 / w)
        w_new = w - step
        if w_new <= 0.0:
            w_new = 0.5 * w
        if abs(w_new - w) <= 4e-16 * abs(w_new):
            w = w_new
            break
        w = w_new
    return w


#: rho_0 = sqrt(1 + exp(W_0(2/e^2) + 2)), the minimiser of l_0 (Lemma "Optimal
#: choice of rho"); the paper prints "approx 3.19".
RHO0 = math.sqrt(1.0 + math.exp(lambert_w0(2.0 / math.e ** 2) + 2.0))


def temperature(beta, R_Q, R_K, n):
    """tau of eq. (kernel-temperature):

        b_0 = log(n) / (beta R_Q R_K) + 2
        rho = b_0 / (2 W_0(b_0 / (2 rho_0)))
        tau = sqrt(rho R_K / R_Q)

    Returns (tau, rho, b_0).

    Reading: if R_Q or R_K is zero the formula divides by zero, but then every
    kernel value exp(beta <q, k>) the method looks at is 1 whatever tau is;
    tau = +inf is returned and the caller runs Alg. 1 with exponent scale 0.
    """
    if not (R_Q > 0.0 and R_K > 0.0):
        return math.inf, math.inf, math.inf
    b0 = math.log(n) / (beta * R_Q * R_K) + 2.0
    rho = b0 / (2.0 * lambert_w0(b0 / (2.0 * RHO0)))
    tau = math.sqrt(rho * R_K / R_Q)
    return tau, rho, b0


# ----------------------------------------------------------------------------
# uniforms: counter-based generator shared (as an algorithm, not as code) with
# the library, so that a bare seed means the same pivot draws on both sides
# ----------------------------------------------------------------------------
def splitmix_uniforms(seed, count, offset=0):
    """u_t = (mix64(seed + (offset+t+1) * 0x9E3779B97F4A7C15) >> 11) * 2^-53,

    mix64 being the SplitMix64 output function (xor-shift 30, multiply
    0xBF58476D1CE4E5B9, xor-shift 27, multiply 0x94D049BB133111EB, xor-shift
    31), all arithmetic modulo 2^64.  Values lie in [0, 1).
    """
    mask = (1 << 64) - 1
    out = np.empty(count, dtype=np.float64)
    for t in range(count):
        zed = (seed + (offset + t + 1) * 0x9E3779B97F4A7C15) & mask
        zed = ((zed ^ (zed >> 30)) * 0xBF58476D1CE4E5B9) & mask
        zed = ((zed ^ (zed >> 27)) * 0x94D049BB133111EB) & mask
        zed = zed ^ (zed >> 31)
        out[t] = (zed >> 11) * (1.0 / 9007199254740992.0)
    return out


# ----------------------------------------------------------------------------
# Alg. 1: randomly pivoted Nystrom
# ----------------------------------------------------------------------------
@dataclass
class RpnysResult:
    S: np.ndarray            # pivots in selection order, length r_eff
    W: np.ndarray            # [r_eff, n] Nystrom weights  M R
    M: np.ndarray            # [r_eff, r_eff] inverse of h(K_S, K_S)
    R: np.ndarray            # [r_eff, n] kernel rows h(K_S, K)
    p: np.ndarray            # final residual diagonal
    T: np.ndarray            # sum(p) seen at each draw, length r_eff
    margin: np.ndarray       # per-draw distance of u*T to the nearest CDF edge, / T
    p_trace: list = field(default_factory=list)   # optional copies of p per step


def rpnys(Kc, beta_tau, r, u, rank_tol=1e-10, keep_p_trace=False):
    """Alg. 1 on the data set Kc with kernel h(x, y) = exp(beta_tau <x, y>).

    State, as in the paper: p (residual diagonal = unnormalised pivot pmf),
    M (inverse of the core kernel matrix, grown by rank-one updates), R (kernel
    rows of the pivots), g.

    Reading (indexing): the listing mixes 0- and 1-based indices.  At the step
    that adds pivot number i (0-based, i = current coreset size) the vector g
    has i+1 entries: g_{<i} = M_{<i,<i} R_{<i,s} (absent for i = 0), g_i = -1,
    all divided by sqrt(p_s) with p_s the residual diagonal at s *before* this
    step's update, which is the g of the inverse-update Proposition.

    Reading (sampling): "s ~ p / sum p" is drawn by inverse CDF from one
    pre-drawn uniform u_i in [0,1) per step: c = inclusive prefix sums of p in
    index order, T = c_{n-1}, s = min{l : c_l > u_i T} (strict, so an index of
    zero mass is never returned); if rounding leaves no such l, the last index
    of positive mass.

    Reading (non-negativity and rank exhaustion): the listing only resets p_s
    "for numerical stability".  Here, after p <- p - delta^2, every entry that
    is no larger than rank_tol times its initial value h(k_l, k_l) is set to
    zero: such a key lies in the span of the coreset features to working
    accuracy.  rank_tol = 0 gives the bare clamp max(p, 0).  The loop stops
    early when sum p <= 0 (the kernel matrix is fully approximated; the paper's
    definitions use the pseudo-inverse there), so fewer than r pivots may be
    returned.
    """
    Kc = np.asarray(Kc, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    n = Kc.shape[0]
    if not (1 <= r <= n):
        raise ValueError("rpnys: need 1 <= r <= n")
    diag0 = np.exp(beta_tau * np.einsum("ld,ld->l", Kc, Kc))
    p = diag0.copy()
    floor = rank_tol * diag0
    M = np.zeros((r, r))
    R = np.zeros((r, n))
    S, Ts, margins, trace = [], [], [], []
    for i in range(r):
        c = np.cumsum(p)
        T = c[-1]
        if not (T > 0.0):
            break
        t = u[i] * T
        s = int(np.searchsorted(c, t, side="right"))      # first l with c_l > t
        if s >= n:
            s = int(np.flatnonzero(p > 0.0)[-1])
        lo = c[s - 1] if s > 0 else 0.0
        margins.append(min(t - lo, c[s] - t) / T)
        Ts.append(T)
        if keep_p_trace:
            trace.append(p.copy())
        # -- update kernel inverse
        g = np.empty(i + 1)
        if i > 0:
            g[:i] = M[:i, :i] @ R[:i, s]
        g[i] = -1.0
        g /= math.sqrt(p[s])
        M[:i + 1, :i + 1] += np.outer(g, g)
        # -- update pivot distribution
        R[i] = np.exp(beta_tau * (Kc @ Kc[s]))
        delta = g @ R[:i + 1]
        p = p - delta * delta
        p[p <= floor] = 0.0
        p[s] = 0.0
        S.append(s)
    k = len(S)
    M = M[:k, :k].copy()
    R = R[:k].copy()
    return RpnysResult(S=np.asarray(S, dtype=np.int64), W=M @ R, M=M, R=R, p=p,
                       T=np.asarray(Ts), margin=np.asarray(margins), p_trace=trace)


# ----------------------------------------------------------------------------
# Alg. 2: CompressKV
# ----------------------------------------------------------------------------
@dataclass
class Coreset:
    idx: np.ndarray      # [r] pivot indices into the n keys, -1 in unused slots
    r_eff: int           # pivots drawn, all bins together
    K_S: np.ndarray      # [r, d]   original (un-recentred) key rows
    V_S: np.ndarray      # [r, d_v] W V
    w: np.ndarray        # [r]      W 1
    tau: float           # B = 1: the temperature; B > 1: that of the first bin (see taus)
    beta_tau: float
    kbar: np.ndarray
    R_K: float
    rp: RpnysResult      # Alg. 1 result of the first (for B = 1: the only) bin
    taus: np.ndarray = None      # [B] temperature of each bin
    R_Ks: np.ndarray = None      # [B] key radius of each bin
    r_effs: np.ndarray = None    # [B] pivots drawn in each bin
    rps: list = None             # [B] Alg. 1 results, pivot indices local to the bin


def compress_kv(K, V, R_Q, beta, r, u, rank_tol=1e-10, keep_p_trace=False, bins=1,
                temperature_n="bin"):
    """Alg. 2: recentre the keys by their row mean (over all n keys), divide the
    rows into B bins, and for each bin take R_K as the largest recentred row
    norm of the bin, tau from eq. (kernel-temperature), and run Alg. 1 on the
    bin's recentred keys with kernel exp(beta <.,.> / tau^2) for r/B pivots.
    The bins' results are concatenated in bin order: slots b r/B .. (b+1) r/B - 1
    belong to bin b.  Returns the original key rows at the pivots (recentred
    rows plus the mean), V_S = W V and w = W 1.

    Readings (the paper's text leaves these open):
      * "Evenly divide (or reshape)": bin b holds the contiguous rows
        b n/B .. (b+1) n/B - 1; B must divide n and r.
      * W = (W^b)_b: Alg. 1 on bin b returns Nystrom weights over that bin's
        keys only, so W is block diagonal and rows b r/B.. of V_S are W^b V^b.
      * The length passed to getTemperature inside the bin loop is written "n";
        Thm. 2 states its guarantee for B > 1 with n/B in place of n, so the
        default (temperature_n="bin") is the bin length; "full" uses n.
      * Step i of bin b consumes uniform u[b r/B + i].

    Unused slots (rank exhaustion in a bin) carry idx = -1 and zero key, value
    and weight, so they add nothing to either sum of Alg. 3.
    """
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    u = np.asarray(u, dtype=np.float64)
    n, d = K.shape
    B = int(bins)
    if B < 1 or n % B or r % B:
        raise ValueError("bins must divide n and r")
    if temperature_n not in ("bin", "full"):
        raise ValueError("temperature_n is 'bin' or 'full'")
    nb, rb = n // B, r // B
    kbar = K.mean(axis=0)
    Kc = K - kbar
    idx = np.full(r, -1, dtype=np.int64)
    K_S = np.zeros((r, d))
    V_S = np.zeros((r, V.shape[1]))
    w = np.zeros(r)
    taus, R_Ks, r_effs, rps, beta_taus = np.zeros(B), np.zeros(B), np.zeros(B, dtype=np.int64), [], []
    for b in range(B):
        rows = slice(b * nb, (b + 1) * nb)
        Kb = Kc[rows]
        R_K = float(np.sqrt(np.einsum("ld,ld->l", Kb, Kb).max()))
        tau, _, _ = temperature(beta, R_Q, R_K, nb if temperature_n == "bin" else n)
        beta_tau = beta / (tau * tau) if math.isfinite(tau) else 0.0
        rp = rpnys(Kb, beta_tau, rb, u[b * rb:(b + 1) * rb], rank_tol=rank_tol, keep_p_trace=keep_p_trace)
        k = len(rp.S)
        slots = slice(b * rb, b * rb + k)
        idx[slots] = b * nb + rp.S
        K_S[slots] = K[b * nb + rp.S]           # == Kc[S] + kbar, without rounding
        V_S[slots] = rp.W @ V[rows]
        w[slots] = rp.W.sum(axis=1)
        taus[b], R_Ks[b], r_effs[b] = tau, R_K, k
        rps.append(rp)
        beta_taus.append(beta_tau)
    return Coreset(idx=idx, r_eff=int(r_effs.sum()), K_S=K_S, V_S=V_S, w=w, tau=float(taus[0]),
                   beta_tau=beta_taus[0], kbar=kbar, R_K=float(R_Ks[0]), rp=rps[0],
                   taus=taus, R_Ks=R_Ks, r_effs=r_effs, rps=rps)


# ----------------------------------------------------------------------------
# Alg. 3: WtdAttn
# ----------------------------------------------------------------------------
def wtd_attn(Q, K_S, V_S, w, v_min, v_max, beta, chunk=4096):
    """A-hat = exp(beta Q K_S^T); O-hat = (A-hat V_S) / (A-hat w) where
    A-hat w > 0, else 0; then clip column j to [v_min_j, v_max_j].

    Each row of A-hat is shifted by its maximum exponent first: a positive
    per-row factor, so neither the ratio nor the sign test changes.
    Reading: "else 0" is applied before the clip, so a row whose normaliser is
    not positive ends at clip(0, v_min, v_max).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K_S = np.asarray(K_S, dtype=np.float64)
    V_S = np.asarray(V_S, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    out = np.empty((Q.shape[0], V_S.shape[1]))
    for a in range(0, Q.shape[0], chunk):
        Z = beta * (Q[a:a + chunk] @ K_S.T)
        Z -= Z.max(axis=1, keepdims=True)
        A = np.exp(Z)
        den = A @ w
        num = A @ V_S
        ok = den > 0.0
        o = np.zeros_like(num)
        o[ok] = num[ok] / den[ok, None]
        out[a:a + chunk] = np.clip(o, v_min, v_max)
    return out


# ----------------------------------------------------------------------------
# Alg. 4: WildCat
# ----------------------------------------------------------------------------
def wildcat(Q, K, V, beta, r, u, rank_tol=1e-10, return_coreset=False, bins=1, temperature_n="bin"):
    """Alg. 4: column-wise value range, query radius R_Q = max row norm of Q,
    CompressKV, WtdAttn.

    Q may be [m, d] or a stack [h, m, d] of query heads that share the keys
    (grouped-query attention).  Reading: the paper does not discuss shared
    key heads; R_Q is then the largest row norm over all query heads of the
    group, and each head attends to the one shared coreset.
    """
    Q = np.asarray(Q, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    v_min = V.min(axis=0)
    v_max = V.max(axis=0)
    Q3 = Q if Q.ndim == 3 else Q[None]
    R_Q = float(np.sqrt(np.einsum("hmd,hmd->hm", Q3, Q3).max()))
    cs = compress_kv(K, V, R_Q, beta, r, u, rank_tol=rank_tol, bins=bins, temperature_n=temperature_n)
    outs = np.stack([wtd_attn(q, cs.K_S, cs.V_S, cs.w, v_min, v_max, beta) for q in Q3])
    out = outs if Q.ndim == 3 else outs[0]
    if return_coreset:
        return out, cs, (v_min, v_max, R_Q)
    return out
