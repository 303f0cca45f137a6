"""The binary32 filter of the search against its own error bound (CPU only).

The HIP search evaluates every candidate in binary32 (k_search), or from
bucketed prefix sums (k_fast), only to decide which candidates are re-evaluated
exactly; the true minimiser of Eq.7 survives if every filter value lies within
half the slack of `keep_threshold` of the exact squared error.  The GPU tests
only observe that the final k* matched.  This test checks the bound itself: it
re-does the filter arithmetic step by step in numpy (binary32 where the kernel
uses binary32) and compares every candidate's value with the oracle's curve on
inputs chosen to stress it.  It shares no code with the kernels: the formulas
are restated here from their definition (u = |w|/m*n, centre step k/L, tail
step (n-k)/L, error in steps t - rne(t)).
"""
import numpy as np
import pytest

from oracle import pwlq_ref as R

F32 = np.float32
EPS_PER_N = 2.0 ** -21          # per-element error allowance of the filter, in units of n
SUM_REL = 3e-5                  # chunked binary32 summation
FAST_REL = 3.0e-11              # prefix-sum arithmetic, times n^2 * count


def half_slack(T, count, n, fast):
    eps = n * EPS_PER_N
    extra = FAST_REL * n * n * count if fast else 0.0
    return SUM_REL * T + 2.0 * eps * np.sqrt(count * T) + count * eps * eps + extra


def to_units(w, n):
    a = np.abs(w.astype(F32))
    m = a.max()
    u = a * (F32(n) / m)                     # two binary32 roundings, as in the kernel
    return np.clip(u, F32(0), F32(n)), m


def filter_elementwise(u, n, bits):
    """k_search's value of every candidate: binary32 t, f = t - rne(t), f*f summed in
    binary32 per region (flushed every 128 elements), scaled by step^2."""
    L = F32(2 ** (bits - 1) - 1)
    k = np.arange(1, n + 1)
    kf = k.astype(F32)
    nk = (n - k).astype(F32)
    rc = L / kf
    with np.errstate(divide="ignore"):
        rt = np.where(k < n, L / nk, F32(0)).astype(F32)
    ct = (-kf * rt).astype(F32)
    stepc, stept = kf / L, nk / L
    sc = np.zeros(n, F32); st = np.zeros(n, F32)
    ac = np.zeros(n, F32); at = np.zeros(n, F32)
    for i, ui in enumerate(np.sort(u)):
        tail = ui > kf
        tc = ui * rc
        tt = (np.float64(ui) * rt.astype(np.float64) + ct.astype(np.float64)).astype(F32)   # fused
        t = np.where(tail, tt, tc)
        f = (t - np.rint(t)).astype(np.float64)
        ac = np.where(tail, ac, (f * f + ac).astype(F32))
        at = np.where(tail, (f * f + at).astype(F32), at)
        if i % 128 == 127:
            sc += ac; st += at; ac[:] = 0; at[:] = 0
    sc += ac; st += at
    return ((stepc * stepc) * sc + (stept * stept) * st).astype(np.float64)


def filter_prefix_sums(u, n, bits):
    """k_fast's value of every candidate: cumulative counts and sums at the half-way
    points of the levels (half-way points in binary32, sums in binary64)."""
    Li = 2 ** (bits - 1) - 1
    Ld = float(Li)
    us = np.sort(u)
    c1 = np.concatenate([[0.0], np.cumsum(us.astype(np.float64))])
    c2 = np.concatenate([[0.0], np.cumsum(us.astype(np.float64) ** 2)])
    S1, S2, K = c1[-1], c2[-1], len(us)
    j = np.arange(Li)
    out = np.empty(n)
    for k in range(1, n + 1):
        kd = float(k)
        half_c = F32(kd / (2.0 * Ld))
        cn = np.searchsorted(us, (2 * j + 1).astype(F32) * half_c, side="right")
        sumC, sumN = c1[cn].sum(), int(((2 * j + 1) * cn).sum())
        nL = int(np.searchsorted(us, F32(k), side="right"))
        cL, s2L = c1[nL], c2[nL]
        s = kd / Ld
        sse = s2L - 2.0 * s * (Ld * cL - sumC) + s * s * (Ld * Ld * nL - sumN)
        if k < n:
            wd = float(n - k)
            half_t = F32(wd / (2.0 * Ld))
            b = ((2 * j + 1).astype(np.float64) * np.float64(half_t) + kd).astype(F32)     # fused
            cn = np.searchsorted(us, b, side="right")
            nt = cn - nL
            sumCt = ((c1[cn] - cL) - kd * nt).sum()
            sumNt = int(((2 * j + 1) * nt).sum())
            ntL = K - nL
            ctL = (S1 - cL) - kd * ntL
            s2t = (S2 - s2L) - 2.0 * kd * (S1 - cL) + kd * kd * ntL
            s = wd / Ld
            sse += s2t - 2.0 * s * (Ld * ctL - sumCt) + s * s * (Ld * Ld * ntL - sumNt)
        out[k - 1] = max(sse, 0.0)
    return out.astype(F32).astype(np.float64)


def adversarial_rows(K, n, bits, rng):
    L = 2 ** (bits - 1) - 1
    rows = {
        "gaussian": rng.standard_normal(K),
        "laplace": rng.laplace(0, 1, K),
        "heavy tail": rng.standard_t(1.5, K),
        "uniform": rng.uniform(-1, 1, K),
        "sparse": rng.standard_normal(K) * (rng.random(K) < 0.05),
        "few values": np.round(rng.standard_normal(K) * 3) / 3,
        "one crowded bucket": np.concatenate([np.full(K - 4, 0.37), [1.0, 0.5, 0.25, 0.125]]),
    }
    # magnitudes exactly half-way between two levels of many candidates: u = (j + 1/2) k / L
    kk = rng.integers(1, n + 1, K)
    jj = rng.integers(0, L, K)
    ties = (jj + 0.5) * kk / L / n
    ties[0] = 1.0
    rows["half-way ties"] = ties * np.sign(rng.standard_normal(K))
    # and right at the breakpoints themselves (region boundary), one ulp to either side too
    edge = rng.integers(1, n + 1, K) / n
    edge = np.nextafter(edge.astype(F32), F32(2) * (rng.random(K) < 0.5)).astype(np.float64)
    edge[0] = 1.0
    rows["on the breakpoints"] = edge
    return rows


@pytest.mark.parametrize("bits,n,K", [(4, 1000, 1024), (2, 257, 700), (8, 500, 2048),
                                      (3, 2000, 1500), (4, 65535, 160), (4, 100, 8192)])
def test_filter_values_stay_within_half_the_slack(bits, n, K):
    rng = np.random.default_rng(bits * 100000 + n)
    worst = {}
    for name, row in adversarial_rows(K, n, bits, rng).items():
        w = row.astype(F32)[None, :]
        ref = R.search(w, bits, n, want_curve=True)
        u, m = to_units(w[0], n)
        assert m == ref["m"][0]
        T = ref["curve"][0] * (float(n) / float(m)) ** 2          # exact curve in candidate units
        for fast, emulate in ((False, filter_elementwise), (True, filter_prefix_sums)):
            F = emulate(u, n, bits)
            allowed = half_slack(T, float(K), n, fast)
            ratio = np.abs(F - T) / allowed
            k_bad = int(np.argmax(ratio))
            assert ratio.max() <= 1.0, (name, "fast" if fast else "plain", k_bad + 1, F[k_bad], T[k_bad],
                                        allowed[k_bad])
            worst[(name, fast)] = float(ratio.max())
    print(f"bits={bits} n={n} K={K}: largest |filter - exact| / allowed = "
          f"{max(worst.values()):.3f} at {max(worst, key=worst.get)}")
