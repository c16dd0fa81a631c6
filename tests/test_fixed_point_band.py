"""Host-side check of the guard band of the optional 16-bit first scoring pass (no GPU needed).

The one-launch decode step can place tokens in histogram bins from 16-bit fixed-point sums F of the lookup tables
("Compressed-Domain Top-k Retrieval": score = sum over the 32 groups of Table[g][Code_g]) and give exact binary32
scores only to the tokens within a band of the threshold bin.  That is exact only if
    F_a - F_b >= D  implies  score_a > score_b
for the binary32 scores the other paths rank by.  The construction (entries rounded to multiples of delta after
subtracting the group minimum; D = 2 (ceil(17 + 1.01 gam / delta) + 1), gam = 31 x 2^-24 x sum_g max_j |T|) is
restated here in numpy binary32 and checked by brute force on random and adversarial tables, together with the
selection rule built on it (bins of 2^sh units, a band of m bins on either side of the threshold bin).
"""
import numpy as np
import pytest

F32 = np.float32


def fixed_point_table(T):
    """T [32, 16] binary32 -> (E [32, 16] integers, inv = 1 / delta, D, sh, base, m), as the kernel builds them."""
    T = T.astype(F32)
    mn, mx = T.min(1, keepdims=True), T.max(1, keepdims=True)
    R = F32((mx - mn).astype(F32).sum(dtype=F32))
    A = F32(np.abs(T).max(1).astype(F32).sum(dtype=F32))
    inv = F32(65495.0) / R if (R > F32(1e-30) and R < F32(3e38)) else F32(0)
    E = np.rint(((T - mn).astype(F32) * inv).astype(F32))
    gam = F32(31.0) * F32(5.9604645e-8) * A
    G = min(float(np.ceil(F32(17.0) + F32(1.01) * gam * inv) + 1.0), 1e6)
    D = 2 * int(G)
    var = float(E.var(1).sum())
    wreq = int(min(9.0 * np.sqrt(var) / 512.0, 60000.0))
    sh = 0 if wreq <= 1 else int(wreq - 1).bit_length()
    base = (int(E.mean(1).sum()) >> sh) - 256
    m = (D - 1 + (1 << sh) - 1) >> sh
    return E.astype(np.int64), inv, D, sh, base, m


def scores_of(T, codes):
    """Binary32 score of every token: the 32 looked-up entries added in ascending group order, as every kernel does."""
    T = T.astype(F32)
    acc = T[0, codes[:, 0]].copy()
    for g in range(1, 32):
        acc = (acc + T[g, codes[:, g]]).astype(F32)
    return acc


def tables():
    rng = np.random.default_rng(11)
    base = rng.standard_normal((32, 16)).astype(F32)
    yield "random", base
    yield "offset", (base + F32(3.0)).astype(F32)
    yield "huge_offset", (base + F32(4000.0)).astype(F32)
    yield "tiny_range", (F32(7.0) + F32(1e-4) * base).astype(F32)
    one = np.zeros((32, 16), F32)
    one[:2] = base[:2] * F32(50.0)
    yield "two_groups", one
    yield "outlier_group", np.concatenate([base[:31], base[31:] * F32(300.0)]).astype(F32)
    # entries sitting just below / above half a unit of delta: the rounding errors of a token's 32 entries line up.
    # delta = 2^-6 exactly: the group ranges are whole units that sum to 65495 units, so that 1 / delta = 64.
    delta = 1.0 / 64.0
    adv = np.zeros((32, 16), np.float64)
    for g in range(32):
        rng_units = 2047 if g < 31 else 65495 - 31 * 2047
        for j in range(1, 15):
            adv[g, j] = (j * (rng_units // 15) + (0.499 if j % 2 == 0 else -0.499)) * delta
        adv[g, 15] = rng_units * delta
    adv = adv.astype(F32)
    yield "aligned_rounding", adv


@pytest.mark.parametrize("name,T", list(tables()), ids=[n for n, _ in tables()])
def test_gap_of_d_units_orders_the_binary32_scores(name, T):
    rng = np.random.default_rng(5)
    L = 6000
    codes = rng.integers(0, 16, size=(L, 32))
    if name == "aligned_rounding":  # half of the tokens take the entries that round up, half those that round down
        codes = np.clip(2 * (codes // 2) + (np.arange(L)[:, None] % 2), 1, 14)
    E, inv, D, sh, base, m = fixed_point_table(T)
    F = E[np.arange(32)[None, :], codes].sum(1)
    assert F.min() >= 0 and F.max() <= 65535, "the sums must fit 16 bits"
    s = scores_of(T, codes).astype(np.float64)
    order = np.argsort(F, kind="stable")
    Fs, ss = F[order], s[order]
    run_max = np.maximum.accumulate(ss)
    # for every token a: the best score among tokens with F <= F_a - D must be below score_a
    lim = np.searchsorted(Fs, Fs - D, side="right")      # tokens [0, lim) have F <= F_a - D
    has = lim > 0
    assert np.all(run_max[lim[has] - 1] < ss[has]), name
    if name == "aligned_rounding":
        # the bound is not vacuous: with this table (sums off by 11 to 14 units either way) smaller gaps do get inverted
        lim2 = np.searchsorted(Fs, Fs - 8, side="right")
        has2 = lim2 > 0
        assert np.any(run_max[lim2[has2] - 1] >= ss[has2])


@pytest.mark.parametrize("name,T", list(tables()), ids=[n for n, _ in tables()])
@pytest.mark.parametrize("k", [1, 37, 600, 5999])
def test_band_selection_equals_exact_top_k(name, T, k):
    rng = np.random.default_rng(9)
    L = 6000
    codes = rng.integers(0, 16, size=(L, 32))
    E, inv, D, sh, base, m = fixed_point_table(T)
    F = E[np.arange(32)[None, :], codes].sum(1)
    s = scores_of(T, codes)
    want = set(np.lexsort((np.arange(L), -s.astype(np.float64)))[:k].tolist())   # score desc, index asc
    bins = np.clip((F >> sh) - base, 0, 511)
    hist = np.bincount(bins, minlength=512)
    from_top = np.cumsum(hist[::-1])[::-1]
    bstar = int(np.max(np.nonzero(from_top >= k)[0]))
    lo_b, hi_b = max(bstar - m, 0), min(bstar + m, 511)
    sure = np.nonzero(bins > hi_b)[0]
    band = np.nonzero((bins >= lo_b) & (bins <= hi_b))[0]
    need = k - len(sure)
    assert 0 <= need <= len(band)
    ranked = band[np.lexsort((band, -s[band].astype(np.float64)))][:need]
    got = set(sure.tolist()) | set(ranked.tolist())
    assert got == want, (name, k, len(sure), len(band))
