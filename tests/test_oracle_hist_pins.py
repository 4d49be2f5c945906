"""Pins for the oracle's histogram mode estimator and for the rule that NaN calibration samples rank last.

The paper (Section 3, "Determination of mode value") names a kernel density estimate looked up for its mode but
gives neither bandwidth nor grid, so this build's stand-in has a definition of its own:

    lo, hi = the ceil(0.001 M)-th and ceil(0.999 M)-th smallest of the M pooled values;
    2048 equal bins of width w = (hi - lo) / 2048 over [lo, hi]; a value v with lo <= v <= hi falls in bin
    floor((v - lo) / w), v == hi in the last bin; values outside are ignored;
    each bin's score is the sum of the counts of the bins b-2 .. b+2 that exist;
    the estimate is lo + (b + 1/2) w for the lowest bin b with the highest score (lo itself when hi <= lo).

Every sample below sits on a grid where lo, hi, w, each bin and each score can be worked out by hand (the
expected values in the asserts are literals with the sums in the comments); `_by_definition` repeats the
derivation in exact rational arithmetic as a check of that hand arithmetic, not of the oracle's code."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from workloads import F16

W = Fraction(1, 64)       # bin width of every case: lo = 0, hi = 32, 2048 bins
OUT_LOW = [-100.0, -50.0, -50.0, -7.0]      # four values below lo: lo is the 5th smallest
OUT_HIGH = [5000.0, 5000.0, 6000.0, 60000.0]  # four values above hi: hi is the (M-4)-th smallest


def _grid_sample(counts, frac, hi_copies, lo_copies=0, empty=()):
    """fp16 sample: `counts[b]` extra values in bin b at offset `frac` of a bin width above the bin's lower edge,
    two background values per bin (at the lower edge; none in the bins listed in `empty`), `lo_copies` extra
    values equal to lo = 0, `hi_copies` values equal to hi = 32, and the eight outliers."""
    vals = []
    for b in range(2048):
        if b not in empty:
            vals += [float(Fraction(b) * W)] * 2
    for b, c in counts.items():
        vals += [float((Fraction(b) + frac) * W)] * c
    vals += [0.0] * lo_copies + [32.0] * hi_copies + OUT_LOW + OUT_HIGH
    a = np.array(vals, dtype=np.float64)
    h = a.astype(np.float16)
    assert np.array_equal(h.astype(np.float64), a), "every value must be exact in fp16"
    rng = np.random.default_rng(7)
    return h[rng.permutation(h.size)].view(np.uint16).reshape(1, -1)


def _by_definition(bits, nbins=2048, box=2, tie="lowest", bin_of=None):
    """The definition in the module docstring in exact rational arithmetic (variants for the negative checks)."""
    v = sorted(Fraction(float(t)) for t in bits.view(np.float16).ravel())
    M = len(v)
    klo, khi = -(-M // 1000), -(-999 * M // 1000)   # ceil(M/1000), ceil(999 M/1000): M avoids near-integers
    lo, hi = v[klo - 1], v[khi - 1]
    w = (hi - lo) / nbins
    cnt = [0] * nbins
    for t in v:
        if lo <= t <= hi:
            b = (t - lo) / w
            b = bin_of(b) if bin_of else b.numerator // b.denominator
            cnt[min(b, nbins - 1)] += 1
    score = [sum(cnt[max(b - box, 0):b + box + 1]) for b in range(nbins)]
    best = max(score)
    cands = [b for b in range(nbins) if score[b] == best]
    b = cands[0] if tie == "lowest" else cands[-1]
    return float(lo + (Fraction(2 * b + 1, 2)) * w)


# ---- case 1: four peaks chosen so that each plausible mistake picks a different one
#   scores (sum of 5 bins) with the background of 2 per bin, i.e. +10:
#     peak A  bins  98..102 = 10 20 40 20 10      -> score(100) = 100 + 10 = 110   <- highest, lowest bin of the tie
#     peak B  bins 398..402 = 30  5 30  5 30      -> score(400) = 100 + 10 = 110   (ties with A; a higher bin)
#     peak C  bins 299..301 = 22 45 22            -> score(300) =  89 + 10 =  99   (wins a 3-bin box: 95 against A's 86;
#                                                                                    wins without smoothing: 47 against 42)
#     peak D  bins 447..453 = 15 each             -> score(450) =  75 + 10 =  85   (wins a 7-bin box: 119 against A's 114)
#   neighbours of A: score(99) = score(101) = 90 + 10 = 100.  Top edge: score(2045) = 2+2+2+2+8 = 16.
#   every peak value sits 3/4 of a bin above its bin's lower edge, so rounding to the nearest edge instead of
#   taking the floor moves each peak up by one bin.
PEAKS = {98: 10, 99: 20, 100: 40, 101: 20, 102: 10,
         398: 30, 399: 5, 400: 30, 401: 5, 402: 30,
         299: 22, 300: 45, 301: 22,
         447: 15, 448: 15, 449: 15, 450: 15, 451: 15, 452: 15, 453: 15}


def _case1():
    X = _grid_sample(PEAKS, Fraction(3, 4), hi_copies=6)
    assert X.size == 4504   # ceil(4.504) = 5 and ceil(4499.496) = 4500 = M - 4: lo = 0, hi = 32
    return X


def test_hist_mode_hand_built_peaks():
    X = _case1()
    eta, _ = oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)
    assert eta == 100.5 / 64          # lo + (100 + 1/2) w = 1.5703125, exact in fp32
    assert eta == _by_definition(X)


def test_hist_mode_plausible_mistakes_give_other_answers():
    """The sample tells the definition from its near misses: each variant lands on another bin."""
    X = _case1()
    right = 100.5 / 64
    assert _by_definition(X, tie="highest") == 400.5 / 64          # highest bin on ties
    assert _by_definition(X, box=1) == 300.5 / 64                   # 3-bin box
    assert _by_definition(X, box=0) == 300.5 / 64                   # no smoothing
    assert _by_definition(X, box=3) in (449.5 / 64, 450.5 / 64, 451.5 / 64)    # 7-bin box (peak D)
    assert _by_definition(X, bin_of=lambda q: int(q + Fraction(1, 2))) == 101.5 / 64   # round instead of floor
    assert _by_definition(X, bin_of=lambda q: -(-q.numerator // q.denominator)) == 101.5 / 64  # ceil
    assert _by_definition(X, nbins=2047) != right and _by_definition(X, nbins=2049) != right
    for wrong in (100.0 / 64, 101.0 / 64, 99.5 / 64):               # lower edge, upper edge, bin below
        assert oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)[0] != wrong


def test_hist_mode_value_equal_to_hi_counts_in_the_last_bin():
    # background 2 per bin and 60 values equal to hi: bin 2047 holds 62.
    #   score(2045) = 2+2+2+2+62 = 70   score(2046) = 2+2+2+62 = 68 (4 bins exist)   score(2047) = 2+2+62 = 66
    # Without the values equal to hi every full window scores 10 and bin 2 would win.
    X = _grid_sample({}, Fraction(0), hi_copies=60)
    assert X.size == 4164   # ceil(4.164) = 5, ceil(4159.836) = 4160 = M - 4
    eta, _ = oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)
    assert eta == 2045.5 / 64
    assert eta == _by_definition(X)


def test_hist_mode_truncated_window_at_the_lower_edge_and_tie():
    # bins 1..6 empty, 40 extra values equal to lo: bin 0 holds 42.
    #   score(0) = score(1) = score(2) = 42 (windows cut at the edge), score(3) = 0, every full window further
    #   up scores 10, score(2045) = 16.  Three bins tie: the lowest wins.
    X = _grid_sample({}, Fraction(0), hi_copies=6, lo_copies=40, empty=range(1, 7))
    assert X.size == 4138   # ceil(4.138) = 5, ceil(4133.862) = 4134 = M - 4
    eta, _ = oracle.calibrate(X, F16, 0.5, oracle.MODE_HIST)
    assert eta == 0.5 / 64
    assert eta == _by_definition(X)
    assert _by_definition(X, tie="highest") == 2.5 / 64


def test_hist_mode_constant_sample_returns_the_constant():
    X = np.full((3, 50), 2.5, dtype=np.float16).view(np.uint16)
    assert oracle.calibrate(X, F16, 0.3, oracle.MODE_HIST) == (2.5, 0.0)


# ---- NaN calibration samples rank above every number (numpy's sort puts them last too)
@pytest.mark.parametrize("s", [0.25, 0.5, 0.8, 0.97])
def test_nan_samples_rank_last_like_numpy_sort(s):
    rng = np.random.default_rng(31)
    a = rng.standard_normal(1000).astype(np.float16)
    a[rng.choice(1000, size=100, replace=False)] = np.nan      # 10 % NaN
    a[:3] = [np.inf, -np.inf, np.inf]
    X = a.view(np.uint16).reshape(4, 250)
    k = int(np.ceil(np.float64(np.float32(s)) * 1000))
    want_tau = np.sort(np.abs(a.astype(np.float32)))[k - 1]     # numpy: NaN last
    eta, tau = oracle.calibrate(X, F16, s, oracle.MODE_ZERO)
    assert eta == 0.0
    assert (np.isnan(tau) and np.isnan(want_tau)) or tau == float(want_tau)
    # s = 0.97 asks for the 970th of 1000 with 900 numbers: the threshold itself is NaN (nothing passes |d| > NaN)
    assert np.isnan(want_tau) == (s > 0.9)


def test_median_with_nan_samples_like_numpy_sort():
    a = np.array([3.0, np.nan, -1.0, 7.0, np.nan, 0.5, 2.0], dtype=np.float16)   # sorted: -1 .5 2 3 7 nan nan
    X = a.view(np.uint16).reshape(1, -1)
    srt = np.sort(a.astype(np.float32))
    assert srt[3] == 3.0
    eta, _ = oracle.calibrate(X, F16, 0.0, oracle.MODE_MEDIAN)
    assert eta == 3.0
    b = np.concatenate([a, np.array([np.nan], dtype=np.float16)])                  # even count: (3 + 7) / 2
    eta, _ = oracle.calibrate(b.view(np.uint16).reshape(1, -1), F16, 0.0, oracle.MODE_MEDIAN)
    assert eta == 5.0
