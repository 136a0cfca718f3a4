"""The single-wavefront selection of the HIP path (csrc/topn.h, wave_topn) rests on two facts
about fp32 arithmetic: bin(v) = int((v - lo) * scale) never decreases with v, and a value one
bin width below the lower edge of bin D is not above any score that falls into bin D or a
higher one.  Both are checked here in numpy's fp32 (IEEE, round to nearest even, as on the
GPU) over score sets of very different magnitudes and spreads; no GPU is involved and nothing
of the library is called."""
import numpy as np
import pytest

BINS = 512


def bins_of(v, lo, hi):
    f = np.float32
    scale = f(BINS - 1) / (f(hi) - f(lo))
    b = ((v.astype(f) - f(lo)) * scale).astype(np.int64)     # truncation, like v_cvt_i32_f32
    return np.minimum(b, BINS - 1), scale


def cases():
    rng = np.random.default_rng(7)
    for offset in (0.0, 1.0, -3.5, 1e3, -1e5, 3e7):
        for spread in (1e-6, 1e-3, 1.0, 40.0, 1e4):
            v = (offset + spread * rng.standard_normal(4096)).astype(np.float32)
            if v.max() > v.min():
                yield offset, spread, v
    # scores one ulp apart, and a set with many repeats
    base = np.float32(2.5)
    yield 2.5, 0.0, np.array([np.nextafter(base, np.float32(9), dtype=np.float32)] * 7 + [base] * 9
                             + [np.nextafter(base, np.float32(0), dtype=np.float32)] * 5, dtype=np.float32)
    yield 0.0, 1.0, np.repeat(rng.standard_normal(64).astype(np.float32), 64)


@pytest.mark.parametrize("offset,spread,v", list(cases()))
def test_bins_never_decrease_with_the_score(offset, spread, v):
    lo, hi = v.min(), v.max()
    b, _ = bins_of(v, lo, hi)
    order = np.argsort(v, kind="stable")
    assert (np.diff(b[order]) >= 0).all()
    assert b.min() >= 0 and b.max() <= BINS - 1


@pytest.mark.parametrize("offset,spread,v", list(cases()))
def test_one_bin_below_the_edge_is_a_lower_bound(offset, spread, v):
    f = np.float32
    lo, hi = v.min(), v.max()
    b, scale = bins_of(v, lo, hi)
    if not np.isfinite(scale) or scale == 0:
        pytest.skip("degenerate range: the kernel takes its radix path")
    for D in (1, 2, 17, 255, 400, BINS - 1):
        members = v[b >= D]
        if members.size == 0:
            continue
        bound = f(lo) + f(D - 1) / scale
        assert bound <= members.min(), (D, bound, members.min())


def test_selection_by_bin_then_exact_rank_equals_a_full_sort():
    """The whole scheme on the host: bin D where the count from the top reaches k, everything
    above kept, the scores of bin D ranked exactly by (score descending, index ascending)."""
    rng = np.random.default_rng(11)
    for n, k in ((1024, 64), (2048, 1), (700, 699), (4096, 256)):
        v = rng.standard_normal(n).astype(np.float32)
        v[rng.integers(0, n, 50)] = v[rng.integers(0, n, 50)]          # exact ties
        b, _ = bins_of(v, v.min(), v.max())
        counts = np.bincount(b, minlength=BINS)[::-1].cumsum()[::-1]    # scores in bin >= D
        D = max(d for d in range(BINS) if counts[d] >= k)
        above = counts[D + 1] if D + 1 < BINS else 0
        inside = [i for i in range(n) if b[i] == D]
        inside.sort(key=lambda i: (-v[i], i))
        kept = sorted([i for i in range(n) if b[i] > D] + inside[:k - above])
        want = sorted(sorted(range(n), key=lambda i: (-v[i], i))[:k])
        assert kept == want
