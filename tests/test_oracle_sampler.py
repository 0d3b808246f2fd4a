"""Pins of the oracle's prioritized sampler (no GPU)."""
import numpy as np
import pytest
from scipy import stats as sps


def test_weight_closed_forms(oracle):
    eps = 0.05
    # v = 1/2 -> sqrt(1/4) + eps; v in {0, 1} -> eps; symmetric in v <-> 1 - v
    w = oracle.weights([1.0, 0.0, 5.0, 1.0, 3.0], [1.0, 5.0, 0.0, 3.0, 1.0], eps)
    assert w[0] == 0.5 + eps
    assert w[1] == eps and w[2] == eps
    assert w[3] == w[4] == pytest.approx(np.sqrt(0.25 * 0.75) + eps, rel=1e-15)
    # the maximum is at v = 1/2
    a = np.linspace(0.1, 9.9, 99).astype(np.float32)
    b = (10.0 - a).astype(np.float32)
    ww = oracle.weights(a, b, eps)
    assert np.argmax(ww) == 49 and ww.max() <= 0.5 + eps + 1e-12
    # depends on alpha, beta only through v
    np.testing.assert_allclose(oracle.weights([2.0], [6.0], eps), oracle.weights([0.5], [1.5], eps))
    # empty entry keeps the bonus only
    assert oracle.weights([0.0], [0.0], eps)[0] == eps


def test_weight_codes_and_cdf(oracle):
    assert oracle.weight_code(0.5) == 1 << 31
    assert oracle.weight_code(0.05) == int(np.floor(0.05 * 2.0 ** 32))
    rng = np.random.default_rng(0)
    a = rng.uniform(0.5, 50, 1000).astype(np.float32)
    b = rng.uniform(0.5, 50, 1000).astype(np.float32)
    w = oracle.weights(a, b, 0.05)
    codes = np.floor(w * 2.0 ** 32).astype(np.uint64)
    assert np.array_equal(oracle.weight_cdf(a, b, 0.05), np.cumsum(codes))


def test_philox_known_answers(oracle):
    # The published known-answer vectors of the generator (tests/golden/philox4x32_10_kat.txt).
    import pathlib
    rows = [ln.split() for ln in (pathlib.Path(__file__).parent / "golden" / "philox4x32_10_kat.txt").read_text().splitlines()
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 3
    for row in rows:
        words = [int(x, 16) for x in row]
        out = oracle.philox4x32_10(words[0:4], words[4:6])
        assert [int(x) for x in out] == words[6:10]


def test_philox_is_a_keyed_bijection_with_good_bits(oracle):
    # Beyond the known answers: determinism, distinct counters give distinct
    # blocks, key and counter both matter, bits are balanced, one flipped input
    # bit flips about half of the output bits.
    key = np.array([7, 9], np.uint32)
    outs = np.array([oracle.philox4x32_10([i, 0, 0, 0], key) for i in range(4096)])
    assert np.array_equal(outs[5], oracle.philox4x32_10([5, 0, 0, 0], key))
    assert len({tuple(o) for o in outs}) == 4096
    assert not np.array_equal(oracle.philox4x32_10([5, 0, 0, 0], [7, 10]), outs[5])
    for pos in range(4):
        c = [0, 0, 0, 0]
        c[pos] = 1
        assert not np.array_equal(oracle.philox4x32_10(c, key), outs[0])
    bits = np.unpackbits(outs.view(np.uint8), axis=1)
    frac = bits.mean(axis=0)
    assert np.all(np.abs(frac - 0.5) < 5 * 0.5 / np.sqrt(4096))
    flips = []
    for i in range(256):
        base = oracle.philox4x32_10([i, 3, 1, 0], key)
        for bit in (0, 7, 31):
            other = oracle.philox4x32_10([i ^ (1 << bit), 3, 1, 0], key)
            flips.append(np.unpackbits((base ^ other).view(np.uint8)).sum())
    assert abs(np.mean(flips) - 64) < 2.0


def test_draw_follows_the_integer_cdf(oracle):
    # slot k, attempt 0: threshold = high 64 bits of (random 64 bits * total)
    rng = np.random.default_rng(3)
    N, B, seed, it = 300, 64, 11, 5
    a = rng.uniform(0.5, 50, N).astype(np.float32)
    b = rng.uniform(0.5, 50, N).astype(np.float32)
    cdf = oracle.weight_cdf(a, b, 0.05)
    total = int(cdf[-1])
    idx = oracle.sample_prompts(a, b, B, 0.05, seed, it, replace=True)
    for k in range(B):
        o = oracle.philox4x32_10([k, 0, it, 0], [seed, 0])
        r = int(o[0]) | (int(o[1]) << 32)
        t = (r * total) >> 64
        assert idx[k] == int(np.searchsorted(cdf, np.uint64(t), side="right"))


def test_equal_trackers_sample_uniformly_and_weighted_matches_chi_square(oracle):
    N = 16
    counts = np.zeros(N)
    a = np.full(N, 0.5, np.float32)
    for seed in range(300):
        idx = oracle.sample_prompts(a, a, 32, 0.05, seed, 0, replace=True)
        counts += np.bincount(idx, minlength=N)
    assert sps.chisquare(counts).pvalue > 1e-3
    # unequal weights: frequencies follow w / sum(w)
    rng = np.random.default_rng(5)
    al = rng.uniform(0.1, 10, N).astype(np.float32)
    be = rng.uniform(0.1, 10, N).astype(np.float32)
    w = oracle.weights(al, be, 0.05)
    counts = np.zeros(N)
    for seed in range(300):
        idx = oracle.sample_prompts(al, be, 64, 0.05, seed, 1, replace=True)
        counts += np.bincount(idx, minlength=N)
    assert sps.chisquare(counts, counts.sum() * w / w.sum()).pvalue > 1e-3
    # a deliberately wrong model (uniform) must be rejected by the same test
    assert sps.chisquare(counts).pvalue < 1e-6


def test_without_replacement_is_successive_sampling(oracle):
    # N = 4, B = 2: P(first = i, second = j) = p_i * p_j / (1 - p_i), i != j
    al = np.array([1.0, 1.0, 9.0, 0.2], np.float32)
    be = np.array([1.0, 4.0, 1.0, 5.0], np.float32)
    w = oracle.weights(al, be, 0.05)
    p = w / w.sum()
    counts = np.zeros((4, 4))
    n = 6000
    for seed in range(n):
        i, j = oracle.sample_prompts(al, be, 2, 0.05, seed, 0, replace=False)
        counts[i, j] += 1
    assert np.all(np.diag(counts) == 0)
    expect = np.array([[0 if i == j else p[i] * p[j] / (1 - p[i]) for j in range(4)]
                       for i in range(4)]) * n
    off = ~np.eye(4, dtype=bool)
    assert sps.chisquare(counts[off], expect[off]).pvalue > 1e-3


def test_without_replacement_distinct_and_permutation(oracle):
    rng = np.random.default_rng(7)
    N = 16
    a = np.full(N, 0.5, np.float32)
    idx, att = oracle.sample_prompts(a, a, 8, 0.05, 0, 0, replace=False, return_attempts=True)
    assert len(set(idx.tolist())) == 8 and att[0] == 0
    full = oracle.sample_prompts(a, a, N, 0.05, 1, 0, replace=False)
    assert sorted(full.tolist()) == list(range(N))
    # the first B' slots do not depend on how many slots follow
    assert np.array_equal(full[:8], oracle.sample_prompts(a, a, 8, 0.05, 1, 0, replace=False))
    # seed and iteration both change the draw
    al = rng.uniform(0.5, 50, 4096).astype(np.float32)
    be = rng.uniform(0.5, 50, 4096).astype(np.float32)
    d0 = oracle.sample_prompts(al, be, 128, 0.05, 7, 0)
    assert not np.array_equal(d0, oracle.sample_prompts(al, be, 128, 0.05, 8, 0))
    assert not np.array_equal(d0, oracle.sample_prompts(al, be, 128, 0.05, 7, 1))
    assert np.array_equal(d0, oracle.sample_prompts(al, be, 128, 0.05, 7, 0))
    with pytest.raises(ValueError):
        oracle.sample_prompts(a, a, N + 1, 0.05, 0, 0, replace=False)


def test_zero_total_weight_draws_nothing(oracle):
    # eps = 0 and every estimate at 0 or 1: all weights vanish; the sampler must refuse, not index past the end
    a = np.array([0.0, 3.0, 0.0, 1.0], np.float32)
    b = np.array([2.0, 0.0, 5.0, 0.0], np.float32)
    assert not oracle.weights(a, b, 0.0).any()
    for replace in (True, False):
        with pytest.raises(RuntimeError):
            oracle.sample_prompts(a, b, 2, 0.0, 0, 0, replace)
    # a single entry with weight keeps everything on it (with replacement)
    a[0], b[0] = 1.0, 1.0
    assert (oracle.sample_prompts(a, b, 5, 0.0, 0, 0, True) == 0).all()
