"""Pins for oracle/sampling.py: the integer generator against big-integer
arithmetic and a published test vector; the noise against Gumbel moments; the
sampler against the categorical distribution it must realise."""
import numpy as np

from oracle import sampling as os_


def _mix_py(z):
    M = (1 << 64) - 1
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M
    return z ^ (z >> 31)


def test_mixer_matches_published_splitmix64_vector():
    # first output of SplitMix64 from state 0 is mix(0x9E3779B97F4A7C15) = 0xE220A8397B1DCDAF
    assert int(os_._mix(np.uint64(0x9E3779B97F4A7C15))) == 0xE220A8397B1DCDAF
    # second and third outputs of the same public sequence
    assert int(os_._mix(np.uint64((2 * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)))) == 0x6E789E6AA1B965F4
    assert int(os_._mix(np.uint64((3 * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)))) == 0x06C45D188009454F


def test_random_bits_match_big_integer_arithmetic():
    M = (1 << 64) - 1
    for seed, seq, step in [(0, 0, 0), (12345, 7, 511), (2 ** 63 + 5, 127, 8191)]:
        key = _mix_py((_mix_py(seed ^ 0x9E3779B97F4A7C15) + ((seq << 32) | step)) & M)
        got = os_.random_bits(seed, seq, step, 50)
        for v in (0, 1, 17, 49):
            assert int(got[v]) == _mix_py((key + v * 0x9E3779B97F4A7C15) & M) >> 32
    # distinct (seq, step) give distinct streams
    assert not np.array_equal(os_.random_bits(1, 2, 3, 64), os_.random_bits(1, 3, 2, 64))


def test_uniform_is_open_interval_and_exact():
    r = np.array([0, 511, 512, 0xFFFFFFFF], dtype=np.uint32)
    u = os_.uniform_from_bits(r)
    assert u.dtype == np.float32
    assert u[0] == np.float32(2.0 ** -24) and u[1] == u[0] and u[2] == np.float32(1.5 * 2.0 ** -23)
    assert u[3] == np.float32(1.0 - 2.0 ** -24) and 0.0 < u.min() and u.max() < 1.0
    assert np.isfinite(os_.gumbel_noise(3, 1, 4, 4096)).all()


def test_gumbel_moments():
    g = np.concatenate([os_.gumbel_noise(9, s, 0, 50000) for s in range(8)]).astype(np.float64)
    assert abs(g.mean() - 0.5772156649) < 0.01           # Euler-Mascheroni
    assert abs(g.var() - np.pi ** 2 / 6) < 0.03
    # distribution function exp(-exp(-x)) at a few points
    for x in (-1.0, 0.0, 1.5):
        assert abs((g <= x).mean() - np.exp(-np.exp(-x))) < 0.005


def test_greedy_is_zero_noise_and_ties_take_lowest_index():
    row = np.array([0.1, 2.0, 2.0, -1.0], dtype=np.float32)
    tok, margin = os_.sample_row(row, 0.0)
    assert tok == 1 and margin == 0.0
    tok2, _ = os_.sample_row(row, 1.0, np.zeros(4, dtype=np.float32))
    assert tok2 == 1
    tok3, m3 = os_.sample_row(np.array([0.0, 1.0, 3.5]), 0.0)
    assert tok3 == 2 and abs(m3 - 2.5) < 1e-7


def test_temperature_divides_logits_before_noise():
    row = np.array([1.0, 0.0], dtype=np.float32)
    noise = np.array([0.0, 1.5], dtype=np.float32)
    assert os_.sample_row(row, 1.0, noise)[0] == 1          # 1.0 vs 1.5
    assert os_.sample_row(row, 0.5, noise)[0] == 0          # 2.0 vs 1.5
    np.testing.assert_allclose(os_.scores(row, 0.5, noise), [2.0, 1.5])


def _chi2(counts, probs):
    n = counts.sum()
    return float(((counts - n * probs) ** 2 / (n * probs)).sum())


def test_sampled_frequencies_follow_softmax():
    """Untruncated categorical at temperature T (actor settings, App. D)."""
    logits = np.array([[2.0, 0.5, -1.0, 0.0, 1.0, -3.0, 0.3, 1.7]], dtype=np.float32)
    N = 20000
    for T in (1.0, 0.6):
        p = np.exp(logits[0].astype(np.float64) / T)
        p /= p.sum()
        counts = np.zeros(8)
        for step in range(N):
            tok, _ = os_.sample(logits, T, seed=42, seq_ids=[step % 5], steps=[step])
            counts[tok[0]] += 1
        # 7 degrees of freedom: P(chi2 > 24.3) = 0.001
        assert _chi2(counts, p) < 24.3, (T, counts, p * N)


def test_shared_noise_mode_overrides_generator():
    logits = np.zeros((2, 16), dtype=np.float32)
    noise = np.zeros((2, 16), dtype=np.float32)
    noise[0, 5] = 1.0
    noise[1, 11] = 1.0
    tok, margin = os_.sample(logits, 1.0, seed=0, seq_ids=[0, 1], steps=[0, 0], noise=noise)
    assert tok.tolist() == [5, 11] and np.allclose(margin, 1.0)
