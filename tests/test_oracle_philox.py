"""Pins for oracle/philox.py: structure and statistics (no known-answer vectors
are available offline; see the module header)."""
import numpy as np

from oracle import philox


def test_counter_blocks_are_distinct():
    # a Philox round is a bijection of the counter for a fixed key, so distinct
    # counters must give distinct 128-bit blocks
    w = philox.philox4x32(12345, np.arange(200_000), step=7, stream=0)
    packed = w.view(np.uint64).reshape(-1, 2)
    assert len({(int(a), int(b)) for a, b in packed}) == packed.shape[0]


def test_streams_steps_seeds_and_subs_do_not_collide():
    base = philox.words(99, 4096, 3, philox.STREAM_INDEX)
    others = [philox.words(99, 4096, 4, philox.STREAM_INDEX),
              philox.words(99, 4096, 3, philox.STREAM_SMOOTH),
              philox.words(100, 4096, 3, philox.STREAM_INDEX),
              philox.words(99 + (1 << 32), 4096, 3, philox.STREAM_INDEX),
              philox.words(99, 4096, 3, philox.STREAM_INDEX, sub=1)]
    for o in others:
        assert np.mean(base == o) < 0.01
    # deterministic
    assert np.array_equal(base, philox.words(99, 4096, 3, philox.STREAM_INDEX))
    # prefix property: element e is word e&3 of block e>>2 whatever n is
    assert np.array_equal(base[:1001], philox.words(99, 1001, 3, philox.STREAM_INDEX))


def test_words_are_uniform_bits():
    w = philox.words(2024, 1 << 18, 0, 0)
    bits = np.unpackbits(w.view(np.uint8))
    assert abs(bits.mean() - 0.5) < 2e-3
    # every one of the 32 bit positions is balanced
    per_bit = [(w >> np.uint32(k)) & np.uint32(1) for k in range(32)]
    assert all(abs(b.mean() - 0.5) < 6e-3 for b in per_bit)
    # serial correlation of successive words
    x = w.astype(np.float64) / 2 ** 32
    assert abs(np.corrcoef(x[:-1], x[1:])[0, 1]) < 0.01


def test_indices_match_exact_integer_definition_and_range():
    for count in (1, 2, 3, 7, 255, 10_000, 1_000_000, 2 ** 32 - 1):
        idx = philox.sample_indices(5, 11, 256, count)
        w = philox.words(5, 256, 11, philox.STREAM_INDEX)
        brute = [(int(x) * count) // (1 << 32) for x in w]      # python big ints
        assert idx.tolist() == brute
        assert idx.min() >= 0 and idx.max() < count


def test_indices_uniform_on_tiny_count():
    count, draws = 7, 0
    hist = np.zeros(count)
    for step in range(400):
        idx = philox.sample_indices(77, step, 256, count)
        hist += np.bincount(idx, minlength=count)
        draws += 256
    expected = draws / count
    chi2 = np.sum((hist - expected) ** 2 / expected)
    assert chi2 < 22.5          # 6 dof, p ~ 0.001


def test_normals_moments_and_box_muller_structure():
    n = 400_000
    z = philox.normals(31337, n, 5, philox.STREAM_SMOOTH)
    assert abs(z.mean()) < 5e-3
    assert abs(z.var() - 1.0) < 1e-2
    assert abs(np.mean(z ** 3)) < 2e-2
    assert abs(np.mean(z ** 4) - 3.0) < 6e-2
    # pairs (z0, z1) of a block come from one (u1, u2): exp(-(z0^2+z1^2)/2) must be
    # a positive multiple of 2^-24 and the angle a multiple of 2 pi 2^-24
    p = z.reshape(-1, 2)[:2000]
    u1 = np.exp(-0.5 * np.sum(p * p, axis=1)) * 2 ** 24
    assert np.all(np.abs(u1 - np.round(u1)) < 1e-4 * np.maximum(u1, 1)) and np.all(np.round(u1) >= 1)
    ang = np.mod(np.arctan2(p[:, 1], p[:, 0]), 2 * np.pi) / (2 * np.pi) * 2 ** 24
    assert np.all(np.abs(ang - np.round(ang)) < 1e-3)
    # element e only depends on e (prefix property)
    assert np.array_equal(z[:999], philox.normals(31337, 999, 5, philox.STREAM_SMOOTH))


def test_mix64_is_injective_on_small_range_and_nonzero():
    vals = {philox.mix64(s, i) for s in range(8) for i in range(256)}
    assert len(vals) == 8 * 256 and 0 not in vals
