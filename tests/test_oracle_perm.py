"""Pins for the permutation generator (Section 3.2): 32-bit xorshift keys, sort carrying indices."""
import os

import numpy as np
import pytest

import oracle

pytestmark = pytest.mark.usefixtures("oracle_lib")
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "perm_known_answers.txt")


def test_is_a_permutation_deterministic_and_seed_dependent():
    for m in [0, 1, 2, 63, 64, 65, 1000, 4097]:
        p = oracle.permutation(5, m)
        assert sorted(p.tolist()) == list(range(m))
        assert np.array_equal(p, oracle.permutation(5, m))
    a, b, c = oracle.permutation(1, 1000), oracle.permutation(2, 1000), oracle.permutation(1, 1000, chunk=1)
    assert not np.array_equal(a, b) and not np.array_equal(a, c)


def test_keys_sorted_with_index_tiebreak():
    m = 300_000          # about m^2 / 2^33 = 10 duplicate keys expected
    perm, keys = oracle.permutation(11, m, want_keys=True)
    ks = keys[perm]
    assert np.all(ks[1:] >= ks[:-1])
    eq = np.nonzero(ks[1:] == ks[:-1])[0]
    assert eq.size > 0, "expected at least one duplicate 32-bit key at this size"
    assert np.all(perm[eq + 1] > perm[eq])
    # the definition again through numpy's stable sort of the keys
    assert np.array_equal(perm, np.argsort(keys, kind="stable").astype(np.uint32))


def test_keys_look_uniform():
    _, keys = oracle.permutation(3, 200_000, want_keys=True)
    assert abs(keys.astype(np.float64).mean() / 2 ** 32 - 0.5) < 0.005
    counts = np.bincount(keys >> 24, minlength=256)
    assert counts.min() > 600 and counts.max() < 970      # expectation 781
    for bit in range(32):
        frac = ((keys >> bit) & 1).mean()
        assert abs(frac - 0.5) < 0.01
    # positions are uniform: mean displacement of a uniform permutation is m/3
    perm = oracle.permutation(3, 200_000)
    disp = np.abs(perm.astype(np.int64) - np.arange(200_000)).mean()
    assert abs(disp / 200_000 - 1 / 3) < 0.01


def test_xorshift_round_is_the_13_17_5_triple():
    """The last stage of the key is four rounds of the (13,17,5) xorshift, a bijection of the
    non-zero 32-bit states; undo it here with the inverse maps and check the pre-image is the
    64->32 fold of the integer mix (an independent re-derivation through inverses, not a re-typing
    of the forward formula)."""
    M = 0xFFFFFFFF

    def inv_shl_xor(x, s):     # inverse of x ^= x << s
        r = x
        for _ in range(32 // s + 1):
            r = x ^ ((r << s) & M)
        return r

    def inv_shr_xor(x, s):     # inverse of x ^= x >> s
        r = x
        for _ in range(32 // s + 1):
            r = x ^ (r >> s)
        return r

    def mix(z):
        z = (z + 0x9E3779B97F4A7C15) & (2 ** 64 - 1)
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & (2 ** 64 - 1)
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & (2 ** 64 - 1)
        return z ^ (z >> 31)

    for seed, chunk, c in [(0, 0, 0), (1, 0, 5), (2 ** 63 + 9, 3, 123456), (77, 15, 999_999)]:
        x = oracle.key(seed, chunk, c)
        for _ in range(4):
            x = inv_shl_xor(x, 5)
            x = inv_shr_xor(x, 17)
            x = inv_shl_xor(x, 13)
        z = mix(seed ^ mix(chunk + 0x632BE59BD9B4E019))
        z = mix((z + c * 0x9E3779B97F4A7C15) & (2 ** 64 - 1))
        fold = (z ^ (z >> 32)) & M
        assert x == (fold if fold != 0 else 0x6C078965)


def test_known_answers():
    """Known-answer vectors written by tests/golden/make_perm_known_answers.py (oracle only)."""
    with open(GOLDEN) as f:
        lines = [l.split() for l in f if l.strip() and not l.startswith("#")]
    assert len(lines) >= 4
    for rec in lines:
        kind, seed, chunk, m = rec[0], int(rec[1]), int(rec[2]), int(rec[3])
        vals = np.array([int(t) for t in rec[4:]], dtype=np.uint32)
        perm, keys = oracle.permutation(seed, m, chunk=chunk, want_keys=True)
        got = keys[: vals.size] if kind == "keys" else perm[: vals.size]
        assert np.array_equal(got, vals)
