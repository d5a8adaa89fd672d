"""Pins for the oracle's random numbers (Philox4x32-10, one 53-bit uniform per
(seed, iteration, token)); the paper's Algorithm 2 only says "sample u ~ U(0,1)"."""
import numpy as np
from scipy import stats

import oracle


def test_known_answer_vectors(golden):
    rows = golden("philox4x32_10_kat.txt")
    assert len(rows) == 3
    for row in rows:
        v = [int(x, 16) for x in row]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in out] == v[6:10]


def test_uniform_is_top_53_bits_of_first_two_words():
    # counter = (token lo, token hi, iteration, 0), key = (seed lo, seed hi)
    for seed, it, tok in [(4631, 1, 0), (2**40 + 17, 7, 123456789), (1, 0, 2**35 + 5),
                          (2**64 - 1, 2**32 - 1, 2**64 - 1)]:
        r = oracle.philox4x32_10([tok & 0xFFFFFFFF, tok >> 32, it, 0],
                                 [seed & 0xFFFFFFFF, seed >> 32])
        bits = ((int(r[0]) << 32) | int(r[1])) >> 11
        assert oracle.uniform(seed, it, tok) == bits / 2.0**53
        assert 0.0 <= oracle.uniform(seed, it, tok) < 1.0


def test_streams_differ_in_every_key_part():
    base = oracle.uniforms(4631, 1, 0, 4096)
    assert len(np.unique(base)) == 4096
    for other in (oracle.uniforms(4632, 1, 0, 4096), oracle.uniforms(4631, 2, 0, 4096),
                  oracle.uniforms(4631, 1, 4096, 4096), oracle.uniforms(4631 + 2**32, 1, 0, 4096),
                  oracle.uniforms(4631, 1, 2**32, 4096)):
        assert not np.any(other == base)
    # the vector call is the scalar call, token by token
    assert base[77] == oracle.uniform(4631, 1, 77)


def test_uniformity():
    n = 1 << 20
    u = oracle.uniforms(4631, 3, 0, n)
    assert abs(u.mean() - 0.5) < 4 * np.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 5e-4
    hist = np.bincount((u * 256).astype(np.int64), minlength=256)
    assert stats.chisquare(hist).pvalue > 1e-4
    # serial pairs
    pair = np.bincount(((u[:-1] * 16).astype(np.int64) * 16 + (u[1:] * 16).astype(np.int64)),
                       minlength=256)
    assert stats.chisquare(pair).pvalue > 1e-4


def test_initial_topics_are_floor_u_times_K():
    K, T = 37, 5000
    z = oracle.init_topics(T, K, 99)
    u = oracle.uniforms(99, 0, 0, T)
    assert np.array_equal(z, np.minimum(np.floor(u * K), K - 1).astype(np.uint16))
    assert stats.chisquare(np.bincount(z, minlength=K)).pvalue > 1e-4
    assert np.all(oracle.init_topics(100, 1, 5) == 0)
