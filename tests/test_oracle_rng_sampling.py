"""Pins for the oracle's random-number and one-hop layers (CPU only).

Philox4x32-10 is pinned by the published known-answer vectors; Floyd's subset algorithm by
the textbook properties (a valid f-subset, uniform over all subsets); one-hop sampling by
the invariants the paper states in Section 4.1.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _kat_rows():
    rows = []
    with open(os.path.join(GOLDEN, "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                w = [int(x, 16) for x in line.replace("->", " ").split()]
                rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        got = oracle.philox4x32_10(ctr, key)
        assert [int(x) for x in got] == want


def _philox_bigint(ctr, key):
    """Second implementation with Python integers, written from the round description:
    two 32x32->64 products, high halves xor'ed with the neighbouring counter word and the key."""
    c = list(ctr)
    k = list(key)
    for r in range(10):
        if r:
            k = [(k[0] + 0x9E3779B9) % 2**32, (k[1] + 0xBB67AE85) % 2**32]
        a = 0xD2511F53 * c[0]
        b = 0xCD9E8D57 * c[2]
        c = [(b >> 32) ^ c[1] ^ k[0], b % 2**32, (a >> 32) ^ c[3] ^ k[1], a % 2**32]
    return c


def test_philox_agrees_with_bigint_version():
    rng = np.random.default_rng(0)
    for _ in range(2000):
        ctr = [int(x) for x in rng.integers(0, 2**32, size=4)]
        key = [int(x) for x in rng.integers(0, 2**32, size=2)]
        assert [int(x) for x in oracle.philox4x32_10(ctr, key)] == _philox_bigint(ctr, key)
    # the known answers also hold for the second implementation (it is not just a mirror)
    for ctr, key, want in _kat_rows():
        assert _philox_bigint(ctr, key) == want


@pytest.mark.parametrize("deg,f", [(5, 2), (6, 5), (7, 1), (40, 15), (1000, 20), (3_000_000_000, 15)])
def test_floyd_returns_a_valid_subset(deg, f):
    for seed in range(50):
        picks = oracle.floyd_positions(deg, f, seed, node=seed * 7 + 1, hop=seed % 3)
        assert len(picks) == f
        assert picks.min() >= 0 and picks.max() < deg
        assert len(set(picks.tolist())) == f


def test_floyd_is_uniform_over_subsets():
    """deg=5, f=2: each of the C(5,2)=10 subsets must appear with frequency 1/10."""
    trials = 40000
    counts = {s: 0 for s in itertools.combinations(range(5), 2)}
    for t in range(trials):
        picks = oracle.floyd_positions(5, 2, seed=12345, node=t, hop=0)
        counts[tuple(sorted(picks.tolist()))] += 1
    expected = trials / 10
    chi2 = sum((c - expected) ** 2 / expected for c in counts.values())
    assert chi2 < 33.7        # chi-square, 9 dof, p = 1e-4


def test_floyd_inclusion_frequency_is_f_over_deg():
    deg, f, trials = 23, 7, 30000
    hits = np.zeros(deg)
    for t in range(trials):
        hits[oracle.floyd_positions(deg, f, seed=t, node=99, hop=1)] += 1
    p = f / deg
    sigma = np.sqrt(trials * p * (1 - p))
    assert np.all(np.abs(hits - trials * p) < 4.5 * sigma)


def test_floyd_streams_differ_by_node_hop_seed_and_direction():
    base = oracle.floyd_positions(10**6, 16, seed=1, node=2, hop=0, dirbit=0).tolist()
    assert base == oracle.floyd_positions(10**6, 16, seed=1, node=2, hop=0, dirbit=0).tolist()
    assert base != oracle.floyd_positions(10**6, 16, seed=2, node=2, hop=0, dirbit=0).tolist()
    assert base != oracle.floyd_positions(10**6, 16, seed=1, node=3, hop=0, dirbit=0).tolist()
    assert base != oracle.floyd_positions(10**6, 16, seed=1, node=2, hop=1, dirbit=0).tolist()
    assert base != oracle.floyd_positions(10**6, 16, seed=1, node=2, hop=0, dirbit=1).tolist()
    assert base != oracle.floyd_positions(10**6, 16, seed=1 << 32, node=2, hop=0, dirbit=0).tolist()


def test_floyd_first_pick_follows_the_documented_word_and_range_reduction():
    """Step s=0 draws word 0 of Philox(counter=(0, node, hop, dir), key=seed halves) and maps
    it to [0, deg-f] by a multiply-high; with nothing picked before, that value is the pick."""
    deg, f, seed, node, hop = 1000, 4, (7 << 32) | 5, 321, 2
    w = oracle.philox4x32_10([0, node, hop, 0], [5, 7])
    picks = oracle.floyd_positions(deg, f, seed, node, hop)
    assert picks[0] == (int(w[0]) * (deg - f + 1)) >> 32


def test_onehop_invariants_on_rmat(rmat16k):
    rp, col = rmat16k["out"]
    g = oracle.Graph(len(rp) - 1, rp, col)
    deg = np.diff(rp)
    rng = np.random.default_rng(1)
    nodes = np.concatenate([rng.integers(0, len(deg), 300), np.argsort(deg)[-20:], np.nonzero(deg == 0)[0][:5]])
    for f in (1, 5, 10, 32):
        for v in nodes:
            v = int(v)
            s = oracle.onehop(g, v, f, seed=9, hop=1)
            adj = col[rp[v]:rp[v + 1]]
            assert len(s) == min(deg[v], f)                    # count = min(deg, fanout)
            assert len(set(s.tolist())) == len(s)              # no duplicates
            assert set(s.tolist()) <= set(adj.tolist())        # every sampled neighbour is a real edge
            if deg[v] <= f:
                assert np.array_equal(s, adj)                  # fewer than f: all returned, as stored


def test_onehop_both_directions_is_out_then_in(rmat16k):
    rp, col = rmat16k["out"]
    rpi, coli = rmat16k["in"]
    g = oracle.Graph(len(rp) - 1, rp, col, rpi, coli)
    g_in_as_out = oracle.Graph(len(rp) - 1, rpi, coli)
    for v in (0, 17, 4000, 16000):
        both = oracle.onehop(g, v, 6, seed=3, hop=0, direction=2)
        out = oracle.onehop(g, v, 6, seed=3, hop=0, direction=0)
        inn = oracle.onehop(g, v, 6, seed=3, hop=0, direction=1)
        assert np.array_equal(both, np.concatenate([out, inn]))
        assert set(inn.tolist()) <= set(coli[rpi[v]:rpi[v + 1]].tolist())
        # the in-stream is its own stream, not the out-stream applied to the reversed graph
        if rpi[v + 1] - rpi[v] > 12:
            assert not np.array_equal(inn, oracle.onehop(g_in_as_out, v, 6, seed=3, hop=0, direction=0))
