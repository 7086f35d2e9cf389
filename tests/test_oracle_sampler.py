"""Pins for the checker's load-adaptive sampler partition (Sec. III-C phase 2)."""
import collections

import numpy as np
import pytest

import oracle


def test_splitmix64_published_values():
    # first outputs for seed 1234567, as listed with the generator's reference code
    rng = oracle.SplitMix64(1234567)
    got = [rng.next() for _ in range(5)]
    assert got == [6457827717110365317, 3203168211198807973, 9817491932198370423,
                   4593380528125082431, 16408922859458223821]


def test_bounded_is_in_range_and_unbiased_enough():
    rng = oracle.SplitMix64(42)
    for n in (1, 2, 3, 7, 1000, 2 ** 40 + 3):
        for _ in range(200):
            assert 0 <= oracle._bounded(rng, n) < n
    counts = collections.Counter(oracle._bounded(rng, 6) for _ in range(60000))
    assert all(abs(c - 10000) < 400 for c in counts.values()) and len(counts) == 6


def test_permutation_is_a_bijection_and_seeded():
    for N in (0, 1, 2, 17, 1000):
        p = oracle.epoch_permutation(N, 7, 3)
        assert sorted(p) == list(range(N))
    a = oracle.epoch_permutation(1000, 7, 3)
    assert a == oracle.epoch_permutation(1000, 7, 3)
    assert a != oracle.epoch_permutation(1000, 7, 4) and a != oracle.epoch_permutation(1000, 8, 3)
    assert oracle.epoch_permutation(10, 1, 1, shuffle=False) == list(range(10))
    # every position is reachable: over many epochs element 0 lands everywhere
    seen = {oracle.epoch_permutation(5, 1, e).index(0) for e in range(200)}
    assert seen == {0, 1, 2, 3, 4}


@pytest.mark.parametrize("N,B,shares", [(50000, 256, [151, 105]), (1000, 96, [40, 30, 26]),
                                        (1024, 128, [80, 48]), (77, 10, [4, 3, 2, 1]), (5, 8, [5, 3])])
@pytest.mark.parametrize("drop_last", [False, True])
def test_partition_properties(N, B, shares, drop_last):
    K = len(shares)
    lists = [oracle.sampler_epoch(N, B, shares, 11, 2, r, True, drop_last) for r in range(K)]
    steps = N // B if drop_last else -(-N // B)
    perm = oracle.epoch_permutation(N, 11, 2)
    for r in range(K):
        assert len(lists[r]) == steps * shares[r]        # b_k samples per global step
    # re-assemble every global batch from the per-device slices: it is the epoch ordering
    for s in range(steps):
        batch = []
        for r in range(K):
            batch += lists[r][s * shares[r]:(s + 1) * shares[r]]
        assert batch == [perm[(s * B + i) % N] for i in range(B)]
    if N % B == 0 or drop_last:
        allidx = [i for l in lists for i in l]
        assert len(set(allidx)) == len(allidx) == steps * B  # no sample twice
    if not drop_last and N > 0:
        assert set(i for l in lists for i in l) >= set(range(N)) or steps * B < N


def test_partition_equal_devices_is_plain_split():
    # equal shares, no shuffle: device r gets positions r*B/K .. of every batch
    got = oracle.sampler_epoch(16, 8, [4, 4], 0, 0, 1, shuffle=False)
    assert got == [4, 5, 6, 7, 12, 13, 14, 15]
    got = oracle.sampler_epoch(10, 8, [6, 2], 0, 0, 1, shuffle=False)      # wraps around
    assert got == [6, 7, 4, 5]
    assert oracle.sampler_epoch(10, 8, [6, 2], 0, 0, 1, shuffle=False, drop_last=True) == [6, 7]
