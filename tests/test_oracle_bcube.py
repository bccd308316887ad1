"""Pins for the oracle's BCube cost model (Section 4.1, equation C_b): reduction to the halving-doubling
model at B = 2, closed forms, digit-wise automorphisms, a hand-worked example."""
import math

import numpy as np
import pytest

import oracle
from gen import clean_hierarchy, random_matrix, random_perms


@pytest.mark.parametrize("n", [2, 4, 8, 64, 1024])
def test_base_2_is_halving_doubling(n):
    c = random_matrix(n, 10 + n, symmetric=False)
    perms = random_perms(n, 6, seed=n)
    assert np.array_equal(oracle.bcube_cost_batch(c, 2, perms), oracle.rd_cost_batch(c, perms))


@pytest.mark.parametrize("n,base", [(4, 4), (16, 4), (64, 4), (256, 4), (1024, 4), (9, 3), (27, 3), (64, 8), (25, 5)])
def test_constant_matrix(n, base):
    k = 13
    c = np.full((n, n), k, dtype=np.int32)
    np.fill_diagonal(c, 0)
    rounds = round(math.log(n, base))
    assert oracle.bcube_cost(c, base, random_perms(n, 1, seed=n)[0]) == k * rounds


def test_hand_worked_n4_b4_and_n16_b4():
    # N = 4, B = 4: one round, every rank talks to every other rank: the cost is the largest off-diagonal entry
    c = np.array([[0, 1, 2, 3], [4, 0, 5, 6], [7, 8, 0, 9], [10, 11, 12, 0]], dtype=np.int32)
    for perm in random_perms(4, 5, seed=1):
        assert oracle.bcube_cost(c, 4, perm) == 12
    # N = 16, B = 4, identity order: round 0 pairs ranks inside {0..3}, {4..7}, ...; round 1 pairs ranks that are
    # equal mod 4.  One large entry inside a round-0 group and one across groups with equal low digit.
    c = np.ones((16, 16), dtype=np.int32)
    np.fill_diagonal(c, 0)
    c[5, 7] = 50        # ranks 5 and 7: same group of four -> round 0
    c[2, 14] = 70       # ranks 2 and 14: both = 2 mod 4 -> round 1
    c[1, 6] = 1000      # ranks 1 and 6 differ in both digits: never exchange
    assert oracle.bcube_cost(c, 4, np.arange(16)) == 50 + 70


@pytest.mark.parametrize("n,base,group", [(16, 4, 4), (64, 4, 4), (64, 4, 16), (64, 8, 8), (27, 3, 9)])
def test_clean_hierarchy_closed_form(n, base, group):
    """Rack-contiguous order, rack size a power of the base: rounds inside a rack cost `intra`, the others `cross`."""
    a, b = 20, 900
    c = clean_hierarchy(n, group, a, b)
    rounds = round(math.log(n, base))
    inner = round(math.log(group, base))
    assert oracle.bcube_cost(c, base, np.arange(n)) == a * inner + b * (rounds - inner)


@pytest.mark.parametrize("n,base", [(16, 4), (64, 4), (27, 3)])
def test_digit_automorphisms(n, base):
    """Adding a constant to one digit (mod B) in every rank id, or permuting the digit positions, maps every
    round's set of exchanges onto a round's set of exchanges."""
    rounds = round(math.log(n, base))
    c = random_matrix(n, 5 + n, symmetric=False)
    rng = np.random.default_rng(n)
    ids = np.arange(n)
    digits = np.stack([(ids // base**i) % base for i in range(rounds)], axis=1)
    for perm in random_perms(n, 3, seed=n):
        want = oracle.bcube_cost(c, base, perm)
        for _ in range(3):
            d2 = digits.copy()
            pos = int(rng.integers(0, rounds))
            d2[:, pos] = (d2[:, pos] + int(rng.integers(1, base))) % base
            new_id = (d2 * base ** np.arange(rounds)).sum(axis=1)
            q = np.empty_like(perm)
            q[new_id] = perm
            assert oracle.bcube_cost(c, base, q) == want
            sigma = rng.permutation(rounds)
            new_id = (digits[:, sigma] * base ** np.arange(rounds)).sum(axis=1)
            q = np.empty_like(perm)
            q[new_id] = perm
            assert oracle.bcube_cost(c, base, q) == want


def test_rejects_n_not_a_power_of_base():
    c = random_matrix(8, 1, symmetric=True)
    with pytest.raises(RuntimeError):
        oracle.bcube_cost_batch(c, 4, random_perms(8, 2, seed=1))


# ------------------------------------------------------------------------------------- size-weighted rounds
@pytest.mark.parametrize("n,base", [(64, 2), (64, 4), (27, 3), (1024, 2), (256, 4)])
def test_unit_weights_are_the_unweighted_model(n, base):
    c = random_matrix(n, 3 + n, symmetric=False)
    perms = random_perms(n, 4, seed=n)
    rounds = round(math.log(n, base))
    assert np.array_equal(oracle.bcube_cost_weighted_batch(c, base, np.ones(rounds), perms),
                          oracle.bcube_cost_batch(c, base, perms))
    if base == 2:
        assert np.array_equal(oracle.bcube_cost_weighted_batch(c, 2, np.ones(rounds), perms), oracle.rd_cost_batch(c, perms))


@pytest.mark.parametrize("n,base", [(16, 2), (64, 2), (64, 4), (81, 3)])
def test_single_round_weight_isolates_that_round(n, base):
    """weight = e_k leaves round k alone: the largest entry over ranks j and their peers in digit k, written
    out with numpy index arithmetic."""
    c = random_matrix(n, 9 + n, symmetric=False)
    rounds = round(math.log(n, base))
    ids = np.arange(n)
    for perm in random_perms(n, 2, seed=n):
        total = 0
        for k in range(rounds):
            stride = base ** k
            digit = (ids // stride) % base
            worst = 0
            for step in range(1, base):
                peer = ids + (((digit + step) % base) - digit) * stride
                worst = max(worst, int(c[perm[ids], perm[peer]].max()))
            w = np.zeros(rounds, dtype=np.int32)
            w[k] = 5
            assert oracle.bcube_cost_weighted_batch(c, base, w, perm[None])[0] == 5 * worst
            total += worst
        assert oracle.bcube_cost_batch(c, base, perm[None])[0] == total


def test_weights_are_linear_and_halving_sizes_closed_form():
    n = 64
    c = random_matrix(n, 2, symmetric=True)
    perms = random_perms(n, 5, seed=9)
    rng = np.random.default_rng(4)
    w1, w2 = rng.integers(0, 1000, size=6), rng.integers(0, 1000, size=6)
    assert np.array_equal(oracle.bcube_cost_weighted_batch(c, 2, w1 + w2, perms),
                          oracle.bcube_cost_weighted_batch(c, 2, w1, perms) + oracle.bcube_cost_weighted_batch(c, 2, w2, perms))
    # halving-doubling on a constant per-byte cost k with S = 2^20 bytes: sum_i k * S / 2^(i+1) = k * S * (1 - 1/N)
    k, S = 3, 1 << 20
    const = np.full((n, n), k, dtype=np.int32)
    np.fill_diagonal(const, 0)
    w = np.array([S >> (i + 1) for i in range(6)])
    assert oracle.bcube_cost_weighted_batch(const, 2, w, perms[:1])[0] == k * S * (n - 1) // n
