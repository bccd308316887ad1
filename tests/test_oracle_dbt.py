"""Pins for the oracle's double-binary-tree cost model (Section 4.1, equation C_dbt): hand-worked trees, the
closed form on a constant matrix (tree height), brute force over explicitly built parent arrays, symmetry."""
import math

import numpy as np
import pytest

import oracle
from gen import random_matrix, random_perms


def inorder_parents(n):
    """Parent of every position of the in-order binary tree on 0..n-1 whose subtree roots are range middles,
    built iteratively with an explicit stack (independent of the oracle's recursion)."""
    parent = [-1] * n
    stack = [(0, n - 1, -1)]
    while stack:
        lo, hi, par = stack.pop()
        if lo > hi:
            continue
        m = (lo + hi) // 2
        parent[m] = par
        stack.append((lo, m - 1, m))
        stack.append((m + 1, hi, m))
    return parent


def brute_tree_cost(c, perm, shift):
    n = len(perm)
    parent = inorder_parents(n)
    worst = 0
    for p in range(n):
        total, q = 0, p
        while parent[q] >= 0:
            total += int(c[perm[(parent[q] + shift) % n], perm[(q + shift) % n]])
            q = parent[q]
        worst = max(worst, total)
    return worst


def test_hand_worked_trees():
    # N = 3: root is rank 1 with children ranks 0 and 2
    c = np.array([[0, 5, 9], [2, 0, 7], [4, 6, 0]], dtype=np.int32)
    ident = np.arange(3)
    assert oracle.dbt_tree_cost(c, ident, 0) == max(c[1, 0], c[1, 2]) == 7
    # second tree: position p holds rank p+1: root is rank 2, children ranks 1 and 0
    assert oracle.dbt_tree_cost(c, ident, 1) == max(c[2, 1], c[2, 0]) == 6
    assert oracle.dbt_cost(c, ident) == 7
    # N = 2: range 0..1, root rank 0, right child rank 1
    c2 = np.array([[0, 3], [8, 0]], dtype=np.int32)
    assert oracle.dbt_tree_cost(c2, np.arange(2), 0) == 3 and oracle.dbt_tree_cost(c2, np.arange(2), 1) == 8
    # N = 7, perfect tree: root 3; children 1 and 5; leaves 0, 2, 4, 6.  One expensive path 3 -> 5 -> 4.
    c7 = np.ones((7, 7), dtype=np.int32)
    np.fill_diagonal(c7, 0)
    c7[3, 5] = 40
    c7[5, 4] = 30
    c7[5, 3] = 999       # child -> parent direction is not used
    c7[3, 4] = 999       # not a tree edge
    assert oracle.dbt_tree_cost(c7, np.arange(7), 0) == 70
    perm = np.array([6, 5, 4, 3, 2, 1, 0])               # reversed order: rank 3 still the root, node ids mirrored
    assert oracle.dbt_tree_cost(c7, perm, 0) == max(c7[3, 5] + max(c7[5, 6], c7[5, 4]), c7[3, 1] + 1) == 70


@pytest.mark.parametrize("n", [2, 3, 4, 5, 7, 8, 15, 16, 17, 63, 64, 100, 1000, 1024])
def test_constant_matrix_gives_tree_height(n):
    k = 11
    c = np.full((n, n), k, dtype=np.int32)
    np.fill_diagonal(c, 0)
    height = math.ceil(math.log2(n + 1)) - 1             # in-order tree with middle roots is height-balanced
    for perm in random_perms(n, 2, seed=n):
        assert oracle.dbt_tree_cost(c, perm, 0) == k * height == oracle.dbt_tree_cost(c, perm, 1)


@pytest.mark.parametrize("n", [2, 3, 4, 6, 7, 8, 13, 31, 32, 64, 200])
def test_against_explicit_paths(n):
    c = random_matrix(n, 30 + n, symmetric=False, lo=0, hi=5000)
    for perm in random_perms(n, 4, seed=n):
        t0, t1 = brute_tree_cost(c, perm, 0), brute_tree_cost(c, perm, 1)
        assert oracle.dbt_tree_cost(c, perm, 0) == t0
        assert oracle.dbt_tree_cost(c, perm, 1) == t1
        assert oracle.dbt_cost(c, perm) == max(t0, t1)


def test_second_tree_is_the_first_on_the_rotated_order():
    n = 20
    c = random_matrix(n, 8, symmetric=False)
    for perm in random_perms(n, 4, seed=3):
        assert oracle.dbt_tree_cost(c, perm, 1) == oracle.dbt_tree_cost(c, np.roll(perm, -1), 0)


@pytest.mark.parametrize("n", [7, 15, 63])
def test_mirror_symmetry_of_perfect_trees(n):
    """N = 2^k - 1: the tree is its own mirror image, so reversing the order keeps the first tree's cost."""
    c = random_matrix(n, n, symmetric=False)
    for perm in random_perms(n, 3, seed=n):
        assert oracle.dbt_tree_cost(c, perm, 0) == oracle.dbt_tree_cost(c, perm[::-1].copy(), 0)


def test_batch_matches_single_calls():
    n = 24
    c = random_matrix(n, 4, symmetric=True)
    perms = random_perms(n, 9, seed=2)
    assert np.array_equal(oracle.dbt_cost_batch(c, perms), [oracle.dbt_cost(c, p) for p in perms])
