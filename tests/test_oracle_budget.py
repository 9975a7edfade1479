"""Pins of the oracle's global block budget (Alg. 1 lines 6-9): hand-worked examples, ties,
agreement with a library sort on tie-free data, monotonicity and minimality of the cut."""
import numpy as np
import pytest

import oracle


def test_hand_worked_two_layers():
    # layer 0: 2 block-rows x 3 blocks, B=4, S=8, K=12, 2:4 ; layer 1: 1 x 2, B=4, S=4, K=8, 2:4
    s0 = np.array([[5.0, 1.0, 3.0], [2.0, 6.0, 4.0]])     # sorted rows: [1,3,5], [2,4,6] -> c0 = [3, 7, 11]
    s1 = np.array([[10.0, 4.0]])                           # sorted: [4, 10]            -> c1 = [4, 10]
    layers = [(8, 12, 2, 4, 4), (4, 8, 2, 4, 4)]
    total = 8 * 12 + 4 * 8                                  # 128 weights, 64 kept after 2:4
    # order: 3 (L0 r0), 4 (L1 r0), 7 (L0 r1), 10 (L1 r1, last of its layer: never), 11 (L0 r2, last)
    # each L0 rank column holds 2 rows x 4 x 4 x 1/2 = 16 kept weights, each L1 column 8
    assert oracle.global_budget(layers, [s0, s1], 0.5) == ([3, 2], 0.5)
    k, ach = oracle.global_budget(layers, [s0, s1], 0.6)            # 64 -> 48 kept: 0.625
    assert k == [2, 2] and ach == 1 - 48 / total
    k, ach = oracle.global_budget(layers, [s0, s1], 0.65)           # -> 40 kept: 0.6875
    assert k == [2, 1] and ach == 1 - 40 / total
    k, ach = oracle.global_budget(layers, [s0, s1], 0.7)            # -> 24 kept: 0.8125
    assert k == [1, 1] and ach == 1 - 24 / total
    k, ach = oracle.global_budget(layers, [s0, s1], 0.99)           # nothing left to prune
    assert k == [1, 1] and ach == 1 - 24 / total


def test_ties_go_by_layer_then_rank():
    s = [np.ones((2, 3)), np.ones((2, 3))]
    layers = [(8, 12, 4, 4, 4), (8, 12, 4, 4, 4)]                   # no N:M part, 96 weights each
    # every rank column sums to 2; order: L0r0, L0r1, (L0r2 is L0's last), L1r0, L1r1
    # (targets sit between the reachable sparsities 1/6, 2/6, 3/6, 4/6)
    assert oracle.global_budget(layers, s, 0.10)[0] == [2, 3]
    assert oracle.global_budget(layers, s, 0.25)[0] == [1, 3]
    assert oracle.global_budget(layers, s, 0.40)[0] == [1, 2]
    assert oracle.global_budget(layers, s, 0.60)[0] == [1, 1]


def test_row_order_is_reverse_of_keep_order():
    # ties inside a row: the block that block_select keeps first (smaller column) is pruned last
    sc = np.array([[2.0, 2.0, 1.0]])
    layers = [(4, 12, 4, 4, 4)]
    k, _ = oracle.global_budget(layers, [sc], 0.6)                  # prune 2 of 3 rank columns
    assert k == [1]
    rp, ci = oracle.block_select(sc, 1, 0)
    assert ci.tolist() == [0]
    k, _ = oracle.global_budget(layers, [sc], 0.3)
    rp, ci = oracle.block_select(sc, k[0], 0)
    assert k == [2] and ci.tolist() == [0, 1]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_against_library_sort_and_minimality(seed):
    rng = np.random.default_rng(seed)
    layers, scores = [], []
    for _ in range(5):
        B = int(rng.choice([16, 32, 64]))
        Sb, Kb = int(rng.integers(1, 5)), int(rng.integers(2, 9))
        n, m = [(1, 4), (2, 4), (2, 8), (4, 8)][int(rng.integers(0, 4))]
        layers.append((Sb * B, Kb * B, n, m, B))
        scores.append(rng.random((Sb, Kb)) * rng.uniform(0.5, 3.0))
    total = sum(S * K for S, K, *_ in layers)
    cols = []
    for l, ((S, K, n, m, B), sc) in enumerate(zip(layers, scores)):
        c = np.sort(sc, axis=1).sum(axis=0)                         # tie-free: library sort is the definition
        assert (np.diff(c) >= 0).all()                              # a layer loses a prefix of its ranks
        cols += [(c[o], l, o, S * B * n / m) for o in range(len(c))]
    cols.sort()
    prev = None
    for target in np.linspace(0.0, 0.98, 25):
        k, ach = oracle.global_budget(layers, scores, float(target))
        kept = sum(S * K * n / m for S, K, n, m, B in layers)
        kk = [sc.shape[1] for sc in scores]
        for c, l, o, wgt in cols:
            if 1 - kept / total >= target:
                break
            if kk[l] <= 1:
                continue
            kept -= wgt
            kk[l] -= 1
        assert k == kk and ach == pytest.approx(1 - kept / total, abs=1e-12)
        assert ach >= target - 1e-12 or all(x == 1 for x in k)
        if prev is not None:
            assert all(a <= b for a, b in zip(k, prev))             # more sparsity never keeps more
        prev = k
