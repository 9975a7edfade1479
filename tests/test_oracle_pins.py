"""Pins of the CPU oracle against things other than itself: brute force on tiny
matrices, hand-written tie cases, closed forms of Sec. 3.1, library fp64
matmul, exact rational sums, the paper's worked index example (Sec. 3.5)."""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2311_14272_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def f32(bits):
    return synth.bf16_bits_to_f32(bits)


# ------------------------------------------------------------------ brute force (joint)
def _masks_joint(S, K, B, n, m, k_row):
    """Every S x K 0/1 mask with <= n ones per aligned m-group and exactly k_row
    whole block columns alive in each block-row (everything else zero)."""
    Sb, Kb = -(-S // B), -(-K // B)
    group_choices = [c for r in range(n + 1) for c in itertools.combinations(range(m), r)]
    ngroups = S * (K // m)
    for blocks in itertools.product(itertools.combinations(range(Kb), k_row), repeat=Sb):
        for pick in itertools.product(group_choices, repeat=ngroups):
            mask = np.zeros((S, K), dtype=np.uint8)
            gi = 0
            for s in range(S):
                for g in range(K // m):
                    for o in pick[gi]:
                        k = g * m + o
                        if (k // B) in blocks[s // B]:
                            mask[s, k] = 1
                    gi += 1
            yield mask


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_brute_force_joint_micro(seed):
    # S=2 rows, K=8, B=4, 2:4 -> 4 groups, 11^4 group picks x 2 block picks.
    S, K, B, n, m, d = 2, 8, 4, 2, 4, 0.5
    rng = np.random.default_rng(100 + seed)
    T = rng.random((S, K)).astype(np.float32) + np.float32(0.01)
    best, best_mask = -1.0, None
    for mask in _masks_joint(S, K, B, n, m, 1):
        v = float((T.astype(np.float64) * mask).sum())
        if v > best:
            best, best_mask = v, mask
    W = synth.f32_to_bf16_bits(np.ones((S, K), dtype=np.float32))
    sel = oracle.select(W, T, n, m, B, d, synth.SAL_GIVEN)
    assert sel.k_row == 1
    got = float((T.astype(np.float64) * sel.mask).sum())
    assert got == pytest.approx(best, rel=1e-12)
    assert (sel.mask == best_mask).all()


def _best_separable(T, B, n, m, k_row):
    """Maximum retained saliency by exhaustive search that only uses the fact
    that the objective is a sum over groups: every <=n subset per group, every
    k_row-subset of block columns per block-row."""
    S, K = T.shape
    Sb, Kb = -(-S // B), -(-K // B)
    T64 = T.astype(np.float64)
    mask = np.zeros((S, K), dtype=np.uint8)
    gbest = np.zeros((S, K), dtype=np.uint8)
    for s in range(S):
        for g0 in range(0, K, m):
            idx = list(range(g0, min(g0 + m, K)))
            bestv, bestc = -1.0, ()
            for r in range(min(n, len(idx)) + 1):
                for c in itertools.combinations(idx, r):
                    v = sum(T64[s, k] for k in c)
                    if v > bestv:
                        bestv, bestc = v, c
            for k in bestc:
                gbest[s, k] = 1
    for bi in range(Sb):
        rows = slice(bi * B, min(S, bi * B + B))
        bestv, bestc = -1.0, None
        for cols in itertools.combinations(range(Kb), k_row):
            v = sum((T64[rows, bj * B:bj * B + B] * gbest[rows, bj * B:bj * B + B]).sum() for bj in cols)
            if v > bestv:
                bestv, bestc = v, cols
        for bj in bestc:
            mask[rows, bj * B:bj * B + B] = gbest[rows, bj * B:bj * B + B]
    return mask


@pytest.mark.parametrize("S,K,B,n,m,d", [(8, 16, 4, 2, 4, 0.5), (8, 16, 4, 1, 4, 0.75), (8, 16, 8, 2, 8, 0.5),
                                          (6, 14, 4, 3, 4, 0.5), (5, 16, 4, 2, 4, 0.25), (8, 24, 8, 4, 8, 0.67)])
def test_brute_force_separable(S, K, B, n, m, d):
    rng = np.random.default_rng(S * 1000 + K * 10 + n)
    T = rng.random((S, K)).astype(np.float32) + np.float32(0.01)
    W = synth.f32_to_bf16_bits(np.ones((S, K), dtype=np.float32))
    sel = oracle.select(W, T, n, m, B, d, synth.SAL_GIVEN)
    expect = _best_separable(T, B, n, m, sel.k_row)
    assert (sel.mask == expect).all()


# ------------------------------------------------------------------ ties, by hand
def test_tie_rules_constant_saliency():
    S, K, B, n, m = 4, 16, 4, 2, 4
    T = np.ones((S, K), dtype=np.float32)
    W = synth.f32_to_bf16_bits(np.ones((S, K), dtype=np.float32))
    sel = oracle.select(W, T, n, m, B, 0.5, synth.SAL_GIVEN)
    # equal saliency: the earlier element of a group wins, the earlier block column wins
    expect_keep = np.tile(np.array([1, 1, 0, 0], dtype=np.uint8), (S, K // 4))
    assert (sel.keep == expect_keep).all()
    assert sel.row_ptr.tolist() == [0, 2] and sel.col_idx.tolist() == [0, 1]
    expect_mask = expect_keep.copy()
    expect_mask[:, 8:] = 0
    assert (sel.mask == expect_mask).all()


def test_tie_rules_partial_ties_and_layer_mode():
    T = np.array([[3, 1, 3, 1, 0, 2, 2, 2]], dtype=np.float32)
    keep = oracle.nm_select(T, 2, 4)
    assert keep.tolist() == [[1, 0, 1, 0, 0, 1, 1, 0]]
    keep1 = oracle.nm_select(T, 1, 4)
    assert keep1.tolist() == [[1, 0, 0, 0, 0, 1, 0, 0]]
    keep8 = oracle.nm_select(T, 3, 8)
    assert keep8.tolist() == [[1, 0, 1, 0, 0, 1, 0, 0]]
    score = np.array([[5.0, 7.0, 7.0, 1.0], [7.0, 0.0, 9.0, 7.0]])
    rp, ci = oracle.block_select(score, 2, 0)
    assert rp.tolist() == [0, 2, 4] and ci.tolist() == [1, 2, 0, 2]
    # whole-grid mode, budget 4: 9, then the 7s in (row, column) order -> (0,1), (0,2), (1,0)
    rp, ci = oracle.block_select(score, 2, 1)
    assert rp.tolist() == [0, 2, 4] and ci.tolist() == [1, 2, 0, 2]
    rp, ci = oracle.block_select(score, 1, 1)   # budget 2: 9 and the first 7 -> (1,2), (0,1)
    assert rp.tolist() == [0, 1, 2] and ci.tolist() == [1, 2]
    score2 = np.array([[9.0, 8.0, 7.0], [1.0, 2.0, 3.0]])
    rp, ci = oracle.block_select(score2, 1, 1)  # budget 2, both in row 0, row 1 empty
    assert rp.tolist() == [0, 2, 2] and ci.tolist() == [0, 1]


def test_short_last_group():
    T = np.array([[1, 2, 3, 4, 9, 8]], dtype=np.float32)      # K = 6, m = 4 -> last group has 2 elements
    assert oracle.nm_select(T, 1, 4).tolist() == [[0, 0, 0, 1, 1, 0]]
    assert oracle.nm_select(T, 2, 4).tolist() == [[0, 0, 1, 1, 1, 1]]
    assert oracle.nm_select(T, 3, 4).tolist() == [[0, 1, 1, 1, 1, 1]]


# ------------------------------------------------------------------ paper's worked value
def test_paper_index_example():
    for line in open(os.path.join(GOLD, "index_example.txt")):
        if line.startswith("#") or not line.strip():
            continue
        m, n, group, expect = line.split()
        m, n, expect = int(m), int(n), int(expect)
        vals = [0.0 if g == "0" else 0.5 for g in group.split(",")]
        B = 4
        W = synth.f32_to_bf16_bits(np.array([vals] + [[0.0] * m] * (B - 1), dtype=np.float32))
        sel = oracle.select(W, None, n, m, B, 1.0, synth.SAL_MAG)
        v, idx, _ = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
        assert v[0, 0, 0] == W[0, vals.index(0.5)]
        assert int(idx[0, 0, 0]) & (m - 1) == expect


def test_k_row_golden():
    for line in open(os.path.join(GOLD, "k_row.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, K, B, d, n, m, kr = line.split()
        assert oracle.k_row(float(d), -(-int(K) // int(B))) == int(kr), name
    assert oracle.k_row(0.01, 10) == 1 and oracle.k_row(1.0, 7) == 7 and oracle.k_row(0.99, 3) == 3


# ------------------------------------------------------------------ invariants on realistic draws
def _pipeline(L, seed=7):
    W, G, X = synth.draw_small(L, seed)
    sel = oracle.select(W, G, L.n, L.m, L.B, L.density, L.sal_kind, L.select_mode)
    return W, G, X, sel


@pytest.mark.parametrize("L", synth.small_cases() + synth.b16_cases(), ids=lambda L: L.name)
def test_mask_invariants(L):
    W, G, X, sel = _pipeline(L)
    S, K, B, n, m = L.S, L.K, L.B, L.n, L.m
    Sb, Kb = -(-S // B), -(-K // B)
    # <= n per aligned group, exactly min(n, len) in the N:M map
    for g0 in range(0, K, m):
        cnt = sel.keep[:, g0:g0 + m].sum(axis=1)
        assert (cnt == min(n, K - g0)).all()
        assert (sel.mask[:, g0:g0 + m].sum(axis=1) <= n).all()
    # block structure
    kept = np.zeros((Sb, Kb), dtype=bool)
    for bi in range(Sb):
        cols = sel.col_idx[sel.row_ptr[bi]:sel.row_ptr[bi + 1]]
        assert (np.diff(cols) > 0).all()
        kept[bi, cols] = True
    if L.select_mode == synth.ROW_UNIFORM:
        assert (np.diff(sel.row_ptr) == sel.k_row).all()
    assert sel.row_ptr[-1] == Sb * sel.k_row
    for bi in range(Sb):
        for bj in range(Kb):
            blk = sel.mask[bi * B:bi * B + B, bj * B:bj * B + B]
            if kept[bi, bj]:
                assert (blk == sel.keep[bi * B:bi * B + B, bj * B:bj * B + B]).all()
            else:
                assert not blk.any()
    # count; closed form of Sec. 3.1 when everything divides
    if S % B == 0 and K % B == 0:
        assert int(sel.mask.sum()) == S * sel.k_row * B * n // m
        sparsity = 1.0 - sel.mask.mean()
        assert sparsity == pytest.approx(1.0 - (sel.k_row * B / K) * (n / m), abs=1e-12)
    # kept blocks beat dropped ones in their row (uniform mode)
    if L.select_mode == synth.ROW_UNIFORM:
        for bi in range(Sb):
            if kept[bi].all():
                continue
            assert sel.score[bi][kept[bi]].min() >= sel.score[bi][~kept[bi]].max()
    else:
        if not kept.all():
            assert sel.score[kept].min() >= sel.score[~kept].max()


def test_saliency_is_one_fp32_product():
    L = synth.small_cases()[0]
    W, G, X = synth.draw_small(L, 3)
    T = oracle.saliency(W, G, synth.SAL_GRAD, L.S, L.K)
    assert (T == np.abs(f32(W) * G)).all() and T.dtype == np.float32
    Tm = oracle.saliency(W, None, synth.SAL_MAG, L.S, L.K)
    assert (Tm == np.abs(f32(W))).all()


def test_magnitude_2_4_matches_argsort():
    rng = np.random.default_rng(5)
    W = synth.f32_to_bf16_bits(rng.standard_normal((32, 64)).astype(np.float32))
    sel = oracle.select(W, None, 2, 4, 32, 1.0, synth.SAL_MAG)
    a = np.abs(f32(W)).reshape(32, 16, 4)
    order = np.argsort(-a, axis=2, kind="stable")       # stable: earlier index wins ties
    expect = np.zeros_like(a, dtype=np.uint8)
    np.put_along_axis(expect, order[:, :, :2], 1, axis=2)
    assert (sel.mask == expect.reshape(32, 64)).all()
    assert (sel.mask == sel.keep).all()                 # density 1: no block dropped


def test_keep_bits_layout():
    keep = np.zeros((2, 70), dtype=np.uint8)
    keep[0, 0] = keep[0, 33] = keep[1, 69] = keep[1, 31] = 1
    bits = oracle.keep_to_bits(keep)
    assert bits.shape == (2, 3)
    assert bits.tolist() == [[1, 2, 0], [1 << 31, 0, 1 << 5]]


# ------------------------------------------------------------------ block score arithmetic
def test_block_score_exact_rational():
    rng = np.random.default_rng(11)
    S, K, B = 16, 24, 8
    T = (rng.random((S, K)) * 10.0 ** rng.integers(-3, 4, (S, K))).astype(np.float32)
    keep = oracle.nm_select(T, 2, 4)
    sc = oracle.block_score(T, keep, B)
    for bi in range(S // B):
        for bj in range(K // B):
            exact = sum(Fraction(float(T[s, k])) for s in range(bi * B, bi * B + B)
                        for k in range(bj * B, bj * B + B) if keep[s, k])
            cnt = int(keep[bi * B:bi * B + B, bj * B:bj * B + B].sum())
            assert abs(Fraction(float(sc[bi, bj])) - exact) <= exact * cnt * Fraction(1, 2 ** 53)


def test_block_score_summation_order_is_fixed():
    # 2^53 + 1 + 1 = 2^53 when added left to right, 2^53 + 2 in any order that adds the ones first.
    B = 4
    big = np.float32(2.0 ** 53)
    T = np.zeros((B, B), dtype=np.float32)
    T[0] = [big, 1, 1, 0]
    keep = np.ones((B, B), dtype=np.uint8)
    assert oracle.block_score(T, keep, B)[0, 0] == 2.0 ** 53            # columns ascending inside a row
    T2 = np.zeros((B, B), dtype=np.float32)
    T2[0] = [1, 1, big, 0]
    assert oracle.block_score(T2, keep, B)[0, 0] == 2.0 ** 53 + 2
    T3 = np.zeros((B, B), dtype=np.float32)                              # rows ascending, row sums first
    T3[0, 0] = big
    T3[1, 0] = 1
    T3[2, 0] = 1
    assert oracle.block_score(T3, keep, B)[0, 0] == 2.0 ** 53
    T4 = np.zeros((B, B), dtype=np.float32)                              # a row is summed before it is added
    T4[0, 0] = big
    T4[1, 0] = 1
    T4[1, 1] = 1
    assert oracle.block_score(T4, keep, B)[0, 0] == 2.0 ** 53 + 2
    keep[0, 0] = 0                                                       # pruned elements do not count
    assert oracle.block_score(T4, keep, B)[0, 0] == 2.0
    # ragged edge: only in-range elements
    T5 = np.ones((5, 6), dtype=np.float32)
    sc = oracle.block_score(T5, np.ones((5, 6), dtype=np.uint8), 4)
    assert sc.tolist() == [[16.0, 8.0], [4.0, 2.0]]


# ------------------------------------------------------------------ pack
@pytest.mark.parametrize("L", synth.small_cases() + synth.b16_cases(), ids=lambda L: L.name)
def test_pack_round_trip_and_sizes(L):
    W, G, X, sel = _pipeline(L, seed=9)
    S, K, B, n, m = L.S, L.K, L.B, L.n, L.m
    vals, idxw, flags = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
    nk = int(sel.row_ptr[-1])
    w = {4: 2, 8: 3}[m]
    assert vals.shape == (nk, B, B * n // m)
    assert idxw.shape == (nk, B, -(-(B * n // m) * w // 32))
    Wd = oracle.unpack(S, K, n, m, B, sel.row_ptr, sel.col_idx, vals, idxw)
    Wm = np.where(sel.mask.astype(bool), W, np.uint16(0))
    # a kept -0.0 keeps its sign bit; both sides are compared as bit patterns
    assert (Wd == Wm).all()
    if S % B == 0 and K % B == 0:
        bits = oracle.metadata_bits(S, K, sel.k_row * B, n, m, B)
        assert bits[2] == vals.size * w                       # S*K'*(n/m)*log2 m  (Sec. 3.1)
        assert bits[2] == S * sel.k_row * B * n / m * w
    # in-group positions ascending inside each group, in range
    slots = B * n // m
    for t in range(min(nk, 3)):
        for r in range(0, B, 7):
            stream = 0
            for x, word in enumerate(idxw[t, r]):
                stream |= int(word) << (32 * x)
            offs = [(stream >> (q * w)) & (m - 1) for q in range(slots)]
            assert stream >> (slots * w) == 0
            for g in range(B // m):
                o = offs[g * n:g * n + n]
                assert all(0 <= x < m for x in o)
    # the 2-of-4 flag against a direct count
    ok = True
    Sb = -(-S // B)
    for bi in range(Sb):
        for bj in sel.col_idx[sel.row_ptr[bi]:sel.row_ptr[bi + 1]]:
            blk = sel.keep[bi * B:bi * B + B, bj * B:min(K, bj * B + B)]
            pad = (-blk.shape[1]) % 4
            blk = np.pad(blk, ((0, 0), (0, pad)))
            if (blk.reshape(blk.shape[0], -1, 4).sum(axis=2) > 2).any():
                ok = False
    assert int(flags[0]) == int(ok)
    if (n, m) in ((1, 4), (2, 4), (1, 8), (2, 8)):
        assert flags[0] == 1
    if (n, m) in ((3, 4), (4, 4)):
        assert flags[0] == 0


def test_pack_hand_written_bits():
    # one 4x4 block, 2:4; row 0 keeps columns 1 and 3 -> positions 1,3 -> bits 0b1101 = 13
    B, n, m = 4, 2, 4
    Wf = np.array([[0, 2, 0, 4], [5, 0, 0, 8], [0, 0, 3, 1], [7, 6, 0, 0]], dtype=np.float32)
    W = synth.f32_to_bf16_bits(Wf)
    sel = oracle.select(W, None, n, m, B, 1.0, synth.SAL_MAG)
    vals, idxw, _ = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
    assert f32(vals[0]).tolist() == [[2, 4], [5, 8], [3, 1], [7, 6]]
    assert idxw[0, :, 0].tolist() == [1 | 3 << 2, 0 | 3 << 2, 2 | 3 << 2, 0 | 1 << 2]
    # m = 8: 3-bit fields, 12 slots per row with B=16, 4:8 -> 36 bits, crosses a word boundary
    rng = np.random.default_rng(2)
    W8 = synth.f32_to_bf16_bits(rng.standard_normal((16, 16)).astype(np.float32))
    s8 = oracle.select(W8, None, 4, 8, 16, 1.0, synth.SAL_MAG)
    v8, i8, _ = oracle.pack(W8, s8.keep, 4, 8, 16, s8.row_ptr, s8.col_idx)
    assert i8.shape == (1, 16, 1)  # 8 slots * 3 bits = 24 bits -> one word
    r = 5
    pos = [k % 8 for k in range(16) if s8.keep[r, k]]
    expect = 0
    for q, p in enumerate(pos):
        expect |= p << (3 * q)
    assert int(i8[0, r, 0]) == expect


def test_two_of_four_flag_counts_aligned_quads():
    # 4:8 is eligible for the 2-of-4 hardware form exactly when no aligned quad of columns holds more
    # than two kept values; the count runs over quads, not over the whole group of eight.
    B, n, m = 8, 4, 8
    big, small = 2.0, 0.5
    even = np.tile(np.array([big, small, small, big, small, big, big, small], dtype=np.float32), (8, 1))
    W = synth.f32_to_bf16_bits(even)                              # two large values in either quad
    sel = oracle.select(W, None, n, m, B, 1.0, synth.SAL_MAG)
    assert sel.keep[0].tolist() == [1, 0, 0, 1, 0, 1, 1, 0]
    assert int(oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)[2][0]) == 1
    skew = even.copy()
    skew[5] = [big, big, big, small, small, small, small, big]  # one row with three in its first quad
    W = synth.f32_to_bf16_bits(skew)
    sel = oracle.select(W, None, n, m, B, 1.0, synth.SAL_MAG)
    assert sel.keep[5].tolist() == [1, 1, 1, 0, 0, 0, 0, 1]
    assert int(oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)[2][0]) == 0


def test_pack_padding_rules():
    # S=3 < B=4 and K=6: block column 1 has columns 4,5 only (short group), row 3 is outside.
    B, n, m = 4, 2, 4
    Wf = np.arange(1, 19, dtype=np.float32).reshape(3, 6)
    W = synth.f32_to_bf16_bits(Wf)
    sel = oracle.select(W, None, n, m, B, 1.0, synth.SAL_MAG)
    vals, idxw, _ = oracle.pack(W, sel.keep, n, m, B, sel.row_ptr, sel.col_idx)
    assert f32(vals[0][:3]).tolist() == [[3, 4], [9, 10], [15, 16]]
    assert idxw[0, :3, 0].tolist() == [2 | 3 << 2] * 3
    assert f32(vals[1][:3]).tolist() == [[5, 6], [11, 12], [17, 18]]
    assert idxw[1, :3, 0].tolist() == [0 | 1 << 2] * 3
    # out-of-range row: zeros with positions 0..n-1
    assert vals[0][3].tolist() == [0, 0] and idxw[0, 3, 0] == (0 | 1 << 2)
    # 1:4 with a 1-element last group (K=5): kept element first, no pads needed; K=5, 2:4: one real + one pad (0, pos 0)
    W5 = synth.f32_to_bf16_bits(np.array([[1, 2, 3, 4, 5]] * 4, dtype=np.float32))
    s5 = oracle.select(W5, None, 2, 4, 4, 1.0, synth.SAL_MAG)
    v5, i5, _ = oracle.pack(W5, s5.keep, 2, 4, 4, s5.row_ptr, s5.col_idx)
    assert f32(v5[1][0]).tolist() == [5, 0] and i5[1, 0, 0] == 0


# ------------------------------------------------------------------ products
@pytest.mark.parametrize("L", synth.small_cases(), ids=lambda L: L.name)
def test_packed_product_equals_dense_masked(L):
    W, G, X, sel = _pipeline(L, seed=4)
    vals, idxw, _ = oracle.pack(W, sel.keep, L.n, L.m, L.B, sel.row_ptr, sel.col_idx)
    nc = min(L.Ncol, 48)
    Y, A = oracle.gemm_masked(W, sel.mask, X, 3, nc)
    Yp = oracle.spmm_packed(L.S, L.K, L.n, L.m, L.B, sel.row_ptr, sel.col_idx, vals, idxw, X, 3, nc)
    assert (Y == Yp).all()
    # library fp64 matmul of the masked weight
    Wm = f32(W).astype(np.float64) * sel.mask
    Xd = f32(X).astype(np.float64)[:, 3:3 + nc]
    ref = Wm @ Xd
    assert np.abs(Y - ref).max() <= 1e-12 * max(1.0, np.abs(ref).max())
    assert np.abs(A - np.abs(Wm) @ np.abs(Xd)).max() <= 1e-12 * max(1.0, np.abs(A).max())


def test_no_pruning_reduces_to_plain_matmul():
    rng = np.random.default_rng(8)
    S, K, N = 64, 96, 40
    W = synth.f32_to_bf16_bits(rng.standard_normal((S, K)).astype(np.float32))
    X = synth.f32_to_bf16_bits(rng.standard_normal((K, N)).astype(np.float32))
    sel = oracle.select(W, None, 4, 4, 32, 1.0, synth.SAL_MAG)
    assert sel.mask.all()
    Y, _ = oracle.gemm_masked(W, sel.mask, X)
    ref = f32(W).astype(np.float64) @ f32(X).astype(np.float64)
    assert np.abs(Y - ref).max() <= 1e-12 * np.abs(ref).max()
    # a transposed operand or a dropped term would not survive this
    assert np.abs(Y - ref).max() < 1e-9 and np.abs(ref).max() > 1.0


def test_block_only_pruning_is_blocked_ell_product():
    rng = np.random.default_rng(9)
    S, K, N, B = 64, 128, 24, 32
    W = synth.f32_to_bf16_bits(rng.standard_normal((S, K)).astype(np.float32))
    X = synth.f32_to_bf16_bits(rng.standard_normal((K, N)).astype(np.float32))
    sel = oracle.select(W, None, 4, 4, B, 0.5, synth.SAL_MAG)
    Wf, Xf = f32(W).astype(np.float64), f32(X).astype(np.float64)
    ref = np.zeros((S, N))
    for bi in range(S // B):
        sums = np.abs(Wf[bi * B:(bi + 1) * B]).reshape(B, K // B, B).sum(axis=(0, 2))
        cols = np.sort(np.argsort(-sums, kind="stable")[:2])
        assert cols.tolist() == sel.col_idx[sel.row_ptr[bi]:sel.row_ptr[bi + 1]].tolist()
        for bj in cols:
            ref[bi * B:(bi + 1) * B] += Wf[bi * B:(bi + 1) * B, bj * B:(bj + 1) * B] @ Xf[bj * B:(bj + 1) * B]
    Y, _ = oracle.gemm_masked(W, sel.mask, X)
    assert np.abs(Y - ref).max() <= 1e-11 * np.abs(ref).max()


# ------------------------------------------------------------------ conv lowering
@pytest.mark.parametrize("C,H,Wd,batch,kh,kw,stride,pad", [(3, 9, 8, 2, 3, 3, 1, 1), (4, 8, 8, 1, 1, 1, 2, 0),
                                                           (2, 11, 11, 2, 7, 7, 2, 3), (5, 6, 7, 3, 1, 1, 1, 0),
                                                           (3, 7, 7, 1, 3, 3, 2, 1)])
def test_im2col_matches_direct_convolution(C, H, Wd, batch, kh, kw, stride, pad):
    rng = np.random.default_rng(C * 100 + H)
    act = synth.f32_to_bf16_bits(rng.standard_normal((C, batch, H, Wd)).astype(np.float32))
    X = oracle.im2col(act, kh, kw, stride, pad)
    Ho, Wo = (H + 2 * pad - kh) // stride + 1, (Wd + 2 * pad - kw) // stride + 1
    assert X.shape == (kh * kw * C, batch * Ho * Wo)
    # window view of the zero-padded input (independent construction)
    a = np.pad(f32(act), ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    win = np.lib.stride_tricks.sliding_window_view(a, (kh, kw), axis=(2, 3))[:, :, ::stride, ::stride]
    # win[c, b, oh, ow, kh, kw] -> rows (kh, kw, c), columns (b, oh, ow)
    expect = win.transpose(4, 5, 0, 1, 2, 3).reshape(kh * kw * C, batch * Ho * Wo)
    assert (f32(X) == expect).all()
    # conv as a product equals the direct correlation sum
    S = 4
    Wt = rng.standard_normal((S, kh, kw, C))
    direct = np.zeros((S, batch, Ho, Wo))
    for x in range(kh):
        for y in range(kw):
            patch = a[:, :, x:x + stride * (Ho - 1) + 1:stride, y:y + stride * (Wo - 1) + 1:stride].astype(np.float64)
            direct += np.einsum("sc,cnhw->snhw", Wt[:, x, y, :], patch)
    viaX = Wt.reshape(S, -1) @ f32(X).astype(np.float64)
    assert np.abs(viaX - direct.reshape(S, -1)).max() < 1e-9
    if kh == 1 and kw == 1 and stride == 1:
        assert (X == act.reshape(C, -1)).all()          # identity for pointwise convs in this layout


def test_metadata_closed_forms():
    # Sec. 3.1 with S=256, K=1024, K'=320 (5 of 16 block columns of 64), 1:4
    # worked by hand: 256*320/(64*64) = 20 kept blocks; floor(log2(320/64)) = floor(log2 5) = 2 bits each -> 40;
    # with ceil(log2(1024/64)) = 4 bits each (every block column addressable) -> 80;
    # 256*320/4 = 20480 kept values, log2(4) = 2 bits each -> 40960
    bits = oracle.metadata_bits(256, 1024, 320, 1, 4, 64)
    assert bits[0] == 40 and bits[1] == 80 and bits[2] == 40960
    # 2:8 in 32x32 blocks, S=64, K=256, K'=128: 8 kept blocks x floor(log2 4) = 2 -> 16; x ceil(log2 8) = 3 -> 24;
    # 64*128*2/8 = 2048 kept values x 3 bits -> 6144
    bits = oracle.metadata_bits(64, 256, 128, 2, 8, 32)
    assert bits[0] == 16 and bits[1] == 24 and bits[2] == 6144


def test_config_shapes():
    for cid in (1, 2, 3, 4):
        wl = synth.config(cid)
        for L in wl.layers:
            assert L.K % L.m == 0
    wl = synth.config(5, batch=2)
    assert len(wl.layers) == 53
    macs = sum(L.S * L.K * (L.Ncol // 2) for L in wl.layers)
    assert abs(macs / 1e9 - 4.087) < 0.01                # ResNet-50 convs, GMAC per image
    assert {(L.n, L.m) for L in wl.layers} <= set(synth.NM_CHOICES)
    assert all(0.2 <= L.density <= 0.8 for L in wl.layers)


def test_epilogue_closed_forms():
    """oracle.epilogue against values worked out by hand: order of the steps (scale before bias
    before residual before ReLU), per-row broadcasting, the scaled error bound."""
    Y = np.array([[1.0, -2.0, 3.0], [-4.0, 5.0, -6.0]])
    A = np.array([[1.0, 2.0, 3.0], [4.0, 5.0, 6.0]])
    scale = np.array([2.0, -0.5], dtype=np.float32)
    bias = np.array([1.0, -1.0], dtype=np.float32)
    res = np.array([[0.0, 10.0, -10.0], [1.0, 1.0, 1.0]])
    out, a = oracle.epilogue(Y, A, scale, bias, res, relu=False)
    assert (out == np.array([[3.0, 7.0, -3.0], [2.0, -2.5, 3.0]])).all()
    assert (a == np.array([[2.0, 4.0, 6.0], [2.0, 2.5, 3.0]])).all()
    out, _ = oracle.epilogue(Y, A, scale, bias, res, relu=True)
    assert (out == np.array([[3.0, 7.0, 0.0], [2.0, 0.0, 3.0]])).all()
    out, a = oracle.epilogue(Y, A)
    assert (out == Y).all() and (a == A).all() and out is not Y
    out, _ = oracle.epilogue(Y, None, relu=True)
    assert (out == np.maximum(Y, 0)).all()
    out, _ = oracle.epilogue(Y, None, bias=bias)
    assert (out == Y + np.array([[1.0], [-1.0]])).all()


def test_maxpool_hand_example():
    """3x3 / stride 2 / pad 1 max-pool of a 4x4 image, worked out by hand (windows clipped at the border)."""
    img = np.array([[1, 2, 3, 4], [5, 6, 7, 8], [-1, -2, -3, -4], [9, 0, 0, -9]], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(img).reshape(1, 1, 4, 4)
    out = synth.bf16_bits_to_f32(oracle.maxpool(bits, 3, 3, 2, 1)).reshape(2, 2)
    # windows: rows {0,1} x cols {0,1}; rows {0,1} x cols {1,2,3}; rows {1,2,3} x cols {0,1}; rows {1,2,3} x cols {1,2,3}
    assert (out == np.array([[6, 8], [9, 8]], dtype=np.float32)).all()
    # 2x2 / stride 2 without padding on an all-negative image: padding must not contribute zeros
    neg = synth.f32_to_bf16_bits(-np.arange(1, 17, dtype=np.float32).reshape(4, 4)).reshape(1, 1, 4, 4)
    out = synth.bf16_bits_to_f32(oracle.maxpool(neg, 2, 2, 2, 0)).reshape(2, 2)
    assert (out == np.array([[-1, -3], [-9, -11]], dtype=np.float32)).all()
    out = synth.bf16_bits_to_f32(oracle.maxpool(neg, 3, 3, 2, 1)).reshape(2, 2)
    assert (out == np.array([[-1, -2], [-5, -6]], dtype=np.float32)).all()
