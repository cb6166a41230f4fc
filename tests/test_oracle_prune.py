"""Pins for the oracle's pruning and packing (CPU only).

Each test checks oracle.prune / oracle.pack against something that is not the
oracle itself: exhaustive subset search, structural invariants the paper fixes
(section 3.1: every column of a tile is kept or pruned as a unit; N of every M),
special cases that reduce to a library routine (T = 1 is conventional row-wise
N:M, section 4.5 configuration 1), and a hand-worked example.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


def _as_ohwi(W, kh=1, kw=1):
    cout, K = W.shape
    return np.ascontiguousarray(W.reshape(cout, kh, kw, K // (kh * kw)), dtype=np.float32)


def _exact_scores(W, r0, r1, cols):
    # weights in these tests are multiples of 1/8 with small magnitude, so every
    # partial sum is exact in binary floating point whatever the order
    return [float(np.abs(W[r0:r1, c].astype(np.float64)).sum()) for c in cols]


def _brute_force_mask(W, n, m, tile):
    cout, K = W.shape
    mask = np.zeros((cout, K), dtype=np.uint8)
    for r0 in range(0, cout, tile):
        r1 = min(r0 + tile, cout)
        for g in range(K // m):
            cols = list(range(g * m, g * m + m))
            sc = _exact_scores(W, r0, r1, cols)
            best_val, best_set = None, None
            # combinations() yields index tuples in lexicographic order, so the
            # first maximiser found is the lexicographically smallest one
            for sub in itertools.combinations(range(m), n):
                v = sum(sc[i] for i in sub)
                if best_val is None or v > best_val:
                    best_val, best_set = v, sub
            for i in best_set:
                mask[r0:r1, g * m + i] = 1
    return mask


@pytest.mark.parametrize("cout,K,n,m,tile", [
    (8, 16, 2, 4, 4), (6, 16, 1, 4, 4), (7, 24, 3, 8, 3), (5, 12, 2, 6, 2),
    (4, 8, 4, 8, 1), (9, 16, 2, 8, 16), (3, 20, 3, 5, 2), (16, 8, 1, 2, 8),
])
def test_selection_is_the_best_subset_brute_force(cout, K, n, m, tile):
    rng = np.random.default_rng(cout * 1000 + K + n)
    # small integer multiples of 1/8: many exact ties, all sums exact
    W = rng.integers(-6, 7, size=(cout, K)).astype(np.float32) / 8.0
    mask, idx, wz = oracle.prune(_as_ohwi(W), n, m, tile)
    ref = _brute_force_mask(W, n, m, tile)
    assert np.array_equal(mask, ref)
    assert np.array_equal(wz.reshape(cout, K), W * ref)


@pytest.mark.parametrize("cout,kh,kw,cin,n,m,tile", [
    (64, 3, 3, 64, 2, 4, 16), (40, 1, 1, 32, 1, 4, 16), (24, 3, 3, 16, 2, 8, 8),
    (33, 3, 1, 8, 4, 8, 32), (10, 1, 1, 64, 1, 8, 3),
])
def test_structural_invariants(cout, kh, kw, cin, n, m, tile):
    rng = np.random.default_rng(7)
    w = rng.standard_normal((cout, kh, kw, cin)).astype(np.float32) * 0.05
    K = kh * kw * cin
    G = K // m
    n_tiles = -(-cout // tile)
    mask, idx, wz = oracle.prune(w, n, m, tile)
    assert mask.shape == (cout, K) and idx.shape == (n_tiles, G, n)
    # exactly N kept in every group of every row
    assert np.all(mask.reshape(cout, G, m).sum(axis=2) == n)
    # one kept set for all rows of a tile
    for j in range(n_tiles):
        rows = mask[j * tile:(j + 1) * tile]
        assert np.all(rows == rows[0])
        # idx lists exactly that set, ascending, inside its group
        kept = np.flatnonzero(rows[0])
        assert np.array_equal(idx[j].reshape(-1), kept)
        for g in range(G):
            assert np.all(idx[j, g] >= g * m) and np.all(idx[j, g] < g * m + m)
            assert np.all(np.diff(idx[j, g]) > 0)
    # closed form for the number of kept weights
    assert int(mask.sum()) == cout * G * n
    # zero filled weights: kept entries untouched bit for bit, others +0
    W = w.reshape(cout, K)
    assert np.array_equal(wz.reshape(cout, K)[mask == 1], W[mask == 1])
    assert np.all(wz.reshape(cout, K)[mask == 0] == 0)
    assert not np.any(np.signbit(wz.reshape(cout, K)[mask == 0]))


def test_tile_one_is_rowwise_magnitude_topn():
    """T = 1 is conventional row-wise N:M (section 4.5, configuration 1):
    per row, per group, the N largest |w|; numpy's stable argsort gives the
    lower index among equals."""
    rng = np.random.default_rng(11)
    cout, K, n, m = 12, 32, 2, 4
    W = (rng.integers(-9, 10, size=(cout, K)) / 16.0).astype(np.float32)
    mask, idx, _ = oracle.prune(_as_ohwi(W), n, m, 1)
    ref = np.zeros_like(mask)
    for r in range(cout):
        for g in range(K // m):
            a = np.abs(W[r, g * m:(g + 1) * m]).astype(np.float64)
            order = np.argsort(-a, kind="stable")[:n]
            ref[r, g * m + order] = 1
    assert np.array_equal(mask, ref)


def test_n_equals_m_keeps_everything():
    rng = np.random.default_rng(3)
    w = rng.standard_normal((10, 3, 3, 4)).astype(np.float32)
    for m in (1, 4, 12):
        mask, idx, wz = oracle.prune(w, m, m, 4)
        assert mask.all()
        assert np.array_equal(wz, w)
        assert np.array_equal(idx.reshape(idx.shape[0], -1),
                              np.tile(np.arange(36, dtype=np.int32), (idx.shape[0], 1)))


def test_group_spanning_the_whole_row():
    """M = K, N = K/2 (Fig. 3c): half of the columns of each tile survive,
    namely those with the largest column norms."""
    rng = np.random.default_rng(5)
    cout, K, tile = 8, 24, 4
    W = rng.standard_normal((cout, K)).astype(np.float32)
    mask, idx, _ = oracle.prune(_as_ohwi(W), K // 2, K, tile)
    for j in range(cout // tile):
        norms = np.abs(W[j * tile:(j + 1) * tile].astype(np.float64)).sum(axis=0)
        kept = np.flatnonzero(mask[j * tile])
        dropped = np.flatnonzero(mask[j * tile] == 0)
        assert kept.size == K // 2
        assert norms[kept].min() > norms[dropped].max()


def test_ties_go_to_the_lower_index():
    W = np.zeros((4, 8), dtype=np.float32)
    W[:, 0:4] = [[1, 1, 1, 1]] * 4            # all equal -> keep columns 0, 1
    W[:, 4:8] = [[0.5, 2, 0.5, 2]] * 4        # clear winners 5, 7
    mask, idx, _ = oracle.prune(_as_ohwi(W), 2, 4, 4)
    assert idx.reshape(-1).tolist() == [0, 1, 5, 7]
    # sign must not matter (L1 norm), zero columns are still "kept" if selected
    W2 = np.zeros((2, 4), dtype=np.float32)
    W2[:, 3] = [-3, 3]
    mask, idx, _ = oracle.prune(_as_ohwi(W2), 2, 4, 2)
    assert idx.reshape(-1).tolist() == [0, 3]
    assert int(mask.sum()) == 4


def test_norm_is_taken_over_the_tile_not_per_row():
    # column 0 is the largest in row 0 only; over the tile column 1 wins
    W = np.array([[4, 3, 0, 0], [0, 3, 0, 0]], dtype=np.float32)
    _, idx, _ = oracle.prune(_as_ohwi(W), 1, 4, 2)
    assert idx.reshape(-1).tolist() == [1]
    _, idx1, _ = oracle.prune(_as_ohwi(W), 1, 4, 1)
    assert idx1.reshape(-1).tolist() == [0, 1]


def test_ragged_last_tile_uses_existing_rows_only():
    W = np.array([[1, 0, 0, 0], [1, 0, 0, 0], [0, 0, 5, 0]], dtype=np.float32)
    mask, idx, _ = oracle.prune(_as_ohwi(W), 1, 4, 2)
    assert idx.reshape(-1).tolist() == [0, 2]
    assert mask.tolist() == [[1, 0, 0, 0], [1, 0, 0, 0], [0, 0, 1, 0]]


def test_repruning_zero_filled_weights_is_idempotent():
    rng = np.random.default_rng(13)
    w = rng.standard_normal((32, 3, 3, 16)).astype(np.float32)
    mask, idx, wz = oracle.prune(w, 2, 4, 8)
    mask2, idx2, wz2 = oracle.prune(wz, 2, 4, 8)
    assert np.array_equal(mask, mask2) and np.array_equal(idx, idx2)
    assert np.array_equal(wz, wz2)


def test_bad_arguments_are_rejected():
    w = np.ones((4, 1, 1, 6), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.prune(w, 2, 4, 2)           # K % M != 0
    with pytest.raises(ValueError):
        oracle.prune(w, 3, 2, 2)           # N > M
    w[1, 0, 0, 2] = np.nan
    with pytest.raises(ValueError):
        oracle.prune(w, 1, 2, 2)


@pytest.mark.parametrize("cout,K,n,m,tile", [(16, 32, 2, 4, 8), (10, 24, 1, 4, 4), (7, 16, 4, 8, 16)])
def test_pack_round_trip(cout, K, n, m, tile):
    """Scattering the compressed values back through the index array gives the
    zero-filled matrix bit for bit (section 2.1: compressed weights + indices)."""
    rng = np.random.default_rng(17)
    W = rng.standard_normal((cout, K)).astype(np.float32)
    mask, idx, wz = oracle.prune(_as_ohwi(W), n, m, tile)
    vals = oracle.pack(_as_ohwi(W), idx, n, m, tile)
    n_tiles = -(-cout // tile)
    assert vals.shape == (n_tiles, K // m * n, tile)
    rebuilt = np.zeros((n_tiles * tile, K), dtype=np.float32)
    for j in range(n_tiles):
        flat = idx[j].reshape(-1)
        for kk, k in enumerate(flat):
            rebuilt[j * tile:(j + 1) * tile, k] = vals[j, kk]
    assert np.array_equal(rebuilt[:cout], wz.reshape(cout, K))
    assert np.all(rebuilt[cout:] == 0)


def test_hand_worked_example():
    """tests/golden/prune_hand_example.txt: a 4x8 matrix pruned 2:4 with T = 2,
    kept sets worked out by hand from the definition in section 3.1."""
    path = os.path.join(HERE, "golden", "prune_hand_example.txt")
    sections, cur = {}, None
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("["):
            cur = line.strip("[]")
            sections[cur] = []
        else:
            sections[cur].append([float(v) for v in line.split()])
    W = np.array(sections["weights"], dtype=np.float32)
    want_idx = np.array(sections["idx"], dtype=np.int32)
    want_mask = np.array(sections["mask"], dtype=np.uint8)
    mask, idx, _ = oracle.prune(_as_ohwi(W), 2, 4, 2)
    assert np.array_equal(idx.reshape(want_idx.shape), want_idx)
    assert np.array_equal(mask, want_mask)
