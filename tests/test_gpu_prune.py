"""nm_prune on the GPU against the CPU oracle: kept indices, mask and packed
values must match bit for bit (section 3.1 selection, section 2.1 format)."""
import numpy as np
import pytest

import oracle
from paper_2507_17301_amd import binding as nm
from gpu_util import say

pytestmark = pytest.mark.gpu

CASES = [
    # cout, kh, kw, cin, n, m, tile
    (64, 3, 3, 64, 2, 4, 16),
    (256, 3, 3, 256, 1, 8, 32),
    (256, 1, 1, 64, 2, 8, 8),
    (100, 3, 3, 24, 4, 8, 16),      # ragged last tile (100 = 6*16 + 4)
    (37, 1, 1, 40, 1, 4, 5),        # odd tile size, ragged
    (64, 7, 7, 3, 1, 1, 16),        # dense stem
    (48, 3, 3, 16, 3, 4, 1),        # T = 1: row-wise N:M
    (32, 3, 3, 32, 144, 288, 8),    # one group spans the whole row (M = K)
    (16, 1, 1, 512, 128, 512, 16),  # M = Cin, beyond one workgroup of columns
    (24, 1, 1, 1200, 100, 300, 24), # M not a power of two
]


def _compare(w, n, m, tile, bf16=False):
    mask, idx, wz = oracle.prune(w, n, m, tile)
    vals = oracle.pack(w, idx, n, m, tile)
    if bf16:
        vals = oracle.round_bf16(vals)
    wp = nm.nm_prune(w, n, m, tile, nm.NM_BF16 if bf16 else nm.NM_F32)
    assert nm.nm_packed_dims(wp) == (idx.shape[0], idx.shape[1], n, idx.shape[1] * n)
    assert np.array_equal(nm.nm_packed_indices(wp), idx)
    assert np.array_equal(nm.nm_packed_mask(wp), mask)
    got = nm.nm_packed_values(wp)
    assert np.array_equal(got.view(np.uint32), vals.view(np.uint32))


@pytest.mark.parametrize("cout,kh,kw,cin,n,m,tile", CASES)
def test_prune_bit_exact_random(cout, kh, kw, cin, n, m, tile):
    say(f"prune random cout={cout} k={kh}x{kw} cin={cin} {n}:{m} T={tile}")
    rng = np.random.default_rng(cout + cin + m)
    w = rng.standard_normal((cout, kh, kw, cin)).astype(np.float32) * 0.05
    _compare(w, n, m, tile)


@pytest.mark.parametrize("cout,kh,kw,cin,n,m,tile", CASES[:5] + CASES[7:8])
def test_prune_bit_exact_with_many_ties(cout, kh, kw, cin, n, m, tile):
    say(f"prune ties cout={cout} k={kh}x{kw} cin={cin} {n}:{m} T={tile}")
    rng = np.random.default_rng(5)
    w = (rng.integers(-2, 3, size=(cout, kh, kw, cin)) / 4.0).astype(np.float32)
    _compare(w, n, m, tile)


def test_prune_bf16_values_are_rounded_after_selection():
    say("prune bf16 values")
    rng = np.random.default_rng(9)
    w = rng.standard_normal((64, 3, 3, 32)).astype(np.float32) * 0.05
    _compare(w, 2, 4, 16, bf16=True)


def test_sums_that_differ_only_in_the_last_bits():
    """Norms are compared in fp64: columns whose fp32 sums would tie must still
    be ordered as the oracle orders them."""
    say("prune near-ties")
    rng = np.random.default_rng(21)
    base = rng.standard_normal((32, 1, 1, 64)).astype(np.float32)
    w = base.copy()
    w[:, 0, 0, 1::4] = base[:, 0, 0, 0::4] * np.float32(1 + 2 ** -23)   # nearly equal columns
    w[:, 0, 0, 2::4] = base[:, 0, 0, 0::4]
    _compare(w, 2, 4, 16)
    _compare(w, 1, 4, 32)
