"""Pins of the oracle's magnitude pruner and of the energy metric."""
import itertools

import numpy as np
import pytest

from oracle import vnm_oracle as o


def f16(x):
    return np.asarray(x, dtype=np.float16).view(np.uint16)


def test_magnitude_units_are_exact_for_every_fp16():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    m = o.magnitude_units(bits)
    vals = bits.view(np.float16).astype(np.float64)
    finite = np.isfinite(vals)
    assert np.array_equal(m[finite], (np.abs(vals[finite]) * 2.0 ** 24).astype(np.int64))   # exact in fp64
    assert (m[~finite] == o.MAG_NONFINITE).all() and m[finite].max() < o.MAG_NONFINITE


def test_hand_example():
    # one 2 x 6 block; column masses 1+1, 9+0, 0+0, 4+4, 2+7, 3+3 -> columns 1, 3, 4, 5 survive
    A = f16([[1, 9, 0, 4, 2, 3],
             [1, 0, 0, 4, 7, 3]])
    mask, kept, total = o.prune(A, 2, 6)
    assert mask.tolist() == [[0, 1, 0, 1, 0, 0],      # row 0 keeps 9 and 4 among (9, 4, 2, 3)
                             [0, 0, 0, 1, 1, 0]]      # row 1 keeps 4 and 7 among (0, 4, 7, 3)
    unit = 1 << 24
    assert kept == (9 + 4 + 4 + 7) * unit and total == 34 * unit
    st, viol = o.check_mask(mask, 2, 6)
    assert st == o.OK


def test_ties_go_to_the_smaller_index():
    A = f16(np.ones((4, 8)))
    mask, kept, total = o.prune(A, 4, 8)
    assert mask.tolist() == [[1, 1, 0, 0, 0, 0, 0, 0]] * 4
    assert kept * 4 == total


def test_is_the_best_legal_choice_by_brute_force():
    rng = np.random.default_rng(5)
    V, M = 2, 6
    A = rng.standard_normal((V, M)).astype(np.float16).view(np.uint16)
    mag = o.magnitude_units(A)
    mask, kept, _ = o.prune(A, V, M)
    # stage 1 by definition: the 4 columns of largest mass; stage 2: best 2 of those per row
    best_cols = max(itertools.combinations(range(M), 4), key=lambda cs: sum(int(mag[:, c].sum()) for c in cs))
    expect = sum(sum(sorted((int(mag[v, c]) for c in best_cols), reverse=True)[:2]) for v in range(V))
    assert kept == expect
    assert set(np.nonzero(mask.any(axis=0))[0]) <= set(best_cols)


@pytest.mark.parametrize("R,K,V,M", [(64, 64, 32, 8), (128, 96, 64, 12), (32, 128, 16, 4), (8, 200, 4, 100)])
def test_pruned_mask_is_legal_dense_enough_and_feeds_compress(R, K, V, M):
    rng = np.random.default_rng(R + M)
    A = (rng.standard_normal((R, K)) * 0.02).astype(np.float16).view(np.uint16)
    mask, kept, total = o.prune(A, V, M)
    assert o.check_mask(mask, V, M)[0] == o.OK
    assert (mask.reshape(R, K // M, M).sum(axis=2) == 2).all()        # exactly N per row and group
    assert 0 < kept <= total
    values, columns, meta = o.compress(A, mask, V, M)
    back = o.decompress(values, columns, meta, R, K, V, M)
    assert np.array_equal(back, np.where(mask != 0, A, 0))
    # energy can only fall when M grows at fixed V (fewer survivors out of more)
    if M * 2 <= K and K % (2 * M) == 0:
        _, kept2, total2 = o.prune(A, V, 2 * M)
        assert total2 == total and kept2 < kept


def test_m4_keeps_top2_of_every_group_of_four():
    rng = np.random.default_rng(9)
    A = rng.standard_normal((8, 16)).astype(np.float16).view(np.uint16)
    mask, kept, _ = o.prune(A, 8, 4)
    mag = o.magnitude_units(A).reshape(8, 4, 4)
    assert kept == int(np.sort(mag, axis=2)[:, :, 2:].sum())


def test_plausible_wrong_rules_give_different_masks_here():
    # column choice by the largest single entry instead of the L1 mass: column 0 (one entry 5,
    # mass 5) would beat the columns of mass 6; the definition drops it
    B = f16([[5, 0, 3, 3, 3, 3],
             [0, 0, 3, 3, 3, 3]])
    m, kept, total = o.prune(B, 2, 6)
    assert m[:, 0].sum() == 0 and m[:, 1].sum() == 0
    assert kept == 12 << 24 and total == 29 << 24
    # per-row top-2 over all M columns (skipping the block stage) would keep the 8 in column 0
    C = f16([[8, 1, 1, 1, 1, 0],
             [0, 3, 3, 3, 3, 0],
             [0, 3, 3, 3, 3, 0],
             [0, 3, 3, 3, 3, 0]])
    m, _, _ = o.prune(C, 4, 6)
    assert m[0, 0] == 0 and m[0].sum() == 2
    # signs do not matter, only magnitudes
    D = f16([[-9, 1, 2, -3, 0, 0]])
    m, _, _ = o.prune(D, 1, 6)
    assert m.tolist() == [[1, 0, 0, 1, 0, 0]]
