"""Pins for the oracle's format half (check_mask / compress / decompress), paper section 3."""
import numpy as np
import pytest

from oracle import vnm_oracle as o
from paper_2310_02065_amd import inputs
from helpers import load_hand_fixture

LEGAL_NIBBLES = {0x4, 0x8, 0xC, 0x9, 0xD, 0xE}   # the six (idx0 < idx1) pairs of a 2:4 group


def test_hand_example_matches_golden():
    fx = load_hand_fixture()
    for fn in (o.compress, o.compress_loops):
        v, c, m = fn(fx["A_bits"], fx["mask"], fx["V"], fx["M"])
        assert np.array_equal(c, fx["columns"])
        assert np.array_equal(v, fx["values"])
        assert np.array_equal(m, fx["meta"])
    for fn in (o.decompress, o.decompress_loops):
        d = fn(fx["values"], fx["columns"], fx["meta"], fx["R"], fx["K"], fx["V"], fx["M"])
        assert np.array_equal(d, np.where(fx["mask"] != 0, fx["A_bits"], 0))


@pytest.mark.parametrize("R,K,V,M", [(256, 256, 64, 8), (128, 320, 32, 10), (256, 512, 128, 32),
                                     (64, 700, 64, 100), (128, 64, 64, 4), (96, 84, 32, 7)])
def test_shapes_invariants_roundtrip(R, K, V, M):
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=7 + M)
    v, c, m = o.compress(A, mask, V, M)
    G = K // M
    # shapes as the paper gives them: values / m-indices R x K/M x 2, column-loc R/V x K/M x 4
    assert v.shape == (R, G, 2) and v.dtype == np.uint16
    assert c.shape == (R // V, G, 4) and c.dtype == np.uint16
    assert m.shape == (R, (G + 7) // 8) and m.dtype == np.uint32
    # column-loc strictly increasing in [0, M)
    assert (np.diff(c.astype(int), axis=-1) > 0).all() and c.max() < M
    # every nibble is one of the six legal pairs; unused nibbles are zero
    nib = np.stack([(m >> (4 * i)) & 0xF for i in range(8)], axis=-1).reshape(R, -1)
    assert set(np.unique(nib[:, :G]).tolist()) <= LEGAL_NIBBLES
    assert (nib[:, G:] == 0).all()
    # structure: <= 4 used columns per block, <= 2 kept entries per row-group, and the random
    # recipe keeps exactly 2 per row-group => 2K/M values per row, none of them padding
    kept = (mask != 0).reshape(R // V, V, G, M)
    assert kept.any(axis=1).sum(-1).max() <= 4 and kept.sum(-1).max() <= 2
    assert (kept.sum(-1) == 2).all()
    # round trip is bit exact, masked-out entries come back as +0
    d = o.decompress(v, c, m, R, K, V, M)
    assert np.array_equal(d, np.where(mask != 0, A, 0))
    # vectorised and loop versions agree; recompressing the expansion changes nothing
    v2, c2, m2 = o.compress_loops(A, mask, V, M) if R * K <= 70000 else (v, c, m)
    assert np.array_equal(v, v2) and np.array_equal(c, c2) and np.array_equal(m, m2)
    v3, c3, m3 = o.compress(d, mask, V, M)
    assert np.array_equal(v, v3) and np.array_equal(c, c3) and np.array_equal(m, m3)


def test_m4_is_plain_2_4():
    # M = 4: every block selects columns (0,1,2,3); V plays no role in the arrays
    A, mask, _ = inputs.gen_problem(128, 64, 8, 64, 4, 1.0, seed=3)
    v64, c64, m64 = o.compress(A, mask, 64, 4)
    v32, c32, m32 = o.compress(A, mask, 32, 4)
    assert (c64 == np.arange(4)).all() and (c32 == np.arange(4)).all()
    assert np.array_equal(v64, v32) and np.array_equal(m64, m32)
    # the nibble is the position pair inside the plain group of 4
    r, g = 5, 3
    pos = np.flatnonzero(mask[r, 4 * g:4 * g + 4])
    assert ((int(m64[r, g // 8]) >> (4 * (g % 8))) & 0xF) == (pos[0] | (pos[1] << 2))


def test_padding_rules_by_hand():
    V, M = 2, 8
    A = (0x4000 + np.arange(2 * 8).reshape(2, 8)).astype(np.uint16)
    # no entry at all: columns 0..3, nibble 0x4, zero values
    mask = np.zeros((2, 8), np.uint8)
    v, c, m = o.compress(A, mask, V, M)
    assert c.tolist() == [[[0, 1, 2, 3]]] and v.tolist() == [[[0, 0]], [[0, 0]]] and m.tolist() == [[4], [4]]
    # one used column (6): columns 0,1,2,6; its row has position 3 kept -> pair (0,3) = 0xC, value slot 1
    mask[1, 6] = 1
    v, c, m = o.compress(A, mask, V, M)
    assert c.tolist() == [[[0, 1, 2, 6]]]
    assert m.tolist() == [[4], [0xC]] and v.tolist() == [[[0, 0]], [[0, int(A[1, 6])]]]
    # two used columns (1, 6) -> 0,1,2,6 ; row 0 keeps column 1 only: pair (0,1) -> 0x4 with value in slot 1
    mask[0, 1] = 1
    v, c, m = o.compress(A, mask, V, M)
    assert c.tolist() == [[[0, 1, 2, 6]]]
    assert m.tolist() == [[4], [0xC]] and v.tolist() == [[[0, int(A[0, 1])]], [[0, int(A[1, 6])]]]
    # three used columns (1, 3, 6) -> 0,1,3,6 ; row 0 keeps 1 and 3 -> positions (1,2) = 0x9
    mask[0, 3] = 1
    v, c, m = o.compress(A, mask, V, M)
    assert c.tolist() == [[[0, 1, 3, 6]]]
    assert m.tolist() == [[9], [0xC]] and v.tolist() == [[[int(A[0, 1]), int(A[0, 3])]], [[0, int(A[1, 6])]]]
    # kept position 0 alone pads with position 1: pair (0,1), value in slot 0
    mask2 = np.zeros((2, 8), np.uint8); mask2[0, 0] = 1
    v, c, m = o.compress(A, mask2, V, M)
    assert m.tolist() == [[4], [4]] and v.tolist() == [[[int(A[0, 0]), 0]], [[0, 0]]]


def test_structure_follows_mask_not_values():
    V, M = 2, 4
    A = np.array([[0x0000, 0x8000, 0x3C00, 0x7E00], [0x0001, 0x0000, 0x0000, 0xFC00]], np.uint16)
    mask = np.array([[1, 1, 0, 0], [0, 0, 1, 1]], np.uint8)
    v, c, m = o.compress(A, mask, V, M)
    assert v.tolist() == [[[0x0000, 0x8000]], [[0x0000, 0xFC00]]]      # +0, -0, +0, -inf kept as bits
    assert m.tolist() == [[0x4], [0xE]]
    d = o.decompress(v, c, m, 2, 4, V, M)
    assert d.tolist() == [[0, 0x8000, 0, 0], [0, 0, 0, 0xFC00]]


def test_illegal_masks():
    V, M, R, K = 4, 8, 8, 24
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=11)
    assert o.check_mask(mask, V, M) == (o.OK, (-1, -1, -1))
    # a fifth column in block (1, 2), written into a row that keeps its own count at 2
    bad = mask.copy()
    blk = bad[4:8, 16:24]
    free_col = int(np.flatnonzero(~blk.any(axis=0))[0])
    r_in = 0
    old = int(np.flatnonzero(blk[r_in])[0])
    blk[r_in, old] = 0; blk[r_in, free_col] = 1
    if blk.any(axis=0).sum() <= 4:         # the moved entry emptied its old column; use another row too
        blk[1, int(np.flatnonzero(blk[1])[0])] = 0; blk[1, old] = 1
    assert blk.any(axis=0).sum() == 5 and blk.sum(axis=1).max() <= 2
    assert o.check_mask(bad, V, M) == (o.ERR_MASK_COLS, (1, 2, -1))
    with pytest.raises(ValueError):
        o.compress(A, bad, V, M)
    # a third entry in row 6 of block (1, 0), inside the block's own 4 columns
    bad = mask.copy()
    blk = bad[4:8, 0:8]
    used = np.flatnonzero(blk.any(axis=0))
    add = [c for c in used if not blk[2, c]][0]
    blk[2, add] = 1
    assert o.check_mask(bad, V, M) == (o.ERR_MASK_ROW, (1, 0, 6))
    # both rules broken in the same block: the column rule is reported
    blk[2, int(np.flatnonzero(~blk.any(axis=0))[0])] = 1
    assert o.check_mask(bad, V, M)[0] == o.ERR_MASK_COLS
    # an earlier block (row-major) with a row violation outranks a later block with a column one
    bad2 = bad.copy()
    blk0 = bad2[0:4, 8:16]
    used = np.flatnonzero(blk0.any(axis=0))
    blk0[3, [c for c in used if not blk0[3, c]][0]] = 1
    assert o.check_mask(bad2, V, M) == (o.ERR_MASK_ROW, (0, 1, 3))


def test_bad_shapes_raise():
    with pytest.raises(ValueError):
        o.check_mask(np.zeros((6, 8), np.uint8), 4, 8)
    with pytest.raises(ValueError):
        o.check_mask(np.zeros((8, 9), np.uint8), 4, 8)
    with pytest.raises(ValueError):
        o.check_mask(np.zeros((8, 6), np.uint8), 4, 3)


def test_planted_mistakes_are_caught_by_the_pins():
    """Each plausible slip, planted in a copy of the expected arrays, breaks a pin above."""
    fx = load_hand_fixture()
    R, K, V, M = fx["R"], fx["K"], fx["V"], fx["M"]
    want = np.where(fx["mask"] != 0, fx["A_bits"], 0)
    # m-index read as an ORIGINAL column id instead of an index into column-loc
    wrong_cols = np.broadcast_to(np.arange(4, dtype=np.uint16), fx["columns"].shape)
    assert not np.array_equal(o.decompress(fx["values"], wrong_cols, fx["meta"], R, K, V, M), want)
    # the two m-indices swapped inside the nibble
    sw = fx["meta"].copy()
    n0, n1 = sw & 0xF, (sw >> 4) & 0xF
    swap = lambda n: ((n & 3) << 2) | (n >> 2)
    sw = (swap(n0) | (swap(n1) << 4)).astype(np.uint32)
    assert not np.array_equal(o.decompress(fx["values"], fx["columns"], sw, R, K, V, M), want)
    # column-loc taken per row-block of the wrong height (V = 1 -> wrong block row)
    shifted = fx["columns"][::-1].copy()
    assert not np.array_equal(o.decompress(fx["values"], shifted, fx["meta"], R, K, V, M), want)
