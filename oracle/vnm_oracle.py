"""Plain, slow, obviously-correct CPU model of the V:N:M format and the product C = A.B.

TEST INFRASTRUCTURE ONLY -- see the package docstring.  Everything here is numpy on the host,
fp64 wherever floating point is involved, and follows the paper's definitions directly:

* the format (paper section 3, "The V:N:M format", figures 2-3): A (R x K) is cut into blocks of
  V rows x M columns; each block keeps 4 of its M columns (vector-wise stage); each row of a
  block keeps at most N=2 of those 4 (the 2:4 stage).  Storage is three arrays: the kept
  `values` (R x K/M x 2), one 2-bit `m-index` per kept value (R x K/M x 2) that addresses the
  FOUR SELECTED columns (not the original M), and `column-loc` (R/V x K/M x 4) naming which 4
  of the M columns were selected.
* the product (paper section 4, figure 4): exactly (A masked) . B -- the format only skips
  structural zeros -- so the oracle expands to a dense masked matrix and multiplies in fp64.

Readings where the paper is silent (order of column-loc entries and of the two m-indices,
padding when fewer than 4 columns / 2 entries are used, word packing of the 2-bit indices):
  - column-loc entries ascending; when a block uses fewer than 4 columns, the smallest unused
    column ids are added until there are 4, and the 4 are sorted;
  - per (row, group) the two m-indices satisfy idx0 < idx1; when fewer than 2 entries are kept
    the smallest unused positions are added and the padded slot stores +0 (0x0000);
  - structure follows the MASK, not the values (a kept entry equal to zero is stored as is);
  - metadata nibble = idx0 | idx1 << 2; eight nibbles per little-endian uint32, group g in bits
    [4*(g%8), 4*(g%8)+3] of word g//8 of its row; unused nibbles are 0.

Pins (tests/test_oracle_*.py): hand-derived golden arrays, compress->decompress round trip,
format invariants, brute-force triple loop on the dense masked matrix, B = identity, all-ones
closed form 2K/M, the M=4 special case against a plain sub-matrix product; for the epilogue
(tests/test_oracle_epilogue.py) tabulated values of the normal distribution, GELU's identities,
minimum and slope bound, and the tanh form's known distance from the definition.
"""
from __future__ import annotations

import numpy as np

N_KEEP = 2          # nonzeros per row per group (the hardware pattern is 2:4)
SEL_COLS = 4        # columns kept per V x M block

OK, ERR_MASK_COLS, ERR_MASK_ROW = "ok", "mask_cols", "mask_row"


def _dims(R, K, V, M):
    if V <= 0 or M < SEL_COLS or R % V or K % M:
        raise ValueError(f"shape not V:N:M-tileable: R={R} K={K} V={V} M={M}")
    return R // V, K // M


# --------------------------------------------------------------------------- mask legality
def check_mask(mask: np.ndarray, V: int, M: int):
    """Section 3: a block may use at most 4 distinct columns and a row at most 2 entries per
    group of M.  Returns (status, (block_row, group, row)).  The first offending block in
    row-major (block_row, group) order is reported; a block breaking both rules reports the
    column rule.  `row` is the first offending absolute row for the row rule, -1 otherwise."""
    R, K = mask.shape
    Rb, G = _dims(R, K, V, M)
    m4 = (mask != 0).reshape(Rb, V, G, M)
    cols_used = m4.any(axis=1).sum(axis=-1)            # (Rb, G)
    per_row = m4.sum(axis=-1)                          # (Rb, V, G)
    bad_cols = cols_used > SEL_COLS
    bad_rows = per_row > N_KEEP
    bad_block = bad_cols | bad_rows.any(axis=1)
    if not bad_block.any():
        return OK, (-1, -1, -1)
    flat = int(np.argmax(bad_block.reshape(-1)))
    b, g = divmod(flat, G)
    if bad_cols[b, g]:
        return ERR_MASK_COLS, (b, g, -1)
    v = int(np.argmax(bad_rows[b, :, g]))
    return ERR_MASK_ROW, (b, g, b * V + v)


# --------------------------------------------------------------------------- compress
def compress(A_bits: np.ndarray, mask: np.ndarray, V: int, M: int):
    """Dense fp16 bit patterns (uint16, R x K) + mask -> (values, columns, meta).

    values  uint16 [R, G, 2]      bit patterns of the kept entries (0x0000 in padded slots)
    columns uint16 [R/V, G, 4]    column-loc, relative ids in [0, M), strictly increasing
    meta    uint32 [R, ceil(G/8)] eight 4-bit (idx0 | idx1<<2) nibbles per word
    Raises ValueError on an illegal mask."""
    status, where = check_mask(mask, V, M)
    if status != OK:
        raise ValueError(f"illegal mask: {status} at (block_row, group, row)={where}")
    R, K = mask.shape
    Rb, G = _dims(R, K, V, M)
    keep = (mask != 0).reshape(Rb, V, G, M)
    A4 = np.ascontiguousarray(A_bits, dtype=np.uint16).reshape(Rb, V, G, M)

    # vector-wise stage: used columns first (ascending), then unused (ascending); first 4; sort.
    used = keep.any(axis=1)                                               # (Rb, G, M)
    order = np.argsort(~used, axis=-1, kind="stable")[..., :SEL_COLS]
    columns = np.sort(order, axis=-1)                                     # (Rb, G, 4)

    # restrict every row to the 4 selected columns
    gather = np.broadcast_to(columns[:, None, :, :], (Rb, V, G, SEL_COLS))
    keep_sel = np.take_along_axis(keep, gather, axis=-1)                  # (Rb, V, G, 4)
    a_sel = np.take_along_axis(A4, gather, axis=-1)

    # 2:4 stage: kept positions first (ascending), then the smallest unused; first 2; sort.
    pos = np.sort(np.argsort(~keep_sel, axis=-1, kind="stable")[..., :N_KEEP], axis=-1)
    v_keep = np.take_along_axis(keep_sel, pos, axis=-1)
    vals = np.where(v_keep, np.take_along_axis(a_sel, pos, axis=-1), np.uint16(0))

    nib = (pos[..., 0] | (pos[..., 1] << 2)).astype(np.uint32).reshape(R, G)
    W = (G + 7) // 8
    nib_pad = np.zeros((R, W * 8), dtype=np.uint32)
    nib_pad[:, :G] = nib
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    meta = np.bitwise_or.reduce(nib_pad.reshape(R, W, 8) << shifts, axis=-1).astype(np.uint32)
    return (vals.astype(np.uint16).reshape(R, G, N_KEEP),
            columns.astype(np.uint16),
            meta)


def compress_loops(A_bits, mask, V, M):
    """The same definition as `compress`, written as explicit loops (small inputs only)."""
    status, where = check_mask(mask, V, M)
    if status != OK:
        raise ValueError(f"illegal mask: {status} at {where}")
    R, K = mask.shape
    Rb, G = _dims(R, K, V, M)
    W = (G + 7) // 8
    values = np.zeros((R, G, 2), np.uint16)
    columns = np.zeros((Rb, G, 4), np.uint16)
    meta = np.zeros((R, W), np.uint32)
    for b in range(Rb):
        for g in range(G):
            S = sorted({c for c in range(M) for v in range(V) if mask[b * V + v, g * M + c]})
            c = 0
            while len(S) < 4:
                if c not in S:
                    S.append(c)
                c += 1
            S.sort()
            columns[b, g] = S
            for v in range(V):
                r = b * V + v
                P = [p for p in range(4) if mask[r, g * M + S[p]]]
                kept = set(P)
                p = 0
                while len(P) < 2:
                    if p not in P:
                        P.append(p)
                    p += 1
                P.sort()
                for t in range(2):
                    values[r, g, t] = A_bits[r, g * M + S[P[t]]] if P[t] in kept else 0
                meta[r, g // 8] |= np.uint32((P[0] | (P[1] << 2)) << (4 * (g % 8)))
    return values, columns, meta


# --------------------------------------------------------------------------- decompress
def unpack_meta(meta: np.ndarray, G: int) -> np.ndarray:
    """uint32 words -> (R, G, 2) array of the two 2-bit m-indices."""
    R, W = meta.shape
    shifts = (4 * np.arange(8, dtype=np.uint32))[None, None, :]
    nib = ((meta[:, :, None] >> shifts) & np.uint32(0xF)).reshape(R, W * 8)[:, :G]
    return np.stack([nib & 3, (nib >> 2) & 3], axis=-1).astype(np.int64)


def decompress(values, columns, meta, R, K, V, M) -> np.ndarray:
    """Section 3: entry t of (row r, group g) lives at column g*M + column_loc[r//V, g, m_index_t]
    -- the m-index addresses the four selected columns.  Returns uint16 bit patterns, R x K,
    +0 everywhere else."""
    Rb, G = _dims(R, K, V, M)
    idx = unpack_meta(meta, G).reshape(Rb, V, G, 2)
    cols = np.broadcast_to(columns.astype(np.int64)[:, None, :, :], (Rb, V, G, SEL_COLS))
    dst = np.take_along_axis(cols, idx, axis=-1)                          # relative column per value
    out = np.zeros((Rb, V, G, M), dtype=np.uint16)
    np.put_along_axis(out, dst, values.reshape(Rb, V, G, 2), axis=-1)
    return out.reshape(R, K)


def decompress_loops(values, columns, meta, R, K, V, M):
    Rb, G = _dims(R, K, V, M)
    out = np.zeros((R, K), np.uint16)
    for r in range(R):
        for g in range(G):
            nib = (int(meta[r, g // 8]) >> (4 * (g % 8))) & 0xF
            for t, p in enumerate((nib & 3, nib >> 2)):
                out[r, g * M + int(columns[r // V, g, p])] = values[r, g, t]
    return out


# --------------------------------------------------------------------------- the product
def f16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(bits, dtype=np.uint16).view(np.float16).astype(np.float64)


def spmm_dense_fp64(A_hat_bits: np.ndarray, B_bits: np.ndarray):
    """C* = A_hat . B and the bound matrix E = |A_hat| . |B|, inputs read exactly from their
    fp16 bit patterns, products and sums in fp64 (a dgemm on the expanded matrix)."""
    A = f16_bits_to_f64(A_hat_bits)
    B = f16_bits_to_f64(B_bits)
    return A @ B, np.abs(A) @ np.abs(B)


def spmm_fp64(values, columns, meta, R, K, V, M, B_bits):
    """Figure 4 / section 4: the V:N:M product is the dense product of the expanded matrix."""
    return spmm_dense_fp64(decompress(values, columns, meta, R, K, V, M), B_bits)


def spmm_bruteforce(A_bits, mask, B_bits):
    """Triple loop straight over the dense masked matrix -- no format involved (tiny inputs)."""
    A = f16_bits_to_f64(A_bits)
    B = f16_bits_to_f64(B_bits)
    R, K = A.shape
    C = B.shape[1]
    out = np.zeros((R, C))
    bound = np.zeros((R, C))
    for i in range(R):
        ks = [k for k in range(K) if mask[i, k]]
        for j in range(C):
            s = 0.0
            e = 0.0
            for k in ks:
                p = float(A[i, k]) * float(B[k, j])
                s += p
                e += abs(p)
            out[i, j] = s
            bound[i, j] = e
    return out, bound


def accept(C_test: np.ndarray, C_star: np.ndarray, E: np.ndarray, elem_tol=1e-2, fro_tol=1e-3):
    """The acceptance rule for a computed product: |C - C*| <= elem_tol * E elementwise (so an
    entry with E = 0 must be exactly 0) and ||C - C*||_F <= fro_tol * ||C*||_F."""
    d = np.abs(np.asarray(C_test, dtype=np.float64) - C_star)
    worst = float(np.max(d - elem_tol * E)) if d.size else 0.0
    num = float(np.sqrt(np.sum(d * d)))
    den = float(np.sqrt(np.sum(C_star * C_star)))
    fro = num / den if den > 0 else (0.0 if num == 0 else np.inf)
    return (worst <= 0.0) and (fro <= fro_tol), {"max_excess": worst, "rel_fro": fro}


# ---------------------------------------------------------------------------------------------
# Fused epilogue of the product: the paper's call is spmm(values, columns, metadata, input, bias)
# (section 7.2, "Case study: sparse LLMs": the sparse layer replaces a linear layer, so the bias
# of the layer is added to every output row = output feature).  An optional GELU follows, in its
# definition x * Phi(x) or in the tanh form transformer code bases use.
GELU_LIPSCHITZ = 1.13          # sup |gelu'(x)| = 1.1289 (at x = sqrt(2)): GELU stretches an error by at most this


def gelu_erf(x: np.ndarray) -> np.ndarray:
    """GELU(x) = x * Phi(x) = x/2 * (1 + erf(x / sqrt 2)), the definition, in fp64."""
    import math
    erf = np.vectorize(math.erf, otypes=[np.float64])
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def gelu_tanh(x: np.ndarray) -> np.ndarray:
    """The tanh form: x/2 * (1 + tanh(sqrt(2/pi) * (x + 0.044715 x^3))), in fp64."""
    x = np.asarray(x, dtype=np.float64)
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x * x * x)))


ACTIVATIONS = {"none": None, "gelu": gelu_erf, "gelu_tanh": gelu_tanh}


def epilogue_fp64(C_star: np.ndarray, E: np.ndarray, bias_bits, activation: str = "none"):
    """Y = act(C* + bias[:, None]).  Returns (Y, E_y): E_y bounds how far Y may move when the
    pre-activation moves by the product's own bound: the magnitude sum grows by |bias| (the add
    is one more rounded term) and an activation stretches it by its Lipschitz constant."""
    Z = np.array(C_star, dtype=np.float64, copy=True)
    Ez = np.array(E, dtype=np.float64, copy=True)
    if bias_bits is not None:
        b = f16_bits_to_f64(np.asarray(bias_bits).reshape(-1))
        if b.shape[0] != Z.shape[0]:
            raise ValueError("bias needs one entry per row of C")
        Z += b[:, None]
        Ez += np.abs(b)[:, None]
    act = ACTIVATIONS[activation]
    if act is None:
        return Z, Ez
    return act(Z), GELU_LIPSCHITZ * Ez


# ---------------------------------------------------------------------------------------------
# Magnitude pruning to V:N:M (section 3, the two pruning stages; section 5, the energy metric).
# The paper does not say how "most significant" is measured for a column of a block; the reading
# taken is the column's L1 mass over the V rows (the sum the energy metric itself is made of), and
# |w| for the per-row stage.  Ties go to the smaller index.  Masses are EXACT: every fp16 is an
# integer multiple of 2^-24, so magnitudes are summed as integers and no rounding order exists.
MAG_NONFINITE = 1 << 40        # Inf / NaN count as more than any finite fp16 (65504 = 2047 * 2^29 units)


def magnitude_units(bits: np.ndarray) -> np.ndarray:
    """|w| of fp16 bit patterns in units of 2^-24, as int64 (exact)."""
    b = np.asarray(bits).astype(np.int64)
    e = (b >> 10) & 31
    f = b & 1023
    normal = (1024 + f) << np.maximum(e - 1, 0)
    return np.where(e == 0, f, np.where(e == 31, MAG_NONFINITE, normal)).astype(np.int64)


def prune(A_bits: np.ndarray, V: int, M: int):
    """One-shot magnitude pruning: per V x M block keep the 4 columns of largest L1 mass, then in
    every row the 2 largest |w| among those 4.  Returns (mask uint8 R x K, kept_mass, total_mass)
    with the masses as Python integers in units of 2^-24 (energy = kept_mass / total_mass)."""
    A_bits = np.asarray(A_bits)
    R, K = A_bits.shape
    Rb, G = _dims(R, K, V, M)
    mag = magnitude_units(A_bits)
    mask = np.zeros((R, K), dtype=np.uint8)
    kept = 0
    for b in range(Rb):
        for g in range(G):
            blk = mag[b * V:(b + 1) * V, g * M:(g + 1) * M]
            mass = blk.sum(axis=0)                                   # exact integers
            order = sorted(range(M), key=lambda c: (-int(mass[c]), c))
            cols = sorted(order[:SEL_COLS])
            for v in range(V):
                row = [(-int(blk[v, c]), p) for p, c in enumerate(cols)]
                for _, p in sorted(row)[:N_KEEP]:
                    mask[b * V + v, g * M + cols[p]] = 1
                    kept += int(blk[v, cols[p]])
    total = int(sum(int(x) for x in mag.sum(axis=1)))
    return mask, kept, total


# ---------------------------------------------------------------------------------------------
# The sparse layer as a linear layer sees it (section 7.2: the V:N:M weight replaces the weight of
# a linear layer; activations arrive token-major, one row of K features per token):
#     Y[t][r] = act( sum_k X[t][k] * A[r][k] + bias[r] ),   Y is tokens x R.
def linear_fp64(values, columns, meta, R, K, V, M, X_bits, bias_bits=None, activation="none"):
    """Returns (Y, E_y), both tokens x R: the product with B = X^T, the epilogue, transposed."""
    X_bits = np.asarray(X_bits)
    if X_bits.ndim != 2 or X_bits.shape[1] != K:
        raise ValueError("X must be tokens x K")
    C_star, E = spmm_fp64(values, columns, meta, R, K, V, M, np.ascontiguousarray(X_bits.T))
    Y, Ey = epilogue_fp64(C_star, E, bias_bits, activation)
    return np.ascontiguousarray(Y.T), np.ascontiguousarray(Ey.T)
