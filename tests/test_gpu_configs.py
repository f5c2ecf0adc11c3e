"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic
variant selection).  Compression is compared bit for bit over the whole matrix; the product is
compared elementwise with the fp64 oracle on all outputs where the oracle finishes in seconds, else
on a sample of rows (every sampled row is a complete row of C, so tile edges in the column
direction are all covered, and rows are drawn from every part of the block-row range)."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vnm_oracle as o
from paper_2310_02065_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def sample_rows(R, V, rng, per_block_row=1):
    """At least one row of every block row (random position inside it, so every 32-row tile position
    occurs), plus the first and last rows of the matrix and of the first block rows."""
    Rb = R // V
    picks = (np.arange(Rb)[:, None] * V + rng.integers(0, V, size=(Rb, per_block_row))).ravel()
    return np.unique(np.concatenate([picks, [0, V - 1, V, R - V, R - 1]]))


def compress_checked(A, mask, V, M):
    A_d = torch.from_numpy(A.view(np.float16)).to(DEV)
    m_d = torch.from_numpy(mask).to(DEV)
    h = binding.venom_compress(A_d, m_d, V, 2, M)
    del A_d, m_d
    v, c, m = binding.venom_export(h)
    torch.cuda.synchronize()
    ov, oc, om = o.compress(A, mask, V, M)
    assert np.array_equal(c.cpu().numpy().view(np.uint16), oc)
    assert np.array_equal(m.cpu().numpy().view(np.uint32), om)
    assert np.array_equal(v.cpu().numpy().view(np.uint16), ov)
    return h, (ov, oc, om)


def check_product_rows(h, arrays, B, R, K, V, M, rows, variant=-1, chunk=8192):
    """The product in the launch configuration the benchmark times, compared on `rows` (all columns)
    with the oracle: the expanded rows times B in fp64, in chunks of rows."""
    ov, oc, om = arrays
    B_d = torch.from_numpy(B.view(np.float16)).to(DEV)
    out = binding.venom_spmm(h, B_d, variant=variant)
    again = binding.venom_spmm(h, B_d, variant=variant)
    torch.cuda.synchronize()
    assert torch.equal(out, again), "the product is not bitwise repeatable"
    worst = None
    for lo in range(0, len(rows), chunk):
        part = rows[lo:lo + chunk]
        if len(part) % V == 0 and part[0] % V == 0 and np.array_equal(part, np.arange(part[0], part[0] + len(part))):
            r0, r1 = int(part[0]), int(part[0]) + len(part)       # whole block rows: expand them in one go
            rows_dense = o.decompress(ov[r0:r1], oc[r0 // V:r1 // V], om[r0:r1], r1 - r0, K, V, M)
        else:
            # expand only the block rows the sampled rows live in
            dense = {}
            for b in np.unique(part // V):
                dense[b] = o.decompress(ov[b * V:(b + 1) * V], oc[b:b + 1], om[b * V:(b + 1) * V], V, K, V, M)
            rows_dense = np.stack([dense[r // V][r % V] for r in part])
        Cs, E = o.spmm_dense_fp64(rows_dense, B)
        got = out[torch.from_numpy(part).to(DEV)].double().cpu().numpy()
        ok, info = o.accept(got, Cs, E)
        assert ok, info
        worst = info
    return out, B_d, worst


def run_config(R, K, C, V, M, sigma, seed, sample_rows=None):
    A, mask, B = inputs.gen_problem(R, K, C, V, M, sigma, seed=seed)
    A_d = torch.from_numpy(A.view(np.float16)).to(DEV)
    m_d = torch.from_numpy(mask).to(DEV)
    h = binding.venom_compress(A_d, m_d, V, 2, M)
    del A_d, m_d
    v, c, m = binding.venom_export(h)
    torch.cuda.synchronize()
    ov, oc, om = o.compress(A, mask, V, M)
    assert np.array_equal(c.cpu().numpy().view(np.uint16), oc)
    assert np.array_equal(m.cpu().numpy().view(np.uint32), om)
    assert np.array_equal(v.cpu().numpy().view(np.uint16), ov)
    del v, c, m
    B_d = torch.from_numpy(B.view(np.float16)).to(DEV)
    out = binding.venom_spmm(h, B_d)
    again = binding.venom_spmm(h, B_d)
    torch.cuda.synchronize()
    assert torch.equal(out, again), "the product is not bitwise repeatable"
    if sample_rows is None:
        rows = np.arange(R)
    else:
        rng = np.random.default_rng(seed)
        rows = np.unique(np.concatenate([rng.choice(R, size=sample_rows, replace=False), [0, V - 1, V, R - V, R - 1]]))
    # oracle on the chosen rows: the expanded rows times B in fp64
    dense = o.decompress(ov, oc, om, R, K, V, M)
    Cs, E = o.spmm_dense_fp64(dense[rows], B)
    got = out[torch.from_numpy(rows).to(DEV)].double().cpu().numpy()
    ok, info = o.accept(got, Cs, E)
    assert ok, info
    # the fused epilogue and the token-major layer view at the same size, same sampled rows (= output features)
    rng = np.random.default_rng(seed + 17)
    bias = rng.standard_normal(R).astype(np.float16)
    bias_d = torch.from_numpy(bias).to(DEV)
    Ys, Ey = o.epilogue_fp64(Cs, E, bias.view(np.uint16)[rows], "gelu")
    fused = binding.venom_spmm(h, B_d, bias=bias_d, activation="gelu")
    ok, info2 = o.accept(fused[torch.from_numpy(rows).to(DEV)].double().cpu().numpy(), Ys, Ey)
    assert ok, info2
    layer = binding.venom_linear(h, B_d.t().contiguous(), bias=bias_d, activation="gelu")
    assert torch.equal(layer, fused.t()), "token-major output differs from the transposed product"
    return info


def test_config0_tiny():
    R, K, C, V, M, s = inputs.CONFIGS["tiny"]
    run_config(R, K, C, V, M, s, inputs.config_seed(0))


def test_config1_bert_base():
    R, K, C, V, M, s = inputs.CONFIGS["bert_base"]
    run_config(R, K, C, V, M, s, inputs.config_seed(1))


def test_config2_bert_large():
    R, K, C, V, M, s = inputs.CONFIGS["bert_large"]
    run_config(R, K, C, V, M, s, inputs.config_seed(2))


def test_config3_gpt3_every_row():
    """All 49152 x 2048 outputs against the oracle (expand + fp64 product, a few block rows at a time),
    then the fused epilogue and the layer view on a sample of rows."""
    R, K, C, V, M, s = inputs.CONFIGS["gpt3"]
    A, mask, B = inputs.gen_problem(R, K, C, V, M, s, seed=inputs.config_seed(3))
    h, arrays = compress_checked(A, mask, V, M)
    del A, mask
    out, B_d, _ = check_product_rows(h, arrays, B, R, K, V, M, np.arange(R), chunk=4096)
    rng = np.random.default_rng(3)
    rows = sample_rows(R, V, rng)
    ov, oc, om = arrays
    dense = np.stack([o.decompress(ov[(r // V) * V:(r // V + 1) * V], oc[r // V:r // V + 1], om[(r // V) * V:(r // V + 1) * V],
                                   V, K, V, M)[r % V] for r in rows])
    Cs, E = o.spmm_dense_fp64(dense, B)
    bias = rng.standard_normal(R).astype(np.float16)
    bias_d = torch.from_numpy(bias).to(DEV)
    Ys, Ey = o.epilogue_fp64(Cs, E, bias.view(np.uint16)[rows], "gelu")
    fused = binding.venom_spmm(h, B_d, bias=bias_d, activation="gelu")
    ok, info = o.accept(fused[torch.from_numpy(rows).to(DEV)].double().cpu().numpy(), Ys, Ey)
    assert ok, info
    layer = binding.venom_linear(h, B_d.t().contiguous(), bias=bias_d, activation="gelu")
    assert torch.equal(layer, fused.t()), "token-major output differs from the transposed product"


# every point of the sparsity sweep: V x M x C.  The matrix (and its compressed form, checked bit for
# bit) is made once per (V, M); the three widths of B follow.
@pytest.mark.parametrize("V", inputs.SWEEP_V)
@pytest.mark.parametrize("M", inputs.SWEEP_M)
def test_config4_every_sweep_point(V, M):
    R, K = inputs.SWEEP_SHAPE
    seed = inputs.config_seed(4) + 7 * M + V
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=seed)
    h, arrays = compress_checked(A, mask, V, M)
    del A, mask
    rng = np.random.default_rng(seed)
    for C in inputs.SWEEP_C:
        B = inputs.gen_B(K, C, seed=seed + C)
        rows = sample_rows(R, V, rng, per_block_row=2 if C <= 2048 else 1)
        check_product_rows(h, arrays, B, R, K, V, M, rows)


def test_many_tiles_per_workgroup_with_a_ragged_last_k_step():
    """More than 512 tiles (every workgroup walks several, odd ones backwards) with K/M not a multiple
    of 8, on every tile width."""
    R, K, C, V, M = 8192, 8400, 4096, 32, 100            # G = 84: the last k-step has 4 of 8 groups
    seed = 77
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=seed)
    h, arrays = compress_checked(A, mask, V, M)
    rows = sample_rows(R, V, np.random.default_rng(seed))
    names = binding.venom_spmm_variants()
    for var in [-1] + [i for i, n in enumerate(names) if n.startswith(f"v{V}_")]:
        check_product_rows(h, arrays, B, R, K, V, M, rows, variant=var)


def test_narrow_tiles_walk_several_tiles_each():
    R, K, C, V, M = 8192, 1024, 2048, 128, 16             # 64 block rows x 16 (128-column) tiles
    seed = 78
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=seed)
    h, arrays = compress_checked(A, mask, V, M)
    rows = sample_rows(R, V, np.random.default_rng(seed), per_block_row=4)
    names = binding.venom_spmm_variants()
    for var in [i for i, n in enumerate(names) if n.startswith(f"v{V}_")]:
        check_product_rows(h, arrays, B, R, K, V, M, rows, variant=var)


# the shape of the paper's column-loc ablation (section 4): 1024 x K x 4096 at V = 128, 2:10 ... 2:100
@pytest.mark.parametrize("M", [10, 20, 40, 100])
@pytest.mark.parametrize("K", [4000, 16000])
def test_column_loc_ablation_shape(M, K):
    R, C, V = 1024, 4096, 128
    seed = 900 + M + K
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=seed)
    h, arrays = compress_checked(A, mask, V, M)
    check_product_rows(h, arrays, B, R, K, V, M, np.arange(R))
