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


def test_config3_gpt3_sampled_rows():
    R, K, C, V, M, s = inputs.CONFIGS["gpt3"]
    run_config(R, K, C, V, M, s, inputs.config_seed(3), sample_rows=768)


@pytest.mark.parametrize("V,M,C", [(64, 4, 256), (128, 8, 2048), (64, 16, 2048), (128, 32, 256),
                                   (64, 64, 2048), (128, 128, 2048), (128, 16, 8192)])
def test_config4_sweep_points_sampled_rows(V, M, C):
    R, K = inputs.SWEEP_SHAPE
    run_config(R, K, C, V, M, 1.0, inputs.config_seed(4) + 7 * M + V + C, sample_rows=256)
