"""GPU parity of venom_linear (token-major activations in, token-major output, fused bias and
activation) against the oracle, through the C ABI."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vnm_oracle as o
from paper_2310_02065_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def setup(R, K, T, V, M, seed):
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=seed)
    rng = np.random.default_rng(seed + 1)
    X = rng.standard_normal((T, K)).astype(np.float16)
    bias = rng.standard_normal(R).astype(np.float16)
    h = binding.venom_compress(torch.from_numpy(A.view(np.float16)).to(DEV), torch.from_numpy(mask).to(DEV), V, 2, M)
    return h, o.compress(A, mask, V, M), X, bias


@pytest.mark.parametrize("R,K,T,V,M", [(256, 384, 264, 128, 8), (384, 1280, 520, 128, 32), (192, 896, 136, 64, 16),
                                       (128, 720, 72, 32, 10), (192, 130 * 4, 8, 96, 4), (64, 1400, 40, 32, 100),
                                       (256, 256, 136, 128, 4), (512, 72, 264, 64, 4)])
@pytest.mark.parametrize("out_dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("activation", ["none", "gelu"])
def test_linear_matches_oracle(R, K, T, V, M, out_dtype, activation):
    h, (ov, oc, om), X, bias = setup(R, K, T, V, M, 40 + R + T)
    for with_bias in (False, True):
        Ys, Ey = o.linear_fp64(ov, oc, om, R, K, V, M, X.view(np.uint16), bias.view(np.uint16) if with_bias else None,
                               activation)
        Y = binding.venom_linear(h, torch.from_numpy(X).to(DEV), bias=torch.from_numpy(bias).to(DEV) if with_bias else None,
                                 activation=activation, out_dtype=out_dtype)
        ok, info = o.accept(Y.double().cpu().numpy(), Ys, Ey)
        assert ok, (with_bias, info)


def test_strided_x_and_y_leave_the_gaps_alone():
    R, K, T, V, M = 256, 512, 200, 64, 8
    h, (ov, oc, om), X, bias = setup(R, K, T, V, M, 7)
    Xbig = torch.zeros((T, K + 6), dtype=torch.float16, device=DEV)       # odd 2-byte offset: unaligned 4-byte reads
    Xbig[:, 3:3 + K] = torch.from_numpy(X).to(DEV)
    Ybig = torch.full((T, R + 12), -7.0, dtype=torch.float16, device=DEV)
    binding.venom_linear(h, Xbig[:, 3:3 + K], out=Ybig[:, 4:4 + R])
    Ys, Ey = o.linear_fp64(ov, oc, om, R, K, V, M, X.view(np.uint16))
    ok, info = o.accept(Ybig[:, 4:4 + R].double().cpu().numpy(), Ys, Ey)
    assert ok, info
    assert bool((Ybig[:, :4] == -7.0).all()) and bool((Ybig[:, 4 + R:] == -7.0).all())


def test_equals_the_column_major_product_bitwise():
    R, K, T, V, M = 256, 768, 128, 128, 16
    h, _, X, bias = setup(R, K, T, V, M, 9)
    X_d = torch.from_numpy(X).to(DEV)
    b_d = torch.from_numpy(bias).to(DEV)
    Y = binding.venom_linear(h, X_d, bias=b_d, activation="gelu_tanh")
    C = binding.venom_spmm(h, X_d.t().contiguous(), bias=b_d, activation="gelu_tanh")
    assert torch.equal(Y, C.t())


def test_argument_errors():
    R, K, T, V, M = 64, 64, 16, 32, 8
    h, _, X, _ = setup(R, K, T, V, M, 3)
    X_d = torch.from_numpy(X).to(DEV)
    with pytest.raises(binding.VenomError) as e:
        binding.venom_linear(h, X_d[:12])                                  # tokens % 8
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED
    with pytest.raises(binding.VenomError) as e:
        binding.venom_linear(h, X_d, scratch=torch.empty(64, dtype=torch.uint8, device=DEV))
    assert e.value.status == binding.VENOM_ERR_WORKSPACE


def test_layer_object_prunes_compresses_and_matches_the_oracle():
    """The layer object (paper's end-to-end section): dense weight -> magnitude pruning -> V:N:M ->
    y = act(x W^T + b), two calls with different token counts through the same object."""
    R, K, V, M = 256, 512, 128, 16
    rng = np.random.default_rng(77)
    W = rng.standard_normal((R, K)).astype(np.float16)
    bias = rng.standard_normal(R).astype(np.float16)
    layer = binding.Spmm.from_dense(torch.from_numpy(W).to(DEV), bias=torch.from_numpy(bias).to(DEV), V=V, N=2, M=M,
                                    activation="gelu")
    mask, _, _ = o.prune(W.view(np.uint16), V, M)
    ov, oc, om = o.compress(W.view(np.uint16), mask, V, M)
    for T in (264, 72):
        X = rng.standard_normal((T, K)).astype(np.float16)
        Y = layer(torch.from_numpy(X).to(DEV))
        Ys, Ey = o.linear_fp64(ov, oc, om, R, K, V, M, X.view(np.uint16), bias.view(np.uint16), "gelu")
        ok, info = o.accept(Y.double().cpu().numpy(), Ys, Ey)
        assert ok, (T, info)
