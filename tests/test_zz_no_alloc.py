"""venom_linear_static (the entry point that allocates nothing: its scratch is a static device array
inside the library) against venom_linear with caller-owned scratch, through the C ABI: two calls
in a row, the second with a smaller input, so stale contents of the shared array would show."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2310_02065_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def layer(R, K, V, M, seed):
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=seed)
    return binding.venom_compress(torch.from_numpy(A.view(np.float16)).to(DEV), torch.from_numpy(mask).to(DEV), V, 2, M)


def test_static_scratch_matches_caller_scratch_on_two_calls_in_a_row():
    rng = np.random.default_rng(11)
    # (R, K, tokens, V, M): a multi-tile layer with a ragged column edge, then a smaller one
    for R, K, T, V, M, act, dt in [(512, 2048, 1096, 128, 16, "gelu", torch.float16),
                                   (256, 640, 136, 64, 8, "none", torch.float32)]:
        h = layer(R, K, V, M, 100 + T)
        X = torch.from_numpy(rng.standard_normal((T, K)).astype(np.float16)).to(DEV)
        bias = torch.from_numpy(rng.standard_normal(R).astype(np.float16)).to(DEV)
        want = binding.venom_linear(h, X, bias=bias, activation=act, out_dtype=dt)
        got = torch.full((T, R), float("nan"), dtype=dt, device=DEV)
        binding.venom_linear_static(h, X, got, bias=bias, activation=act)
        torch.cuda.synchronize()
        assert torch.equal(got, want), (R, K, T)


def test_static_scratch_rejects_sizes_beyond_the_array():
    limit = binding.venom_linear_static_max_bytes()
    assert limit == 64 << 20
    R, K, V, M = 64, 4096, 32, 8
    h = layer(R, K, V, M, 5)
    T = limit // (2 * K) + 8                      # K * T * 2 bytes just beyond the array
    X = torch.zeros((T, K), dtype=torch.float16, device=DEV)
    out = torch.empty((T, R), dtype=torch.float16, device=DEV)
    with pytest.raises(binding.VenomError) as e:
        binding.venom_linear_static(h, X, out)
    assert e.value.status == binding.VENOM_ERR_WORKSPACE
    T = limit // (2 * K)                          # exactly the array: accepted
    X = torch.zeros((T, K), dtype=torch.float16, device=DEV)
    out = torch.full((T, R), 1.0, dtype=torch.float16, device=DEV)
    binding.venom_linear_static(h, X, out)
    torch.cuda.synchronize()
    assert bool((out == 0).all())
