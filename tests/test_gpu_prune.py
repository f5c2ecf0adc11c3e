"""GPU parity of venom_prune (magnitude pruning to V:N:M + the energy masses) against the oracle:
integer work, so everything is compared bit for bit."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vnm_oracle as o
from paper_2310_02065_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run(A_bits, V, M):
    A_d = torch.from_numpy(np.ascontiguousarray(A_bits).view(np.float16)).to(DEV)
    mask, kept, total = binding.venom_prune(A_d, V, 2, M)
    torch.cuda.synchronize()
    return A_d, mask, kept, total


@pytest.mark.parametrize("R,K,V,M", [(256, 256, 64, 8), (256, 384, 128, 32), (96, 360, 32, 10), (64, 1400, 32, 100),
                                     (128, 336, 64, 7), (64, 64, 16, 4), (8, 2048, 4, 1024), (130, 520, 13, 5)])
def test_mask_and_masses_match_the_oracle_bit_for_bit(R, K, V, M):
    rng = np.random.default_rng(R * 7 + M)
    A = (rng.standard_normal((R, K)) * 0.02).astype(np.float16).view(np.uint16)
    omask, okept, ototal = o.prune(A, V, M)
    _, mask, kept, total = run(A, V, M)
    assert np.array_equal(mask.cpu().numpy(), omask)
    assert sum(int(x) for x in kept.cpu().tolist()) == okept
    assert sum(int(x) for x in total.cpu().tolist()) == ototal
    assert abs(binding.venom_energy(kept, total) - okept / ototal) <= 2.0 ** -52 * (okept / ototal)


def test_ties_zeros_and_special_values():
    V, M = 8, 8
    A = np.zeros((16, 32), dtype=np.float16)
    A[:8, :8] = 1.0                                # all equal: smallest indices win
    A[:8, 8:16] = 0.0                              # all zero: still exactly two kept per row
    A[8:, :8] = np.float16(6e-8)                   # subnormals count
    A[8:, 5] = np.float16(1.2e-7)
    A[8:, 16:24] = 1.0
    A[9, 18] = np.inf                              # non-finite outranks everything
    A[10, 23] = np.nan
    A[11, 17] = -65504.0
    bits = A.view(np.uint16)
    omask, okept, ototal = o.prune(bits, V, M)
    _, mask, kept, total = run(bits, V, M)
    assert np.array_equal(mask.cpu().numpy(), omask)
    assert sum(int(x) for x in kept.cpu().tolist()) == okept and sum(int(x) for x in total.cpu().tolist()) == ototal
    assert (mask.cpu().numpy().reshape(16, 4, 8).sum(axis=2) == 2).all()


def test_strided_input_and_pipeline_into_compress_and_product():
    R, K, C, V, M = 256, 512, 128, 128, 16
    rng = np.random.default_rng(3)
    big = (rng.standard_normal((R, K + 24)) * 0.05).astype(np.float16)
    big_d = torch.from_numpy(big).to(DEV)
    A_d = big_d[:, 8:8 + K]                        # row stride K + 24
    mask, kept, total = binding.venom_prune(A_d, V, 2, M)
    A = np.ascontiguousarray(big[:, 8:8 + K]).view(np.uint16)
    omask, okept, ototal = o.prune(A, V, M)
    assert np.array_equal(mask.cpu().numpy(), omask)
    h = binding.venom_compress(A_d, mask, V, 2, M)   # legal by construction
    B = rng.standard_normal((K, C)).astype(np.float16)
    out = binding.venom_spmm(h, torch.from_numpy(B).to(DEV))
    ov, oc, om = o.compress(A, omask, V, M)
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B.view(np.uint16))
    ok, info = o.accept(out.double().cpu().numpy(), Cs, E)
    assert ok, info


def test_full_size_properties():
    # GPT-3 FFN-up sized matrix: too large for the oracle's loops; check what holds at any size
    R, K, V, M = 49152, 12288, 128, 32
    g = torch.Generator(device=DEV).manual_seed(20231002)
    A_d = (torch.randn((R, K), generator=g, device=DEV, dtype=torch.float32) * 0.02).to(torch.float16)
    mask, kept, total = binding.venom_prune(A_d, V, 2, M)
    torch.cuda.synchronize()
    per_group = mask.view(R, K // M, M).sum(dim=2, dtype=torch.int32)
    assert bool((per_group == 2).all())
    cols_used = (mask.view(R // V, V, K // M, M).sum(dim=1, dtype=torch.int32) > 0).sum(dim=2)
    assert bool((cols_used <= 4).all())
    # sampled block rows against the oracle: the mask and the exact integer masses of the whole block row
    for b in (0, 77, R // V - 1):
        rows = slice(b * V, (b + 1) * V)
        bits = A_d[rows].cpu().numpy().view(np.uint16)
        omask, okept, ototal = o.prune(bits, V, M)
        assert np.array_equal(mask[rows].cpu().numpy(), omask)
        assert int(kept[b]) == okept and int(total[b]) == ototal
    # the energy of the whole matrix is the ratio of the exact sums
    e = binding.venom_energy(kept, total)
    ek, et = sum(int(x) for x in kept.cpu().tolist()), sum(int(x) for x in total.cpu().tolist())
    assert abs(e - ek / et) <= 2.0 ** -52 * e
    # masses against a plain torch recomputation on the kept / all entries (fp64 sum of exact multiples of 2^-24)
    tot = float(A_d.abs().double().sum()) * 2.0 ** 24
    assert abs(tot - sum(int(x) for x in total.cpu().tolist())) <= 1e-9 * tot


def test_argument_errors():
    L = binding.lib()
    assert L.venom_prune(None, 8, 8, 8, 4, 2, 4, None, 8, None, None, None) == binding.VENOM_ERR_INVALID_ARG
    assert L.venom_prune(None, 8, 8, 9, 4, 2, 4, None, 8, None, None, None) == binding.VENOM_ERR_SHAPE
    assert L.venom_prune(None, 8, 8, 8, 4, 3, 4, None, 8, None, None, None) == binding.VENOM_ERR_UNSUPPORTED
