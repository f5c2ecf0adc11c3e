"""GPU parity of the product (venom_spmm) against the fp64 CPU oracle on the same seeded inputs.

Tolerance (stated by the benchmark spec, derived from fp16 inputs with fp32 accumulation and one rounding
to fp16): |C - C*| <= 1e-2 * (|A|.|B|) elementwise and ||C - C*||_F <= 1e-3 * ||C*||_F."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import vnm_oracle as o
from paper_2310_02065_amd import binding, inputs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_dev_f16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.float16)).to(DEV)


def compress_dev(A, mask, V, M):
    return binding.venom_compress(to_dev_f16(A), torch.from_numpy(mask).to(DEV), V, 2, M)


def check(C_dev, Cs, E):
    ok, info = o.accept(C_dev.double().cpu().numpy(), Cs, E)
    assert ok, info
    return info


def variants_for(V, M=None, R=None):
    """Tile variants that serve a matrix of block height V.  At M = 4 every block selects all four
    columns, so the library packs the matrix 128 rows high whenever R allows, whatever V is."""
    if M == 4 and R is not None and R % 128 == 0:
        V = 128
    names = binding.venom_spmm_variants()
    return [i for i, n in enumerate(names) if n.startswith(f"v{V}_")]


CASES = [
    # R, K, C, V, M          several tiles in every dimension, ragged column tails, odd step counts
    (256, 256, 64, 64, 8),            # the tiny config (C narrower than any tile)
    (256, 384, 264, 128, 8),          # C = one full tile + 8 columns
    (384, 1280, 520, 128, 32),        # 3 block rows, G = 40 (5 k-steps, odd)
    (192, 896, 136, 64, 16),          # G = 56 (7 k-steps)
    (128, 720, 72, 32, 10),           # 2:10, G = 72
    (64, 1400, 40, 32, 100),          # 2:100, G = 14: ragged last k-step
    (128, 336, 96, 64, 7),            # 2:7, G = 48
    (256, 64, 128, 128, 4),           # plain 2:4, G = 16
    (512, 200, 520, 128, 4),          # plain 2:4, G = 50 (ragged)
    (256, 96, 264, 64, 4),            # plain 2:4 at V = 64, R a multiple of 128: runs on the 128-row tiles
    (256, 136, 72, 32, 4),            # the same at V = 32
    (192, 64, 72, 64, 4),             # plain 2:4 at V = 64 where R is not a multiple of 128: 64-row tiles
    (384, 64, 72, 128, 4),            # three block rows
    (192, 512, 136, 96, 8),           # V = 96 (three 32-row tiles), two block rows
]


@pytest.mark.parametrize("R,K,C,V,M", CASES)
@pytest.mark.parametrize("out_dtype", [torch.float16, torch.float32])
def test_spmm_matches_oracle_all_variants(R, K, C, V, M, out_dtype):
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=500 + R + K + M)
    h = compress_dev(A, mask, V, M)
    ov, oc, om = o.compress(A, mask, V, M)
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B)
    Bd = to_dev_f16(B)
    for var in [-1] + variants_for(V, M, R):
        out = torch.full((R, C), float("nan"), dtype=out_dtype, device=DEV)
        binding.venom_spmm(h, Bd, out=out, variant=var)
        torch.cuda.synchronize()
        check(out, Cs, E)


def test_identity_B_reproduces_expanded_matrix_exactly():
    # products by 1 and sums with 0 are exact in any precision: pins gather + decode bit for bit
    R, K, V, M = 256, 512, 128, 16
    A, mask, _ = inputs.gen_problem(R, K, 8, V, M, 1.0, seed=3)
    h = compress_dev(A, mask, V, M)
    eye = torch.eye(K, dtype=torch.float16, device=DEV)
    want = np.where(mask != 0, A, 0).astype(np.uint16)
    for var in [-1] + variants_for(V, M, R):
        out = binding.venom_spmm(h, eye, variant=var)
        torch.cuda.synchronize()
        got = out.cpu().numpy().view(np.uint16)
        # -0 * 1 + 0 = +0 in the accumulator: compare numerically equal bit patterns modulo the sign of zero
        assert np.array_equal(np.where(got == 0x8000, 0, got), np.where(want == 0x8000, 0, want))


def test_all_ones_counts():
    R, K, C, V, M = 128, 1024, 64, 64, 32
    _, mask, _ = inputs.gen_problem(R, K, C, V, M, 1.0, seed=4)
    ones = np.ones((R, K), np.float16).view(np.uint16)
    h = compress_dev(ones, mask, V, M)
    out = binding.venom_spmm(h, torch.ones((K, C), dtype=torch.float16, device=DEV), out_dtype=torch.float32)
    torch.cuda.synchronize()
    assert (out == 2 * K // M).all()


def test_strided_B_and_C_and_repeatability():
    R, K, C, V, M = 256, 512, 200, 64, 8
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=8)
    h = compress_dev(A, mask, V, M)
    ov, oc, om = o.compress(A, mask, V, M)
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B)
    Bbig = torch.randn((K, C + 56), dtype=torch.float16, device=DEV)
    Bbig[:, :C] = to_dev_f16(B)
    Cbig = torch.full((R, C + 24), 7.0, dtype=torch.float16, device=DEV)
    binding.venom_spmm(h, Bbig[:, :C], out=Cbig[:, :C])
    torch.cuda.synchronize()
    check(Cbig[:, :C], Cs, E)
    assert (Cbig[:, C:] == 7.0).all()          # nothing written past the logical width
    again = torch.empty_like(Cbig)
    binding.venom_spmm(h, Bbig[:, :C], out=again[:, :C])
    torch.cuda.synchronize()
    assert torch.equal(again[:, :C], Cbig[:, :C])   # bitwise repeatable


def test_argument_errors():
    R, K, C, V, M = 64, 64, 64, 32, 8
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=2)
    h = compress_dev(A, mask, V, M)
    Bd = to_dev_f16(B)
    with pytest.raises(binding.VenomError) as e:      # C_cols not a multiple of 8
        binding.venom_spmm(h, Bd[:, :60].contiguous())
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED
    with pytest.raises(binding.VenomError) as e:      # misaligned B
        binding.venom_spmm(h, Bd[:, 4:60])
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED
    with pytest.raises(binding.VenomError) as e:      # a variant built for another V
        binding.venom_spmm(h, Bd, variant=[i for i, n in enumerate(binding.venom_spmm_variants()) if n.startswith("v128_")][0])
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED
    h8 = compress_dev(*inputs.gen_problem(40, 48, 8, 8, 6, 1.0, seed=1)[:2], 8, 6)
    with pytest.raises(binding.VenomError) as e:      # V not a multiple of 32
        binding.venom_spmm(h8, torch.zeros((48, 8), dtype=torch.float16, device=DEV))
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED


@pytest.mark.parametrize("activation", ["none", "gelu", "gelu_tanh"])
@pytest.mark.parametrize("out_dtype", [torch.float16, torch.float32])
@pytest.mark.parametrize("R,K,C,V,M", [(256, 384, 264, 128, 8), (192, 896, 136, 64, 16), (128, 720, 72, 32, 10),
                                       (256, 128, 264, 128, 4)])
def test_fused_bias_and_activation(R, K, C, V, M, out_dtype, activation):
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=900 + R + M)
    rng = np.random.default_rng(77 + R)
    bias = rng.standard_normal(R).astype(np.float16)
    h = compress_dev(A, mask, V, M)
    ov, oc, om = o.compress(A, mask, V, M)
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B)
    for with_bias in (True, False):
        if not with_bias and activation == "none":
            continue                      # the plain product is covered above
        Ys, Ey = o.epilogue_fp64(Cs, E, bias.view(np.uint16) if with_bias else None, activation)
        bias_d = torch.from_numpy(bias).to(DEV) if with_bias else None
        for v in variants_for(V, M, R):
            out = binding.venom_spmm(h, to_dev_f16(B), out_dtype=out_dtype, variant=v, bias=bias_d,
                                     activation=activation)
            ok, info = o.accept(out.float().cpu().numpy().astype(np.float64), Ys, Ey)
            assert ok, (binding.venom_spmm_variants()[v], with_bias, info)


def test_zero_product_returns_activation_of_bias_exactly_in_fp32():
    R, K, C, V, M = 128, 256, 64, 128, 8
    A, mask, _ = inputs.gen_problem(R, K, C, V, M, 1.0, seed=11)
    h = compress_dev(A, mask, V, M)
    B0 = torch.zeros((K, C), dtype=torch.float16, device=DEV)
    bias = np.linspace(-3, 3, R).astype(np.float16)
    out = binding.venom_spmm(h, B0, out_dtype=torch.float32, bias=torch.from_numpy(bias).to(DEV))
    assert np.array_equal(out.cpu().numpy(), np.repeat(bias.astype(np.float32)[:, None], C, axis=1))
    outg = binding.venom_spmm(h, B0, out_dtype=torch.float32, bias=torch.from_numpy(bias).to(DEV), activation="gelu")
    ref = o.gelu_erf(bias.astype(np.float64))
    assert np.abs(outg.cpu().numpy()[:, 0] - ref).max() < 2e-6
    assert (outg.cpu().numpy() == outg.cpu().numpy()[:, :1]).all()


def test_epilogue_argument_errors():
    R, K, C, V, M = 64, 64, 64, 32, 8
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=5)
    h = compress_dev(A, mask, V, M)
    out = torch.empty((R, C), dtype=torch.float16, device=DEV)
    L = binding.lib()
    import ctypes
    st = L.venom_spmm_bias_act(h.ptr, ctypes.c_void_p(to_dev_f16(B).data_ptr()), C, C, None, 7,
                               ctypes.c_void_p(out.data_ptr()), C, 0, -1, None)
    assert st == binding.VENOM_ERR_INVALID_ARG
    bias = torch.zeros(R + 8, dtype=torch.float16, device=DEV)
    st = L.venom_spmm_bias_act(h.ptr, ctypes.c_void_p(to_dev_f16(B).data_ptr()), C, C,
                               ctypes.c_void_p(bias.data_ptr() + 2), 0, ctypes.c_void_p(out.data_ptr()), C, 0, -1, None)
    assert st == binding.VENOM_ERR_UNSUPPORTED


def test_nonexistent_trailing_groups_never_touch_B():
    # K/M = 14 groups: the last k-step of every tile has 2 padded groups, whose gathered rows are
    # placeholders.  Whatever sits in B at the placeholder row (row 0) must not leak into C.
    R, K, C, V, M = 64, 1400, 136, 32, 100
    for seed in range(50):
        A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=seed)
        if not mask[:, 0].any():
            break
    else:
        pytest.skip("no seed leaves column 0 unused")
    Bh = B.view(np.float16).copy()
    Bh[0, :] = np.inf
    Bh[0, 1::2] = np.nan
    h = compress_dev(A, mask, V, M)
    ov, oc, om = o.compress(A, mask, V, M)
    B0 = Bh.copy()
    B0[0, :] = 0                                        # row 0 is not selected: the product ignores it
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B0.view(np.uint16))
    for v in variants_for(V):
        for dt in (torch.float16, torch.float32):
            out = binding.venom_spmm(h, torch.from_numpy(Bh).to(DEV), out_dtype=dt, variant=v)
            assert bool(torch.isfinite(out).all()), binding.venom_spmm_variants()[v]
            check(out, Cs, E)


def test_product_replays_inside_a_captured_graph():
    # venom_spmm allocates nothing and clears nothing, so it can be captured; every replay is
    # compared with the eager result, with eager work and synchronisations in between.
    R, K, C, V, M = 384, 1280, 520, 128, 32
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=61)
    h = compress_dev(A, mask, V, M)
    B_d = to_dev_f16(B)
    bias = torch.randn(R, device=DEV).half()
    eager = binding.venom_spmm(h, B_d, bias=bias, activation="gelu")      # also the first-launch set-up
    eager_plain = binding.venom_spmm(h, B_d)
    out = torch.empty_like(eager)
    out_plain = torch.empty_like(eager)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        binding.venom_spmm(h, B_d, out=out, bias=bias, activation="gelu")
        binding.venom_spmm(h, B_d, out=out_plain)
    for rep in range(4):
        out.fill_(float("nan"))
        out_plain.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, eager) and torch.equal(out_plain, eager_plain), rep
        again = binding.venom_spmm(h, B_d)                                 # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(again, eager_plain)


def test_runs_on_the_stream_it_is_given():
    R, K, C, V, M = 256, 512, 264, 128, 16
    A, mask, B = inputs.gen_problem(R, K, C, V, M, 1.0, seed=71)
    side = torch.cuda.Stream()                       # default priority
    B_d = to_dev_f16(B)
    A_d = to_dev_f16(A)
    m_d = torch.from_numpy(mask).to(DEV)
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        h = binding.venom_compress(A_d, m_d, V, 2, M)          # uses the current (side) stream
        out = binding.venom_spmm(h, B_d)
        gate = torch.cuda.Event()
        gate.record(side)
    # an explicit stream argument, while another stream is current
    out2 = torch.empty_like(out)
    binding.venom_spmm(h, B_d, out=out2, stream=side)
    side.synchronize()
    ov, oc, om = o.compress(A, mask, V, M)
    Cs, E = o.spmm_fp64(ov, oc, om, R, K, V, M, B)
    check(out, Cs, E)
    assert torch.equal(out, out2)


def test_k_equal_zero_is_refused_not_run():
    A = torch.zeros((128, 0), dtype=torch.float16, device=DEV)
    mask = torch.zeros((128, 0), dtype=torch.uint8, device=DEV)
    h = binding.venom_compress(A, mask, 128, 2, 8)
    out = torch.full((128, 64), 3.0, dtype=torch.float16, device=DEV)
    with pytest.raises(binding.VenomError) as e:
        binding.venom_spmm(h, torch.zeros((0, 64), dtype=torch.float16, device=DEV), out=out)
    assert e.value.status == binding.VENOM_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())


def test_matrix_instruction_probe_runs():
    sink = torch.zeros(1, dtype=torch.float32, device=DEV)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    binding.venom_probe_smfmac_rate(200, sink)
    a.record()
    binding.venom_probe_smfmac_rate(2000, sink)
    b.record()
    torch.cuda.synchronize()
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    tflops = 2000 * 8 * 32768 * 16 * cus / (a.elapsed_time(b) * 1e-3) / 1e12
    assert 500 < tflops < 2600, tflops      # useful FLOP/s of the instruction alone: below the 2.5 PFLOP/s spec peak
