"""Y stored as bfloat16 or IEEE half (fusedmm_execute_bf16y / fusedmm_execute_f16y): the GPU must
compute, in fp32 arithmetic, the same function of the ROUNDED inputs as the oracle does in fp64.  The
rounding itself (fusedmm_to_bf16 / fusedmm_to_f16) is checked bit for bit against a round-to-nearest-even
written independently in numpy (bfloat16) and against numpy's own float16 conversion (half)."""
import numpy as np
import pytest

import oracle
from paper_2011_06391_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


def bf16_bits_rne(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep = u >> 16
    rest = u & 0xFFFF
    up = (rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1))
    return (keep + up).astype(np.uint16)


def widen(bits: np.ndarray) -> np.ndarray:
    return (bits.astype(np.uint32) << 16).view(np.float32)


def test_rounding_kernel_bit_exact(B):
    rng = np.random.default_rng(1)
    a = np.concatenate([(rng.normal(size=100000) * 10.0 ** rng.integers(-20, 20, 100000)).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38], np.float32)])
    # exact ties in both directions
    ties = (np.array([0x3F808000, 0x3F818000, 0xBF808000, 0xBF818000], dtype=np.uint32)).view(np.float32)
    a = np.concatenate([a, ties]).astype(np.float32)
    assert np.isfinite(a[:100000]).all()
    src = torch.from_numpy(a).cuda()
    dst = torch.zeros(len(a), dtype=torch.int16, device="cuda")
    B.fusedmm_to_bf16(dst, src, len(a))
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint16)
    np.testing.assert_array_equal(got, bf16_bits_rne(a))
    assert widen(got[-4:]).tolist() == [1.0, 1.015625, -1.0, -1.015625]  # ties go to the even neighbour
    nan = torch.tensor([float("nan")], device="cuda")
    out = torch.zeros(1, dtype=torch.int16, device="cuda")
    B.fusedmm_to_bf16(out, nan, 1)
    assert np.isnan(widen(out.cpu().numpy().view(np.uint16)))[0]


def test_half_rounding_kernel_bit_exact(B):
    rng = np.random.default_rng(2)
    a = np.concatenate([(rng.normal(size=100000) * 10.0 ** rng.integers(-9, 6, 100000)).astype(np.float32),
                        np.array([0.0, -0.0, 1.0, 65504.0, 65519.9, 65520.0, 1e6, -1e6, 6.0e-8, 5.96e-8, 2.9e-8, 3.1e-8,
                                  np.inf, -np.inf], np.float32),
                        # exact ties between neighbouring halves around 1.0 (spacing 2^-10)
                        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, -(1.0 + 2.0 ** -11)], np.float32)]).astype(np.float32)
    src = torch.from_numpy(a).cuda()
    dst = torch.zeros(len(a), dtype=torch.int16, device="cuda")
    B.fusedmm_to_f16(dst, src, len(a))
    torch.cuda.synchronize()
    got = dst.cpu().numpy().view(np.uint16)
    with np.errstate(over="ignore"):
        want = a.astype(np.float16).view(np.uint16)   # IEEE round to nearest even, subnormals kept, overflow to inf
    np.testing.assert_array_equal(got, want)
    assert got.view(np.float16)[-3:].tolist() == [1.0, 1.001953125, -1.0]
    nan = torch.tensor([float("nan")], device="cuda")
    out = torch.zeros(1, dtype=torch.int16, device="cuda")
    B.fusedmm_to_f16(out, nan, 1)
    assert np.isnan(out.cpu().numpy().view(np.float16))[0]


@pytest.mark.parametrize("d", (32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 16, 72, 136, 392, 600))
@pytest.mark.parametrize("pattern", ("one_minus_sigmoid", "gcn", "tdist", "general"))
def test_half_storage_parity(B, pattern, d):
    rng = np.random.default_rng(41 + d)
    g = synth.rmat(11, (1 << 10) * 24, seed=190 + d)
    m = n = g.m
    X = rng.uniform(-0.6, 0.6, (m, d)).astype(np.float32)
    Y = rng.uniform(-0.6, 0.6, (n, d)).astype(np.float32)
    Y[5, :4] = [1e-7, -3e-8, 6.2e-5, 70000.0]      # half subnormals and an overflow to infinity ...
    vals = rng.uniform(-1, 1, g.nnz).astype(np.float32)
    with np.errstate(over="ignore"):
        bits = Y.astype(np.float16).view(np.uint16)
    Yr = bits.view(np.float16).astype(np.float32)    # what the GPU will see
    assert np.isinf(Yr[5, 3])
    Yr[5, 3] = Y[5, 3] = 0.25                       # ... checked above as a conversion; keep the parity data finite
    bits = Yr.astype(np.float16).view(np.uint16)
    assert np.abs(Yr - Y).max() < 0.6 * 2 ** -11
    if pattern == "general":
        names, oaop, gaop = ("SUB", "NOOP", "SIGMOID", "MUL_Y"), "AMEAN", "MEAN"
        Zr, S, _ = oracle.unfused_general(g.rowptr, g.colidx, vals, X, Yr, names, oaop, alpha=0.3)
        ops = B.make_ops(*names, aop=gaop, alpha=0.3)
    else:
        Zr, S, _ = oracle.unfused(g.rowptr, g.colidx, vals, X, Yr, pattern, alpha=0.3)
        ops = B.fusedmm_ops_preset(pattern)
        ops.alpha = 0.3
    rp, ci = torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda()
    Xd, Yd, vd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), torch.from_numpy(vals).cuda()
    Yh = torch.zeros((n, d), dtype=torch.int16, device="cuda")
    B.fusedmm_to_f16(Yh, Yd, n * d)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Yh.cpu().numpy().view(np.uint16), bits)
    for options in ({"column_classes": 1}, {"column_classes": 16, "tile_row_min": 64, "split_row_min": 128}):
        plan = B.Plan(m, n, rp, ci, options)
        plan.reserve(d)
        Z = torch.full((m, d), float("nan"), dtype=torch.float32, device="cuda")
        plan.execute_f16y(ops, None if pattern == "gcn" else Xd, Yh, Z, vd)
        torch.cuda.synchronize()
        err, am, viol = oracle.compare(Z.cpu().numpy(), Zr, S)
        assert viol == 0 and err <= TOL, f"{pattern} d={d} {options}: err {err:.3e} at {am}, viol {viol}"
        Z32 = torch.empty_like(Z)
        plan.execute(ops, None if pattern == "gcn" else Xd, torch.from_numpy(Yr).cuda(), Z32, vd)
        torch.cuda.synchronize()
        # the fp32 entry point on the widened matrix computes the same sums in another order
        e32, _, _ = oracle.compare(Z.cpu().numpy(), Z32.cpu().numpy().astype(np.float64), S)
        assert e32 <= TOL
        plan.close()


@pytest.mark.parametrize("d", (32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 8, 16, 24, 40, 80, 200, 264, 504, 600))
@pytest.mark.parametrize("pattern", ("one_minus_sigmoid", "gcn", "tdist", "fr", "general"))
def test_bf16_storage_parity(B, pattern, d):
    rng = np.random.default_rng(31 + d)
    g = synth.rmat(11, (1 << 10) * 24, seed=90 + d)   # skewed: packed rows, wave rows, chunks, tiles
    m = n = g.m
    X = rng.uniform(-0.6, 0.6, (m, d)).astype(np.float32)
    Y = rng.uniform(-0.6, 0.6, (n, d)).astype(np.float32)
    vals = rng.uniform(-1, 1, g.nnz).astype(np.float32)
    bits = bf16_bits_rne(Y)
    Yr = widen(bits)                       # what the GPU will see
    assert np.abs(Yr - Y).max() < 0.6 * 2 ** -8
    if pattern == "general":
        onames, oaop, gnames, gaop = ("SUB", "NOOP", "SIGMOID", "MUL_Y"), "AMAX", ("SUB", "NOOP", "SIGMOID", "MUL_Y"), "MAX"
        Zr, S, _ = oracle.unfused_general(g.rowptr, g.colidx, vals, X, Yr, onames, oaop, alpha=0.3)
        ops = B.make_ops(*gnames, aop=gaop, alpha=0.3)
    else:
        Zr, S, _ = oracle.unfused(g.rowptr, g.colidx, vals, X, Yr, pattern, alpha=0.3)
        ops = B.fusedmm_ops_preset(pattern)
        ops.alpha = 0.3
    rp, ci = torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda()
    Xd, Yd, vd = torch.from_numpy(X).cuda(), torch.from_numpy(Y).cuda(), torch.from_numpy(vals).cuda()
    Yb = torch.zeros((n, d), dtype=torch.int16, device="cuda")
    B.fusedmm_to_bf16(Yb, Yd, n * d)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(Yb.cpu().numpy().view(np.uint16), bits)
    for options in ({"column_classes": 1}, {"column_classes": 16, "tile_row_min": 64, "split_row_min": 128}):
        plan = B.Plan(m, n, rp, ci, options)
        plan.reserve(d)
        Z = torch.full((m, d), float("nan"), dtype=torch.float32, device="cuda")
        plan.execute_bf16y(ops, None if pattern == "gcn" else Xd, Yb, Z, vd)
        torch.cuda.synchronize()
        err, am, viol = oracle.compare(Z.cpu().numpy(), Zr, S)
        assert viol == 0 and err <= TOL, f"{pattern} d={d} {options}: err {err:.3e} at {am}, viol {viol}"
        # the fp32 entry point on the widened matrix computes the same sums in another order
        Z32 = torch.empty_like(Z)
        plan.execute(ops, None if pattern == "gcn" else Xd, torch.from_numpy(Yr).cuda(), Z32, vd)
        torch.cuda.synchronize()
        e32, _, _ = oracle.compare(Z.cpu().numpy(), Z32.cpu().numpy().astype(np.float64), S)
        assert e32 <= TOL
        plan.close()


@pytest.mark.parametrize("d,ld", ((40, 48), (8, 16), (200, 256), (264, 272)))
def test_two_byte_rows_narrower_than_their_pitch(B, d, ld):
    """Rows of Y that are d elements wide in a matrix ld apart, with NaN in every element beyond d (and X, Z
    likewise wider than d): nothing beyond d may be read into the result or written."""
    rng = np.random.default_rng(7 + d)
    g = synth.rmat(11, (1 << 10) * 24, seed=400 + d)
    m = n = g.m
    X = rng.uniform(-0.6, 0.6, (m, d)).astype(np.float32)
    Y = (rng.uniform(0.05, 0.6, (n, d)) * rng.choice((-1.0, 1.0), (n, d))).astype(np.float32)
    Y = widen(bf16_bits_rne(Y))   # exactly representable in bfloat16, and (away from zero) in half as well
    Zr, S, _ = oracle.unfused(g.rowptr, g.colidx, None, X, Y, "sigmoid")
    rp, ci = torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda()
    Xw = torch.full((m, ld), float("nan"), dtype=torch.float32, device="cuda")
    Xw[:, :d] = torch.from_numpy(X).cuda()
    Zw = torch.full((m, ld), 7.0, dtype=torch.float32, device="cuda")
    ops = B.fusedmm_ops_preset("sigmoid")
    for fmt, entry in (("bf16", B.fusedmm_execute_bf16y), ("f16", B.fusedmm_execute_f16y)):
        if fmt == "bf16":
            Yw = torch.full((n, ld), 0x7FC0, dtype=torch.int16, device="cuda")          # bfloat16 NaN
            Yw[:, :d] = torch.from_numpy(bf16_bits_rne(Y).view(np.int16)).cuda()
        else:
            Yw = torch.full((n, ld), 0x7E00, dtype=torch.int16, device="cuda")          # half NaN
            Yw[:, :d] = torch.from_numpy(Y.astype(np.float16).view(np.int16)).cuda()   # bfloat16 values fit half here
            assert np.array_equal(Y.astype(np.float16).astype(np.float32), Y)
        for options in ({"column_classes": 1}, {"column_classes": 16, "tile_row_min": 64, "split_row_min": 128}):
            plan = B.Plan(m, n, rp, ci, options)
            plan.reserve(d)
            Zw.fill_(7.0)
            entry(plan._plan, ops, d, None, Xw, ld, Yw, ld, Zw, ld)
            torch.cuda.synchronize()
            out = Zw.cpu().numpy()
            assert (out[:, d:] == 7.0).all(), f"{fmt} d={d}: written beyond d"
            err, am, viol = oracle.compare(out[:, :d].copy(), Zr, S)
            assert viol == 0 and err <= TOL, f"{fmt} d={d} ld={ld} {options}: err {err:.3e} at {am}, viol {viol}"
            plan.close()


def test_bf16_argument_checks(B):
    g = synth.rmat(8, 1024, seed=3)
    rp, ci = torch.from_numpy(g.rowptr).cuda(), torch.from_numpy(g.colidx).cuda()
    plan = B.Plan(g.m, g.n, rp, ci)
    ops = B.fusedmm_ops_preset("sigmoid")
    for d, ld, expect in ((44, 48, B.FUSEDMM_ERR_UNSUPPORTED_DIM), (1032, 1032, B.FUSEDMM_ERR_UNSUPPORTED_DIM),
                          (64, 66, B.FUSEDMM_ERR_INVALID_ARG), (48, 52, B.FUSEDMM_ERR_INVALID_ARG)):
        X = torch.zeros((g.m, d), dtype=torch.float32, device="cuda")
        Yb = torch.zeros((g.n, ld), dtype=torch.int16, device="cuda")
        Z = torch.zeros((g.m, d), dtype=torch.float32, device="cuda")
        for entry in (B.fusedmm_execute_bf16y, B.fusedmm_execute_f16y):
            with pytest.raises(B.FusedMMError) as ei:
                entry(plan._plan, ops, d, None, X, d, Yb, ld, Z, d)
            assert ei.value.status == expect
    plan.close()
