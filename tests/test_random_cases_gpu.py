"""Seeded random differential tests: random shapes, degree mixes, schedules (every plan option),
patterns and op tuples against the oracle.  Each case is small, but between them they hit the
thresholds from both sides (rows exactly at small_row_max / split_row_min / tile_row_min, chunk
lengths at multiples of 64 and 256, more column classes than columns, classes without entries)."""
import os

import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
PATTERNS = ("sigmoid", "one_minus_sigmoid", "gcn", "tdist", "fr")
# (binding names, binding AOP, oracle names, oracle AOP)
TUPLES = [
    (("MUL", "RSUM", "SCAL", "MUL_T"), "SUM", ("MUL", "RSUM", "SCAL", "MUL_T"), "ASUM"),
    (("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"), "MAX", ("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"), "AMAX"),
    (("SUB", "NOOP", "SIGMOID", "MUL_T"), "MIN", ("SUB", "NOOP", "SIGMOID", "MUL_T"), "AMIN"),
    (("ADD", "SUMSQ", "INV_1P", "SEL2ND"), "MAX", ("ADD", "SUMSQ", "INV1P", "SEL2ND"), "AMAX"),
    (("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"), "MEAN", ("SEL2ND", "NOOP", "EDGE_VALUE", "MUL_Y"), "AMEAN"),
    (("MUL", "RSUM", "SIGMOID", "MUL_Y"), "MEAN", ("MUL", "RSUM", "SIGMOID", "MUL_Y"), "AMEAN"),
]


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


ALPHA = float(np.float32(0.21))   # alpha travels as fp32 in the op struct: the oracle gets the same value


def make_case(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 400))
    n = int(rng.integers(1, 3000))
    opts = {
        "small_row_max": int(rng.choice([1, 2, 7, 16, 32, 33])),
        "split_row_min": int(rng.choice([16, 63, 64, 65, 256])),
        "chunk_edges": int(rng.choice([256, 512, 1024])),
        "column_classes": int(rng.choice([1, 8, 16, 64, 512])),
        "tile_row_min": int(rng.choice([8, 17, 64, 128])),
        "host_threads": int(rng.choice([0, 1, 3, 64])),
    }
    specials = [0, 1, opts["small_row_max"], opts["small_row_max"] + 1, opts["split_row_min"], opts["split_row_min"] + 1,
                opts["tile_row_min"] - 1, opts["tile_row_min"], 63, 64, 65, 255, 256, 257, 511, 512, 513, 1024, 1025, 2500]
    degs = np.where(rng.random(m) < 0.3, rng.choice(specials, m), rng.integers(0, 40, m))
    degs = np.where(rng.random(m) < 0.15, 0, degs).astype(np.int64)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(degs)
    nnz = int(rowptr[-1])
    if rng.random() < 0.5:  # columns concentrated in a narrow band: most classes stay empty
        lo = int(rng.integers(0, n))
        colidx = (lo + rng.integers(0, max(1, n // 7), nnz)) % n
    else:
        colidx = rng.integers(0, n, nnz)
    colidx = colidx.astype(np.int32)
    sorted_cols = rng.random() < 0.8
    if sorted_cols:
        for u in range(m):
            colidx[rowptr[u]:rowptr[u + 1]].sort()
    d = int(rng.choice([32, 64, 128, 256, 512, 32, 64, 128, 256, 512, 4, 36, 100, 200, 300, 508, 13, 50, 97, 301, 511, 768, 1024, 1433,
                        1, 2, 3, 5, 7, 8, 16, 24, 40, 96, 264, 600, 2048]))
    share = rng.random() < 0.3 and m <= n
    ld = d + int(rng.choice([0, 0, 4, 12, 1, 3]))     # rows need no alignment beyond one float
    Yb = rng.uniform(-0.7, 0.7, (n, ld)).astype(np.float32)
    Xb = Yb[:m] if share else rng.uniform(-0.7, 0.7, (m, ld)).astype(np.float32)
    vals = rng.uniform(-1, 1, max(1, nnz)).astype(np.float32)[:nnz]
    fmt = str(rng.choice(["f32", "f32", "bf16", "f16"]))
    if d % 8 != 0 or d > 1024 or ld % 8 != 0:
        # 2-byte storage of Y exists for multiples of 8 up to 1024 and 16-byte aligned rows; elsewhere every third case
        # that asked for it runs in double precision instead
        fmt = "f64" if fmt != "f32" and seed % 3 == 0 else "f32"
    if fmt in ("f32", "f64") and rng.random() < 0.1:
        opts["general_kernel_only"] = 1
    return m, n, d, rowptr, colidx, vals, Xb, Yb, share, opts, fmt


def rounded(Y, fmt):
    """Y as the kernel sees it after fusedmm_to_bf16 / fusedmm_to_f16 (round to nearest even)."""
    if fmt == "f16":
        return Y.astype(np.float16).astype(np.float32)
    u = np.ascontiguousarray(Y, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep, rest = u >> 16, u & 0xFFFF
    keep = keep + ((rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1)))
    return (keep.astype(np.uint32) << 16).view(np.float32)


@pytest.mark.parametrize("seed", range(int(os.environ.get("FUSEDMM_RANDOM_CASES", "150"))))
def test_random_case(B, seed):
    m, n, d, rowptr, colidx, vals, Xb, Yb, share, opts, fmt = make_case(1000 + seed)
    rng = np.random.default_rng(seed)
    X, Y = np.ascontiguousarray(Xb[:, :d]), np.ascontiguousarray(Yb[:, :d])
    if fmt in ("bf16", "f16"):
        Y = rounded(Y, fmt)          # x_u stays fp32 even where X and Y share storage
    if seed % 3 == 2:
        gnames, gaop, onames, oaop = TUPLES[(seed // 3) % len(TUPLES)]
        Zr, S, _ = oracle.unfused_general(rowptr, colidx, vals, X, Y, onames, oaop, alpha=ALPHA)
        ops = B.make_ops(*gnames, aop=gaop, alpha=ALPHA)
        what = f"{gnames}/{gaop}"
    else:
        pattern = PATTERNS[int(rng.integers(0, len(PATTERNS)))]
        Zr, S, _ = oracle.unfused(rowptr, colidx, vals, X, Y, pattern, alpha=ALPHA)
        ops = B.fusedmm_ops_preset(pattern)
        ops.alpha = ALPHA
        what = pattern
    rp = torch.from_numpy(rowptr).cuda()
    ci = torch.from_numpy(colidx).cuda()
    Yd = torch.from_numpy(Yb).cuda()
    Xd = Yd[:m] if share else torch.from_numpy(Xb).cuda()
    vd = torch.from_numpy(vals).cuda()
    Zb = torch.full((m, Yb.shape[1]), np.nan, dtype=torch.float32, device="cuda")
    plan = B.Plan(m, n, rp, ci, opts)
    plan.reserve(d)
    if fmt == "f64":
        plan.reserve_f64(d)
        Zb = torch.full((m, Yb.shape[1]), np.nan, dtype=torch.float64, device="cuda")
        Y64 = Yd.double()
        plan.execute_f64(ops, (Y64[:m] if share else Xd.double())[:, :d], Y64[:, :d], Zb[:, :d], vd.double())
    elif fmt == "f32":
        plan.execute(ops, Xd[:, :d], Yd[:, :d], Zb[:, :d], vd)
    else:
        Yh = torch.zeros((n, Yb.shape[1]), dtype=torch.int16, device="cuda")
        (B.fusedmm_to_bf16 if fmt == "bf16" else B.fusedmm_to_f16)(Yh, Yd, Yh.numel())
        (plan.execute_bf16y if fmt == "bf16" else plan.execute_f16y)(ops, Xd[:, :d], Yh[:, :d], Zb[:, :d], vd)
    torch.cuda.synchronize()
    out = Zb.cpu().numpy()
    err, am, viol = oracle.compare(out[:, :d], Zr, S)
    info = f"seed {seed} {what} {fmt} m={m} n={n} d={d} nnz={len(colidx)} opts={opts} stats={plan.stats()}"
    assert viol == 0, info
    assert err <= (1e-12 if fmt == "f64" else TOL), f"{info}: max rel err {err:.3e} at {am}"
    assert np.isnan(out[:, d:]).all(), info  # padding columns untouched
    counts = torch.zeros(max(1, len(colidx)), dtype=torch.int32, device="cuda")
    # the indexing of the kernel that ran: 0 = the general one, 1 = the fp32 schedule, 2 = its double-precision instances
    general = opts.get("general_kernel_only", 0)
    plan.edge_visits(d, 0 if general else (2 if fmt == "f64" else 1), counts)
    torch.cuda.synchronize()
    if len(colidx):
        c = counts[:len(colidx)].cpu().numpy()
        assert c.min() == 1 and c.max() == 1, info
    plan.close()
