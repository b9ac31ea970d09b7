"""Every valid op tuple of the selector (4 VOP x 26 valid ROP/SOP pairs x 3 MOP x 4 AOP = 1248) against the
oracle, on a small pattern that reaches every bin of the schedule, at dimensions with instances of their own
(32, 128), between instance sizes on the masked instances (20; 6, 13, 27, 97, 301: rows that end inside a
16-byte piece; 700 on the 1024 instance, 1100 on the 2048 instance), two of the one-lane-per-entry kernels (2, 3), on the
general kernel (6, 27, 97, 128 with the plan told to use nothing else: its lane-group widths and register counts), with Y stored as bfloat16 / half
(narrow loads at 32, wide ones at 64 and 128), and in double precision on the specialised schedule (32, 256, and
20 on the masked instance; bound 1e-12).  A dispatch slip -- a tuple
recognised as a pattern it is not, a step skipped at run time -- cannot hide among hand-picked cases."""
import itertools

import numpy as np
import pytest

import oracle

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-4
TOL64 = 1e-12
ALPHA = float(np.float32(0.37))   # alpha travels as fp32 in the op struct: the oracle gets the same value
ONAME = {"NORM2": "NORM", "INV_1P": "INV1P"}
OAOP = {"SUM": "ASUM", "MAX": "AMAX", "MIN": "AMIN", "MEAN": "AMEAN"}


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


def all_valid_tuples(B):
    for vop, rop, sop, mop, aop in itertools.product(B.VOP, B.ROP, B.SOP, B.MOP, B.AOP):
        if (sop == "EDGE_VALUE") and rop != "NOOP":
            continue
        yield vop, rop, sop, mop, aop


def rounded(Y, fmt):
    if fmt == "f16":
        return Y.astype(np.float16).astype(np.float32)
    if fmt == "bf16":
        u = np.ascontiguousarray(Y, dtype=np.float32).view(np.uint32).astype(np.uint64)
        keep, rest = u >> 16, u & 0xFFFF
        keep = keep + ((rest > 0x8000) | ((rest == 0x8000) & ((keep & 1) == 1)))
        return (keep.astype(np.uint32) << 16).view(np.float32)
    return Y


@pytest.mark.parametrize("d,fmt", [(32, "f32"), (20, "f32"), (6, "f32"), (128, "f32"), (32, "bf16"), (64, "f16"),
                                   (128, "bf16"), (128, "f16"),
                                   # rows that end inside a 16-byte piece (ragged instances), the 1024 instance at 700,
                                   # the 2048 instance at 1100
                                   (2, "f32"), (3, "f32"), (13, "f32"), (27, "f32"), (97, "f32"), (301, "f32"),
                                   (700, "f32"), (1100, "f32"), (32, "f64"), (20, "f64"), (256, "f64"),
                                   # the general kernel at dimensions the wide kernels would take
                                   (6, "general"), (27, "general"), (97, "general"), (128, "general")])
def test_every_valid_tuple(B, d, fmt):
    rng = np.random.default_rng(2024 + d)
    m, n = 48, 90
    degs = rng.integers(0, 9, m)
    degs[[0, 7]] = 0
    degs[5], degs[20], degs[33], degs[47] = 40, 70, 300, 600     # wave rows, chunks, tiles under the options below
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(degs)
    colidx = rng.integers(0, n, rowptr[-1]).astype(np.int32)
    for u in range(m):
        colidx[rowptr[u]:rowptr[u + 1]].sort()
    vals = rng.uniform(-1.0, 1.0, len(colidx)).astype(np.float32)
    # x - y >= 0 and everything positive: no scaling step comes near the pole of 1/(1+s)
    Xs = rng.uniform(0.30, 0.50, (m, d)).astype(np.float32)
    Ys = rng.uniform(0.05, 0.25, (n, d)).astype(np.float32)
    # ROP = RMUL: the product of d factors must stay inside fp32's normal range for every VOP, so that it is
    # compared as a number.  Up to d = 32 one pair of matrices does (factors near 1 for SEL2ND and SUB, 2 for
    # MUL, 3 for ADD); for longer rows every VOP gets operands that put its own factors near 1.
    if d <= 32:
        Xp = rng.uniform(1.9, 2.1, (m, d)).astype(np.float32)
        Yp = rng.uniform(0.9, 1.1, (n, d)).astype(np.float32)
        rmul_sets = {v: ("Xp", "Yp") for v in B.VOP}
        mats = {"Xp": Xp, "Yp": Yp}
    else:
        mats = {"Xone": rng.uniform(0.98, 1.02, (m, d)).astype(np.float32),     # MUL: x * y near 1 (SEL2ND: y)
                "Xtwo": rng.uniform(1.98, 2.02, (m, d)).astype(np.float32),     # SUB: x - y near 1
                "Xhalf": rng.uniform(0.49, 0.51, (m, d)).astype(np.float32),    # ADD: x + y near 1
                "Yone": rng.uniform(0.98, 1.02, (n, d)).astype(np.float32),
                "Yhalf": rng.uniform(0.49, 0.51, (n, d)).astype(np.float32)}
        rmul_sets = {"MUL": ("Xone", "Yone"), "SEL2ND": ("Xone", "Yone"), "SUB": ("Xtwo", "Yone"), "ADD": ("Xhalf", "Yhalf")}
    mats["Xs"] = Xs
    mats["Ys"] = Ys
    for k in [k for k in mats if k.startswith("Y")]:
        mats[k] = rounded(mats[k], fmt)      # what the kernels see when Y is stored in 2 bytes
    rp, ci, vd = (torch.from_numpy(a).cuda() for a in (rowptr, colidx, vals))
    dev = {k: torch.from_numpy(v).cuda() for k, v in mats.items()}
    general = fmt == "general"
    if general:
        fmt = "f32"
    plan = B.Plan(m, n, rp, ci, {"small_row_max": 4, "split_row_min": 32, "chunk_edges": 256, "column_classes": 8,
                                 "tile_row_min": 64, "feature_dim_hint": d, "general_kernel_only": int(general)})
    plan.reserve(d)
    st = plan.stats()
    assert st["tiled_rows"] > 0 and st["wave_rows"] > 0 and st["packed_rows"] > 0
    Z = torch.empty((m, d), dtype=torch.float64 if fmt == "f64" else torch.float32, device="cuda")
    if fmt == "f64":
        plan.reserve_f64(d)
        dev64 = {k: v.double() for k, v in dev.items()}
        vd64 = vd.double()
    elif fmt != "f32":
        for k in [k for k in mats if k.startswith("Y")]:
            h = torch.zeros((n, d), dtype=torch.int16, device="cuda")
            (B.fusedmm_to_bf16 if fmt == "bf16" else B.fusedmm_to_f16)(h, dev[k], n * d)
            dev[k + "h"] = h
    failures, count = [], 0
    for vop, rop, sop, mop, aop in all_valid_tuples(B):
        xk, yk = rmul_sets[vop] if rop == "RMUL" else ("Xs", "Ys")
        X, Y, Xd, Yd = mats[xk], mats[yk], dev[xk], dev[yk]
        names = (vop, ONAME.get(rop, rop), ONAME.get(sop, sop), mop)
        Zr, S, _ = oracle.unfused_general(rowptr, colidx, vals, X, Y, names, OAOP[aop], alpha=ALPHA)
        ops = B.make_ops(vop, rop, sop, mop, aop=aop, alpha=ALPHA)
        Z.fill_(float("nan"))
        Xarg = None if vop == "SEL2ND" else Xd
        if fmt == "f32":
            plan.execute(ops, Xarg, Yd, Z, vd)
        elif fmt == "f64":
            plan.execute_f64(ops, None if vop == "SEL2ND" else dev64[xk], dev64[yk], Z, vd64)
        else:
            Yh = dev[yk + "h"]
            (plan.execute_bf16y if fmt == "bf16" else plan.execute_f16y)(ops, Xarg, Yh, Z, vd)
        torch.cuda.synchronize()
        Zg = Z.cpu().numpy()
        # results below fp32's range (a sigmoid of several hundred): the double oracle still holds 1e-200,
        # fp32 holds 0; there the rule is "nothing but such a tiny number", not a relative error
        tiny = S < 1e-30
        assert (np.abs(Zg[tiny]) <= 1e-30).all()
        # the product itself is always a normal number here: compared as such, never as 0 = 0 (short rows with
        # factors 2 and 3 reach products of hundreds, whose 1 - sigmoid is legitimately below fp32's range)
        if rop == "RMUL" and (d > 32 or sop != "ONE_MINUS_SIGMOID"):
            assert not (tiny & (S > 0)).any(), (vop, rop, sop, mop, aop)
        S = np.where(tiny, 0.0, S)
        Zg = np.where(tiny, 0.0, Zg)
        Zr = np.where(tiny, 0.0, Zr)
        err, am, viol = oracle.compare(Zg if fmt == "f64" else Zg.astype(np.float32), Zr, S)
        count += 1
        if viol != 0 or not err <= (TOL64 if fmt == "f64" else TOL):
            failures.append(f"{(vop, rop, sop, mop, aop)}: err {err:.3e} at {am}, viol {viol}")
    plan.close()
    assert count == 1248
    assert not failures, f"d={d} {fmt}: {len(failures)} of {count} tuples differ from the oracle, first: {failures[:5]}"
