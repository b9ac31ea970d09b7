"""fusedmm_execute_static_scratch -- the entry point that allocates nothing -- against fusedmm_execute.

Same kernels, same schedule, same order of every sum: the two must agree bit for bit (which is inside the
parity bound of the other GPU tests, 1e-4 of the sum of |terms|).  Two calls in a row share the one static
array, the second on a smaller input; the plans are created with a small dimension hint, so their own
scratch could not serve these calls at all."""
import numpy as np
import pytest

from paper_2011_06391_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU (torch.cuda.is_available() is False)")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def one_case(B, scale, pairs, d, pattern, seed, general=False):
    g = synth.rmat(scale, pairs, seed=seed)
    X = synth.fill_uniform((g.m, d), seed + 1, -0.5, 0.5)
    rp, ci, Xd = dev(g.rowptr), dev(g.colidx), dev(X)
    options = {"small_row_max": 8, "split_row_min": 64, "chunk_edges": 256, "column_classes": 8, "tile_row_min": 48,
               "feature_dim_hint": 32, "general_kernel_only": int(general)}
    plan_ref = B.Plan(g.m, g.n, rp, ci, options)
    plan_ref.reserve(d)
    plan = B.Plan(g.m, g.n, rp, ci, options)      # never reserved beyond 32: only the static scratch can serve d
    stats = plan.stats()
    assert stats["split_rows"] > 0 and stats["partials"] > 0
    ops = B.fusedmm_ops_preset(pattern)
    Z_ref = torch.full((g.m, d), float("nan"), dtype=torch.float32, device="cuda")
    plan_ref.execute(ops, Xd, Xd, Z_ref)
    Z = torch.full((g.m, d), float("nan"), dtype=torch.float32, device="cuda")
    if d > 32 and not general:
        with pytest.raises(B.FusedMMError) as ei:   # the ordinary entry point refuses: nothing reserved for d
            plan.execute(ops, Xd, Xd, Z)
        assert ei.value.status == B.FUSEDMM_ERR_NOT_RESERVED
    B.fusedmm_execute_static_scratch(plan._plan, ops, d, None, Xd, d, Xd, d, Z, d)
    torch.cuda.synchronize()
    assert torch.isfinite(Z).all().item()
    assert torch.equal(Z, Z_ref), f"scale {scale} d={d} {pattern}: static-scratch result differs from fusedmm_execute"
    plan.close()
    plan_ref.close()
    return stats


def test_two_calls_in_a_row_second_one_smaller(B):
    big = one_case(B, 13, (1 << 12) * 16, 128, "tdist", 601)
    small = one_case(B, 10, (1 << 9) * 16, 64, "one_minus_sigmoid", 602)
    assert small["partials"] < big["partials"]
    # and once more through a ragged instance (d not a multiple of 4), the largest instance (masked), the general
    # kernel (a plan that asks for it), whose segments use the same array, and through the one-lane-per-entry
    # kernels (partial rows 16 floats apart)
    one_case(B, 11, (1 << 10) * 16, 50, "fr", 603)
    one_case(B, 11, (1 << 10) * 16, 1100, "fr", 606)
    one_case(B, 11, (1 << 10) * 16, 300, "fr", 607, general=True)
    one_case(B, 11, (1 << 10) * 16, 3, "fr", 604)
    one_case(B, 12, (1 << 11) * 16, 16, "sigmoid", 605)


def test_sizes_beyond_the_static_scratch_are_refused(B):
    """5 000 rows of 64 sorted entries spread over all columns: 8 partial rows each under 8 column classes,
    40 000 partial rows of 2 KiB at d = 512 = 78 MiB, beyond the 64 MiB array."""
    m, n, d, deg = 5000, 4096, 512, 64
    rowptr = np.arange(m + 1, dtype=np.int64) * deg
    colidx = np.tile((np.arange(deg, dtype=np.int32) * (n // deg)), m)
    rp, ci = dev(rowptr), dev(colidx)
    plan = B.Plan(m, n, rp, ci, {"column_classes": 8, "tile_row_min": 64, "feature_dim_hint": 32})
    s = plan.stats()
    assert s["partials"] * d * 4 > B.FUSEDMM_STATIC_SCRATCH_BYTES
    X = torch.zeros((m, d), dtype=torch.float32, device="cuda")
    Y = torch.zeros((n, d), dtype=torch.float32, device="cuda")
    Z = torch.full((m, d), 3.0, dtype=torch.float32, device="cuda")
    ops = B.fusedmm_ops_preset("sigmoid")
    with pytest.raises(B.FusedMMError) as ei:
        B.fusedmm_execute_static_scratch(plan._plan, ops, d, None, X, d, Y, d, Z, d)
    assert ei.value.status == B.FUSEDMM_ERR_SCRATCH_LIMIT
    assert "scratch" in B.fusedmm_status_string(B.FUSEDMM_ERR_SCRATCH_LIMIT)
    torch.cuda.synchronize()
    assert (Z == 3.0).all().item()          # nothing was launched
    # the same plan at d = 32 fits (40 000 x 128 B) and runs
    X32, Y32 = X[:, :32].contiguous(), Y[:, :32].contiguous()
    Z32 = torch.full((m, 32), float("nan"), dtype=torch.float32, device="cuda")
    B.fusedmm_execute_static_scratch(plan._plan, ops, 32, None, X32, 32, Y32, 32, Z32, 32)
    torch.cuda.synchronize()
    assert (Z32 == 0).all().item()          # sigmoid(0) * 0
    plan.close()
