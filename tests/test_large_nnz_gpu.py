"""More than 2^31 stored entries: every offset into colidx / values must be 64-bit.  The oracle cannot run a
matrix of this size, so the checks are properties that hold at any size: every stored entry visited exactly
once (both kernels' indexing), and a GCN sum over integer data against its closed form, bit for bit.  The
short, the empty and the hub rows sit at the end of the matrix, behind entry 2^31."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

D = 32


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


@pytest.fixture(autouse=True)
def release_cached_memory():
    """These tests hold tens of GB; hand them back so the library's own allocations in later tests find room."""
    yield
    torch.cuda.empty_cache()


def build_pattern():
    """Row u holds deg[u] entries at columns first[u] + k * step[u], k = 0 .. deg[u]-1 (sorted, distinct)."""
    m, n = (1 << 20) + 6000, 3_200_000
    u = np.arange(m, dtype=np.int64)
    deg = 2048 + (u % 64)
    tail = u >= (1 << 20)
    deg[tail] = u[tail] % 70                          # packed rows and rows without entries
    deg[tail & (u % 5 == 0)] = 80 + u[tail & (u % 5 == 0)] % 400   # one wavefront each
    deg[tail & (u % 11 == 0)] = 0
    deg[m - 3] = 3_000_000                            # a hub, cut into many chunks
    step = np.ones(m, dtype=np.int64)
    spread = (u % 16 == 3) & (deg > 0)
    step[spread] = n // deg[spread]                   # these rows reach every column class
    first = np.where(step == 1, (u * 7919) % (n - deg), 0)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(deg)
    return m, n, deg, step, first, rowptr


def closed_form(deg, step, first):
    """z_u[j] = sum_k ((first + k*step + j) mod 4): k runs through the residues mod 4 in turn."""
    j = np.arange(D, dtype=np.int64)[None, :]
    Z = np.zeros((len(deg), D), dtype=np.int64)
    for r in range(4):
        cnt = (deg + 3 - r) // 4
        Z += cnt[:, None] * ((first[:, None] + r * step[:, None] + j) % 4)
    assert Z.max() < (1 << 24)                        # every partial sum is an integer fp32 holds exactly
    return Z.astype(np.float32)


def test_offsets_beyond_2_to_31(B):
    m, n, deg, step, first, rowptr = build_pattern()
    nnz = int(rowptr[-1])
    assert nnz > (1 << 31) and rowptr[1 << 20] > (1 << 31) and (deg[1 << 20:] == 0).any()
    rp = torch.from_numpy(rowptr).cuda()
    rows = torch.repeat_interleave(torch.arange(m, dtype=torch.int32, device="cuda"), torch.from_numpy(deg).cuda())
    assert rows.numel() == nnz
    k = torch.arange(nnz, dtype=torch.int64, device="cuda") - rp[rows.long()]
    ci = (torch.from_numpy(first).cuda()[rows.long()] + k * torch.from_numpy(step).cuda()[rows.long()]).to(torch.int32)
    del rows, k
    assert int(ci.max()) < n and int(ci.min()) >= 0
    plan = B.Plan(m, n, rp, ci, {"tile_row_min": 128})   # (a pattern this dense would tile from 64 entries: no wave rows)
    st = plan.stats()
    assert st["tiled_rows"] > 0 and st["wave_rows"] > 0 and st["packed_rows"] > 0 and st["column_classes"] > 1

    counts = torch.zeros(nnz, dtype=torch.int32, device="cuda")
    for fast in (True, False):
        counts.zero_()
        plan.edge_visits(D, fast, counts)
        torch.cuda.synchronize()
        assert bool((counts == 1).all()), f"fast_path={fast}: {int((counts != 1).sum())} entries not visited exactly once"
    del counts

    Y = ((torch.arange(n, device="cuda")[:, None] + torch.arange(D, device="cuda")[None, :]) % 4).float()
    vals = torch.ones(nnz, dtype=torch.float32, device="cuda")
    Z = torch.full((m, D), float("nan"), dtype=torch.float32, device="cuda")
    plan.execute("gcn", None, Y, Z, vals)
    torch.cuda.synchronize()
    Zg = Z.cpu().numpy()
    plan.close()
    assert np.array_equal(Zg, closed_form(deg, step, first))


def test_operand_offsets_beyond_4_gib(B):
    """X, Y and Z of 6.5 GB each (3.2 M rows of 512 floats): row offsets in bytes need more than 32 bits.  A GCN sum
    and a tuple that reads X (s = sum_j (x_uj - y_vj), w = s * y_v), on integer data, against closed forms."""
    d, m = 512, 3_200_000
    n = m
    u = np.arange(m, dtype=np.int64)
    deg = u % 3
    long_rows = u % 5000 == 7
    deg[long_rows] = 3000
    step = np.ones(m, dtype=np.int64)
    step[long_rows] = n // 3000
    first = np.where(step == 1, (u * 7919) % (n - deg), 0)
    rowptr = np.zeros(m + 1, dtype=np.int64)
    rowptr[1:] = np.cumsum(deg)
    nnz = int(rowptr[-1])
    rp, degd, stepd, firstd = (torch.from_numpy(a).cuda() for a in (rowptr, deg, step, first))
    rows = torch.repeat_interleave(torch.arange(m, dtype=torch.int64, device="cuda"), degd)
    k = torch.arange(nnz, dtype=torch.int64, device="cuda") - rp[rows]
    ci = (firstd[rows] + k * stepd[rows]).to(torch.int32)
    del rows, k
    assert int(ci.max()) * d * 4 > (1 << 32)
    j = torch.arange(d, device="cuda")
    Y = ((torch.arange(n, device="cuda")[:, None] + j[None, :]) % 4).float()
    X = torch.zeros((m, d), dtype=torch.float32, device="cuda")
    X[:, 0] = (torch.arange(m, device="cuda") % 3).float()          # sum_j x_uj = u mod 3
    vals = torch.ones(nnz, dtype=torch.float32, device="cuda")
    Z = torch.empty((m, d), dtype=torch.float32, device="cuda")
    plan = B.Plan(m, n, rp, ci, {"feature_dim_hint": d})

    def gcn_block(lo, hi):      # sum_k ((first + k*step + j) mod 4), rows lo .. hi-1
        out = torch.zeros((hi - lo, d), dtype=torch.int64, device="cuda")
        for r in range(4):
            cnt = (degd[lo:hi] + 3 - r) // 4
            out += cnt[:, None] * ((firstd[lo:hi, None] + r * stepd[lo:hi, None] + j[None, :]) % 4)
        return out

    row_sum_y = (d // 4) * 6                                         # sum_j y_vj for any v: d is a multiple of 4
    for ops, scale in (("gcn", None), (B.make_ops("SUB", "RSUM", "NOOP", "MUL_Y"), "x")):
        Z.fill_(float("nan"))
        plan.execute(ops, None if scale is None else X, Y, Z, vals if scale is None else None)
        torch.cuda.synchronize()
        for lo in range(0, m, 400_000):
            hi = min(m, lo + 400_000)
            want = gcn_block(lo, hi)
            if scale is not None:
                want = want * ((torch.arange(lo, hi, device="cuda") % 3) - row_sum_y)[:, None]
            assert int(want.abs().max()) < (1 << 24)
            assert torch.equal(Z[lo:hi], want.float()), f"{ops if scale is None else 'SUB/RSUM tuple'}: rows {lo}..{hi}"
    plan.close()
