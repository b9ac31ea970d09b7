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
    plan = B.Plan(m, n, rp, ci)
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
