"""Minibatch embedding epoch (fusedmm_minibatch_*) against the oracle's epoch, through the C ABI.

Bound per element of the embedding after an epoch: |X_gpu - X_ref| <= 1e-4 * S + 2^-22 * |X_ref|,
S = lr * (sum of |terms| of the two FusedMM calls that produced the element's update): the parity
tolerance of the kernels, scaled by the learning rate, plus one rounding of the stored fp32 value.
"""
import numpy as np
import pytest

import oracle
from paper_2011_06391_amd import synth

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    if not torch.cuda.is_available():
        pytest.fail("GPU tests need a GPU")
    from paper_2011_06391_amd import binding
    binding.load()
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def negatives_for(n, batch_rows, s, seed):
    nb = (n + batch_rows - 1) // batch_rows
    return np.random.default_rng(seed).integers(0, n, (nb, s)).astype(np.int32)


def check_epoch(Xg, Xr, S, what):
    bound = 1e-4 * S + 2.0 ** -22 * np.abs(Xr)
    excess = np.abs(Xg.astype(np.float64) - Xr.astype(np.float64)) - bound
    assert excess.max() <= 0, f"{what}: |dX| exceeds the bound by {excess.max():.3e} at {np.unravel_index(excess.argmax(), excess.shape)}"


def graph_with_hub(n, seed, hub_degree):
    """Erdos-Renyi pattern plus one vertex adjacent to hub_degree others (a split row inside a batch)."""
    g = synth.erdos_renyi(n, 4 * n, seed)
    rng = np.random.default_rng(seed)
    hub = n // 3
    others = rng.choice(n, hub_degree, replace=False).astype(np.int32)
    src = np.repeat(np.arange(n, dtype=np.int32), g.degrees())
    pairs_s = np.concatenate([src, np.full(hub_degree, hub, np.int32)])
    pairs_d = np.concatenate([g.colidx, others])
    keep = pairs_s != pairs_d
    return synth.csr_from_pairs(n, pairs_s[keep], pairs_d[keep], None, True), hub


@pytest.mark.parametrize("n,d,batch_rows,s", [(1000, 64, 256, 5), (2708, 128, 256, 5), (300, 20, 64, 0), (517, 32, 517, 3),
                                              (130, 256, 1000, 2), (400, 50, 128, 4), (400, 3, 128, 4)])
def test_epoch_matches_oracle(B, n, d, batch_rows, s):
    g, hub = graph_with_hub(n, 11 + n, min(n - 1, 700))
    assert g.degrees()[hub] >= min(n - 3, 700)   # a long row inside one batch (the hub may draw itself: dropped)
    X0 = synth.fill_uniform((n, d), 5 + d, -0.5, 0.5)
    neg = negatives_for(n, batch_rows, s, 3)
    lr = 0.02
    rp, ci = dev(g.rowptr), dev(g.colidx)
    mb = B.Minibatch(n, rp, ci, batch_rows, dev(neg) if s else None)
    info = mb.info()
    assert info["n_batches"] == (n + batch_rows - 1) // batch_rows
    X = dev(X0)
    with pytest.raises(B.FusedMMError) as ei:   # an epoch never allocates: the result buffer must be reserved first
        mb.epoch(X, lr)
    assert ei.value.status == B.FUSEDMM_ERR_NOT_RESERVED
    mb.reserve(d)
    mb.epoch(X, lr)
    torch.cuda.synchronize()
    X1 = X.cpu().numpy()
    Xr, S = oracle.embedding_epoch(g.rowptr, g.colidx, X0, batch_rows, neg.reshape(info["n_batches"], s), lr)
    check_epoch(X1, Xr, S, f"epoch 1 n={n} d={d}")
    assert np.abs(X1 - X0).max() > 1e-3
    # second epoch: the oracle starts from what the GPU stored, so errors are not compounded
    mb.epoch(X, lr)
    torch.cuda.synchronize()
    Xr2, S2 = oracle.embedding_epoch(g.rowptr, g.colidx, X1, batch_rows, neg.reshape(info["n_batches"], s), lr)
    check_epoch(X.cpu().numpy(), Xr2, S2, f"epoch 2 n={n} d={d}")
    mb.close()


def test_epoch_leading_dimension_and_isolated_vertices(B):
    n, d, batch_rows, s = 400, 64, 128, 4
    g = synth.erdos_renyi(n, 300, 77)        # sparse: many vertices without neighbours
    assert (g.degrees() == 0).sum() > 20
    wide = synth.fill_uniform((n, d + 32), 9, -0.5, 0.5)
    neg = negatives_for(n, batch_rows, s, 5)
    mb = B.Minibatch(n, dev(g.rowptr), dev(g.colidx), batch_rows, dev(neg))
    Xw = dev(wide)
    mb.reserve(d)
    mb.epoch(Xw[:, :d], 0.05)
    torch.cuda.synchronize()
    out = Xw.cpu().numpy()
    Xr, S = oracle.embedding_epoch(g.rowptr, g.colidx, wide[:, :d], batch_rows, neg, 0.05)
    check_epoch(out[:, :d], Xr, S, "strided")
    assert np.array_equal(out[:, d:], wide[:, d:])     # columns beyond d untouched
    mb.close()


def test_epoch_replayed_from_a_hip_graph(B):
    """An epoch allocates nothing after reserve(), so it can be captured; every replay must equal the
    eager epoch bit for bit (the launches are deterministic)."""
    n, d, batch_rows, s = 1500, 128, 256, 5
    g, _ = graph_with_hub(n, 21, 600)
    X0 = synth.fill_uniform((n, d), 13, -0.5, 0.5)
    neg = negatives_for(n, batch_rows, s, 8)
    mb = B.Minibatch(n, dev(g.rowptr), dev(g.colidx), batch_rows, dev(neg))
    mb.reserve(d)
    Xe = dev(X0)
    eager = []
    for _ in range(3):
        mb.epoch(Xe, 0.02)
        torch.cuda.synchronize()
        eager.append(Xe.clone())
    Xg = dev(X0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        mb.epoch(Xg, 0.02)              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    Xg.copy_(dev(X0))
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        mb.epoch(Xg, 0.02)
    Xg.copy_(dev(X0))                    # capture does not execute
    for i in range(3):
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Xg, eager[i]), f"replay {i} differs from the eager epoch"
        _ = (Xe + 1).sum().item()        # unrelated eager work between replays
    del graph
    mb.close()


def test_minibatch_argument_errors(B):
    n = 100
    g = synth.erdos_renyi(n, 200, 3)
    rp, ci = dev(g.rowptr), dev(g.colidx)
    bad = negatives_for(n, 32, 2, 1)
    bad[1, 0] = n                        # outside [0, n)
    with pytest.raises(B.FusedMMError) as ei:
        B.Minibatch(n, rp, ci, 32, dev(bad))
    assert ei.value.status == B.FUSEDMM_ERR_INVALID_ARG
    with pytest.raises(ValueError):
        B.Minibatch(n, rp, ci, 32, dev(negatives_for(n, 50, 2, 1)))
    with pytest.raises(B.FusedMMError):
        B.fusedmm_minibatch_create(n, g.nnz, rp, ci, 0, 0, None)
    mb = B.Minibatch(n, rp, ci, 32, None)
    with pytest.raises(TypeError):
        mb.epoch(torch.zeros((n + 1, 32), device="cuda"), 0.1)
    mb.close()
