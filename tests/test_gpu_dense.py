"""GPU parity of the dense side of a layer (projection on the matrix cores, its transposed product and weight
gradient, the GAT feature gradient) against the CPU fp64 oracle, and of a whole GAT layer chained through them."""
import numpy as np
import pytest
import torch

import oracle
from parity import compare, down, f16, rand_graph, up

pytestmark = pytest.mark.gpu


def padded(a, ld, dev, fill=0.0):
    """Device copy of a inside rows of pitch ld; returns (view of the data, whole buffer)."""
    buf = torch.full((a.shape[0], ld), fill, dtype=torch.float16, device=dev)
    buf[:, :a.shape[1]] = up(a, dev)
    return buf[:, :a.shape[1]], buf


def check_f32(name, got, ref, sabs, rel=2e-5):
    err = np.abs(got.astype(np.float64) - ref)
    bound = rel * sabs + 1e-30
    assert np.all(err <= bound), f"{name}: worst error {err.max():.3e} against bound {bound[np.argmax(err - bound)]:.3e}"


LINEAR_CASES = [  # n, K, F, transposed weight, extra pitch of X, extra pitch of Y
    (1000, 64, 64, False, 0, 0), (333, 8, 8, False, 8, 0), (1, 16, 40, False, 0, 8), (4097, 128, 128, False, 0, 0),
    (700, 608, 64, False, 0, 0), (300, 1024, 256, False, 8, 8), (5000, 64, 7, False, 0, 1), (129, 72, 36, False, 0, 4),
    (1000, 64, 64, True, 0, 0), (257, 40, 96, True, 8, 0), (300, 1024, 200, True, 0, 0), (127, 24, 2, True, 0, 6),
    (2000, 64, 300, False, 0, 4),
]


@pytest.mark.parametrize("n,K,F,trans,px,py", LINEAR_CASES)
def test_linear_shapes(hgnn, dev, n, K, F, trans, px, py):
    print(f"linear n={n} K={K} F={F} trans={trans} px={px} py={py}", flush=True)
    r = np.random.default_rng(n + 3 * K + 7 * F)
    X = f16(r.standard_normal((n, K)))
    W = f16(r.standard_normal((F, K) if trans else (K, F)) / np.sqrt(K))
    ref, sabs = oracle.linear(X, W, trans=trans, want_sabs=True)
    Xd, _ = padded(X, K + px, dev)
    ldy = (F + py + 7) // 8 * 8
    Ybuf = torch.full((n, ldy), 7.0, dtype=torch.float16, device=dev)
    Wd = up(W, dev)
    hgnn.hgnn_linear(Xd, Wd, Ybuf[:, :F], trans_w=trans)
    got = down(Ybuf)
    compare("linear", got[:, :F], ref, sabs)
    assert np.all(got[:, F:] == 7.0), "columns beyond F were touched"
    # a weight with a pitch of its own gives the same bits
    Wp = torch.zeros((W.shape[0], W.shape[1] + 5), dtype=torch.float16, device=dev)
    Wp[:, :W.shape[1]] = Wd
    Y2 = torch.full((n, ldy), 7.0, dtype=torch.float16, device=dev)
    hgnn.hgnn_linear(Xd, Wp[:, :W.shape[1]], Y2[:, :F], trans_w=trans)
    assert np.array_equal(down(Y2).view(np.uint16), got.view(np.uint16))


def test_linear_identity_and_zero_rows(hgnn, dev):
    n, K = 777, 96
    r = np.random.default_rng(5)
    X = f16(r.standard_normal((n, K)))
    Xd = up(X, dev)
    Y = torch.empty((n, K), dtype=torch.float16, device=dev)
    hgnn.hgnn_linear(Xd, torch.eye(K, dtype=torch.float16, device=dev), Y)
    assert np.array_equal(down(Y).view(np.uint16), X.view(np.uint16))
    # n = 0 is a no-op; bad shapes are refused on the host
    hgnn.hgnn_linear(Xd[:0], torch.eye(K, dtype=torch.float16, device=dev), Y[:0])
    with pytest.raises(hgnn.HgnnError) as e:
        hgnn.hgnn_linear(Xd[:, :20], torch.zeros((20, 8), dtype=torch.float16, device=dev), Y[:, :8])
    assert e.value.status == hgnn.HGNN_EUNSUPPORTED  # K % 8 != 0
    with pytest.raises(hgnn.HgnnError) as e:
        hgnn.hgnn_linear(Xd, torch.zeros((K, 8), dtype=torch.float16, device=dev), Y[:, :8], F=16)
    assert e.value.status == hgnn.HGNN_EINVAL  # weight pitch smaller than F


WGRAD_CASES = [(1000, 64, 64), (17, 8, 8), (50000, 64, 64), (3000, 128, 72), (100, 200, 136), (16385, 16, 256), (5, 64, 64)]


@pytest.mark.parametrize("n,K,F", WGRAD_CASES)
def test_linear_wgrad_shapes(hgnn, dev, n, K, F):
    print(f"wgrad n={n} K={K} F={F}", flush=True)
    r = np.random.default_rng(n + K + F)
    X, dY = f16(r.standard_normal((n, K))), f16(r.standard_normal((n, F)))
    ref, sabs = oracle.linear_wgrad(X, dY, want_sabs=True)
    Xd, _ = padded(X, K + 8, dev)
    dYd, _ = padded(dY, F + 16, dev)
    ws = torch.empty(hgnn.hgnn_linear_wgrad_workspace(K, F), dtype=torch.uint8, device=dev)
    dWbuf = torch.full((K, F + 3), 7.0, dtype=torch.float32, device=dev)
    hgnn.hgnn_linear_wgrad(Xd, dYd, dWbuf[:, :F], ws)
    got = down(dWbuf)
    check_f32("wgrad", got[:, :F], ref, sabs)
    assert np.all(got[:, F:] == 7.0)
    # the same bits on a second run (fixed summation order), with a dirty workspace
    ws.fill_(0xff)
    dW2 = torch.empty((K, F), dtype=torch.float32, device=dev)
    hgnn.hgnn_linear_wgrad(Xd, dYd, dW2, ws)
    assert np.array_equal(down(dW2).view(np.uint32), got[:, :F].view(np.uint32))


def test_linear_wgrad_errors(hgnn, dev):
    X = torch.zeros((64, 64), dtype=torch.float16, device=dev)
    dW = torch.zeros((64, 64), dtype=torch.float32, device=dev)
    small = torch.empty(1024, dtype=torch.uint8, device=dev)
    with pytest.raises(hgnn.HgnnError) as e:
        hgnn.hgnn_linear_wgrad(X, X, dW, small)
    assert e.value.status == hgnn.HGNN_EINVAL and "workspace" in str(e.value)
    # no rows: the gradient is zero
    ws = torch.empty(hgnn.hgnn_linear_wgrad_workspace(64, 64), dtype=torch.uint8, device=dev)
    dW.fill_(5.0)
    hgnn.hgnn_linear_wgrad(X[:0], X[:0], dW, ws)
    assert np.all(down(dW) == 0)


@pytest.mark.parametrize("n,H,D", [(1000, 1, 64), (333, 4, 16), (5000, 3, 8), (64, 8, 64), (40000, 1, 8), (257, 2, 128)])
def test_gat_feature_grad_shapes(hgnn, dev, n, H, D):
    print(f"feature grad n={n} H={H} D={D}", flush=True)
    F = H * D
    r = np.random.default_rng(n + H + D)
    dV, hfeat = f16(r.standard_normal((n, F))), f16(r.standard_normal((n, F)))
    d_el, d_er = f16(0.3 * r.standard_normal((n, H))), f16(0.3 * r.standard_normal((n, H)))
    a_l, a_r = f16(0.5 * r.standard_normal(F)), f16(0.5 * r.standard_normal(F))
    dh_ref, dal_ref, dar_ref, sl, sr = oracle.gat_feature_grad(dV, d_el, d_er, a_l, a_r, hfeat, H)
    mag = (np.abs(dV.astype(np.float64)) + np.abs(np.repeat(d_el.astype(np.float64), D, 1) * a_l.astype(np.float64)) +
           np.abs(np.repeat(d_er.astype(np.float64), D, 1) * a_r.astype(np.float64)))
    dVd, _ = padded(dV, F + 8, dev)
    hd, _ = padded(hfeat, F + 16, dev)
    dhbuf = torch.full((n, F + 8), 7.0, dtype=torch.float16, device=dev)
    da_l = torch.full((F,), 7.0, dtype=torch.float32, device=dev)
    da_r = torch.full((F,), 7.0, dtype=torch.float32, device=dev)
    ws = torch.empty(hgnn.hgnn_gat_feature_grad_workspace(H, D), dtype=torch.uint8, device=dev)
    ws.fill_(0xff)
    hgnn.hgnn_gat_feature_grad(H, D, dVd, up(d_el, dev), up(d_er, dev), up(a_l, dev), up(a_r, dev), hd, dhbuf[:, :F],
                               da_l, da_r, ws)
    got = down(dhbuf)
    compare("dh", got[:, :F], dh_ref, mag)
    assert np.all(got[:, F:] == 7.0)
    check_f32("da_l", down(da_l), dal_ref, sl)
    check_f32("da_r", down(da_r), dar_ref, sr)


def test_gat_layer_forward_and_backward_chain(hgnn, dev):
    """h = X W; out = GAT aggregation of (h, h); then every gradient of L = <dOut, out>.  The oracle chain rounds to
    fp16 where the device stores fp16 (h, dV, d_el, d_er, dh) and nowhere else."""
    V, K, H, D = 1500, 40, 2, 16
    F = H * D
    rowptr, col = rand_graph(V, V, 9, 123, hubs=((3, 2500), (900, 400)), empties=(0, 77))
    r = np.random.default_rng(9)
    X = f16(r.standard_normal((V, K)))
    W = f16(r.standard_normal((K, F)) / np.sqrt(K))
    a_l, a_r = f16(0.3 * r.standard_normal(F)), f16(0.3 * r.standard_normal(F))
    dOut = f16(r.standard_normal((V, F)))
    # ---- oracle chain
    h64, h_sabs = oracle.linear(X, W, want_sabs=True)
    h16 = h64.astype(np.float16)
    out_ref, lse_ref, out_sabs = oracle.gat_forward(rowptr, col, h16, h16, a_l, a_r, H)
    dV_ref, del_ref, der_ref = oracle.gat_backward(rowptr, col, h16, h16, a_l, a_r, dOut, H)
    dh_ref, dal_ref, dar_ref, sl, sr = oracle.gat_feature_grad(dV_ref.astype(np.float16), del_ref.astype(np.float16),
                                                               der_ref.astype(np.float16), a_l, a_r, h16, H)
    dh16 = dh_ref.astype(np.float16)
    dX_ref, dX_sabs = oracle.linear(dh16, W, trans=True, want_sabs=True)
    dW_ref, dW_sabs = oracle.linear_wgrad(X, dh16, want_sabs=True)
    # ---- device chain
    g = hgnn.Csr(up(rowptr, dev), up(col, dev))
    p = hgnn.hgnn_plan_create(g, 128, F, H)
    gt = hgnn.hgnn_transpose(g)
    pt = hgnn.hgnn_plan_create(gt, 128, F, H)
    Xd, Wd, ald, ard, dOutd = up(X, dev), up(W, dev), up(a_l, dev), up(a_r, dev), up(dOut, dev)
    half = lambda *s: torch.empty(s, dtype=torch.float16, device=dev)
    h, out, dV, d_el, d_er, dh, dX = half(V, F), half(V, F), half(V, F), half(V, H), half(V, H), half(V, F), half(V, K)
    lse = torch.empty((V, H), dtype=torch.float32, device=dev)
    dW = torch.empty((K, F), dtype=torch.float32, device=dev)
    da_l, da_r = torch.empty(F, dtype=torch.float32, device=dev), torch.empty(F, dtype=torch.float32, device=dev)
    ws = torch.empty(max(hgnn.hgnn_linear_wgrad_workspace(K, F), hgnn.hgnn_gat_feature_grad_workspace(H, D)),
                     dtype=torch.uint8, device=dev)
    hgnn.hgnn_linear(Xd, Wd, h)
    hgnn.hgnn_gat_forward_fused(g, p, H, D, h, h, ald, ard, out, lse)
    hgnn.hgnn_gat_backward_fused(g, p, gt, pt, H, D, h, h, ald, ard, out, lse, dOutd, dV, d_el, d_er)
    hgnn.hgnn_gat_feature_grad(H, D, dV, d_el, d_er, ald, ard, h, dh, da_l, da_r, ws)
    hgnn.hgnn_linear(dh, Wd, dX, trans_w=True)
    hgnn.hgnn_linear_wgrad(Xd, dh, dW, ws)
    compare("layer h", down(h), h64, h_sabs)
    compare("layer out", down(out), out_ref, out_sabs)
    # gradients: the device's own fp16 intermediates differ from the oracle's by a rounding each, which the
    # cancelling sums behind d_el / d_er amplify; rel-L2 bands as for the fused backward on its own
    rel = lambda a, b: np.linalg.norm(a.astype(np.float64) - b) / np.linalg.norm(b)
    assert rel(down(dh), dh_ref) < 5e-3
    assert rel(down(dX), dX_ref) < 5e-3
    assert rel(down(dW), dW_ref) < 5e-3
    assert rel(down(da_l), dal_ref) < 2e-2 and rel(down(da_r), dar_ref) < 2e-2
    hgnn.hgnn_plan_destroy(p)
    hgnn.hgnn_plan_destroy(pt)


def test_dense_at_dense_degree_size(hgnn, dev):
    """The projection and the weight gradient at the vertex count and width of the dense-degree workload
    (233 000 x 64 -> 64): sampled rows of Y, the whole of dW."""
    n, K, F = 233000, 64, 64
    r = np.random.default_rng(2024)
    X = f16(r.standard_normal((n, K)))
    W = f16(r.standard_normal((K, F)) / 8)
    G = f16(r.standard_normal((n, F)))
    Xd, Gd, Wd = up(X, dev), up(G, dev), up(W, dev)
    Y = torch.empty((n, F), dtype=torch.float16, device=dev)
    hgnn.hgnn_linear(Xd, Wd, Y)
    rows = np.unique(np.concatenate([r.integers(0, n, 4000), [0, 127, 128, n - 129, n - 1]]))
    ref, sabs = oracle.linear(X[rows], W, want_sabs=True)
    compare("linear full", down(Y)[rows], ref, sabs)
    ws = torch.empty(hgnn.hgnn_linear_wgrad_workspace(K, F), dtype=torch.uint8, device=dev)
    dW = torch.empty((K, F), dtype=torch.float32, device=dev)
    hgnn.hgnn_linear_wgrad(Xd, Gd, dW, ws)
    dref, dsabs = oracle.linear_wgrad(X, G, want_sabs=True)
    check_f32("wgrad full", down(dW), dref, dsabs)
