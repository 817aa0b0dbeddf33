"""Shared helpers of the GPU parity tests: device upload, random graphs and the comparison rule."""
import numpy as np
import torch

import workloads as wl

REL_L2 = 5e-3      # ||y - ref||_2 / ||ref||_2
REL_ELEM = 2e-2    # elementwise relative error
FP16_MAX = 65504.0


CANCEL_LOG = []  # one entry per compare() call that took the cancelling branch: (name, true ratio, ||ref|| / ||sabs||)


def compare(name, got16, ref, sabs=None, rel_l2=REL_L2, rel_elem=REL_ELEM, check_finite=True, allow_cancel=False):
    """got16: numpy float16 from the GPU; ref: float64 oracle values; sabs: oracle's sum of |terms|
    (natural magnitude).  Elementwise rule: |y - ref| <= rel_elem*|ref| + 2^-11 * sabs, i.e. the stated
    relative bound plus one fp16 rounding at the magnitude the sum passed through (a pure relative
    bound cannot be met next to zero by any fp16 output).  Norm rule: ||y - ref|| <= rel_l2 * ||ref||, except where
    ||ref|| <= 2^-8 ||sabs|| (the result is a near-complete cancellation): there ||y - ref|| <= 2^-11 ||sabs||.
    That branch is only taken where the ratio fails and only with allow_cancel=True (the randomized sweep passes it;
    everything else, the five configurations included, is held to the ratio), it is
    recorded in CANCEL_LOG, and the returned dict carries `cancelled` and the true ratio `rel_l2` it replaced.
    Entries whose fp64 value does not fit fp16
    are excluded from the value checks and must be +-inf with the right sign."""
    got = got16.astype(np.float64)
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    fits = np.abs(ref) <= FP16_MAX
    if check_finite:
        bad = ~np.isfinite(got) & (np.abs(ref) <= FP16_MAX * (1 - 2.0 ** -10))
        assert not bad.any(), f"{name}: {int(bad.sum())} non-finite outputs where the exact value fits fp16"
        fits &= np.isfinite(got)  # within a rounding step of the largest finite value either outcome is legitimate
    over = np.abs(ref) >= 65520.0 * (1 + 2.0 ** -10)  # clearly beyond the range: must be inf of the right sign
    if over.any():
        assert np.all(np.isinf(got[over]) & (np.sign(got[over]) == np.sign(ref[over]))), f"{name}: overflow entries"
    over = np.abs(ref) > FP16_MAX
    g, r = got[fits], ref[fits]
    if r.size == 0:
        return {"rel_l2": 0.0, "max_rel": 0.0, "n_over": int(over.sum()), "cancelled": False}
    denom = np.linalg.norm(r)
    l2 = np.linalg.norm(g - r) / denom if denom > 0 else np.linalg.norm(g - r)
    cancelled = False
    if l2 > rel_l2 and allow_cancel and sabs is not None and denom <= (2.0 ** -8) * np.linalg.norm(sabs[fits]):
        # the ratio fails, and the exact result is what is left after at least 8 bits of its terms have cancelled (down
        # to exactly zero for some inputs): one fp16 rounding at the magnitude of the terms, which no fp16 path can
        # avoid, is then 2^-3 of the result or more, and a ratio to the result's norm measures the input, not the
        # kernel.  There the error must stay below that one rounding, in norm as it must element by element
        snorm = np.linalg.norm(sabs[fits])
        assert np.linalg.norm(g - r) <= (2.0 ** -11) * snorm, f"{name}: cancelling result off"
        cancelled = True
        CANCEL_LOG.append((name, float(l2), float(denom / snorm) if snorm > 0 else 0.0))
        print(f"[parity] {name}: norm rule replaced by the cancelling bound (||ref||/||sum|terms||| = {CANCEL_LOG[-1][2]:.2e}); "
              f"the ratio it replaced: {l2:.3e}", flush=True)
    else:
        assert l2 <= rel_l2, f"{name}: rel-L2 {l2:.3e} > {rel_l2}"
    floor = (2.0 ** -11) * (sabs[fits] if sabs is not None else np.abs(r)) + 2.0 ** -24
    err = np.abs(g - r)
    viol = err > rel_elem * np.abs(r) + floor
    assert not viol.any(), (f"{name}: {int(viol.sum())} elements beyond tolerance; worst abs err "
                            f"{err[viol].max():.3e} at ref {r[viol][np.argmax(err[viol])]:.3e}")
    nz = np.abs(r) > 0
    strict = np.max(err[nz] / np.abs(r[nz])) if nz.any() else 0.0
    return {"rel_l2": float(l2), "max_rel": float(strict), "n_over": int(over.sum()), "cancelled": cancelled}


_WS = {}


def spmm_plain(hgnn, g, edge_val, H, X, Y, workspace=True, **kw):
    """hgnn_spmm with the workspace its long rows want (one buffer per size, kept for the session);
    workspace=False runs the call without one (every long row on a single wavefront)."""
    F = kw.get("F") or X.shape[1]
    ws = None
    if workspace:
        need = hgnn.hgnn_spmm_workspace(g.nrows, g.ncols, g.nnz, F)
        if need:
            ws = _WS.get(need)
            if ws is None:
                ws = _WS[need] = torch.empty(need, dtype=torch.uint8, device=X.device)
    hgnn.hgnn_spmm(g, edge_val, H, X, Y, workspace=ws, **kw)


def sample_rows(rowptr, n, seed, extra_top=8):
    """n random rows plus the extra_top longest rows (hubs), sorted unique."""
    rng = np.random.default_rng(seed)
    V = rowptr.size - 1
    deg = np.diff(rowptr)
    pick = rng.integers(0, V, size=min(n, V))
    top = np.argsort(deg)[-extra_top:]
    return np.unique(np.concatenate([pick, top])).astype(np.int32)


def up(a, dev):
    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def down(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def rand_graph(V, ncols, avg_deg, seed, hubs=(), empties=()):
    r = np.random.default_rng(seed)
    deg = r.poisson(avg_deg, size=V)
    for i, d in hubs:
        deg[i] = d
    for i in empties:
        deg[i] = 0
    rowptr = np.concatenate([[0], np.cumsum(deg)]).astype(np.int32)
    col = r.integers(0, ncols, size=int(rowptr[-1])).astype(np.int32)
    for i in range(V):  # ascending inside a row
        col[rowptr[i]:rowptr[i + 1]].sort()
    return rowptr, col


def f16(a):
    return wl.to_f16(np.asarray(a, dtype=np.float64))
