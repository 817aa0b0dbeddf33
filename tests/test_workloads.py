"""The seeded input generators: determinism, structure and distribution checks (CPU only)."""
import numpy as np

import workloads as wl

M64 = (1 << 64) - 1


def py_rnd_u64(seed, ctr):
    z = (seed + (ctr + 1) * 0x9E3779B97F4A7C15) & M64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & M64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & M64
    return z ^ (z >> 31)


def test_counter_rng_matches_python_twin():
    lib = wl._load()
    for seed in (0, 1, wl.seed_for(4, 1), M64):
        for ctr in (0, 1, 2, 12345678901, M64 - 1):
            assert lib.wl_rnd_u64(seed, ctr) == py_rnd_u64(seed, ctr)


def test_f16_conversion_is_rne():
    r = np.random.default_rng(5)
    x = r.standard_normal(300000) * np.exp(r.uniform(-20, 12, 300000))
    with np.errstate(over="ignore"):
        ref = x.astype(np.float16)
    assert np.array_equal(wl.to_f16(x).view(np.uint16), ref.view(np.uint16))


def test_tensor_distributions_and_determinism():
    a = wl.normal_f16((4096, 64), 77)
    b = wl.normal_f16((4096, 64), 77)
    assert np.array_equal(a.view(np.uint16), b.view(np.uint16))
    a64 = a.astype(np.float64)
    assert abs(a64.mean()) < 0.01 and abs(a64.std() - 1.0) < 0.01
    u = wl.uniform_f16((4096, 64), 78, -8.0, 8.0).astype(np.float64)
    assert u.min() >= -8 and u.max() <= 8 and abs(u.mean()) < 0.05 and abs(u.std() - 16 / np.sqrt(12)) < 0.05
    s = wl.normal_f16((2000, 16), 79, 0.0, 0.1).astype(np.float64)
    assert abs(s.std() - 0.1) < 0.005


def check_csr(rowptr, col, V):
    assert rowptr[0] == 0 and rowptr[-1] == col.size and np.all(np.diff(rowptr) >= 0)
    assert col.min() >= 0 and col.max() < V
    row = np.repeat(np.arange(V), np.diff(rowptr))
    same = row[1:] == row[:-1]
    assert np.all(col[1:][same] >= col[:-1][same])  # ascending inside a row


def test_config1_shape():
    w = wl.gcn_tiny()
    assert w.V == 4096 and w.E == 32768 + 4096 and w.F == 64
    check_csr(w.rowptr, w.col, w.V)
    row = np.repeat(np.arange(w.V), np.diff(w.rowptr))
    assert np.all(np.bincount(row[row == w.col], minlength=w.V) >= 1)  # a self-loop per vertex
    deg_r = np.diff(w.rowptr)
    deg_c = np.bincount(w.col, minlength=w.V)
    ref = (1.0 / np.sqrt(deg_r[row].astype(np.float64) * deg_c[w.col])).astype(np.float16)
    assert np.array_equal(ref.view(np.uint16), w.tensors["w"].view(np.uint16))
    w2 = wl.gcn_tiny()
    assert np.array_equal(w.col, w2.col) and np.array_equal(w.tensors["X"].view(np.uint16), w2.tensors["X"].view(np.uint16))


def test_rmat_has_hubs_and_keeps_duplicates():
    w = wl.gin_overflow(scale=14, avg_degree=16)
    assert w.E == 16 << 14
    check_csr(w.rowptr, w.col, w.V)
    deg = np.diff(w.rowptr)
    assert deg.max() > 50 * deg.mean()          # power-law hubs
    assert (deg == 0).mean() > 0.2              # and many isolated rows
    row = np.repeat(np.arange(w.V), deg)
    key = row.astype(np.int64) * w.V + w.col
    assert np.unique(key).size < key.size       # duplicates were kept
    wp = wl.gin_overflow(scale=14, avg_degree=16, positive=True)
    assert wp.tensors["X"].min() >= 0 and np.array_equal(wp.col, w.col)


def test_rmat_vertex_limit_and_lognormal():
    rowptr, col = wl.rmat_graph(12, 20000, 9, V=3000)
    assert rowptr.size == 3001 and col.size == 20000
    check_csr(rowptr, col, 3000)
    rowptr, col = wl.lognormal_graph(2000, 200000, 11)
    check_csr(rowptr, col, 2000)
    deg = np.diff(rowptr)
    assert deg.min() >= 1 and deg.sum() == 200000
    ln = np.log(deg[deg > 3])
    assert 0.8 < ln.std() < 1.2                 # sigma = 1 in log space
