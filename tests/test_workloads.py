"""Seeded input generators: same seed => same bytes (whatever the thread count), patterns are
well-formed (sorted, duplicate-free, symmetric where promised, no self-loops), random access into
the dense streams agrees with bulk generation."""
import hashlib

import numpy as np
import scipy.sparse as sp

import workloads as wl


def digest(g):
    return hashlib.sha256(g.rowptr.tobytes() + g.colidx.tobytes()).hexdigest()


def well_formed(g, symmetric):
    assert g.rowptr[0] == 0 and np.all(np.diff(g.rowptr) >= 0) and g.rowptr[-1] == len(g.colidx)
    assert g.colidx.min(initial=0) >= 0 and g.colidx.max(initial=0) < g.n_cols
    for i in range(min(g.n_rows, 2000)):
        row = g.colidx[g.rowptr[i]:g.rowptr[i + 1]]
        assert np.all(np.diff(row) > 0)
        assert not np.any(row == i) or not symmetric  # no self-loops in the square generators
    if symmetric:
        A = sp.csr_matrix((np.ones(len(g.colidx)), g.colidx, g.rowptr), shape=(g.n_rows, g.n_cols))
        assert (A != A.T).nnz == 0 and A.diagonal().sum() == 0


def test_generators_are_deterministic_and_well_formed():
    tiny = wl.CONFIGS["tiny"].graph()
    assert digest(tiny) == "aba8462a928a4e088dd5f5b6e278636ad9283d5969430548b66541c937dc30b7"
    well_formed(tiny, True)
    cl = wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99)
    assert (cl.nnz, digest(cl)[:16]) == (141014, "317f67ff6e4e2728")
    well_formed(cl, True)
    rm = wl.rmat(12, 30000, 0.57, 0.19, 0.19, 5)
    assert (rm.nnz, digest(rm)[:16]) == (49420, "7e5f41b35ef29989")
    well_formed(rm, True)
    rb = wl.row_block(500, 4000, 6000, 2.5, 200.0, 1.6, 17)
    assert (rb.nnz, digest(rb)[:16]) == (3305, "a04bcfe3d60300ae")
    well_formed(rb, False)
    assert digest(wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99)) == digest(cl)  # and again: same bytes


def test_chung_lu_degrees_follow_the_requested_shape():
    g = wl.chung_lu(20000, 2.0e6, 2.1, 4000.0, 7)
    d = np.diff(g.rowptr)
    assert abs(d.mean() - 100.0) < 5.0          # target average degree (truncation loses a little)
    assert d.max() > 20 * d.mean()              # heavy tail
    assert np.median(d) < d.mean()              # skewed


def test_dense_streams_random_access_and_statistics():
    cfg = wl.CONFIGS["tiny"]
    X = cfg.features(4096)
    assert X.dtype == np.float32 and X.shape == (4096, 64)
    assert X[0, :4].tolist() == [0.8507335782051086, -0.5963334441184998, 1.762925148010254, -0.4891006052494049]
    # element (r, c) is element r*64 + c of the stream, wherever the window starts
    part = wl.normal_f32(cfg.seed + 0x100, 0, (3, 64), first=1000 * 64)
    assert np.array_equal(part, X[1000:1003])
    assert abs(X.mean()) < 0.01 and abs(X.std() - 1.0) < 0.01
    assert cfg.labels(8).tolist() == [0, 2, 1, 5, 0, 4, 3, 2]
    W = cfg.weights()
    a = np.sqrt(6.0 / (64 + 16))
    assert W[0].shape == (64, 16) and np.all(np.abs(W[0]) <= a) and abs(W[0].std() - a / np.sqrt(3)) < 0.01
