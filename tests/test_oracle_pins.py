"""Pins for the CPU oracle: every oracle function is checked against something other than
itself -- dense brute force written with numpy matrix algebra, closed forms, invariants the
paper states, scipy / numpy / torch-autograd as independent opinions, a hand-computed
worked example, and central finite differences for the backward chain.  CPU only."""
import math
import os

import numpy as np
import pytest
import scipy.sparse as sp

import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))


# ----------------------------------------------------------------------------
# helpers (test-side, independent of the oracle's code)
# ----------------------------------------------------------------------------

def random_pattern(n, m, density, rng, symmetric=True, self_loops=False):
    A = rng.random((n, m)) < density
    if symmetric:
        assert n == m
        A = np.triu(A, 1)
        A = A | A.T
    if n == m and not self_loops:
        np.fill_diagonal(A, False)
    if self_loops:
        idx = rng.choice(min(n, m), size=max(1, min(n, m) // 3), replace=False)
        A[idx, idx] = True
    S = sp.csr_matrix(A.astype(np.float64))
    S.sort_indices()
    return A, S.indptr.astype(np.int32), S.indices.astype(np.int32)


def dense_symnorm(A):
    """D^-1/2 (A+I) D^-1/2 by explicit dense matrix products."""
    n = A.shape[0]
    At = (A | np.eye(n, dtype=bool)).astype(np.float64)
    d = At.sum(axis=1)
    Dm = np.diag(1.0 / np.sqrt(d))
    return Dm @ At @ Dm, At, d


def to_dense(n_rows, n_cols, rowptr, colidx, val):
    D = np.zeros((n_rows, n_cols))
    for i in range(n_rows):
        for k in range(rowptr[i], rowptr[i + 1]):
            D[i, colidx[k]] += val[k]
    return D


# ----------------------------------------------------------------------------
# normalisation
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("n,density,sym,loops", [(1, 0.0, True, False), (7, 0.3, True, False),
                                                   (33, 0.15, True, True), (64, 0.1, False, False),
                                                   (40, 0.0, True, False), (25, 1.0, True, False)])
def test_normalize_dense_bruteforce(ref, n, density, sym, loops):
    rng = np.random.default_rng(n * 7 + int(density * 100))
    A, rp, ci = random_pattern(n, n, density, rng, symmetric=sym, self_loops=loops)
    rp2, ci2, val = ref.csr_normalize(n, n, rp, ci)
    want, At, d = dense_symnorm(A)
    got = to_dense(n, n, rp2, ci2, val)
    # pattern: exactly A united with the diagonal, each entry once, columns ascending
    assert np.array_equal(got != 0, At != 0)
    assert rp2[-1] == int(At.sum())
    for i in range(n):
        row = ci2[rp2[i]:rp2[i + 1]]
        assert np.all(np.diff(row) > 0)
    np.testing.assert_allclose(got, want, rtol=1e-15, atol=0)


def test_normalize_worked_example(ref):
    """Path graph 0-1-2 with hand-derived entries and product (tests/golden/path3_symnorm.txt)."""
    entries, Y = [], []
    for line in open(os.path.join(HERE, "golden", "path3_symnorm.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        if tok[0] == "Y":
            Y.append([float(tok[1]), float(tok[2])])
        else:
            entries.append((int(tok[0]), int(tok[1]), float(tok[2])))
    rp = np.array([0, 1, 3, 4], dtype=np.int32)
    ci = np.array([1, 0, 2, 1], dtype=np.int32)
    rp2, ci2, val = ref.csr_normalize(3, 3, rp, ci)
    got = [(i, int(ci2[k]), val[k]) for i in range(3) for k in range(rp2[i], rp2[i + 1])]
    assert [(g[0], g[1]) for g in got] == [(e[0], e[1]) for e in entries]
    np.testing.assert_allclose([g[2] for g in got], [e[2] for e in entries], rtol=2e-16)
    X = np.array([[1.0, 2.0], [3.0, 4.0], [5.0, 6.0]])
    np.testing.assert_allclose(ref.spmm(ref.OP_N, 3, 3, rp2, ci2, val, X), np.array(Y), rtol=4e-16)


def test_normalize_symmetric_values_bitwise_and_eigenvector(ref):
    g = wl.erdos_renyi(500, 0.02, 11)
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx)
    S = sp.csr_matrix((val, ci, rp), shape=(500, 500))
    T = S.T.tocsr()
    T.sort_indices()
    assert np.array_equal(T.indices, ci) and np.array_equal(T.data.view(np.int64), val.view(np.int64))
    # closed form valid for every graph: A^ sqrt(d) = sqrt(d), d counted with the self-loop
    d = np.diff(rp).astype(np.float64)
    y = ref.spmm(ref.OP_N, 500, 500, rp, ci, val, np.sqrt(d)[:, None])
    np.testing.assert_allclose(y[:, 0], np.sqrt(d), rtol=1e-13)
    # spectral bound ||A^ x|| <= ||x||
    x = np.random.default_rng(0).standard_normal((500, 3))
    y = ref.spmm(ref.OP_N, 500, 500, rp, ci, val, x)
    assert np.all(np.linalg.norm(y, axis=0) <= np.linalg.norm(x, axis=0) * (1 + 1e-12))


@pytest.mark.parametrize("n,k", [(16, 1), (31, 3), (8, 7)])  # 2k-regular circulant; k=7,n=8.. complete-ish
def test_normalize_regular_graph(ref, n, k):
    A = np.zeros((n, n), dtype=bool)
    for i in range(n):
        for s in range(1, k + 1):
            A[i, (i + s) % n] = A[(i + s) % n, i] = True
    np.fill_diagonal(A, False)
    deg = int(A[0].sum())
    S = sp.csr_matrix(A.astype(float))
    S.sort_indices()
    rp, ci, val = ref.csr_normalize(n, n, S.indptr.astype(np.int32), S.indices.astype(np.int32))
    assert np.all(val == 1.0 / (deg + 1))
    y = ref.spmm(ref.OP_N, n, n, rp, ci, val, np.full((n, 2), 3.0))
    np.testing.assert_allclose(y, 3.0, rtol=1e-15)


def test_normalize_isolated_vertex_and_existing_loop(ref):
    # vertex 2 isolated; vertex 0 already has a self-loop: it must stay a single entry
    rp = np.array([0, 2, 3, 3], dtype=np.int32)
    ci = np.array([0, 1, 0], dtype=np.int32)
    rp2, ci2, val = ref.csr_normalize(3, 3, rp, ci)
    assert rp2.tolist() == [0, 2, 4, 5] and ci2.tolist() == [0, 1, 0, 1, 2]
    assert val[4] == 1.0
    np.testing.assert_allclose(val[:4], 0.5, rtol=0)


def test_normalize_mean_mode_constant_features(ref):
    """Eq. 2: every vertex averages its in-neighbours, so A^T_mean * c1 = c1."""
    rng = np.random.default_rng(5)
    A, rp, ci = random_pattern(48, 48, 0.12, rng, symmetric=False)
    rp2, ci2, val = ref.csr_normalize(48, 48, rp, ci, mode=ref.NORM_MEAN_IN)
    D = to_dense(48, 48, rp2, ci2, val)
    At = (A | np.eye(48, dtype=bool)).astype(float)
    np.testing.assert_allclose(D, At / At.sum(axis=0, keepdims=True), rtol=1e-15)
    y = ref.spmm(ref.OP_T, 48, 48, rp2, ci2, val, np.full((48, 3), 2.5))
    np.testing.assert_allclose(y, 2.5, rtol=1e-14)
    # exactly representable case: ring with self-loop has column count 3? use 4-cycle pairs -> count 2
    rp = np.array([0, 1, 2], dtype=np.int32)
    ci = np.array([1, 0], dtype=np.int32)
    rp2, ci2, val = ref.csr_normalize(2, 2, rp, ci, mode=ref.NORM_MEAN_IN)
    assert np.all(val == 0.5)
    y = ref.spmm(ref.OP_T, 2, 2, rp2, ci2, val, np.full((2, 1), 7.0))
    assert np.all(y == 7.0)


def test_normalize_rectangular_block_with_given_degrees(ref):
    rng = np.random.default_rng(9)
    A, rp, ci = random_pattern(12, 40, 0.2, rng, symmetric=False)
    dr = rng.integers(1, 50, size=12).astype(np.float64)
    dc = rng.integers(1, 50, size=40).astype(np.float64)
    rp2, ci2, val = ref.csr_normalize(12, 40, rp, ci, deg_row=dr, deg_col=dc)
    At = A.copy()
    At[np.arange(12), np.arange(12)] = True
    want = At / np.sqrt(np.outer(dr, dc))
    np.testing.assert_allclose(to_dense(12, 40, rp2, ci2, val), want, rtol=1e-15)


def test_validate_rejects_bad_csr(ref):
    ok = ref.csr_validate(2, 2, np.array([0, 1, 2]), np.array([1, 0]))
    assert ok == 0
    assert ref.csr_validate(2, 2, np.array([0, 2, 2]), np.array([1, 0])) != 0  # unsorted
    assert ref.csr_validate(2, 2, np.array([0, 2, 2]), np.array([1, 1])) != 0  # duplicate
    assert ref.csr_validate(2, 2, np.array([0, 1, 2]), np.array([1, 2])) != 0  # out of range
    assert ref.csr_validate(2, 2, np.array([0, 2, 1]), np.array([0, 1])) != 0  # non-monotone


# ----------------------------------------------------------------------------
# SpMM
# ----------------------------------------------------------------------------

def _small_graph(ref, n=57, density=0.1, seed=3, mode=None, symmetric=True):
    rng = np.random.default_rng(seed)
    A, rp, ci = random_pattern(n, n, density, rng, symmetric=symmetric)
    rp2, ci2, val = ref.csr_normalize(n, n, rp, ci, mode=ref.NORM_SYM if mode is None else mode)
    return rp2, ci2, val, to_dense(n, n, rp2, ci2, val)


@pytest.mark.parametrize("F", [1, 3, 16, 41])
def test_spmm_dense_bruteforce_and_scipy(ref, F):
    n = 57
    rp, ci, val, D = _small_graph(ref, n)
    X = np.random.default_rng(F).standard_normal((n, F))
    Y = ref.spmm(ref.OP_N, n, n, rp, ci, val, X)
    np.testing.assert_allclose(Y, D @ X, rtol=1e-13, atol=1e-14)
    S = sp.csr_matrix((val, ci, rp), shape=(n, n))
    np.testing.assert_allclose(Y, S @ X, rtol=1e-13, atol=1e-14)
    # transpose op against the dense transpose, non-symmetric operator
    rp, ci, val, D = _small_graph(ref, n, mode=ref.NORM_MEAN_IN, symmetric=False, seed=4)
    assert not np.allclose(D, D.T)
    np.testing.assert_allclose(ref.spmm(ref.OP_T, n, n, rp, ci, val, X), D.T @ X, rtol=1e-13, atol=1e-14)


def test_spmm_rectangular(ref):
    rng = np.random.default_rng(12)
    A, rp, ci = random_pattern(20, 70, 0.1, rng, symmetric=False)
    val = rng.standard_normal(len(ci))
    D = to_dense(20, 70, rp, ci, val)
    X = rng.standard_normal((70, 5))
    G = rng.standard_normal((20, 5))
    np.testing.assert_allclose(ref.spmm(ref.OP_N, 20, 70, rp, ci, val, X), D @ X, rtol=1e-13, atol=1e-14)
    np.testing.assert_allclose(ref.spmm(ref.OP_T, 20, 70, rp, ci, val, G), D.T @ G, rtol=1e-13, atol=1e-14)
    # adjoint identity <A X, G> = <X, A^T G>
    lhs = np.sum(ref.spmm(ref.OP_N, 20, 70, rp, ci, val, X) * G)
    rhs = np.sum(X * ref.spmm(ref.OP_T, 20, 70, rp, ci, val, G))
    assert abs(lhs - rhs) <= 1e-12 * max(1.0, abs(lhs))


def test_spmm_structural_invariants(ref):
    g = wl.erdos_renyi(300, 0.03, 21)
    n = g.n_rows
    rp, ci, val = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    rng = np.random.default_rng(1)
    X = rng.standard_normal((n, 24))
    X2 = rng.standard_normal((n, 24))
    Y = ref.spmm(ref.OP_N, n, n, rp, ci, val, X)
    # symmetric operator: transpose op gives bit-identical output
    YT = ref.spmm(ref.OP_T, n, n, rp, ci, val, X)
    assert np.array_equal(Y, YT)
    # linearity
    Y2 = ref.spmm(ref.OP_N, n, n, rp, ci, val, X2)
    np.testing.assert_allclose(ref.spmm(ref.OP_N, n, n, rp, ci, val, 2 * X - 3 * X2), 2 * Y - 3 * Y2,
                               rtol=1e-12, atol=1e-13)
    # feature columns are independent ("SpMM scales each feature dimension independently")
    Y8 = ref.spmm(ref.OP_N, n, n, rp, ci, val, X[:, :8])
    assert np.array_equal(Y8, Y[:, :8])
    # empty graph: A^ is the identity
    rpe, cie, vale = ref.csr_normalize(n, n, np.zeros(n + 1, np.int32), np.zeros(0, np.int32))
    assert np.array_equal(ref.spmm(ref.OP_N, n, n, rpe, cie, vale, X), X)
    # vertex relabelling commutes with the product (section "Permutation")
    perm = rng.permutation(n)
    inv = np.argsort(perm)
    S = sp.csr_matrix((val, ci, rp), shape=(n, n))
    Sp = S[inv][:, inv].tocsr()
    Sp.sort_indices()
    Xp = np.empty_like(X)
    Xp[perm] = X
    Yp = ref.spmm(ref.OP_N, n, n, Sp.indptr, Sp.indices, Sp.data, Xp)
    np.testing.assert_allclose(Yp[perm], Y, rtol=1e-12, atol=1e-13)


def test_spmm_column_panel_accumulate(ref):
    """Stage-wise C += A^{ij} H^j over column panels equals the unsplit product (1-D row scheme)."""
    g = wl.erdos_renyi(200, 0.05, 33)
    n = g.n_rows
    rp, ci, val = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    X = np.random.default_rng(2).standard_normal((n, 7))
    S = sp.csr_matrix((val, ci, rp), shape=(n, n))
    Y = np.zeros((n, 7))
    bounds = [0, 50, 51, 130, 200]
    for a, b in zip(bounds[:-1], bounds[1:]):
        P = S[:, a:b].tocsr()
        P.sort_indices()
        ref.spmm(ref.OP_N, n, b - a, P.indptr, P.indices, P.data, X[a:b], beta=1.0, Y=Y)
    np.testing.assert_allclose(Y, ref.spmm(ref.OP_N, n, n, rp, ci, val, X), rtol=1e-12, atol=1e-13)


def test_transpose_matches_scipy(ref):
    rng = np.random.default_rng(8)
    A, rp, ci = random_pattern(30, 45, 0.15, rng, symmetric=False)
    val = rng.standard_normal(len(ci))
    rpt, cit, vat = ref.csr_transpose(30, 45, rp, ci, val)
    T = sp.csr_matrix((val, ci, rp), shape=(30, 45)).T.tocsr()
    T.sort_indices()
    assert np.array_equal(rpt, T.indptr) and np.array_equal(cit, T.indices) and np.array_equal(vat, T.data)


# ----------------------------------------------------------------------------
# GeMM, ReLU, loss
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (17, 5, 9), (64, 33, 70)])
def test_gemm_against_numpy(ref, M, N, K):
    rng = np.random.default_rng(M + N + K)
    A, B = rng.standard_normal((M, K)), rng.standard_normal((K, N))
    want = A @ B
    np.testing.assert_allclose(ref.gemm(ref.OP_N, ref.OP_N, A, B), want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref.gemm(ref.OP_T, ref.OP_N, np.ascontiguousarray(A.T), B), want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(ref.gemm(ref.OP_N, ref.OP_T, A, np.ascontiguousarray(B.T)), want, rtol=1e-12, atol=1e-13)
    C0 = rng.standard_normal((M, N))
    got = ref.gemm(ref.OP_N, ref.OP_N, A, B, beta=1.0, Cmat=C0.copy())
    np.testing.assert_allclose(got, C0 + want, rtol=1e-12, atol=1e-13)
    # identity and one-hot weights
    assert np.array_equal(ref.gemm(ref.OP_N, ref.OP_N, A, np.eye(K)), A)


def test_relu_and_mask(ref):
    Z = np.array([[-1.0, 0.0, 2.0], [3.0, -0.0, -5.0]])
    assert np.array_equal(ref.relu(Z), np.array([[0.0, 0.0, 2.0], [3.0, 0.0, 0.0]]))
    G = np.full((2, 3), 7.0)
    assert np.array_equal(ref.relu_bwd(Z, G), np.array([[0.0, 0.0, 7.0], [7.0, 0.0, 0.0]]))


@pytest.mark.parametrize("C", [8, 41, 47])
def test_softmax_ce_closed_forms(ref, C):
    rng = np.random.default_rng(C)
    n = 37
    labels = rng.integers(0, C, size=n).astype(np.int32)
    # zero logits -> loss = ln C exactly (up to rounding), gradient (1/C - onehot)/n
    loss, dZ = ref.softmax_ce(np.zeros((n, C)), labels)
    assert abs(loss - math.log(C)) < 1e-15 * 4
    want = np.full((n, C), 1.0 / C)
    want[np.arange(n), labels] -= 1.0
    np.testing.assert_allclose(dZ, want / n, rtol=1e-14)
    Z = rng.standard_normal((n, C)) * 5
    loss, dZ = ref.softmax_ce(Z, labels)
    # rows of the gradient sum to zero; shift invariance
    np.testing.assert_allclose(dZ.sum(axis=1), 0.0, atol=1e-16)
    loss2, dZ2 = ref.softmax_ce(Z + 1000.0, labels)
    assert abs(loss - loss2) < 1e-10
    np.testing.assert_allclose(dZ, dZ2, atol=1e-12)
    # third opinion
    import torch

    tl = torch.nn.functional.cross_entropy(torch.from_numpy(Z), torch.from_numpy(labels.astype(np.int64)))
    assert abs(tl.item() - loss) < 1e-12


# ----------------------------------------------------------------------------
# layers, epoch, gradients
# ----------------------------------------------------------------------------

def _setup_model(ref, n, dims, seed, mode=None, symmetric=True, density=0.15):
    rng = np.random.default_rng(seed)
    A, rp, ci = random_pattern(n, n, density, rng, symmetric=symmetric)
    rp2, ci2, val = ref.csr_normalize(n, n, rp, ci, mode=ref.NORM_SYM if mode is None else mode)
    X = rng.standard_normal((n, dims[0]))
    Ws = [rng.standard_normal((dims[l], dims[l + 1])) * math.sqrt(2.0 / (dims[l] + dims[l + 1]))
          for l in range(len(dims) - 1)]
    labels = rng.integers(0, dims[-1], size=n).astype(np.int32)
    return rp2, ci2, val, X, Ws, labels


def test_order_rule(ref):
    assert ref.order(100, 256) == ref.SPMM_FIRST
    assert ref.order(256, 256) == ref.GEMM_FIRST  # tie -> GeMM first
    assert ref.order(602, 128) == ref.GEMM_FIRST


def test_layer_forward_orders_agree_with_dense(ref):
    n, dims = 40, (12, 20)
    rp, ci, val, X, Ws, _ = _setup_model(ref, n, dims, 1)
    D = to_dense(n, n, rp, ci, val)
    want = np.maximum(D @ X @ Ws[0], 0.0)
    a = ref.layer_fwd(n, rp, ci, val, X, Ws[0], ref.GEMM_FIRST, True)
    b = ref.layer_fwd(n, rp, ci, val, X, Ws[0], ref.SPMM_FIRST, True)
    np.testing.assert_allclose(a, want, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(b, want, rtol=1e-12, atol=1e-13)
    c = ref.layer_fwd(n, rp, ci, val, X, Ws[0], ref.GEMM_FIRST, False)
    np.testing.assert_allclose(c, D @ X @ Ws[0], rtol=1e-12, atol=1e-13)


def _torch_epoch(rp, ci, val, X, Ws, labels, n):
    import torch

    S = sp.csr_matrix((val, ci, rp), shape=(n, n)).tocoo()
    A = torch.sparse_coo_tensor(np.vstack([S.row, S.col]), S.data, (n, n), dtype=torch.float64).coalesce()
    H = torch.from_numpy(X)
    Wt = [torch.from_numpy(w.copy()).requires_grad_(True) for w in Ws]
    for l, w in enumerate(Wt):
        H = torch.sparse.mm(A, H @ w)
        if l + 1 < len(Wt):
            H = torch.relu(H)
    loss = torch.nn.functional.cross_entropy(H, torch.from_numpy(labels.astype(np.int64)))
    loss.backward()
    return loss.item(), [w.grad.numpy() for w in Wt], H.detach().numpy()


@pytest.mark.parametrize("dims,mode,sym", [((9, 6, 4), None, True), ((5, 11, 7, 3), None, True),
                                            ((6, 6, 5), "mean", False), ((4, 9, 3), "mean", False)])
def test_epoch_against_torch_autograd_and_orders(ref, dims, mode, sym):
    n = 35
    m = ref.NORM_MEAN_IN if mode == "mean" else ref.NORM_SYM
    rp, ci, val, X, Ws, labels = _setup_model(ref, n, dims, sum(dims), mode=m, symmetric=sym)
    loss_t, WG_t, logits_t = _torch_epoch(rp, ci, val, X, Ws, labels, n)
    L = len(Ws)
    seen = []
    for orders in (None, [ref.GEMM_FIRST] * L, [ref.SPMM_FIRST] * L):
        loss, WG, logits = ref.epoch(n, rp, ci, val, X, labels, Ws, orders=orders, want_logits=True)
        assert abs(loss - loss_t) < 1e-12
        np.testing.assert_allclose(logits, logits_t, rtol=1e-11, atol=1e-12)
        for a, b in zip(WG, WG_t):
            np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-13)
        seen.append(WG)
    # the two associations agree to rounding ("Order of Computation")
    for a, b in zip(seen[1], seen[2]):
        np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-14)


@pytest.mark.parametrize("order_name", ["gemm_first", "spmm_first"])
@pytest.mark.parametrize("mode", ["sym", "mean"])
def test_epoch_gradients_finite_differences(ref, order_name, mode):
    n, dims = 24, (7, 10, 5)
    m = ref.NORM_MEAN_IN if mode == "mean" else ref.NORM_SYM
    rp, ci, val, X, Ws, labels = _setup_model(ref, n, dims, 77, mode=m, symmetric=(mode == "sym"))
    o = ref.GEMM_FIRST if order_name == "gemm_first" else ref.SPMM_FIRST
    orders = [o] * 2
    _, WG, _ = ref.epoch(n, rp, ci, val, X, labels, Ws, orders=orders)
    rng = np.random.default_rng(0)
    h = 1e-6
    for l in range(2):
        for _ in range(6):
            a, b = rng.integers(0, dims[l]), rng.integers(0, dims[l + 1])
            Wp = [w.copy() for w in Ws]
            Wm = [w.copy() for w in Ws]
            Wp[l][a, b] += h
            Wm[l][a, b] -= h
            lp, _, _ = ref.epoch(n, rp, ci, val, X, labels, Wp, orders=orders)
            lm, _, _ = ref.epoch(n, rp, ci, val, X, labels, Wm, orders=orders)
            fd = (lp - lm) / (2 * h)
            assert abs(fd - WG[l][a, b]) <= 1e-6 * max(abs(fd), 1e-3), (l, a, b, fd, WG[l][a, b])


def test_layer_bwd_input_gradient_finite_differences(ref):
    """H_G of a middle layer: perturb the layer input, watch sum(H_out * R)."""
    n, d_in, d_out = 20, 6, 8
    rp, ci, val, X, Ws, _ = _setup_model(ref, n, (d_in, d_out), 5, mode=ref.NORM_MEAN_IN, symmetric=False)
    R = np.random.default_rng(3).standard_normal((n, d_out))
    for o in (ref.GEMM_FIRST, ref.SPMM_FIRST):
        out = ref.layer_fwd(n, rp, ci, val, X, Ws[0], o, True)
        WG, HG, ZG = ref.layer_bwd(n, rp, ci, val, X, out, R, Ws[0], o, True)
        rng = np.random.default_rng(4)
        for _ in range(8):
            i, f = rng.integers(0, n), rng.integers(0, d_in)
            h = 1e-6
            Xp, Xm = X.copy(), X.copy()
            Xp[i, f] += h
            Xm[i, f] -= h
            fp = np.sum(ref.layer_fwd(n, rp, ci, val, Xp, Ws[0], o, True) * R)
            fm = np.sum(ref.layer_fwd(n, rp, ci, val, Xm, Ws[0], o, True) * R)
            fd = (fp - fm) / (2 * h)
            assert abs(fd - HG[i, f]) <= 1e-6 * max(abs(fd), 1e-3)


def test_zero_weights_give_ln_c(ref):
    cfg = wl.CONFIGS["tiny"]
    g = cfg.graph()
    n = g.n_rows
    rp, ci, val = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    X = cfg.features(n).astype(np.float64)
    Ws = [np.zeros((64, 16)), np.zeros((16, 8))]
    loss, WG, _ = ref.epoch(n, rp, ci, val, X, cfg.labels(n), Ws)
    assert abs(loss - math.log(8)) < 1e-12  # 4096-term running sum
    assert all(np.all(w == 0) for w in WG[:1])  # dead ReLUs block the first layer's gradient


def test_tiny_config_epoch_against_torch(ref):
    cfg = wl.CONFIGS["tiny"]
    g = cfg.graph()
    n = g.n_rows
    rp, ci, val = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    X = cfg.features(n).astype(np.float64)
    Ws = [w.astype(np.float64) for w in cfg.weights()]
    labels = cfg.labels(n)
    loss, WG, _ = ref.epoch(n, rp, ci, val, X, labels, Ws)
    loss_t, WG_t, _ = _torch_epoch(rp, ci, val, X, Ws, labels, n)
    assert abs(loss - loss_t) < 1e-12
    for a, b in zip(WG, WG_t):
        np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-14)


def test_epoch_with_injected_relu_decisions(ref):
    """Handing the oracle its own ReLU' decisions changes nothing; flipping one decision at
    (u, b) of the hidden layer changes exactly the gradient paths through unit b."""
    n, dims = 30, (6, 9, 4)
    rp, ci, val, X, Ws, labels = _setup_model(ref, n, dims, 123)
    loss, WG, _ = ref.epoch(n, rp, ci, val, X, labels, Ws)
    H1 = ref.layer_fwd(n, rp, ci, val, X, Ws[0], ref.order(6, 9), True)
    own = (H1 > 0).astype(np.uint8)
    loss2, WG2, _ = ref.epoch(n, rp, ci, val, X, labels, Ws, relu_masks=[own])
    assert loss == loss2
    for a, b in zip(WG, WG2):
        assert np.array_equal(a, b)
    flipped = own.copy()
    u, b = 5, 2
    flipped[u, b] ^= 1
    _, WG3, _ = ref.epoch(n, rp, ci, val, X, labels, Ws, relu_masks=[flipped])
    assert np.array_equal(WG3[1], WG[1])                 # last layer's gradient does not see the mask
    changed = np.any(WG3[0] != WG[0], axis=0)
    assert changed[b] and not np.any(np.delete(changed, b))


def test_adam_against_closed_form_and_torch(ref):
    import torch

    rng = np.random.default_rng(4)
    W0 = rng.standard_normal((13, 7))
    grads = [rng.standard_normal((13, 7)) * 10.0 ** rng.integers(-4, 2) for _ in range(4)]
    # first step from zero moments: the bias-corrected ratio is g / (|g| + eps) exactly
    W, m, v = W0.copy(), np.zeros_like(W0), np.zeros_like(W0)
    ref.adam_step(W, grads[0], m, v, 1, lr=0.05, eps=1e-8)
    np.testing.assert_allclose(W, W0 - 0.05 * grads[0] / (np.abs(grads[0]) + 1e-8), rtol=1e-12)
    # several steps against torch's optimiser in fp64
    Wt = torch.from_numpy(W0.copy()).requires_grad_(True)
    opt = torch.optim.Adam([Wt], lr=0.05, betas=(0.9, 0.999), eps=1e-8)
    W, m, v = W0.copy(), np.zeros_like(W0), np.zeros_like(W0)
    for t, g in enumerate(grads, start=1):
        Wt.grad = torch.from_numpy(g.copy())
        opt.step()
        ref.adam_step(W, g, m, v, t, lr=0.05)
        np.testing.assert_allclose(W, Wt.detach().numpy(), rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------------------
# bfloat16 copy of the gathered operand (extension beyond the paper's fp32)
# ----------------------------------------------------------------------------

def _f32_from_bits(bits):
    return np.array(bits, dtype=np.uint32).view(np.float32)


def test_bf16_round_worked_values(ref):
    """Hand-worked roundings.  bfloat16 keeps 7 fraction bits, so its step at 1.0 is 2^-7."""
    cases = [
        (1.0, 0x3F80),
        (1.0 + 2.0 ** -8, 0x3F80),                 # tie between 1 and 1+2^-7: even fraction (0) wins
        (1.0 + 2.0 ** -8 + 2.0 ** -23, 0x3F81),    # just above the tie
        (1.0 + 2.0 ** -7 + 2.0 ** -8, 0x3F82),     # tie between fractions 1 and 2: even (2) wins
        (-(1.0 + 2.0 ** -8), 0xBF80),              # sign does not change the choice
        (0.0, 0x0000),
        (-0.0, 0x8000),
        (np.inf, 0x7F80),
        (-np.inf, 0xFF80),
        (3.0, 0x4040),
        (0.1, 0x3DCD),                             # 0.1f = 0x3DCCCCCD: low half 0xCCCD > 0x8000 -> up
    ]
    x = np.array([c[0] for c in cases], dtype=np.float32)
    codes, values = ref.bf16_round(x)
    assert [int(c) for c in codes] == [c[1] for c in cases]
    assert np.array_equal(values.view(np.uint32), codes.astype(np.uint32) << 16)
    # largest finite float32 is more than half a step above the largest finite bfloat16 -> infinity;
    # the largest bfloat16 itself and anything below its upper tie stay finite
    big = _f32_from_bits([0x7F7FFFFF, 0x7F7F0000, 0x7F7F7FFF, 0x7F7F8000])
    codes, _ = ref.bf16_round(big)
    assert [int(c) for c in codes] == [0x7F80, 0x7F7F, 0x7F7F, 0x7F80]
    # subnormal float32: same rule on the bit pattern (steps are uniform there)
    sub = _f32_from_bits([0x00000001, 0x00008000, 0x00008001, 0x00018000, 0x807FFFFF])
    codes, _ = ref.bf16_round(sub)
    assert [int(c) for c in codes] == [0x0000, 0x0000, 0x0001, 0x0002, 0x8080]
    # NaN stays NaN
    codes, values = ref.bf16_round(_f32_from_bits([0x7FC00000, 0x7F800001, 0xFFFFFFFF]))
    assert np.all(np.isnan(values))


def test_bf16_round_against_integer_rule_and_torch(ref):
    """Every upper half-word with the low half-words around the tie, plus random bit patterns:
    compared with the rule stated on integers (magnitude m = q*2^16 + r: round q up iff r > 2^15, or
    r == 2^15 and q odd) and with torch's float32 -> bfloat16 conversion."""
    import torch

    hi = np.arange(1 << 16, dtype=np.uint32) << 16
    lows = np.array([0x0000, 0x0001, 0x7FFF, 0x8000, 0x8001, 0xFFFF], dtype=np.uint32)
    bits = (hi[:, None] | lows[None, :]).ravel()
    rng = np.random.default_rng(11)
    bits = np.concatenate([bits, rng.integers(0, 1 << 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)])
    x = bits.view(np.float32)
    codes, values = ref.bf16_round(x)
    finite = np.isfinite(x)
    mag = (bits & 0x7FFFFFFF).astype(np.int64)
    q, r = mag >> 16, mag & 0xFFFF
    q = q + ((r > 0x8000) | ((r == 0x8000) & (q & 1 == 1)))
    want = ((bits >> 31).astype(np.int64) << 15) | q
    assert np.array_equal(codes[finite].astype(np.int64), want[finite])
    t = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(codes[finite], t[finite])
    assert np.all(np.isnan(values[np.isnan(x)]))
    assert np.array_equal(values[np.isinf(x)], x[np.isinf(x)])
    # properties of a rounding: idempotent, monotone, within half a step (at most 2^-8 relative for normal values)
    again, _ = ref.bf16_round(values)
    assert np.array_equal(again[finite], codes[finite])
    xs = np.sort(x[finite])
    _, vs = ref.bf16_round(xs)
    assert np.all(vs[1:] >= vs[:-1])
    normal = finite & (np.abs(x) >= 2.0 ** -126) & np.isfinite(values)
    err = np.abs(values[normal].astype(np.float64) - x[normal].astype(np.float64))
    assert np.all(err <= 2.0 ** -8 * np.abs(x[normal].astype(np.float64)))


def _numpy_epoch_bf16(rp, ci, val, X, Ws, labels, n, orders):
    """The bfloat16-gather epoch re-composed from scipy / numpy products, with torch's conversion as
    the rounding: every SpMM sees its dense operand rounded float64 -> float32 -> bfloat16."""
    import torch

    def q(M):
        t = torch.from_numpy(np.ascontiguousarray(M, dtype=np.float32)).to(torch.bfloat16)
        return t.to(torch.float64).numpy()

    A = sp.csr_matrix((val, ci, rp), shape=(n, n))
    L = len(Ws)
    H = [X]
    for l in range(L):
        Z = A @ q(H[l] @ Ws[l]) if orders[l] == 0 else (A @ q(H[l])) @ Ws[l]
        H.append(np.maximum(Z, 0.0) if l + 1 < L else Z)
    Z = H[L]
    lse = np.log(np.exp(Z - Z.max(axis=1, keepdims=True)).sum(axis=1)) + Z.max(axis=1)
    loss = float(np.mean(lse - Z[np.arange(n), labels]))
    G = np.exp(Z - lse[:, None])
    G[np.arange(n), labels] -= 1.0
    G /= n
    WG = [None] * L
    for l in range(L - 1, -1, -1):
        if l + 1 < L:
            G = G * (H[l + 1] > 0)
        if orders[l] == 0:
            T = A.T @ q(G)
            WG[l] = H[l].T @ T
            G = T @ Ws[l].T
        else:
            WG[l] = (A @ q(H[l])).T @ G
            G = A.T @ q(G @ Ws[l].T) if l > 0 else None
    return loss, WG


@pytest.mark.parametrize("dims,mode,sym", [((9, 6, 4), None, True), ((5, 11, 7, 3), None, True),
                                            ((6, 6, 5), "mean", False), ((4, 9, 3), "mean", False)])
def test_epoch_bf16_against_numpy_recomposition(ref, dims, mode, sym):
    n = 37
    m = ref.NORM_MEAN_IN if mode == "mean" else ref.NORM_SYM
    rp, ci, val, X, Ws, labels = _setup_model(ref, n, dims, 7 + sum(dims), mode=m, symmetric=sym)
    L = len(Ws)
    auto = [ref.order(dims[l], dims[l + 1]) for l in range(L)]
    for orders in (None, [ref.GEMM_FIRST] * L, [ref.SPMM_FIRST] * L):
        loss, WG, own_f, own_b = ref.epoch_bf16(n, rp, ci, val, X, labels, Ws, orders=orders)
        want_loss, want_WG = _numpy_epoch_bf16(rp, ci, val, X, Ws, labels, n, auto if orders is None else orders)
        assert abs(loss - want_loss) < 1e-12
        for a, b in zip(WG, want_WG):
            np.testing.assert_allclose(a, b, rtol=1e-10, atol=1e-13)
        # it is a perturbation of the fp32-operand epoch of the size of the rounding step, not equal to it
        loss32, WG32, _ = ref.epoch(n, rp, ci, val, X, labels, Ws, orders=orders)
        assert loss != loss32 and abs(loss - loss32) < 2e-2 * abs(loss32)
        for a, b in zip(WG, WG32):
            assert np.max(np.abs(a - b)) < 5e-2 * np.max(np.abs(b))


def test_epoch_bf16_recorded_and_injected_operands(ref):
    n, dims = 33, (6, 10, 4)
    rp, ci, val, X, Ws, labels = _setup_model(ref, n, dims, 99)
    orders = [ref.SPMM_FIRST, ref.GEMM_FIRST]
    loss, WG, own_f, own_b = ref.epoch_bf16(n, rp, ci, val, X, labels, Ws, orders=orders)
    # the recorded operands are the roundings of what the chain feeds its SpMMs
    assert own_f[0].shape == (n, 6) and own_f[1].shape == (n, 4) and own_b[0] is None and own_b[1].shape == (n, 4)
    assert np.array_equal(own_f[0], ref.bf16_round(X.astype(np.float32))[0])
    _, xq = ref.bf16_round(X.astype(np.float32))
    A = sp.csr_matrix((val, ci, rp), shape=(n, n))
    H1 = np.maximum((A @ xq.astype(np.float64)) @ Ws[0], 0.0)
    assert np.array_equal(own_f[1], ref.bf16_round((H1 @ Ws[1]).astype(np.float32))[0])
    # handing the oracle its own roundings changes nothing
    loss2, WG2, f2, b2 = ref.epoch_bf16(n, rp, ci, val, X, labels, Ws, orders=orders, fwd_codes=own_f, bwd_codes=own_b)
    assert loss2 == loss and all(np.array_equal(a, b) for a, b in zip(WG, WG2))
    assert all(np.array_equal(a, b) for a, b in zip(own_f, f2))
    # an all-zero operand for the last layer's forward SpMM gives zero logits: loss = ln C exactly
    zero = [None, np.zeros((n, 4), dtype=np.uint16)]
    loss3, _, f3, _ = ref.epoch_bf16(n, rp, ci, val, X, labels, Ws, orders=orders, fwd_codes=zero)
    assert abs(loss3 - math.log(4.0)) < 1e-15
    assert np.array_equal(f3[1], own_f[1])  # what is recorded is still the oracle's own rounding
    # moving one operand entry by one bfloat16 step moves the result, by about that step's share
    bumped = [own_f[0].copy(), None]
    bumped[0][3, 2] += 1
    loss4, _, _, _ = ref.epoch_bf16(n, rp, ci, val, X, labels, Ws, orders=orders, fwd_codes=bumped)
    assert loss4 != loss and abs(loss4 - loss) < 1e-3


# ----------------------------------------------------------------------------------------------
# the arithmetic behind the GeMM extension on the bfloat16 matrix instructions: facts about fp32
# numbers, checked here in numpy, that the tolerance of its GPU tests rests on (no product code)
# ----------------------------------------------------------------------------------------------

def _three_pieces(x):
    """x (fp32) -> its upper 16 bits, the upper 16 bits of what that leaves, and the rest"""
    top = (x.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    r1 = x - top
    mid = (r1.view(np.uint32) & np.uint32(0xFFFF0000)).view(np.float32)
    low = r1 - mid
    return top, mid, low


def test_fp32_is_the_exact_sum_of_three_bfloat16_pieces():
    rng = np.random.default_rng(12)
    bits = rng.integers(0, 2 ** 32, size=2_000_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x) & (np.abs(x) > 2.0 ** -100) & (np.abs(x) < 2.0 ** 100)]
    x = np.concatenate([x, np.float32([1.0, -1.0, 1.0 + 2.0 ** -23, 2.0 - 2.0 ** -23, 3.0, 0.1, 1e-30, -7e29, 0.0])])
    top, mid, low = _three_pieces(x)
    with np.errstate(over="ignore"):
        # every piece is a bfloat16 number (its lower 16 bits are zero) ...
        for piece in (top, mid, low):
            assert np.all((piece.view(np.uint32) & np.uint32(0xFFFF)) == 0)
        # ... the three add up to x exactly, and both subtractions were exact in fp32
        assert np.array_equal(top.astype(np.float64) + mid.astype(np.float64) + low.astype(np.float64), x.astype(np.float64))
        assert np.array_equal((x.astype(np.float64) - top.astype(np.float64)).astype(np.float32).astype(np.float64),
                              x.astype(np.float64) - top.astype(np.float64))
    ax = np.abs(x.astype(np.float64))
    assert np.all(np.abs(mid) <= 2.0 ** -7 * ax) and np.all(np.abs(low) <= 2.0 ** -15 * ax)


def test_six_of_nine_piece_products_lose_less_than_2_to_minus_21():
    rng = np.random.default_rng(13)
    a = rng.standard_normal(1_000_000).astype(np.float32)
    b = (rng.standard_normal(1_000_000) * 37.0).astype(np.float32)
    a0, a1, a2 = (p.astype(np.float64) for p in _three_pieces(a))
    b0, b1, b2 = (p.astype(np.float64) for p in _three_pieces(b))
    kept = a2 * b0 + a0 * b2 + a1 * b1 + a1 * b0 + a0 * b1 + a0 * b0   # each term exact: 8 x 8 significand bits
    exact = a.astype(np.float64) * b.astype(np.float64)
    lost = np.abs(exact - kept)
    assert np.all(lost <= 2.0 ** -21 * np.abs(exact))
    assert lost.mean() <= 2.0 ** -23 * np.abs(exact).mean()  # on average a fraction of one fp32 rounding
    # a product of two pieces has at most 16 significand bits: exact in the fp32 the matrix unit adds in
    p = (a1 * b1)
    assert np.array_equal(p.astype(np.float32).astype(np.float64), p)
