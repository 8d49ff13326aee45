"""GPU parity: every entry point of the C-ABI library against the fp64 CPU oracle, element by
element on the same seeded inputs.  Integer and index results must match bit for bit; fp32
results must satisfy, per output row,  max|got - ref| <= 1e-4 * max|ref|  (the tolerance the
build's target states), with the oracle fed the same fp32 inputs widened to fp64."""
import sys

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu

TOL = 1e-4


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def mg():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2110_08688_amd as m

    m.binding.lib()  # fails loudly if libmggcn.so is missing
    return m


@pytest.fixture(scope="module")
def dev():
    import torch

    return torch.device("cuda:0")


def to_dev(a, dev):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def row_err(got, want):
    """per-row max-norm relative error; rows whose reference is exactly zero must be zero"""
    got = np.asarray(got, dtype=np.float64)
    num = np.abs(got - want).max(axis=1) if want.shape[1] else np.zeros(want.shape[0])
    den = np.abs(want).max(axis=1) if want.shape[1] else np.ones(want.shape[0])
    zero = den == 0
    assert np.all(num[zero] == 0), "rows with an exactly-zero reference must be exactly zero"
    return np.where(zero, 0.0, num / np.maximum(den, 1e-300))


def assert_rows_close(got, want, tol=TOL, what="", pre=None):
    """pre: for an output that went through the fused ReLU, the reference's pre-activation rows.
    ReLU is exact and 1-Lipschitz, so the rounding error of relu(z) is that of the product z, and it
    is measured against the row of z (the row of relu(z) may have lost its largest entries)."""
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    if pre is not None:
        num = np.abs(np.asarray(got, dtype=np.float64) - want).max(axis=1)
        den = np.abs(pre).max(axis=1)
        assert np.all(num[den == 0] == 0)
        e = np.where(den == 0, 0.0, num / np.maximum(den, 1e-300))
    else:
        e = row_err(got, want)
    worst = int(np.argmax(e)) if e.size else -1
    assert e.size == 0 or e[worst] <= tol, f"{what}: row {worst} rel err {e[worst]:.3e} > {tol}"
    return float(e.max()) if e.size else 0.0


def normalized(ref, g, mode=None):
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx,
                                    mode=ref.NORM_SYM if mode is None else mode)
    return rp, ci, val.astype(np.float32)  # the values the GPU path holds


def adversarial_pattern(n=300, seed=5):
    """empty rows, a row holding most entries, a full column, isolated vertices, ragged size"""
    rng = np.random.default_rng(seed)
    rows = [set() for _ in range(n)]
    hub = 7
    for j in range(n):
        if j != hub and j % 3:
            rows[hub].add(j); rows[j].add(hub)
    for _ in range(4 * n):
        a, b = rng.integers(0, n, 2)
        if a != b and a % 11 and b % 11:  # every 11th vertex stays isolated (unless tied to the hub)
            rows[a].add(int(b)); rows[b].add(int(a))
    rowptr = np.zeros(n + 1, np.int32)
    col = []
    for i in range(n):
        c = sorted(rows[i])
        col += c
        rowptr[i + 1] = len(col)
    return wl.Pattern(n, n, rowptr, np.array(col, np.int32))


# ----------------------------------------------------------------------------------------------
# a0: normalisation and transpose -- bit exact
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("case", ["tiny", "adversarial", "powerlaw", "empty", "loops"])
@pytest.mark.parametrize("mode", ["sym", "mean"])
def test_csr_normalize_bit_exact(mg, dev, ref, case, mode):
    say(f"[normalize] case={case} mode={mode}")
    if case == "tiny":
        g = wl.CONFIGS["tiny"].graph()
    elif case == "adversarial":
        g = adversarial_pattern()
    elif case == "powerlaw":
        g = wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99)
    elif case == "empty":
        g = wl.Pattern(77, 77, np.zeros(78, np.int32), np.zeros(0, np.int32))
    else:  # some self-loops already present, non-symmetric pattern
        rng = np.random.default_rng(3)
        A = rng.random((129, 129)) < 0.05
        A[np.arange(0, 129, 4), np.arange(0, 129, 4)] = True
        import scipy.sparse as sp

        S = sp.csr_matrix(A.astype(np.float32)); S.sort_indices()
        g = wl.Pattern(129, 129, S.indptr.astype(np.int32), S.indices.astype(np.int32))
    m = ref.NORM_MEAN_IN if mode == "mean" else ref.NORM_SYM
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx, mode=m)
    grp, gci, gval = mg.mggcn_csr_normalize(g.n_rows, g.n_cols, to_dev(g.rowptr, dev), to_dev(g.colidx, dev),
                                            mode=mg.NORM_MEAN_IN if mode == "mean" else mg.NORM_SYM_SELFLOOP,
                                            validate=True)
    assert np.array_equal(grp.cpu().numpy(), rp)
    assert np.array_equal(gci.cpu().numpy(), ci)
    assert np.array_equal(gval.cpu().numpy().view(np.int32), val.astype(np.float32).view(np.int32))


def test_csr_normalize_rectangular_block(mg, dev, ref):
    g = wl.row_block(500, 4000, 6000, 2.5, 200.0, 1.6, 17)
    rng = np.random.default_rng(1)
    dr = rng.integers(1, 3000, g.n_rows).astype(np.int32)
    dc = rng.integers(1, 3000, g.n_cols).astype(np.int32)
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx, deg_row=dr, deg_col=dc)
    grp, gci, gval = mg.mggcn_csr_normalize(g.n_rows, g.n_cols, to_dev(g.rowptr, dev), to_dev(g.colidx, dev),
                                            deg_row=to_dev(dr, dev), deg_col=to_dev(dc, dev))
    assert np.array_equal(grp.cpu().numpy(), rp) and np.array_equal(gci.cpu().numpy(), ci)
    assert np.array_equal(gval.cpu().numpy().view(np.int32), val.astype(np.float32).view(np.int32))


def test_csr_normalize_rejects_malformed(mg, dev):
    rp = to_dev(np.array([0, 2, 3], np.int32), dev)
    for bad in ([1, 0, 1], [0, 0, 1], [0, 5, 1]):  # unsorted, duplicate, out of range
        with pytest.raises(mg.MggcnError) as ei:
            mg.mggcn_csr_normalize(2, 2, rp, to_dev(np.array(bad, np.int32), dev), validate=True)
        assert ei.value.code == mg.binding.E_BAD_CSR


def test_graph_create_rejects_malformed(mg, dev):
    """a handle is only made of offsets that start at 0 and never decrease and of column indices
    inside the matrix: no product can then gather outside its operand"""
    ones = to_dev(np.ones(3, np.float32), dev)
    good_rp = to_dev(np.array([0, 2, 3], np.int32), dev)
    cases = [([0, 2, 3], [0, 2, 1]),    # column 2 of a 2 x 2 matrix
             ([0, 2, 3], [0, -1, 1]),   # negative column
             ([1, 2, 3], [0, 1, 1]),    # offsets do not start at 0
             ([0, 3, 2], [0, 1, 1])]    # offsets decrease
    for rp, ci in cases:
        with pytest.raises(mg.MggcnError) as ei:
            mg.Graph(2, 2, to_dev(np.array(rp, np.int32), dev), to_dev(np.array(ci, np.int32), dev), ones, F_max=8)
        assert ei.value.code == mg.binding.E_BAD_CSR, (rp, ci)
    # the transposed operator is checked as well
    with pytest.raises(mg.MggcnError) as ei:
        mg.Graph(2, 2, good_rp, to_dev(np.array([0, 1, 1], np.int32), dev), ones,
                 transpose=(good_rp, to_dev(np.array([0, 1, 7], np.int32), dev), ones), F_max=8)
    assert ei.value.code == mg.binding.E_BAD_CSR
    G = mg.Graph(2, 2, good_rp, to_dev(np.array([0, 1, 1], np.int32), dev), ones, F_max=8)
    Y = mg.mggcn_spmm(G, mg.OP_N, to_dev(np.array([[1.0], [10.0]], np.float32), dev))
    assert np.array_equal(Y.cpu().numpy(), np.array([[11.0], [10.0]], np.float32))


@pytest.mark.parametrize("shape", [(30, 45, 0.15), (1000, 700, 0.02), (64, 64, 0.0)])
def test_csr_transpose_exact(mg, dev, ref, shape):
    n, m, dens = shape
    say(f"[transpose] {shape}")
    rng = np.random.default_rng(n)
    import scipy.sparse as sp

    S = sp.random(n, m, density=dens, format="csr", random_state=7, dtype=np.float32)
    S.sort_indices()
    rp, ci, va = S.indptr.astype(np.int32), S.indices.astype(np.int32), S.data.astype(np.float32)
    rpt, cit, vat = ref.csr_transpose(n, m, rp, ci, va.astype(np.float64))
    g = mg.mggcn_csr_transpose(n, m, to_dev(rp, dev), to_dev(ci, dev), to_dev(va, dev))
    assert np.array_equal(g[0].cpu().numpy(), rpt) and np.array_equal(g[1].cpu().numpy(), cit)
    assert np.array_equal(g[2].cpu().numpy(), vat.astype(np.float32))


def test_csr_transpose_many_tiles_passes_and_a_hub_column(mg, dev, ref):
    """The counting sort behind the transpose at sizes that span many sort tiles with a ragged last one,
    column counts that need two, three and four 8-bit passes, a column that every row holds (its run of
    equal keys crosses hundreds of tiles: stability keeps the rows ascending) and empty columns."""
    rng = np.random.default_rng(3)
    for n, m, per_row in ((40_000, 200, 6), (9_001, 70_000, 40), (3_000, 20_000_000, 25)):
        say(f"[transpose big] {n} x {m}, ~{per_row} per row")
        rows = []
        rp = np.zeros(n + 1, np.int64)
        for i in range(n):
            c = np.unique(np.concatenate([rng.integers(0, m, per_row), [7]]))  # column 7 in every row
            rows.append(c)
            rp[i + 1] = rp[i] + len(c)
        ci = np.concatenate(rows).astype(np.int32)
        rp = rp.astype(np.int32)
        va = wl.normal_f32(11, n, (len(ci),))
        rpt, cit, vat = ref.csr_transpose(n, m, rp, ci, va.astype(np.float64))
        g = mg.mggcn_csr_transpose(n, m, to_dev(rp, dev), to_dev(ci, dev), to_dev(va, dev))
        assert np.array_equal(g[0].cpu().numpy(), rpt) and np.array_equal(g[1].cpu().numpy(), cit)
        assert np.array_equal(g[2].cpu().numpy(), vat.astype(np.float32))
        g2 = mg.mggcn_csr_transpose(n, m, to_dev(rp, dev), to_dev(ci, dev), to_dev(va, dev))
        assert all(np.array_equal(a.cpu().numpy(), b.cpu().numpy()) for a, b in zip(g, g2))


# ----------------------------------------------------------------------------------------------
# a2 / a6: SpMM
# ----------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def spmm_graphs(mg, dev, ref):
    """name -> (pattern, rp, ci, val32, Graph)"""
    out = {}
    pats = {
        "tiny": wl.CONFIGS["tiny"].graph(),
        "adversarial": adversarial_pattern(),
        "powerlaw": wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99),  # rows longer than a segment
        "rmat": wl.rmat(12, 30000, 0.57, 0.19, 0.19, 5),        # many isolated vertices, hubs
    }
    for name, g in pats.items():
        rp, ci, val = normalized(ref, g)
        G = mg.Graph(g.n_rows, g.n_cols, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=640)
        out[name] = (g, rp, ci, val, G)
    return out


@pytest.mark.parametrize("F", [1, 3, 8, 16, 41, 47, 64, 100, 128, 256, 602])
@pytest.mark.parametrize("name", ["tiny", "adversarial", "powerlaw", "rmat"])
def test_spmm_forward(mg, dev, ref, spmm_graphs, name, F):
    say(f"[spmm N] graph={name} F={F}")
    g, rp, ci, val, G = spmm_graphs[name]
    n = g.n_rows
    X = wl.normal_f32(1234 + F, 1, (n, F))
    want = ref.spmm(ref.OP_N, n, n, rp, ci, val.astype(np.float64), X.astype(np.float64))
    got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
    if F >= 8:
        assert_rows_close(got, want, what=f"spmm {name} F={F}")
    else:
        # With one or three columns the row norm is (nearly) a single entry, and a sum of signed
        # terms that cancels makes |err| / |y| ill-conditioned whatever the kernel does.  Use the
        # forward error bound of a dot product instead: |err| <= 1e-5 * (|A^| |X|) row-wise.
        scale = ref.spmm(ref.OP_N, n, n, rp, ci, np.abs(val).astype(np.float64), np.abs(X).astype(np.float64))
        err = np.abs(got - want).max(axis=1)
        assert np.all(err <= 1e-5 * scale.max(axis=1)), f"spmm {name} F={F}: {err.max():.3e}"
    # symmetric operator: the transposed product is the same numbers
    got_t = mg.mggcn_spmm(G, mg.OP_T, to_dev(X, dev)).cpu().numpy()
    assert np.array_equal(got, got_t)


@pytest.mark.parametrize("F,ldx,ldy", [(41, 48, 64), (41, 41, 41), (47, 50, 47), (100, 112, 100), (128, 130, 129),
                                       (5, 8, 12)])
def test_spmm_leading_dimensions_and_padding_untouched(mg, dev, ref, spmm_graphs, F, ldx, ldy):
    import torch

    say(f"[spmm ld] F={F} ldx={ldx} ldy={ldy}")
    g, rp, ci, val, G = spmm_graphs["powerlaw"]
    n = g.n_rows
    Xp = wl.normal_f32(77, 2, (n, ldx))
    Xd = to_dev(Xp, dev)
    Yd = torch.full((n, ldy), 123.0, device=dev)
    mg.mggcn_spmm(G, mg.OP_N, Xd[:, :F], Y=Yd[:, :F])
    want = ref.spmm(ref.OP_N, n, n, rp, ci, val.astype(np.float64), Xp[:, :F].astype(np.float64))
    Y = Yd.cpu().numpy()
    assert_rows_close(Y[:, :F], want, what="ld")
    assert np.all(Y[:, F:] == 123.0), "columns beyond F must not be written"


def test_spmm_degenerate_shapes(mg, dev, ref):
    """no rows, no columns of features, a single vertex, one row holding every entry (cut into many
    segments, in single-pass and in panelled form), a matrix with no entries at all"""
    import torch

    # no rows / a single isolated vertex
    for n in (0, 1):
        rp = np.zeros(n + 1, np.int32)
        ci = np.zeros(0, np.int32)
        grp, gci, gval = mg.mggcn_csr_normalize(n, n, to_dev(rp, dev), to_dev(ci, dev))
        assert gci.numel() == n and (n == 0 or gval.item() == 1.0)
        G = mg.Graph(n, n, grp, gci, gval, F_max=8)
        Y = mg.mggcn_spmm(G, mg.OP_N, torch.ones((n, 8), device=dev))
        assert Y.shape == (n, 8) and (n == 0 or bool((Y == 1.0).all()))
    # F = 0 is a no-op
    g = wl.CONFIGS["tiny"].graph()
    rp, ci, val = normalized(ref, g)
    G = mg.Graph(g.n_rows, g.n_cols, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=16)
    mg.mggcn_spmm(G, mg.OP_N, torch.zeros((g.n_rows, 16), device=dev), F=0, Y=torch.zeros((g.n_rows, 16), device=dev))
    # a matrix without entries: Y = beta * Y, epilogue applied
    n = 300
    z = mg.Graph(n, n, to_dev(np.zeros(n + 1, np.int32), dev), to_dev(np.zeros(0, np.int32), dev),
                 to_dev(np.zeros(0, np.float32), dev), F_max=8)
    Y0 = wl.normal_f32(1, 1, (n, 8))
    Yd = to_dev(Y0, dev)
    mg.mggcn_spmm(z, mg.OP_N, torch.ones((n, 8), device=dev), beta=1.0, epilogue=mg.EPI_RELU, Y=Yd)
    assert np.array_equal(Yd.cpu().numpy(), np.maximum(Y0, 0.0))
    mg.mggcn_spmm(z, mg.OP_N, torch.ones((n, 8), device=dev), Y=Yd)
    assert bool((Yd == 0).all())
    # one row with every entry: 60,000 entries -> 30 segments of a cut row; the other rows are empty
    n, m, F = 5, 60000, 24
    rp = np.array([0, 0, m, m, m, m], np.int32)
    ci = np.arange(m, dtype=np.int32)
    va = wl.normal_f32(2, 1, (m,))
    X = wl.normal_f32(2, 2, (m, F))
    want = ref.spmm(ref.OP_N, n, m, rp, ci, va.astype(np.float64), X.astype(np.float64))
    scale = np.abs(va).astype(np.float64) @ np.abs(X).astype(np.float64)
    d = [to_dev(a, dev) for a in (rp, ci, va)]
    t = mg.mggcn_csr_transpose(n, m, *d)
    for P in (0, 1, 5):
        G = mg.Graph(n, m, *d, transpose=t, F_max=F, n_panels=P)
        got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
        assert np.all(got[[0, 2, 3, 4]] == 0)
        assert np.all(np.abs(got[1] - want[1]) <= 1e-5 * scale.max()), f"P={P}"
        # the transposed operator: every output row is one entry times one row of the operand
        R = wl.normal_f32(2, 3, (n, F))
        got_t = mg.mggcn_spmm(G, mg.OP_T, to_dev(R, dev)).cpu().numpy()
        np.testing.assert_allclose(got_t, va[:, None].astype(np.float64) * R[1][None, :], rtol=1e-6, atol=0)


def test_spmm_rejects_overlapping_operands(mg, dev, spmm_graphs):
    import torch

    g, rp, ci, val, G = spmm_graphs["tiny"]
    buf = torch.zeros((g.n_rows, 64), device=dev)
    with pytest.raises(mg.MggcnError):
        mg.mggcn_spmm(G, mg.OP_N, buf[:, :16], Y=buf[:, :16])          # the same rows
    with pytest.raises(mg.MggcnError):
        mg.mggcn_spmm(G, mg.OP_N, buf[:, :16], Y=buf[:, 32:48])        # interleaved columns of one buffer
    other = torch.zeros((g.n_rows, 16), device=dev)
    mg.mggcn_spmm(G, mg.OP_N, buf[:, :16], Y=other)                    # disjoint: fine


@pytest.mark.parametrize("name", ["adversarial", "powerlaw"])
@pytest.mark.parametrize("F", [16, 100])
def test_spmm_accumulate_and_epilogues(mg, dev, ref, spmm_graphs, name, F):
    say(f"[spmm epi] graph={name} F={F}")
    g, rp, ci, val, G = spmm_graphs[name]
    n = g.n_rows
    X = wl.normal_f32(9, 3, (n, F))
    Y0 = wl.normal_f32(9, 4, (n, F))
    v64 = val.astype(np.float64)
    base = ref.spmm(ref.OP_N, n, n, rp, ci, v64, X.astype(np.float64))
    # beta = 1
    got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), beta=1.0, Y=to_dev(Y0, dev)).cpu().numpy()
    want = ref.spmm(ref.OP_N, n, n, rp, ci, v64, X.astype(np.float64), beta=1.0, Y=Y0.astype(np.float64))
    assert_rows_close(got, want, what="beta=1")
    # fused ReLU: compare against the oracle's ReLU of the GPU's own pre-activation decision
    got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), epilogue=mg.EPI_RELU).cpu().numpy()
    plain = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
    assert np.array_equal(got, np.maximum(plain, 0.0))
    assert_rows_close(got, ref.relu(base), what="relu", pre=base)
    # in-place ReLU' mask: Y_old > 0 keeps the product, else 0
    got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), epilogue=mg.EPI_RELU_MASK, Y=to_dev(Y0, dev)).cpu().numpy()
    assert np.array_equal(got, np.where(Y0 > 0, plain, 0.0).astype(np.float32))


def test_spmm_transpose_nonsymmetric_and_rectangular(mg, dev, ref):
    say("[spmm T] mean-normalised directed graph, and a rectangular block")
    rng = np.random.default_rng(21)
    import scipy.sparse as sp

    S = sp.random(900, 900, density=0.02, format="csr", random_state=3, dtype=np.float32)
    S.setdiag(0); S.eliminate_zeros(); S.sort_indices()
    rp, ci, val = ref.csr_normalize(900, 900, S.indptr.astype(np.int32), S.indices.astype(np.int32),
                                    mode=ref.NORM_MEAN_IN)
    v32 = val.astype(np.float32)
    d = [to_dev(a, dev) for a in (rp, ci, v32)]
    t = mg.mggcn_csr_transpose(900, 900, *d)
    G = mg.Graph(900, 900, *d, transpose=t, F_max=64)
    X = wl.normal_f32(5, 5, (900, 33))
    for op, rop in ((mg.OP_N, ref.OP_N), (mg.OP_T, ref.OP_T)):
        want = ref.spmm(rop, 900, 900, rp, ci, v32.astype(np.float64), X.astype(np.float64))
        got = mg.mggcn_spmm(G, op, to_dev(X, dev)).cpu().numpy()
        assert_rows_close(got, want, what=f"mean op={op}")
    # rectangular row block with given degrees
    g = wl.row_block(700, 5000, 9000, 2.5, 300.0, 1.6, 4)
    dr = rng.integers(1, 500, g.n_rows).astype(np.int32)
    dc = rng.integers(1, 500, g.n_cols).astype(np.int32)
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx, deg_row=dr, deg_col=dc)
    v32 = val.astype(np.float32)
    d = [to_dev(a, dev) for a in (rp, ci, v32)]
    t = mg.mggcn_csr_transpose(g.n_rows, g.n_cols, *d)
    G = mg.Graph(g.n_rows, g.n_cols, *d, transpose=t, F_max=128)
    X = wl.normal_f32(6, 6, (g.n_cols, 128))
    Gr = wl.normal_f32(6, 7, (g.n_rows, 128))
    want = ref.spmm(ref.OP_N, g.n_rows, g.n_cols, rp, ci, v32.astype(np.float64), X.astype(np.float64))
    assert_rows_close(mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy(), want, what="block N")
    want = ref.spmm(ref.OP_T, g.n_rows, g.n_cols, rp, ci, v32.astype(np.float64), Gr.astype(np.float64))
    assert_rows_close(mg.mggcn_spmm(G, mg.OP_T, to_dev(Gr, dev)).cpu().numpy(), want, what="block T")


def test_spmm_is_deterministic_and_segment_length_invariant(mg, dev, ref, spmm_graphs):
    g, rp, ci, val, G = spmm_graphs["powerlaw"]
    n = g.n_rows
    Xd = to_dev(wl.normal_f32(8, 8, (n, 128)), dev)
    a = mg.mggcn_spmm(G, mg.OP_N, Xd).cpu().numpy()
    b = mg.mggcn_spmm(G, mg.OP_N, Xd).cpu().numpy()
    assert np.array_equal(a, b)
    want = ref.spmm(ref.OP_N, n, n, rp, ci, val.astype(np.float64), Xd.cpu().numpy().astype(np.float64))
    for seg in (8, 64, 100000):
        G2 = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128, seg_len=seg)
        assert_rows_close(mg.mggcn_spmm(G2, mg.OP_N, Xd).cpu().numpy(), want, what=f"seg_len={seg}")


@pytest.mark.parametrize("name", ["adversarial", "powerlaw", "rmat"])
@pytest.mark.parametrize("P,seg", [(2, 0), (7, 0), (16, 16), (64, 0)])
def test_spmm_column_panels(mg, dev, ref, spmm_graphs, name, P, seg):
    """Column-panel passes (the stage loop C += A^{ij} H^j on one GPU) give the unsplit product,
    with beta, the fused ReLU and cut rows handled once per row."""
    say(f"[spmm panels] graph={name} P={P} seg_len={seg}")
    g, rp, ci, val, _ = spmm_graphs[name]
    n = g.n_rows
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128, seg_len=seg, n_panels=P)
    v64 = val.astype(np.float64)
    for F in (41, 128):
        X = wl.normal_f32(55, F, (n, F))
        Y0 = wl.normal_f32(56, F, (n, F))
        want = ref.spmm(ref.OP_N, n, n, rp, ci, v64, X.astype(np.float64))
        got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
        assert_rows_close(got, want, what=f"panels F={F}")
        assert np.array_equal(got, mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy())
        got_relu = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), epilogue=mg.EPI_RELU).cpu().numpy()
        assert np.array_equal(got_relu, np.maximum(got, 0.0))
        acc = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), beta=1.0, Y=to_dev(Y0, dev)).cpu().numpy()
        assert_rows_close(acc, want + Y0.astype(np.float64), what=f"panels beta F={F}")
        masked = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), epilogue=mg.EPI_RELU_MASK, Y=to_dev(Y0, dev)).cpu().numpy()
        assert_rows_close(masked, np.where(Y0 > 0, want, 0.0), what=f"panels mask F={F}")


def test_spmm_many_rows_without_entries(mg, dev, ref):
    """The transposed product of a row block with far more columns than entries: most of its output rows hold no
    entry.  With beta = 0 they are written by the fill kernel (zeros whatever the epilogue), with beta = 1 they
    stay; widths with 16-, 8- and 4-byte lanes, a padded and an unaligned output, panels."""
    import torch

    g = wl.row_block(3000, 400_000, 60_000, 2.5, 300.0, 1.6, 11)
    say(f"[spmm rows without entries] {g.n_rows} x {g.n_cols}, {g.nnz} entries")
    rng = np.random.default_rng(12)
    dr = rng.integers(1, 500, g.n_rows).astype(np.int32)
    dc = rng.integers(1, 500, g.n_cols).astype(np.int32)
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx, deg_row=dr, deg_col=dc)
    v32 = val.astype(np.float32)
    d = [to_dev(a, dev) for a in (rp, ci, v32)]
    t = mg.mggcn_csr_transpose(g.n_rows, g.n_cols, *d)
    empty = np.diff(t[0].cpu().numpy()) == 0
    assert empty.sum() > 300_000, "the case must hold enough rows without entries for the fill kernel to be chosen"
    for panels in (0, 4):
        G = mg.Graph(g.n_rows, g.n_cols, *d, transpose=t, F_max=128, n_panels=panels)
        for F, ld, shift in ((128, 128, 0), (41, 48, 0), (41, 41, 0), (6, 8, 0), (33, 36, 1)):
            U = wl.normal_f32(20 + F, 1, (g.n_rows, F))
            want = ref.spmm(ref.OP_T, g.n_rows, g.n_cols, rp, ci, v32.astype(np.float64), U.astype(np.float64))
            Y0 = wl.normal_f32(20 + F, 2, (g.n_cols, ld))
            flat = torch.full((g.n_cols * ld + shift,), 5.0, dtype=torch.float32, device=dev)
            Yd = flat[shift:].view(g.n_cols, ld)  # shift = 1: rows start on odd 4-byte boundaries
            for beta, epi in ((0.0, mg.EPI_NONE), (0.0, mg.EPI_RELU), (0.0, mg.EPI_RELU_MASK), (1.0, mg.EPI_NONE)):
                Yd.copy_(to_dev(Y0, dev))
                mg.mggcn_spmm(G, mg.OP_T, to_dev(U, dev), beta=beta, epilogue=epi, Y=Yd[:, :F])
                got = Yd.cpu().numpy()
                exp = want + (Y0[:, :F].astype(np.float64) if beta else 0.0)
                if epi == mg.EPI_RELU:
                    exp = np.maximum(exp, 0.0)
                if epi == mg.EPI_RELU_MASK:
                    exp = np.where(Y0[:, :F] > 0, exp, 0.0)
                assert_rows_close(got[:, :F], exp, pre=want if epi != mg.EPI_NONE else None,
                                  what=f"P={panels} F={F} ld={ld} beta={beta} epi={epi}")
                if beta == 0.0:
                    assert not got[empty][:, :F].any(), "rows without entries must be exactly zero"
                else:
                    assert np.array_equal(got[empty][:, :F], Y0[empty][:, :F]), "beta = 1 leaves rows without entries as they are"
                assert np.array_equal(got[:, F:], Y0[:, F:]), "padding columns must not be written"
            if shift:
                assert float(flat[0]) == 5.0


# ----------------------------------------------------------------------------------------------
# a1 / a7 / a8: GeMM
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (200, 16, 64), (4097, 8, 16), (1000, 41, 128), (777, 128, 602),
                                   (513, 256, 100), (300, 47, 256), (129, 130, 33)])
def test_gemm_nn_nt(mg, dev, ref, M, N, K):
    say(f"[gemm NN/NT] {M}x{N}x{K}")
    A = wl.normal_f32(M + N, 11, (M, K))
    Bm = wl.normal_f32(M + K, 12, (K, N))
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    got = mg.mggcn_gemm(mg.OP_N, mg.OP_N, to_dev(A, dev), to_dev(Bm, dev)).cpu().numpy()
    assert_rows_close(got, want, what="NN")
    got = mg.mggcn_gemm(mg.OP_N, mg.OP_T, to_dev(A, dev), to_dev(np.ascontiguousarray(Bm.T), dev)).cpu().numpy()
    assert_rows_close(got, want, what="NT")
    got = mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(np.ascontiguousarray(A.T), dev), to_dev(Bm, dev)).cpu().numpy()
    assert_rows_close(got, want, what="TN small K")


@pytest.mark.parametrize("M,N,K", [(602, 128, 30001), (128, 41, 9999), (16, 8, 4097), (100, 256, 20000)])
def test_gemm_tn_split_k(mg, dev, ref, M, N, K):
    """weight-gradient shape: the inner dimension is the (long) vertex axis"""
    say(f"[gemm TN split-K] {M}x{N}x{K}")
    H = wl.normal_f32(K, 13, (K, M))
    T = wl.normal_f32(K, 14, (K, N))
    want = ref.gemm(ref.OP_T, ref.OP_N, H.astype(np.float64), T.astype(np.float64))
    a = mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    assert_rows_close(a, want, what="TN")
    b = mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    assert np.array_equal(a, b), "split-K reduction must be reproducible"


@pytest.mark.parametrize("M,N,K", [(70001, 128, 96), (40000, 192, 100), (300, 256, 64), (129, 384, 2052),
                                   (128, 64, 68)])
def test_gemm_aligned_operands_all_forms(mg, dev, ref, M, N, K):
    """Rows that start on 16-byte boundaries take the kernel with buffer-addressed loads: 128 x 128 tiles for N a
    multiple of 128, 128 x 64 otherwise; more tiles than resident workgroups (each walks several, and ids that only
    pad the grid are skipped), a ragged last row tile, a ragged last k-step, all four operand forms, every epilogue."""
    say(f"[gemm aligned] {M}x{N}x{K}")
    A = wl.normal_f32(M + N, 31, (M, K))
    Bm = wl.normal_f32(M + K, 32, (K, N))
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    Mp = (M + 3) // 4 * 4   # the transposed A needs rows of a multiple of four floats
    At = np.zeros((K, Mp), dtype=np.float32)
    At[:, :M] = A.T
    Ad, Bd, Atd, Btd = to_dev(A, dev), to_dev(Bm, dev), to_dev(At, dev)[:, :M], to_dev(np.ascontiguousarray(Bm.T), dev)
    plain = mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad, Bd).cpu().numpy()
    assert_rows_close(plain, want, what="NN")
    assert_rows_close(mg.mggcn_gemm(mg.OP_N, mg.OP_T, Ad, Btd).cpu().numpy(), want, what="NT")
    assert_rows_close(mg.mggcn_gemm(mg.OP_T, mg.OP_N, Atd, Bd).cpu().numpy(), want, what="TN")
    assert_rows_close(mg.mggcn_gemm(mg.OP_T, mg.OP_T, Atd, Btd).cpu().numpy(), want, what="TT")
    C0 = wl.normal_f32(M, 33, (M, N))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad, Bd, epilogue=mg.EPI_RELU, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), np.maximum(plain, 0))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad, Bd, epilogue=mg.EPI_RELU_MASK, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), np.where(C0 > 0, plain, 0).astype(np.float32))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad, Bd, beta=1.0, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), plain + C0)
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad, Bd, beta=1.0, epilogue=mg.EPI_RELU, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), np.maximum(plain + C0, 0))


@pytest.mark.parametrize("M,N,K", [(128, 256, 50001), (256, 128, 33333), (100, 64, 40000)])
def test_gemm_tn_split_k_aligned(mg, dev, ref, M, N, K):
    """the weight gradient on aligned operands: split inner dimension whose last part ends in a ragged k-step"""
    say(f"[gemm TN split-K aligned] {M}x{N}x{K}")
    H = wl.normal_f32(K, 34, (K, M))
    T = wl.normal_f32(K, 35, (K, N))
    want = ref.gemm(ref.OP_T, ref.OP_N, H.astype(np.float64), T.astype(np.float64))
    a = mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    assert_rows_close(a, want, what="TN")
    b = mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    assert np.array_equal(a, b), "split-K reduction must be reproducible"
    C0 = wl.normal_f32(M, 36, (M, N))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev), beta=1.0, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), a + C0)


def test_gemm_very_long_rows_of_c(mg, dev, ref):
    """Rows of C (and of A) 2^21 floats apart: offsets inside a wavefront's block of C no longer fit the 32-bit
    lane offsets of the buffer stores, so the epilogue takes its 64-bit form and the operands the checked loaders."""
    import torch

    M, N, K, ld = 130, 64, 96, 1 << 21
    say(f"[gemm long rows] {M}x{N}x{K} ld {ld}")
    A = wl.normal_f32(5, 41, (M, K))
    Bm = wl.normal_f32(5, 42, (K, N))
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    Abig = torch.zeros((M, ld), dtype=torch.float32, device=dev)
    Abig[:, :K] = to_dev(A, dev)
    Cbig = torch.full((M, ld), 7.0, dtype=torch.float32, device=dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Abig[:, :K], to_dev(Bm, dev), Cm=Cbig[:, :N])
    assert_rows_close(Cbig[:, :N].cpu().numpy(), want, what="long rows")
    assert bool((Cbig[:, N:N + 64] == 7.0).all()) and bool((Cbig[:, -64:] == 7.0).all()), "padding columns must not be written"
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Abig[:, :K], to_dev(Bm, dev), epilogue=mg.EPI_RELU, Cm=Cbig[:, :N])
    assert_rows_close(Cbig[:, :N].cpu().numpy(), np.maximum(want, 0), pre=want, what="long rows, ReLU")


def test_gemm_degenerate_shapes(mg, dev, ref):
    """empty outputs are no-ops; an empty inner dimension leaves epilogue(beta * C)"""
    import torch

    A = torch.ones((0, 5), device=dev)
    B = torch.ones((5, 7), device=dev)
    assert mg.mggcn_gemm(mg.OP_N, mg.OP_N, A, B).shape == (0, 7)
    assert mg.mggcn_gemm(mg.OP_N, mg.OP_N, torch.ones((4, 5), device=dev), torch.ones((5, 0), device=dev)).shape == (4, 0)
    C0 = wl.normal_f32(9, 1, (37, 11))
    for beta, epi, want in [(0.0, mg.EPI_NONE, np.zeros_like(C0)), (1.0, mg.EPI_NONE, C0),
                            (1.0, mg.EPI_RELU, np.maximum(C0, 0.0))]:
        Cd = to_dev(C0, dev)
        mg.mggcn_gemm(mg.OP_N, mg.OP_N, torch.ones((37, 0), device=dev), torch.ones((0, 11), device=dev), beta=beta,
                      epilogue=epi, Cm=Cd)
        assert np.array_equal(Cd.cpu().numpy(), want), (beta, epi)
    # a single element, and a single row times a wide matrix
    one = mg.mggcn_gemm(mg.OP_N, mg.OP_N, torch.full((1, 1), 3.0, device=dev), torch.full((1, 1), -2.0, device=dev))
    assert one.item() == -6.0
    a, b = wl.normal_f32(9, 2, (1, 300)), wl.normal_f32(9, 3, (300, 513))
    got = mg.mggcn_gemm(mg.OP_N, mg.OP_N, to_dev(a, dev), to_dev(b, dev)).cpu().numpy()
    assert_rows_close(got, ref.gemm(ref.OP_N, ref.OP_N, a.astype(np.float64), b.astype(np.float64)), what="1 x 513")


def test_gemm_epilogues_beta_and_strides(mg, dev, ref):
    import torch

    M, N, K = 333, 41, 100
    A = wl.normal_f32(1, 15, (M, 112))      # ld 112 > K
    Bm = wl.normal_f32(1, 16, (K, N))       # ld 41: unaligned rows
    C0 = wl.normal_f32(1, 17, (M, 48))
    Ad, Bd = to_dev(A, dev), to_dev(Bm, dev)
    want = ref.gemm(ref.OP_N, ref.OP_N, A[:, :K].astype(np.float64), Bm.astype(np.float64))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, Cm=Cd[:, :N])
    C = Cd.cpu().numpy()
    assert_rows_close(C[:, :N], want, what="strided")
    assert np.array_equal(C[:, N:], C0[:, N:]), "padding columns must not be written"
    plain = C[:, :N].copy()
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, beta=1.0, Cm=Cd[:, :N])
    assert_rows_close(Cd.cpu().numpy()[:, :N], want + C0[:, :N].astype(np.float64), what="beta")
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, epilogue=mg.EPI_RELU, Cm=Cd[:, :N])
    assert np.array_equal(Cd.cpu().numpy()[:, :N], np.maximum(plain, 0))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, epilogue=mg.EPI_RELU_MASK, Cm=Cd[:, :N])
    assert np.array_equal(Cd.cpu().numpy()[:, :N], np.where(C0[:, :N] > 0, plain, 0).astype(np.float32))


# ----------------------------------------------------------------------------------------------
# a4 / a5: loss, ReLU'
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,C,ld", [(4096, 8, 16), (1001, 41, 48), (333, 47, 47), (50, 100, 100), (7, 1, 4),
                                     (513, 256, 256), (300, 512, 512), (64, 513, 520), (100, 600, 600), (33, 17, 17)])
def test_softmax_ce(mg, dev, ref, n, C, ld):
    say(f"[softmax_ce] n={n} C={C} ld={ld}")
    Zp = wl.normal_f32(n, 20, (n, ld)) * 3
    labels = wl.labels_i32(n, 21, n, C)
    loss, dZ = ref.softmax_ce(Zp[:, :C].astype(np.float64), labels)
    Zd = to_dev(Zp, dev)
    gl, gd = mg.mggcn_softmax_ce(Zd[:, :C], to_dev(labels, dev))  # in place
    assert abs(gl.item() - loss) <= 1e-5 * abs(loss) + 1e-7
    out = Zd.cpu().numpy()
    assert_rows_close(out[:, :C], dZ, tol=1e-4 if C > 1 else 1.0, what="dlogits")
    assert np.array_equal(out[:, C:], Zp[:, C:])


def test_relu_bwd(mg, dev):
    act = wl.normal_f32(3, 22, (500, 48))
    G = wl.normal_f32(3, 23, (500, 64))
    Gd = to_dev(G, dev)
    mg.mggcn_relu_bwd(to_dev(act, dev)[:, :41], Gd[:, :41])
    want = G.copy()
    want[:, :41] = np.where(act[:, :41] > 0, G[:, :41], 0)
    assert np.array_equal(Gd.cpu().numpy(), want)


# ----------------------------------------------------------------------------------------------
# layers and epoch
# ----------------------------------------------------------------------------------------------

def gpu_relu_decisions(mg, model, Xd, Wd):
    """ReLU' decisions (activation > 0) of the hidden layers as the device takes them: the same
    forward calls, hence the same bits, as inside mggcn_epoch."""
    import torch

    masks, H = [], Xd
    for l in range(model.L - 1):
        d = model.dims[l + 1]
        out = torch.empty((H.shape[0], (d + 15) // 16 * 16), device=H.device)[:, :d]
        mg.mggcn_layer_fwd(model, l, H, Wd[l], relu=True, H_out=out)
        masks.append((out > 0).cpu().numpy().astype(np.uint8))
        H = out
    return masks


def oracle_preactivations(ref, n, rp, ci, v64, X64, W64s, r_orders):
    """The oracle's own fp64 pre-activations Z of the hidden layers (the forward chain of Eq. 5-7)."""
    Zs, H = [], X64
    for l in range(len(W64s) - 1):
        Z = ref.layer_fwd(n, rp, ci, v64, H, W64s[l], r_orders[l], False)
        Zs.append(Z)
        H = np.maximum(Z, 0.0)
    return Zs


def assert_relu_decisions_agree(masks, Zs, what=""):
    """The device's ReLU' decisions that the oracle's backward pass is handed must be the oracle's own
    except where the pre-activation is zero to within fp32 rounding: at most 1e-5 of the entries
    (three for a small matrix) may differ, and each of those has |z| <= 1e-5 of its row's largest
    entry (of the matrix's largest entry for rows narrower than 8, whose own norm may cancel)."""
    total = 0
    assert len(masks) == len(Zs)
    for l, (m, Z) in enumerate(zip(masks, Zs)):
        assert m.shape == Z.shape
        diff = (Z > 0) != m.astype(bool)
        nd = int(np.count_nonzero(diff))
        total += nd
        assert nd <= max(3, 1e-5 * m.size), f"{what} layer {l}: {nd} of {m.size} ReLU' decisions differ from the oracle's"
        if nd:
            rowmax = np.abs(Z).max(axis=1)
            scale = rowmax if Z.shape[1] >= 8 else np.full_like(rowmax, np.abs(Z).max())
            r, c = np.nonzero(diff)
            worst = float((np.abs(Z[r, c]) / np.maximum(scale[r], 1e-300)).max())
            assert worst <= 1e-5, f"{what} layer {l}: a differing decision sits at |z| = {worst:.2e} of its row"
    return total


def _model_inputs(ref, g, dims, seed):
    rp, ci, val = normalized(ref, g)
    n = g.n_rows
    X = wl.normal_f32(seed, 30, (n, dims[0]))
    Ws = [wl.glorot_f32(seed, 40 + l, dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    labels = wl.labels_i32(seed, 50, n, dims[-1])
    return rp, ci, val, X, Ws, labels


@pytest.mark.parametrize("d_in,d_out", [(64, 16), (20, 100), (41, 41)])
@pytest.mark.parametrize("order", ["gemm_first", "spmm_first"])
def test_layer_fwd_bwd(mg, dev, ref, d_in, d_out, order):
    say(f"[layer] {d_in}->{d_out} {order}")
    g = wl.chung_lu(2000, 60e3, 2.1, 700.0, 3)
    rp, ci, val, X, Ws, _ = _model_inputs(ref, g, (d_in, d_out), 1)
    n = g.n_rows
    o = mg.ORDER_GEMM_FIRST if order == "gemm_first" else mg.ORDER_SPMM_FIRST
    ro = ref.GEMM_FIRST if order == "gemm_first" else ref.SPMM_FIRST
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128)
    model = mg.Model(G, (d_in, d_out), orders=[o])
    assert model.order(0) == o
    Xd, Wd = to_dev(X, dev), to_dev(Ws[0], dev)
    v64, X64, W64 = val.astype(np.float64), X.astype(np.float64), Ws[0].astype(np.float64)
    out = mg.mggcn_layer_fwd(model, 0, Xd, Wd, relu=True)
    pre = ref.layer_fwd(n, rp, ci, v64, X64, W64, ro, False)
    want = ref.layer_fwd(n, rp, ci, v64, X64, W64, ro, True)
    assert np.array_equal(want, np.maximum(pre, 0.0))
    out_h = out.cpu().numpy()
    assert_rows_close(out_h, want, what="fwd", pre=pre)
    # backward with the GPU's own saved activation as the mask source (identical inputs)
    R = wl.normal_f32(2, 31, (n, d_out))
    WG, HG = mg.mggcn_layer_bwd(model, 0, Xd, out, to_dev(R, dev), Wd, need_input_grad=True)
    WG_r, HG_r, _ = ref.layer_bwd(n, rp, ci, v64, X64, out_h.astype(np.float64), R.astype(np.float64), W64, ro, True)
    assert_rows_close(WG.cpu().numpy(), WG_r, what="W_G")
    assert_rows_close(HG.cpu().numpy(), HG_r, what="H_G")


@pytest.mark.parametrize("cfg_name,dims,orders", [
    ("tiny", None, None),
    ("tiny", (64, 100, 32, 8), None),            # SpMM-first then GeMM-first layers
    ("tiny", (64, 16, 8), "spmm_first"),
    ("small_powerlaw", (50, 128, 41), None),
])
def test_epoch(mg, dev, ref, cfg_name, dims, orders):
    say(f"[epoch] {cfg_name} dims={dims} orders={orders}")
    if cfg_name == "tiny":
        g = wl.CONFIGS["tiny"].graph()
        dims = dims or wl.CONFIGS["tiny"].dims
    else:
        g = wl.chung_lu(5000, 300e3, 2.1, 2500.0, 8)
    n = g.n_rows
    rp, ci, val, X, Ws, labels = _model_inputs(ref, g, dims, 7)
    L = len(dims) - 1
    ords = None if orders is None else [mg.ORDER_SPMM_FIRST] * L
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128)
    model = mg.Model(G, dims, orders=ords)
    Xd, Wd = to_dev(X, dev), [to_dev(w, dev) for w in Ws]
    loss, WG = mg.mggcn_epoch(model, Xd, to_dev(labels, dev), Wd)
    loss2, WG2 = mg.mggcn_epoch(model, Xd, to_dev(labels, dev), Wd)
    # Whether a hidden activation that is zero to within rounding counts as "on" is a discrete
    # decision: the oracle's backward pass takes the device's fp32 decisions (one flipped entry
    # would otherwise move a whole column of a weight gradient by far more than rounding).
    masks = gpu_relu_decisions(mg, model, Xd, Wd)
    r_ords = [ref.SPMM_FIRST if model.order(l) == mg.ORDER_SPMM_FIRST else ref.GEMM_FIRST for l in range(L)]
    assert_relu_decisions_agree(masks, oracle_preactivations(ref, n, rp, ci, val.astype(np.float64), X.astype(np.float64),
                                                             [w.astype(np.float64) for w in Ws], r_ords), "epoch")
    rl, rWG, _ = ref.epoch(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws],
                           orders=None if ords is None else [ref.SPMM_FIRST] * L, relu_masks=masks)
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    assert loss.item() == loss2.item()
    for l in range(L):
        a = WG[l].cpu().numpy()
        assert np.array_equal(a, WG2[l].cpu().numpy()), "epoch must be reproducible bit for bit"
        assert_rows_close(a, rWG[l], what=f"W_G[{l}]")
        # the order rule
        want_order = mg.ORDER_SPMM_FIRST if (ords is not None or dims[l] < dims[l + 1]) else mg.ORDER_GEMM_FIRST
        assert model.order(l) == want_order


def test_epoch_random_cases(mg, dev, ref):
    """Seeded random models on small random graphs: depth 1-4, widths 1-150 (so both orders of the
    rule, ties, ragged tiles and single-column layers occur), forced orders, both normalisations."""
    rng = np.random.default_rng(77)
    for case in range(14):
        n = int(rng.integers(40, 1500))
        L = int(rng.integers(1, 5))
        dims = tuple(int(x) for x in rng.choice([1, 2, 7, 16, 33, 41, 64, 100, 150], size=L + 1))
        forced = [None, "gemm", "spmm"][int(rng.integers(0, 3))]
        mean = bool(rng.integers(0, 2))
        say(f"[epoch random {case}] n={n} dims={dims} forced={forced} mean={mean}")
        g = wl.chung_lu(n, float(n * rng.integers(3, 40)), 2.2, float(n) / 2, 1000 + case)
        mode = ref.NORM_MEAN_IN if mean else ref.NORM_SYM
        rp, ci, val = normalized(ref, g, mode=mode)
        X = wl.normal_f32(case, 30, (n, dims[0]))
        Ws = [wl.glorot_f32(case, 40 + l, dims[l], dims[l + 1]) for l in range(L)]
        labels = wl.labels_i32(case, 50, n, dims[-1])
        d = [to_dev(a, dev) for a in (rp, ci, val)]
        t = mg.mggcn_csr_transpose(n, n, *d) if mean else None   # mean normalisation is not symmetric
        G = mg.Graph(n, n, *d, transpose=t, F_max=max(dims))
        ords = None if forced is None else [mg.ORDER_GEMM_FIRST if forced == "gemm" else mg.ORDER_SPMM_FIRST] * L
        model = mg.Model(G, dims, orders=ords)
        Xd, Wd = to_dev(X, dev), [to_dev(w, dev) for w in Ws]
        loss, WG = mg.mggcn_epoch(model, Xd, to_dev(labels, dev), Wd)
        masks = gpu_relu_decisions(mg, model, Xd, Wd)
        r_ords = [ref.SPMM_FIRST if model.order(l) == mg.ORDER_SPMM_FIRST else ref.GEMM_FIRST for l in range(L)]
        assert_relu_decisions_agree(masks, oracle_preactivations(ref, n, rp, ci, val.astype(np.float64), X.astype(np.float64),
                                                                 [w.astype(np.float64) for w in Ws], r_ords), f"case {case}")
        rl, rWG, _ = ref.epoch(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                               [w.astype(np.float64) for w in Ws], orders=r_ords, relu_masks=masks)
        assert abs(loss.item() - rl) <= 1e-5 * max(abs(rl), 1e-3), (case, loss.item(), rl)
        for l in range(L):
            got = WG[l].cpu().numpy()
            # a weight gradient row is a sum over all vertices of signed terms: compare against the
            # largest row of the matrix (rows that cancel to ~0 are ill-conditioned by themselves)
            scale = np.abs(rWG[l]).max()
            assert np.abs(got - rWG[l]).max() <= 1e-4 * max(scale, 1e-30), f"case {case} W_G[{l}]"


def test_epoch_with_cached_input(mg, dev, ref):
    """MGGCN_MODEL_CACHE_INPUT: A^ X formed once, first layer without any SpMM in either pass;
    the same gradients as the oracle evaluating that layer in the (A^ X) W association."""
    g = wl.chung_lu(4000, 200e3, 2.1, 1500.0, 21)
    dims = (50, 24, 7)
    n = g.n_rows
    rp, ci, val, X, Ws, labels = _model_inputs(ref, g, dims, 11)
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=64)
    model = mg.Model(G, dims, flags=mg.MODEL_CACHE_INPUT)
    assert model.order(0) == mg.ORDER_SPMM_FIRST and model.order(1) == mg.ORDER_GEMM_FIRST
    Xd, Wd, ld = to_dev(X, dev), [to_dev(w, dev) for w in Ws], to_dev(labels, dev)
    with pytest.raises(mg.MggcnError):
        mg.mggcn_epoch(model, None, ld, Wd)  # cache not filled yet
    model.cache_input(Xd)
    loss, WG = mg.mggcn_epoch(model, None, ld, Wd)
    loss2, WG2 = mg.mggcn_epoch(model, None, ld, Wd)  # the cache survives an epoch
    masks = gpu_relu_decisions(mg, model, Xd, Wd)
    assert_relu_decisions_agree(masks, oracle_preactivations(ref, n, rp, ci, val.astype(np.float64), X.astype(np.float64),
                                                             [w.astype(np.float64) for w in Ws],
                                                             [ref.SPMM_FIRST, ref.GEMM_FIRST]), "cached input")
    rl, rWG, _ = ref.epoch(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws], orders=[ref.SPMM_FIRST, ref.GEMM_FIRST],
                           relu_masks=masks)
    # the cached first layer takes no gradient with respect to X: its shared temporary has no room for it
    with pytest.raises(mg.MggcnError):
        mg.mggcn_layer_bwd(model, 0, Xd, None, to_dev(wl.normal_f32(3, 3, (n, dims[1])), dev), Wd[0], need_input_grad=True)
    wg0, hg0 = mg.mggcn_layer_bwd(model, 0, Xd, None, to_dev(wl.normal_f32(3, 3, (n, dims[1])), dev), Wd[0],
                                  need_input_grad=False)
    assert hg0 is None
    P = ref.spmm(ref.OP_N, n, n, rp, ci, val.astype(np.float64), X.astype(np.float64))
    assert_rows_close(wg0.cpu().numpy(), P.T @ wl.normal_f32(3, 3, (n, dims[1])).astype(np.float64), what="cached layer_bwd W_G")
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl) and loss.item() == loss2.item()
    for l in range(2):
        assert np.array_equal(WG[l].cpu().numpy(), WG2[l].cpu().numpy())
        assert_rows_close(WG[l].cpu().numpy(), rWG[l], what=f"cached W_G[{l}]")


def test_epoch_mean_aggregation_in_the_papers_arrangement(mg, dev, ref):
    """Eq. 1-2: the paper's layer multiplies by the transpose of the column-normalised matrix, i.e. it
    averages H over the in-neighbours of each vertex.  The handle is therefore created with A^^T as
    the matrix and A^ as its transpose; every row of the operator then sums to 1."""
    import scipy.sparse as sp

    n, dims = 1500, (40, 24, 9)
    S = sp.random(n, n, density=0.01, format="csr", random_state=12, dtype=np.float32)
    S.setdiag(0); S.eliminate_zeros(); S.sort_indices()
    rp, ci, val = ref.csr_normalize(n, n, S.indptr.astype(np.int32), S.indices.astype(np.int32), mode=ref.NORM_MEAN_IN)
    v32 = val.astype(np.float32)
    rpt, cit, vt = ref.csr_transpose(n, n, rp, ci, v32.astype(np.float64))
    assert not (np.array_equal(rpt, rp) and np.array_equal(cit, ci)), "the test needs a non-symmetric pattern"
    ones = ref.spmm(ref.OP_N, n, n, rpt, cit, vt, np.ones((n, 1)))
    assert np.abs(ones - 1.0).max() <= 1e-6, "rows of A^^T (in-neighbour averages) must sum to 1"
    d = [to_dev(a, dev) for a in (rp, ci, v32)]
    t = mg.mggcn_csr_transpose(n, n, *d)
    G = mg.Graph(n, n, *t, transpose=tuple(d), F_max=max(dims))  # (matrix, transpose) = (A^^T, A^)
    X = wl.normal_f32(31, 30, (n, dims[0]))
    Ws = [wl.glorot_f32(31, 40 + l, dims[l], dims[l + 1]) for l in range(2)]
    labels = wl.labels_i32(31, 50, n, dims[-1])
    model = mg.Model(G, dims)
    Xd, Wd = to_dev(X, dev), [to_dev(w, dev) for w in Ws]
    loss, WG = mg.mggcn_epoch(model, Xd, to_dev(labels, dev), Wd)
    masks = gpu_relu_decisions(mg, model, Xd, Wd)
    r_ords = [ref.SPMM_FIRST if model.order(l) == mg.ORDER_SPMM_FIRST else ref.GEMM_FIRST for l in range(2)]
    W64 = [w.astype(np.float64) for w in Ws]
    assert_relu_decisions_agree(masks, oracle_preactivations(ref, n, rpt, cit, vt, X.astype(np.float64), W64, r_ords), "mean")
    rl, rWG, _ = ref.epoch(n, rpt, cit, vt, X.astype(np.float64), labels, W64, orders=r_ords, relu_masks=masks)
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    for l in range(2):
        assert_rows_close(WG[l].cpu().numpy(), rWG[l], what=f"mean aggregation W_G[{l}]")
    # first layer forward = relu(mean over in-neighbours of (X W)): a constant feature matrix stays constant
    c = mg.mggcn_spmm(G, mg.OP_N, to_dev(np.full((n, 4), 2.5, np.float32), dev)).cpu().numpy()
    assert np.abs(c - 2.5).max() <= 1e-5


def test_adam_step(mg, dev, ref):
    import torch

    W0 = wl.normal_f32(3, 60, (602, 128))
    W = W0.astype(np.float64).copy()
    m, v = np.zeros_like(W), np.zeros_like(W)
    Wd = to_dev(W0, dev)
    md, vd = torch.zeros_like(Wd), torch.zeros_like(Wd)
    for t in range(1, 6):
        g = wl.normal_f32(3, 60 + t, (602, 128)) * 10.0 ** (t - 4)
        ref.adam_step(W, g.astype(np.float64), m, v, t, lr=0.01)
        mg.mggcn_adam_step(Wd, to_dev(g, dev), md, vd, t, lr=0.01)
        assert_rows_close(Wd.cpu().numpy(), W, tol=1e-5, what=f"adam step {t}")
    with pytest.raises(mg.MggcnError):
        mg.mggcn_adam_step(Wd, Wd, md, vd, 0)


def test_epoch_can_be_captured_in_a_hip_graph(mg, dev, ref):
    """mggcn_epoch only enqueues kernels on the given stream (no allocation, copy, memset or
    synchronisation), so a caller may capture it in a HIP graph.  Replayed several times, with eager
    epochs and synchronisations in between, every replay must give the eager result bit for bit."""
    import torch

    g = wl.chung_lu(5000, 300e3, 2.1, 2500.0, 8)
    dims = (50, 128, 41)
    n = g.n_rows
    rp, ci, val, X, Ws, labels = _model_inputs(ref, g, dims, 7)
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128)
    for flags in (0, mg.MODEL_GATHER_BF16):
        model = mg.Model(G, dims, flags=flags)
        Xd, Wd, ld = to_dev(X, dev), [to_dev(w, dev) for w in Ws], to_dev(labels, dev)
        WG = [torch.empty_like(w) for w in Wd]
        loss = torch.empty(1, device=dev)

        def step():
            mg.mggcn_epoch(model, Xd, ld, Wd, W_Gs=WG, loss=loss)

        step()
        torch.cuda.synchronize()
        want_loss, want = loss.clone(), [w.clone() for w in WG]
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()  # warm-up on the capture stream
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for r in range(4):
            for w in WG:
                w.fill_(float("nan"))
            loss.fill_(float("nan"))
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(loss, want_loss), f"flags={flags} replay {r}: loss differs"
            assert all(torch.equal(a, b) for a, b in zip(WG, want)), f"flags={flags} replay {r}: W_G differs"
            step()  # eager work between replays
            torch.cuda.synchronize()
            assert torch.equal(loss, want_loss)
        del graph


def test_training_trajectory(mg, dev, ref):
    """Ten full training steps (epoch + Adam on every layer) on the tiny configuration, the same ten
    in the oracle: the loss falls, and the two loss curves stay together.  (Adam's first steps move
    every weight by about +-lr whatever the size of its gradient, so weights whose gradient is zero
    to within rounding may step the other way; the comparison is therefore on the loss and on the
    weights to within a few lr, not per entry to 1e-4.)"""
    import torch

    cfg = wl.CONFIGS["tiny"]
    g = cfg.graph()
    n, dims = g.n_rows, cfg.dims
    L = len(dims) - 1
    rp, ci, val = normalized(ref, g)
    X, Ws, labels = cfg.features(n), cfg.weights(), cfg.labels(n)
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=64)
    model = mg.Model(G, dims)
    Xd, ld = to_dev(X, dev), to_dev(labels, dev)
    Wd = [to_dev(w, dev) for w in Ws]
    md, vd = [torch.zeros_like(w) for w in Wd], [torch.zeros_like(w) for w in Wd]
    Wr = [w.astype(np.float64) for w in Ws]
    mr, vr = [np.zeros_like(w) for w in Wr], [np.zeros_like(w) for w in Wr]
    v64, X64 = val.astype(np.float64), X.astype(np.float64)
    lr, steps = 0.01, 10
    gl, rl = [], []
    for t in range(1, steps + 1):
        loss, WG = mg.mggcn_epoch(model, Xd, ld, Wd)
        gl.append(loss.item())
        r_loss, rWG, _ = ref.epoch(n, rp, ci, v64, X64, labels, Wr)
        rl.append(r_loss)
        for l in range(L):
            mg.mggcn_adam_step(Wd[l], WG[l], md[l], vd[l], t, lr=lr)
            ref.adam_step(Wr[l], rWG[l], mr[l], vr[l], t, lr=lr)
    say("[training] gpu losses", [round(x, 5) for x in gl])
    assert gl[-1] < gl[0] - 0.01 and all(b < a for a, b in zip(gl, gl[1:])), "the loss must fall (labels are random: slowly)"
    for a, b in zip(gl, rl):
        assert abs(a - b) <= 2e-4 * abs(b), (gl, rl)
    for l in range(L):
        assert np.abs(Wd[l].cpu().numpy() - Wr[l]).max() <= 3 * lr


def test_spmm_random_cases(mg, dev, ref):
    """Seeded random small problems: rectangular shapes, random densities, widths, leading
    dimensions, ops, beta, epilogues, segment lengths and panel counts."""
    import scipy.sparse as sp
    import torch

    rng = np.random.default_rng(2024)
    for case in range(40):
        nr, nc = int(rng.integers(1, 400)), int(rng.integers(1, 400))
        dens = float(rng.choice([0.0, 0.01, 0.1, 0.5]))
        S = sp.random(nr, nc, density=dens, format="csr", random_state=int(rng.integers(1 << 30)), dtype=np.float32)
        S.sort_indices()
        rp, ci, va = S.indptr.astype(np.int32), S.indices.astype(np.int32), S.data.astype(np.float32)
        F = int(rng.choice([1, 2, 5, 8, 16, 33, 41, 64, 100, 128, 130, 300]))
        ldx, ldy = F + int(rng.integers(0, 9)), F + int(rng.integers(0, 9))
        op = int(rng.integers(0, 2))
        beta = float(rng.integers(0, 2))
        epi = int(rng.choice([mg.EPI_NONE, mg.EPI_RELU, mg.EPI_RELU_MASK])) if beta == 0 else int(rng.choice([mg.EPI_NONE, mg.EPI_RELU]))
        seg, P = int(rng.choice([0, 8, 50])), int(rng.choice([0, 1, 3, 8]))
        say(f"[spmm random {case}] {nr}x{nc} dens={dens} F={F} ldx={ldx} ldy={ldy} op={op} beta={beta} epi={epi} seg={seg} P={P}")
        d = [to_dev(a, dev) for a in (rp, ci, va)]
        t = mg.mggcn_csr_transpose(nr, nc, *d)
        G = mg.Graph(nr, nc, *d, transpose=t, F_max=max(F, 1), seg_len=seg, n_panels=P)
        xin, yout = (nc, nr) if op == mg.OP_N else (nr, nc)
        Xp = wl.normal_f32(case, 1, (xin, ldx))
        Y0 = wl.normal_f32(case, 2, (yout, ldy))
        Yd = to_dev(Y0, dev)
        mg.mggcn_spmm(G, op, to_dev(Xp, dev)[:, :F], beta=beta, epilogue=epi, Y=Yd[:, :F])
        got = Yd.cpu().numpy()
        want = ref.spmm(op, nr, nc, rp, ci, va.astype(np.float64), Xp[:, :F].astype(np.float64), beta=beta,
                        Y=Y0[:, :F].astype(np.float64).copy())
        if epi == mg.EPI_RELU:
            want = np.maximum(want, 0.0)
        elif epi == mg.EPI_RELU_MASK:
            want = np.where(Y0[:, :F] > 0, want, 0.0)
        scale = ref.spmm(op, nr, nc, rp, ci, np.abs(va).astype(np.float64), np.abs(Xp[:, :F]).astype(np.float64))
        scale = scale + beta * np.abs(Y0[:, :F])
        err = np.abs(got[:, :F] - want)
        # forward error bound of the row sums (random sparse values cancel, so compare against |A||X|)
        assert np.all(err <= 1e-5 * np.maximum(scale.max(axis=1, keepdims=True), 1e-30)), f"case {case}: {err.max()}"
        assert np.array_equal(got[:, F:], Y0[:, F:])


# ----------------------------------------------------------------------------------------------
# the SpMM's segment tables against their definition written out in numpy
# ----------------------------------------------------------------------------------------------

def expected_tables(rp, ci, n_cols, P, seg_len):
    """Row segments by the rule the header states: every row is cut at the P equal column-panel boundaries,
    every non-empty (row, panel) range (an empty row: one empty range in panel 0) into pieces of at most seg_len
    entries of equal size; panel-major, longest first, row order (then piece order) among equal lengths."""
    FIRST, LAST = 1 << 30, 1 << 29
    n = len(rp) - 1
    width = -(-max(n_cols, 1) // P)
    tasks = [[] for _ in range(P)]
    fix = [[] for _ in range(P)]
    slots = [0] * P
    for i in range(n):
        cols = ci[rp[i]:rp[i + 1]]
        cut = [int(rp[i])] + [int(rp[i] + np.searchsorted(cols, min((c + 1) * width, n_cols), side="left")) for c in range(P - 1)] \
            + [int(rp[i + 1])]
        ne = [p for p in range(P) if cut[p + 1] > cut[p]]
        first, last = (ne[0], ne[-1]) if ne else (0, 0)
        for p in range(first, last + 1):
            lo, ln = cut[p], cut[p + 1] - cut[p]
            if ln == 0 and not (p == first and first == last):
                continue
            flags = (FIRST if p == first else 0) | (LAST if p == last else 0)
            if ln <= seg_len:
                tasks[p].append((i, lo, ln, flags, -1))
            else:
                nseg = -(-ln // seg_len)
                piece = -(-ln // nseg)
                fix[p].append((i, slots[p], nseg, flags))
                for s in range(nseg):
                    k0 = lo + s * piece
                    k1 = min(lo + ln, k0 + piece)
                    tasks[p].append((i, k0, k1 - k0, 0, slots[p]))
                    slots[p] += 1
    out_t, out_f, tb, fb = [], [], [0], [0]
    for p in range(P):
        order = sorted(range(len(tasks[p])), key=lambda k: -tasks[p][k][2])  # stable: generation order inside a length
        out_t += [tasks[p][k] for k in order]
        out_f += fix[p]
        tb.append(len(out_t))
        fb.append(len(out_f))
    return out_t, tb, out_f, fb, max(slots)


@pytest.mark.parametrize("name", ["adversarial", "powerlaw", "rect"])
def test_segment_tables_match_their_definition(mg, dev, ref, name):
    if name == "adversarial":
        g = adversarial_pattern()
    elif name == "powerlaw":
        g = wl.chung_lu(1500, 90e3, 2.1, 900.0, 5)
    else:
        g = wl.row_block(400, 3000, 5000, 2.5, 200.0, 1.6, 3)
    nr, nc = g.n_rows, g.n_cols
    kw = {}
    if nr != nc:
        kw = dict(deg_row=np.full(nr, 3.0), deg_col=np.full(nc, 2.0))
    rp, ci, val = ref.csr_normalize(nr, nc, g.rowptr, g.colidx, **kw)
    v32 = val.astype(np.float32)
    d = [to_dev(a, dev) for a in (rp, ci, v32)]
    rpt, cit, vt = ref.csr_transpose(nr, nc, rp, ci, v32.astype(np.float64))
    t = [to_dev(a, dev) for a in (rpt, cit, vt.astype(np.float32))]
    for P, seg in ((0, 0), (1, 8), (5, 16), (64, 0), (3, 40)):
        say(f"[tables] {name} n_panels={P} seg_len={seg}")
        G = mg.Graph(nr, nc, *d, transpose=tuple(t), F_max=8, n_panels=P, seg_len=seg)
        S = seg if seg else 2048
        for op, (a_rp, a_ci, a_nc) in ((mg.OP_N, (rp, ci, nc)), (mg.OP_T, (rpt, cit, nr))):
            form = 0
            while True:
                tab = G.tables(op, form)
                want_t, tb, want_f, fb, n_slots = expected_tables(a_rp, a_ci, a_nc, tab["n_panels"], S)
                got = tab["tasks"].numpy()
                assert tab["task_begin"] == tb and tab["fix_begin"] == fb, (form, tab["task_begin"], tb)
                exp = np.array([(r, k0, ln | fl, sl) for r, k0, ln, fl, sl in want_t], dtype=np.int64).reshape(-1, 4)
                assert np.array_equal(got.astype(np.int64) & 0xFFFFFFFF, exp & 0xFFFFFFFF), f"{name} P={P} op={op} form={form}"
                expf = np.array(want_f, dtype=np.int64).reshape(-1, 4)
                assert np.array_equal(tab["fix"].numpy().astype(np.int64) & 0xFFFFFFFF, expf & 0xFFFFFFFF)
                assert tab["n_slots"] == n_slots
                if form == 0:
                    assert tab["n_panels"] == 1
                form += 1
                if form > tab["n_forms"]:
                    break
            if P > 1:
                assert G.tables(op, 1)["n_panels"] == P
