"""GPU parity of the 64-bit-row-offset entry points (matrices of 2^31 entries and more).

Small graphs go through both forms and must give the same bits as the 32-bit one (and so match the
oracle); one banded circulant graph with 2.18e9 entries -- generated on the device, every value and
every output row known in closed form -- exercises entry offsets beyond 2^31 for real."""
import sys

import numpy as np
import pytest

import workloads as wl

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def mg():
    import torch

    assert torch.cuda.is_available(), "these tests need the MI355X"
    import paper_2110_08688_amd as m

    m.binding.lib()
    return m


@pytest.fixture(scope="module")
def dev():
    import torch

    return torch.device("cuda:0")


def to_dev(a, dev):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


@pytest.mark.parametrize("name", ["tiny", "powerlaw", "rect"])
@pytest.mark.parametrize("mode", ["sym", "mean"])
def test_wide_offsets_give_the_same_bits(mg, dev, ref, name, mode):
    import torch

    say(f"[wide small] {name} {mode}")
    if name == "tiny":
        g = wl.CONFIGS["tiny"].graph()
    elif name == "powerlaw":
        g = wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99)
    else:
        g = wl.row_block(500, 4000, 6000, 2.5, 200.0, 1.6, 17)
    nr, nc = g.n_rows, g.n_cols
    kw = {}
    rkw = {}
    if name == "rect":
        rng = np.random.default_rng(1)
        dr = rng.integers(1, 3000, nr).astype(np.int32)
        dc = rng.integers(1, 3000, nc).astype(np.int32)
        kw = dict(deg_row=to_dev(dr, dev), deg_col=to_dev(dc, dev))
        rkw = dict(deg_row=dr, deg_col=dc)
    m = mg.NORM_MEAN_IN if mode == "mean" else mg.NORM_SYM_SELFLOOP
    rp32, ci32, v32 = mg.mggcn_csr_normalize(nr, nc, to_dev(g.rowptr, dev), to_dev(g.colidx, dev), mode=m,
                                             validate=True, **kw)
    rp64, ci64, v64 = mg.mggcn_csr_normalize(nr, nc, to_dev(g.rowptr.astype(np.int64), dev), to_dev(g.colidx, dev),
                                             mode=m, validate=True, **kw)
    assert rp64.dtype == torch.int64
    assert torch.equal(rp64, rp32.to(torch.int64)) and torch.equal(ci64, ci32)
    assert torch.equal(v64.view(torch.int32), v32.view(torch.int32))
    rp, ci, val = ref.csr_normalize(nr, nc, g.rowptr, g.colidx, mode=ref.NORM_MEAN_IN if mode == "mean" else ref.NORM_SYM,
                                    **rkw)
    assert np.array_equal(rp64.cpu().numpy(), rp.astype(np.int64)) and np.array_equal(ci64.cpu().numpy(), ci)
    assert np.array_equal(v64.cpu().numpy().view(np.int32), val.astype(np.float32).view(np.int32))
    t32 = mg.mggcn_csr_transpose(nr, nc, rp32, ci32, v32)
    t64 = mg.mggcn_csr_transpose(nr, nc, rp64, ci64, v64)  # the 64-bit entry point
    assert t64[0].dtype == torch.int64
    assert torch.equal(t64[0], t32[0].to(torch.int64)) and torch.equal(t64[1], t32[1])
    assert torch.equal(t64[2].view(torch.int32), t32[2].view(torch.int32))
    rpt, cit, vt = ref.csr_transpose(nr, nc, rp, ci, val.astype(np.float32).astype(np.float64))
    assert np.array_equal(t32[0].cpu().numpy(), rpt) and np.array_equal(t32[1].cpu().numpy(), cit)
    assert np.array_equal(t32[2].cpu().numpy(), vt.astype(np.float32))
    F = 41
    for P, seg in [(0, 0), (1, 16), (7, 0)]:
        G32 = mg.Graph(nr, nc, rp32, ci32, v32, transpose=t32, F_max=F, n_panels=P, seg_len=seg)
        G64 = mg.Graph(nr, nc, rp64, ci64, v64, transpose=t64, F_max=F, n_panels=P, seg_len=seg)
        for op, rows_in in [(mg.OP_N, nc), (mg.OP_T, nr)]:
            X = to_dev(wl.normal_f32(5, op, (rows_in, F)), dev)
            a = mg.mggcn_spmm(G32, op, X)
            b = mg.mggcn_spmm(G64, op, X)
            assert torch.equal(a, b)
            v = val.astype(np.float32).astype(np.float64)
            Xh = X.cpu().numpy().astype(np.float64)
            want = ref.spmm(op, nr, nc, rp, ci, v, Xh)
            scale = ref.spmm(op, nr, nc, rp, ci, np.abs(v), np.abs(Xh))
            err = np.abs(b.cpu().numpy() - want).max(axis=1)
            assert np.all(err <= 1e-5 * np.maximum(scale.max(axis=1), 1e-30))  # forward error bound of the row sums
            Xb = mg.mggcn_f32_to_bf16(X)
            assert torch.equal(mg.mggcn_spmm_bf16(G32, op, Xb), mg.mggcn_spmm_bf16(G64, op, Xb))


def test_wide_rejects_what_it_cannot_hold(mg, dev):
    import torch

    # a row count that only 32-bit offsets cannot express goes through; 2^32 entries are refused
    rp = torch.tensor([0, 1 << 32], dtype=torch.int64, device=dev)
    ci = torch.zeros(1, dtype=torch.int32, device=dev)
    va = torch.zeros(1, dtype=torch.float32, device=dev)
    with pytest.raises(mg.MggcnError) as e:
        mg.Graph(1, 1, rp, ci, va)
    assert e.value.code == mg.binding.E_OVERFLOW
    rp = torch.tensor([0, 2, 1], dtype=torch.int64, device=dev)
    with pytest.raises(mg.MggcnError) as e:
        mg.Graph(2, 2, rp, ci, va)
    assert e.value.code == mg.binding.E_BAD_CSR


def test_wide_two_billion_entries_closed_form(mg, dev):
    """Circulant band graph: vertex i is joined to i +- 1 .. i +- k (mod n).  Every row of A~ has
    2k+1 entries, so every value of A^ is 1/(2k+1), and (A^ X)[i] is the mean of X over the cyclic
    window around i: known for every row from one prefix sum.  n = 2^21, k = 520: 2,183,135,232
    entries, more than 2^31, so the normalisation, the segment tables and the kernels all work
    with entry offsets that do not fit 31 bits."""
    import torch

    n, k, F = 1 << 21, 520, 64
    w = 2 * k
    say(f"[wide big] n={n} k={k}: {n * (w + 1)} entries with the diagonal")
    assert n * (w + 1) > (1 << 31)
    offs = torch.cat([torch.arange(-k, 0, device=dev), torch.arange(1, k + 1, device=dev)])  # ascending, no 0
    colidx_in = torch.empty(n * w, dtype=torch.int32, device=dev)
    step = 1 << 17
    for r0 in range(0, n, step):  # rows in chunks: the wrapped rows at both ends need a sort
        rows = torch.arange(r0, min(n, r0 + step), device=dev)
        c = (rows[:, None] + offs[None, :]) % n
        if r0 < k or r0 + step > n - k:
            c = torch.sort(c, dim=1).values
        colidx_in[r0 * w:(r0 + rows.numel()) * w] = c.reshape(-1).to(torch.int32)
    del c, rows
    rowptr_in = torch.arange(n + 1, dtype=torch.int64, device=dev) * w
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, rowptr_in, colidx_in, validate=True)
    del colidx_in
    assert rowptr.dtype == torch.int64 and int(rowptr[-1].item()) == n * (w + 1)
    assert torch.equal(rowptr, torch.arange(n + 1, dtype=torch.int64, device=dev) * (w + 1))
    expect = np.float32(1.0 / np.sqrt(float(w + 1) * float(w + 1)))
    assert bool((val == float(expect)).all()), "every entry of A^ is 1/(2k+1)"
    # pattern: row i holds i and its 2k neighbours, ascending (checked on the first, last and some middle rows)
    for i in [0, 1, k, n // 2, n - k - 1, n - 1]:
        row = colidx[i * (w + 1):(i + 1) * (w + 1)].cpu().numpy().astype(np.int64)
        want = np.sort((i + np.arange(-k, k + 1)) % n)
        assert np.array_equal(row, want), f"row {i}"
    say("[wide big] normalised; building the segment tables")
    X = wl.normal_f32(2021, 1, (n, F))
    ext = np.concatenate([X[-k:], X, X[:k]]).astype(np.float64)
    cs = np.concatenate([np.zeros((1, F)), np.cumsum(ext, axis=0)])
    want = (cs[w + 1:] - cs[:n]) / float(w + 1)   # window sum over ext[i .. i+2k]
    del ext, cs
    Xd = to_dev(X, dev)
    for P in (1, 0):  # single pass, then the automatic panel choice (reads the column indices back)
        G = mg.Graph(n, n, rowptr, colidx, val, F_max=F, n_panels=P)
        say(f"[wide big] n_panels={P}: {G.panels(F)} passes at F={F}")
        for op in (mg.OP_N, mg.OP_T):
            Y = mg.mggcn_spmm(G, op, Xd).cpu().numpy()
            err = np.abs(Y - want).max(axis=1)
            den = np.abs(want).max(axis=1)
            worst = float((err / np.maximum(den, 1e-300)).max())
            say(f"[wide big] P={P} op={op}: max row rel err {worst:.3e}")
            # a mean of 1041 N(0,1) values cancels to ~0.03: bound the error by the row's |A^||X| instead
            assert np.all(err <= 1e-5 * np.abs(X).max()), "forward error bound"
        del G
