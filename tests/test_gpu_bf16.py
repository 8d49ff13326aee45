"""GPU parity of the bfloat16-gather extension: the conversion kernel bit for bit, the SpMM with a
bfloat16 operand against the fp64 oracle fed the same rounded values (same per-row bound as the
fp32 product), and layers / epochs of a model created with MODEL_GATHER_BF16.

Chain-level comparisons hand the oracle the device's discrete decisions -- its ReLU' masks and the
bfloat16 operands of its SpMMs -- because a value within fp32 rounding of a rounding boundary goes
to one neighbour on the device and may go to the other in fp64; the test then checks separately
that those operands are the roundings of (nearly) the oracle's own values."""
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

    m.binding.lib()
    return m


@pytest.fixture(scope="module")
def dev():
    import torch

    return torch.device("cuda:0")


def to_dev(a, dev):
    import torch

    return torch.from_numpy(np.ascontiguousarray(a)).to(dev)


def codes_of(t):
    """int16 device tensor of bit patterns -> uint16 numpy"""
    return t.cpu().numpy().view(np.uint16)


def values_of(codes):
    return (codes.astype(np.uint32) << 16).view(np.float32)


def row_err(got, want):
    got = np.asarray(got, dtype=np.float64)
    num = np.abs(got - want).max(axis=1)
    den = np.abs(want).max(axis=1)
    zero = den == 0
    assert np.all(num[zero] == 0), "rows with an exactly-zero reference must be exactly zero"
    return np.where(zero, 0.0, num / np.maximum(den, 1e-300))


def assert_rows_close(got, want, tol=TOL, what=""):
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    e = row_err(got, want)
    worst = int(np.argmax(e)) if e.size else -1
    assert e.size == 0 or e[worst] <= tol, f"{what}: row {worst} rel err {e[worst]:.3e} > {tol}"


def normalized(ref, g, mode=None):
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx,
                                    mode=ref.NORM_SYM if mode is None else mode)
    return rp, ci, val.astype(np.float32)


# ----------------------------------------------------------------------------------------------
# conversion: bit exact
# ----------------------------------------------------------------------------------------------

@pytest.mark.parametrize("rows,cols,lds,ldd", [(1000, 128, 128, 128), (333, 41, 48, 48), (77, 47, 47, 51),
                                               (5, 1, 1, 1), (4096, 8, 16, 8), (0, 16, 16, 16)])
def test_f32_to_bf16_bit_exact(mg, dev, ref, rows, cols, lds, ldd):
    import torch

    say(f"[f32->bf16] {rows}x{cols} lds={lds} ldd={ldd}")
    src = wl.normal_f32(5, 70, (max(rows, 1), lds))[:rows]
    src = src * np.exp2(wl.uniform_f32(5, 71, (max(rows, 1), lds), -30.0, 30.0)[:rows]).astype(np.float32)
    if rows >= 5 and cols >= 1:
        special = np.array([0x3F808000, 0x3F818000, 0x3F808001, 0x7F7FFFFF, 0x7F7F7FFF, 0x00008000, 0x00018000,
                            0x80000001, 0x7F800000, 0xFF800000, 0x7FC00000, 0x7F800001, 0x00000000, 0x80000000],
                           dtype=np.uint32).view(np.float32)
        flat = src.reshape(-1)
        flat[: min(len(special), flat.size)] = special[: flat.size]
    sd = to_dev(src, dev)
    dd = torch.full((max(rows, 1), ldd), -21846, dtype=torch.int16, device=dev)[:rows]  # 0xAAAA
    mg.mggcn_f32_to_bf16(sd[:, :cols], dst=dd[:, :cols])
    got = codes_of(dd)
    want, _ = ref.bf16_round(np.ascontiguousarray(src[:, :cols]))
    assert np.array_equal(got[:, :cols], want)
    assert np.all(got[:, cols:] == 0xAAAA), "columns beyond cols must not be written"


# ----------------------------------------------------------------------------------------------
# SpMM with a bfloat16 operand
# ----------------------------------------------------------------------------------------------

def adversarial_pattern(n=300, seed=5):
    rng = np.random.default_rng(seed)
    rows = [set() for _ in range(n)]
    hub = 7
    for j in range(n):
        if j != hub and j % 3:
            rows[hub].add(j); rows[j].add(hub)
    for _ in range(4 * n):
        a, b = rng.integers(0, n, 2)
        if a != b and a % 11 and b % 11:
            rows[a].add(int(b)); rows[b].add(int(a))
    rowptr = np.zeros(n + 1, np.int32)
    col = []
    for i in range(n):
        c = sorted(rows[i])
        col += c
        rowptr[i + 1] = len(col)
    return wl.Pattern(n, n, rowptr, np.array(col, np.int32))


@pytest.fixture(scope="module")
def graphs(mg, dev, ref):
    out = {}
    pats = {
        "tiny": wl.CONFIGS["tiny"].graph(),
        "adversarial": adversarial_pattern(),
        "powerlaw": wl.chung_lu(3001, 150e3, 2.1, 1500.0, 99),
        "rmat": wl.rmat(12, 30000, 0.57, 0.19, 0.19, 5),
    }
    for name, g in pats.items():
        rp, ci, val = normalized(ref, g)
        G = mg.Graph(g.n_rows, g.n_cols, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=640)
        out[name] = (g, rp, ci, val, G)
    return out


def check_spmm(ref, op, nr, nc, rp, ci, val, Xq, got, F, beta=0.0, Y0=None, epi=None, what=""):
    want = ref.spmm(op, nr, nc, rp, ci, val.astype(np.float64), Xq.astype(np.float64), beta=beta,
                    Y=None if Y0 is None else Y0.astype(np.float64).copy())
    if epi == "relu":
        want = np.maximum(want, 0.0)
    elif epi == "mask":
        want = np.where(Y0 > 0, want, 0.0)
    if F >= 8 and beta == 0.0 and epi is None:
        assert_rows_close(got, want, what=what)
    else:  # narrow rows / accumulation: forward error bound of the row sums, as for the fp32 product
        scale = ref.spmm(op, nr, nc, rp, ci, np.abs(val).astype(np.float64), np.abs(Xq).astype(np.float64))
        if Y0 is not None:
            scale = scale + beta * np.abs(Y0)
        err = np.abs(got - want).max(axis=1)
        assert np.all(err <= 1e-5 * np.maximum(scale.max(axis=1), 1e-30)), f"{what}: {err.max():.3e}"


@pytest.mark.parametrize("F", [1, 3, 8, 16, 41, 47, 64, 100, 128, 256, 602])
@pytest.mark.parametrize("name", ["tiny", "adversarial", "powerlaw", "rmat"])
def test_spmm_bf16(mg, dev, ref, graphs, name, F):
    say(f"[spmm bf16] graph={name} F={F}")
    g, rp, ci, val, G = graphs[name]
    n = g.n_rows
    X = wl.normal_f32(4321 + F, 1, (n, F))
    Xb = mg.mggcn_f32_to_bf16(to_dev(X, dev))           # padded leading dimension: the wide path
    codes = codes_of(Xb)
    want_codes, Xq = ref.bf16_round(X)
    assert np.array_equal(codes, want_codes)
    got = mg.mggcn_spmm_bf16(G, mg.OP_N, Xb).cpu().numpy()
    check_spmm(ref, ref.OP_N, n, n, rp, ci, val, Xq, got, F, what=f"spmm bf16 {name} F={F}")
    got_t = mg.mggcn_spmm_bf16(G, mg.OP_T, Xb).cpu().numpy()
    assert np.array_equal(got, got_t)
    # against the fp32 product the difference is the rounding of X: at most 2^-8 of |A^||X| per row
    full = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
    scale = ref.spmm(ref.OP_N, n, n, rp, ci, np.abs(val).astype(np.float64), np.abs(X).astype(np.float64))
    assert np.all(np.abs(got - full).max(axis=1) <= (2.0 ** -8 + 1e-5) * np.maximum(scale.max(axis=1), 1e-30))


@pytest.mark.parametrize("F,ldx,ldy", [(41, 48, 64), (41, 41, 41), (47, 50, 47), (100, 104, 100), (128, 136, 129),
                                       (5, 8, 12), (16, 16, 18)])
def test_spmm_bf16_leading_dimensions(mg, dev, ref, graphs, F, ldx, ldy):
    """aligned and unaligned operands (the element-by-element path), padding untouched"""
    import torch

    say(f"[spmm bf16 ld] F={F} ldx={ldx} ldy={ldy}")
    g, rp, ci, val, G = graphs["powerlaw"]
    n = g.n_rows
    Xp = wl.normal_f32(78, 2, (n, ldx))
    Xb = torch.empty((n, ldx), dtype=torch.int16, device=dev)
    mg.mggcn_f32_to_bf16(to_dev(Xp, dev), dst=Xb)
    _, Xq = ref.bf16_round(Xp)
    Yd = torch.full((n, ldy), 123.0, device=dev)
    mg.mggcn_spmm_bf16(G, mg.OP_N, Xb[:, :F], Y=Yd[:, :F])
    Y = Yd.cpu().numpy()
    check_spmm(ref, ref.OP_N, n, n, rp, ci, val, Xq[:, :F], Y[:, :F], F, what="ld")
    assert np.all(Y[:, F:] == 123.0), "columns beyond F must not be written"


@pytest.mark.parametrize("name", ["adversarial", "powerlaw", "rmat"])
@pytest.mark.parametrize("P,seg,F", [(1, 0, 100), (7, 0, 128), (16, 16, 41), (64, 0, 16)])
def test_spmm_bf16_panels_accumulate_epilogues(mg, dev, ref, graphs, name, P, seg, F):
    say(f"[spmm bf16 panels] graph={name} P={P} seg={seg} F={F}")
    g, rp, ci, val, _ = graphs[name]
    n = g.n_rows
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=F, seg_len=seg, n_panels=P)
    X = wl.normal_f32(99 + P, 3, (n, F))
    Xb = mg.mggcn_f32_to_bf16(to_dev(X, dev))
    _, Xq = ref.bf16_round(X)
    Y0 = wl.normal_f32(99 + P, 4, (n, F))
    for beta, epi, epi_name in [(0.0, mg.EPI_NONE, None), (1.0, mg.EPI_NONE, None), (0.0, mg.EPI_RELU, "relu"),
                                (1.0, mg.EPI_RELU, "relu"), (0.0, mg.EPI_RELU_MASK, "mask")]:
        Yd = to_dev(Y0, dev)
        mg.mggcn_spmm_bf16(G, mg.OP_N, Xb, beta=beta, epilogue=epi, Y=Yd)
        check_spmm(ref, ref.OP_N, n, n, rp, ci, val, Xq, Yd.cpu().numpy(), F, beta=beta, Y0=Y0, epi=epi_name,
                   what=f"beta={beta} epi={epi_name}")
    a = mg.mggcn_spmm_bf16(G, mg.OP_N, Xb).cpu().numpy()
    b = mg.mggcn_spmm_bf16(G, mg.OP_N, Xb).cpu().numpy()
    assert np.array_equal(a, b), "run-to-run bit equality"


def test_spmm_bf16_nonsymmetric_and_rectangular(mg, dev, ref):
    g = wl.row_block(700, 5000, 9000, 2.5, 300.0, 1.6, 23)
    rng = np.random.default_rng(2)
    dr = rng.integers(1, 3000, g.n_rows).astype(np.int32)
    dc = rng.integers(1, 3000, g.n_cols).astype(np.int32)
    rp, ci, val = ref.csr_normalize(g.n_rows, g.n_cols, g.rowptr, g.colidx, deg_row=dr, deg_col=dc)
    val = val.astype(np.float32)
    d = [to_dev(a, dev) for a in (rp, ci, val)]
    t = mg.mggcn_csr_transpose(g.n_rows, g.n_cols, *d)
    G = mg.Graph(g.n_rows, g.n_cols, *d, transpose=t, F_max=64)
    for op, rows_in, F in [(mg.OP_N, g.n_cols, 64), (mg.OP_T, g.n_rows, 24)]:
        say(f"[spmm bf16 rect] op={op} F={F}")
        X = wl.normal_f32(7 + op, 5, (rows_in, F))
        Xb = mg.mggcn_f32_to_bf16(to_dev(X, dev))
        _, Xq = ref.bf16_round(X)
        got = mg.mggcn_spmm_bf16(G, op, Xb).cpu().numpy()
        check_spmm(ref, op, g.n_rows, g.n_cols, rp, ci, val, Xq, got, F, what=f"rect op={op}")


def test_spmm_bf16_argument_errors(mg, dev, graphs):
    import torch

    g, rp, ci, val, G = graphs["tiny"]
    Xb = torch.zeros((g.n_rows, 16), dtype=torch.int16, device=dev)
    with pytest.raises(mg.MggcnError):
        mg.mggcn_spmm_bf16(G, 5, Xb)
    with pytest.raises(mg.MggcnError):
        mg.mggcn_spmm_bf16(G, mg.OP_N, Xb, beta=0.5)
    with pytest.raises(mg.MggcnError):
        mg.mggcn_spmm_bf16(G, mg.OP_N, Xb, F=4096)


# ----------------------------------------------------------------------------------------------
# model with MODEL_GATHER_BF16
# ----------------------------------------------------------------------------------------------

def _model_inputs(ref, g, dims, seed):
    rp, ci, val = normalized(ref, g)
    n = g.n_rows
    X = wl.normal_f32(seed, 30, (n, dims[0]))
    Ws = [wl.glorot_f32(seed, 40 + l, dims[l], dims[l + 1]) for l in range(len(dims) - 1)]
    labels = wl.labels_i32(seed, 50, n, dims[-1])
    return rp, ci, val, X, Ws, labels


def manual_epoch(mg, model, Xd, labels_d, Wd, cached=False):
    """The call sequence of mggcn_epoch issued layer by layer (same kernels on same-shaped buffers,
    hence the same bits), reading back what the device decided on the way: the ReLU' masks and the
    bfloat16 operand of every SpMM.  -> (loss, W_G list, masks, fwd_codes, bwd_codes)"""
    import torch

    L, dims, n = model.L, model.dims, Xd.shape[0]
    pad = lambda d: (d + 15) // 16 * 16
    acts = [torch.empty((n, pad(dims[l + 1])), device=Xd.device)[:, : dims[l + 1]] for l in range(L)]
    fwd, bwd, masks = [None] * L, [None] * L, []
    H = Xd
    for l in range(L):
        first = model.order(l) == mg.ORDER_SPMM_FIRST
        mg.mggcn_layer_fwd(model, l, H, Wd[l], relu=l + 1 < L, H_out=acts[l])
        if not (cached and l == 0):
            fwd[l] = codes_of(model.gather_operand(dims[l] if first else dims[l + 1]))
        if l + 1 < L:
            masks.append((acts[l] > 0).cpu().numpy().astype(np.uint8))
        H = acts[l]
    loss, _ = mg.mggcn_softmax_ce(acts[L - 1], labels_d)
    WG = [None] * L
    for l in range(L - 1, -1, -1):
        first = model.order(l) == mg.ORDER_SPMM_FIRST
        H_in = acts[l - 1] if l > 0 else Xd
        WG[l], _ = mg.mggcn_layer_bwd(model, l, H_in, None, acts[l], Wd[l], need_input_grad=l > 0,
                                      H_G=acts[l - 1] if l > 0 else None, hg_relu_mask=True)
        if not first:
            bwd[l] = codes_of(model.gather_operand(dims[l + 1]))
        elif l > 0:
            bwd[l] = codes_of(model.gather_operand(dims[l]))
    return loss, WG, masks, fwd, bwd


def assert_bf16_relu_decisions_agree(ref, n, rp, ci, v64, W64s, r_orders, fwd_codes, masks, what):
    """The ReLU' decisions handed to the oracle, bounded as in the fp32 tests: the oracle's fp64
    pre-activation of every hidden layer, formed from the same bfloat16 operand the device gathered,
    must take the same decision except at entries that are zero to within fp32 rounding."""
    from test_gpu_parity import assert_relu_decisions_agree

    Zs = []
    for l in range(len(W64s) - 1):
        P = ref.spmm(ref.OP_N, n, n, rp, ci, v64, values_of(fwd_codes[l]).astype(np.float64))
        Zs.append(P if r_orders[l] == ref.GEMM_FIRST else ref.gemm(ref.OP_N, ref.OP_N, P, W64s[l]))
    return assert_relu_decisions_agree(masks, Zs, what)


def assert_operands_are_roundings(dev_codes, own_codes, what):
    """The device's operand is the rounding of its fp32 value, the oracle's that of its fp64 value: they
    agree except where the value sits within fp32 rounding of a boundary (then they are neighbours)."""
    a, b = values_of(dev_codes).astype(np.float64), values_of(own_codes).astype(np.float64)
    assert np.all(np.isfinite(a))
    scale = np.abs(b).max() if b.size else 0.0
    # neighbours differ by one step: 2^-7 relative at most (2^-8 .. 2^-7); near zero allow fp32 noise
    ok = np.abs(a - b) <= 2.0 ** -7 * np.maximum(np.abs(a), np.abs(b)) + 1e-6 * scale
    assert np.all(ok), f"{what}: operand off by more than one bfloat16 step"
    frac = float(np.mean(dev_codes != own_codes)) if dev_codes.size else 0.0
    assert frac <= 5e-3, f"{what}: {frac:.2%} of the operand rounded differently"
    return frac


def run_epoch_case(mg, dev, ref, g, dims, orders, seed, cached=False):
    n = g.n_rows
    rp, ci, val, X, Ws, labels = _model_inputs(ref, g, dims, seed)
    L = len(dims) - 1
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=128)
    flags = mg.MODEL_GATHER_BF16 | (mg.MODEL_CACHE_INPUT if cached else 0)
    model = mg.Model(G, dims, orders=orders, flags=flags)
    Xd, Wd, ld = to_dev(X, dev), [to_dev(w, dev) for w in Ws], to_dev(labels, dev)
    x_codes = None
    if cached:
        model.cache_input(Xd)
        x_codes = codes_of(model.gather_operand(dims[0]))
    loss, WG = mg.mggcn_epoch(model, None if cached else Xd, ld, Wd)
    loss2, WG2 = mg.mggcn_epoch(model, None if cached else Xd, ld, Wd)
    mloss, mWG, masks, fwd, bwd = manual_epoch(mg, model, Xd, ld, Wd, cached=cached)
    if cached:
        fwd[0] = x_codes
    assert loss.item() == loss2.item() == mloss.item()
    for l in range(L):
        assert np.array_equal(WG[l].cpu().numpy(), WG2[l].cpu().numpy()), "epoch must be reproducible bit for bit"
        assert np.array_equal(WG[l].cpu().numpy(), mWG[l].cpu().numpy()), "layer-by-layer epoch differs"
    r_orders = [ref.SPMM_FIRST if model.order(l) == mg.ORDER_SPMM_FIRST else ref.GEMM_FIRST for l in range(L)]
    assert_bf16_relu_decisions_agree(ref, n, rp, ci, val.astype(np.float64), [w.astype(np.float64) for w in Ws], r_orders,
                                     fwd, masks, "bf16 epoch")
    rl, rWG, own_f, own_b = ref.epoch_bf16(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                                           [w.astype(np.float64) for w in Ws], orders=r_orders, relu_masks=masks,
                                           fwd_codes=fwd, bwd_codes=bwd)
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl), (loss.item(), rl)
    for l in range(L):
        assert_rows_close(WG[l].cpu().numpy(), rWG[l], what=f"W_G[{l}]")
        assert fwd[l] is not None
        assert_operands_are_roundings(fwd[l], own_f[l], f"fwd operand {l}")
        assert (bwd[l] is None) == (own_b[l] is None)
        if bwd[l] is not None:
            assert_operands_are_roundings(bwd[l], own_b[l], f"bwd operand {l}")
    # and it is the fp32 epoch up to the rounding of the gathered operands
    rl32, _, _ = ref.epoch(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws], orders=r_orders)
    assert abs(loss.item() - rl32) <= 1e-2 * abs(rl32)


@pytest.mark.parametrize("cfg_name,dims,orders", [
    ("tiny", None, None),
    ("tiny", (64, 100, 32, 8), None),
    ("tiny", (64, 16, 8), "spmm_first"),
    ("small_powerlaw", (50, 128, 41), None),
])
def test_epoch_bf16(mg, dev, ref, cfg_name, dims, orders):
    say(f"[epoch bf16] {cfg_name} dims={dims} orders={orders}")
    if cfg_name == "tiny":
        g = wl.CONFIGS["tiny"].graph()
        dims = dims or wl.CONFIGS["tiny"].dims
    else:
        g = wl.chung_lu(5000, 300e3, 2.1, 2500.0, 8)
    L = len(dims) - 1
    ords = None if orders is None else [mg.ORDER_SPMM_FIRST] * L
    run_epoch_case(mg, dev, ref, g, dims, ords, 7)


def test_epoch_bf16_with_cached_input(mg, dev, ref):
    say("[epoch bf16] cached input")
    g = wl.chung_lu(4000, 200e3, 2.1, 1500.0, 21)
    run_epoch_case(mg, dev, ref, g, (50, 24, 7), None, 11, cached=True)


def test_epoch_bf16_random_cases(mg, dev, ref):
    """Seeded random models with bfloat16 gathers: depths 1-3, mixed widths, forced orders."""
    rng = np.random.default_rng(78)
    for case in range(8):
        n = int(rng.integers(200, 1500))
        L = int(rng.integers(1, 4))
        dims = tuple(int(x) for x in rng.choice([8, 16, 33, 41, 64, 100], size=L + 1))
        forced = [None, mg.ORDER_GEMM_FIRST, mg.ORDER_SPMM_FIRST][int(rng.integers(0, 3))]
        say(f"[epoch bf16 random {case}] n={n} dims={dims} forced={forced}")
        g = wl.chung_lu(n, float(n * rng.integers(5, 40)), 2.2, float(n) / 2, 2000 + case)
        run_epoch_case(mg, dev, ref, g, dims, None if forced is None else [forced] * L, 100 + case)


def test_model_bf16_flag_errors(mg, dev, ref):
    g = wl.CONFIGS["tiny"].graph()
    rp, ci, val = normalized(ref, g)
    G = mg.Graph(g.n_rows, g.n_cols, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=64)
    plain = mg.Model(G, (64, 16, 8))
    with pytest.raises(mg.MggcnError):
        plain.gather_operand(16)
    with pytest.raises(mg.MggcnError):
        mg.Model(G, (64, 16, 8), flags=64)
    half = mg.Model(G, (64, 16, 8), flags=mg.MODEL_GATHER_BF16)  # GeMM first twice: SpMM widths 16 and 8
    assert half.gather_operand(16).shape == (g.n_rows, 16)
    for width in (0, 17, 64):  # the copy holds the widest SpMM operand, nothing wider
        with pytest.raises(mg.MggcnError):
            half.gather_operand(width)


@pytest.mark.parametrize("F", [100, 256, 602])
def test_spmm_automatic_panels_and_feature_slices(mg, dev, ref, F):
    """Automatic mode on a graph dense enough to get panel forms, with the per-panel target shrunk
    to 1 MiB so that a small operand already takes several panels and, at the wider widths,
    several feature slices -- the path a wide operand takes on the 233K-vertex graph."""
    say(f"[spmm auto panels] F={F}")
    g = wl.chung_lu(3000, 600e3, 2.1, 1500.0, 41)
    rp, ci, val = normalized(ref, g)
    n = g.n_rows
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=F, panel_mib=1)
    # the fp32 target is 3/4 of the setting, feature slices are cut for 2/3 of that; 200 entries per
    # row afford 4 panels; 7 MiB at F=602 then also takes 4 feature slices
    assert G.panels(602) == 16 and G.panels(100) == 2 and G.panels(16) == 1
    X = wl.normal_f32(55 + F, 6, (n, F))
    Y0 = wl.normal_f32(55 + F, 7, (n, F))
    want = ref.spmm(ref.OP_N, n, n, rp, ci, val.astype(np.float64), X.astype(np.float64))
    got = mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev)).cpu().numpy()
    assert_rows_close(got, want, what=f"fp32 auto F={F}")
    Yd = to_dev(Y0, dev)
    mg.mggcn_spmm(G, mg.OP_N, to_dev(X, dev), beta=1.0, epilogue=mg.EPI_RELU, Y=Yd)
    check_spmm(ref, ref.OP_N, n, n, rp, ci, val, X, Yd.cpu().numpy(), F, beta=1.0, Y0=Y0, epi="relu", what="fp32 auto acc")
    Xb = mg.mggcn_f32_to_bf16(to_dev(X, dev))
    _, Xq = ref.bf16_round(X)
    got = mg.mggcn_spmm_bf16(G, mg.OP_N, Xb).cpu().numpy()
    check_spmm(ref, ref.OP_N, n, n, rp, ci, val, Xq, got, F, what=f"bf16 auto F={F}")
