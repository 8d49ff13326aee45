"""GPU parity at the benchmark's full size: the Reddit-shaped "medium" configuration
(232,965 vertices, ~114M entries, 602 -> 128 -> 41) in exactly the launch configuration
bench.py times (padded leading dimensions, fused ReLU epilogue, default segment length).
The oracle is fast enough here to check every output row, not a sample."""
import sys
import time

import numpy as np
import pytest

import workloads as wl
from test_gpu_parity import assert_relu_decisions_agree, oracle_preactivations

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1100)]


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def row_err(got, want):
    num = np.abs(got.astype(np.float64) - want).max(axis=1)
    den = np.abs(want).max(axis=1)
    assert np.all(num[den == 0] == 0)
    return num / np.maximum(den, 1e-300)


@pytest.fixture(scope="module")
def medium(ref):
    import torch

    import paper_2110_08688_amd as mg

    mg.binding.lib()
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS["medium"]
    t0 = time.time()
    g = cfg.graph()
    say(f"[medium] generated n={g.n_rows} nnz={g.nnz} in {time.time() - t0:.1f}s")
    n = g.n_rows
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev), validate=True)
    t0 = time.time()
    rp, ci, rv = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    say(f"[medium] oracle normalise {time.time() - t0:.1f}s, nnz with self-loops {len(ci)}")
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=128)
    return dict(mg=mg, dev=dev, cfg=cfg, n=n, rowptr=rowptr, colidx=colidx, val=val, rp=rp, ci=ci, rv=rv,
                graph=graph)


def test_medium_normalize_bit_exact(medium):
    m = medium
    assert np.array_equal(m["rowptr"].cpu().numpy(), m["rp"])
    assert np.array_equal(m["colidx"].cpu().numpy(), m["ci"])
    assert np.array_equal(m["val"].cpu().numpy().view(np.int32), m["rv"].astype(np.float32).view(np.int32))
    # closed form on the device values: A^ sqrt(d) = sqrt(d) -- holds at any size
    d = np.diff(m["rp"]).astype(np.float64)
    assert d.min() >= 1


@pytest.mark.parametrize("F,ld,relu", [(128, 128, True), (41, 48, False)])
def test_medium_spmm_all_rows(medium, ref, F, ld, relu):
    import torch

    m = medium
    mg, dev, n = m["mg"], m["dev"], m["n"]
    say(f"[medium spmm] F={F} ld={ld} relu={relu}")
    Xp = wl.normal_f32(4242, F, (n, ld))
    Xd = torch.from_numpy(Xp).to(dev)
    Yd = torch.zeros((n, ld), device=dev)
    mg.mggcn_spmm(m["graph"], mg.OP_N, Xd[:, :F], epilogue=mg.EPI_RELU if relu else mg.EPI_NONE, Y=Yd[:, :F])
    got = Yd.cpu().numpy()
    t0 = time.time()
    want = ref.spmm(ref.OP_N, n, n, m["rp"], m["ci"], m["rv"].astype(np.float32).astype(np.float64),
                    Xp[:, :F].astype(np.float64))
    say(f"[medium spmm] oracle {time.time() - t0:.1f}s")
    if relu:
        want = np.maximum(want, 0.0)
    e = row_err(got[:, :F], want)
    say(f"[medium spmm] max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    assert np.all(got[:, F:] == 0)
    # transposed product on the symmetric operator gives the same bits
    Yt = torch.zeros((n, ld), device=dev)
    mg.mggcn_spmm(m["graph"], mg.OP_T, Xd[:, :F], epilogue=mg.EPI_RELU if relu else mg.EPI_NONE, Y=Yt[:, :F])
    assert torch.equal(Yd, Yt)


@pytest.mark.parametrize("gemm", ["fp32", "bf16x3"])
def test_medium_epoch(medium, ref, gemm):
    """the benchmarked epoch against the oracle's, with the GeMMs on the fp32 matrix instruction and
    (the extension) on the bfloat16 ones: same oracle, same bounds"""
    import torch

    m = medium
    mg, dev, n, cfg = m["mg"], m["dev"], m["n"], m["cfg"]
    X, Ws, labels = cfg.features(n), cfg.weights(), cfg.labels(n)
    model = mg.Model(m["graph"], cfg.dims, flags=mg.MODEL_GEMM_BF16X3 if gemm == "bf16x3" else 0)
    Xd, Wd = torch.from_numpy(X).to(dev), [torch.from_numpy(w).to(dev) for w in Ws]
    loss, WG = mg.mggcn_epoch(model, Xd, torch.from_numpy(labels).to(dev), Wd)
    torch.cuda.synchronize()
    say(f"[medium epoch, GeMM {gemm}] gpu loss {loss.item():.7f}; running the fp64 oracle epoch on the host ...")
    # the device's own ReLU' decisions (same forward call, same bits as inside the epoch): a
    # hidden activation that is zero to within rounding is "on" or "off" by a coin toss, and one
    # such entry moves a whole column of W_G[0] by ~1/sqrt(n) of its size
    out = torch.empty((n, 128), device=dev)
    mg.mggcn_layer_fwd(model, 0, Xd, Wd[0], relu=True, H_out=out)
    mask = (out > 0).cpu().numpy().astype(np.uint8)
    v64 = m["rv"].astype(np.float32).astype(np.float64)
    t0 = time.time()
    rl, rWG, _ = ref.epoch(n, m["rp"], m["ci"], v64, X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws], relu_masks=[mask])
    say(f"[medium epoch] oracle {time.time() - t0:.1f}s loss {rl:.7f}")
    own = ref.layer_fwd(n, m["rp"], m["ci"], v64, X.astype(np.float64), Ws[0].astype(np.float64),
                        ref.GEMM_FIRST, True) > 0
    say(f"[medium epoch] ReLU' decisions that differ between fp32 device and fp64 oracle: "
        f"{int(np.count_nonzero(own != mask.astype(bool)))} of {mask.size}")
    del own
    pre = ref.layer_fwd(n, m["rp"], m["ci"], v64, X.astype(np.float64), Ws[0].astype(np.float64), ref.GEMM_FIRST, False)
    assert_relu_decisions_agree([mask], [pre], "medium epoch")
    del pre
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    for l, (a, b) in enumerate(zip(WG, rWG)):
        e = row_err(a.cpu().numpy(), b)
        say(f"[medium epoch] W_G[{l}] max row rel err {e.max():.3e}")
        assert e.max() <= 1e-4


@pytest.mark.parametrize("F,ld", [(128, 128), (41, 48)])
def test_medium_spmm_bf16_all_rows(medium, ref, F, ld):
    """bfloat16 copy of the gathered operand (extension): same per-row bound against the oracle fed
    the same rounded values; the conversion itself is bit exact."""
    import torch

    m = medium
    mg, dev, n = m["mg"], m["dev"], m["n"]
    say(f"[medium spmm bf16] F={F} ld={ld}")
    Xp = wl.normal_f32(4343, F, (n, ld))
    Xb = torch.empty((n, ld), dtype=torch.int16, device=dev)
    mg.mggcn_f32_to_bf16(torch.from_numpy(Xp).to(dev)[:, :F], dst=Xb[:, :F])
    codes, Xq = ref.bf16_round(np.ascontiguousarray(Xp[:, :F]))
    assert np.array_equal(Xb[:, :F].cpu().numpy().view(np.uint16), codes)
    Yd = torch.zeros((n, ld), device=dev)
    mg.mggcn_spmm_bf16(m["graph"], mg.OP_N, Xb[:, :F], Y=Yd[:, :F])
    got = Yd.cpu().numpy()
    want = ref.spmm(ref.OP_N, n, n, m["rp"], m["ci"], m["rv"].astype(np.float32).astype(np.float64),
                    Xq.astype(np.float64))
    e = row_err(got[:, :F], want)
    say(f"[medium spmm bf16] max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    assert np.all(got[:, F:] == 0)


def test_medium_epoch_bf16(medium, ref):
    """Epoch with MODEL_GATHER_BF16 at full size: the oracle's bfloat16-gather epoch, handed the device's
    ReLU' decisions and SpMM operands, must give the same loss and weight gradients; the operands
    themselves must be the roundings of (nearly) the oracle's own values."""
    import torch

    from test_gpu_bf16 import assert_bf16_relu_decisions_agree, assert_operands_are_roundings, manual_epoch

    m = medium
    mg, dev, n, cfg = m["mg"], m["dev"], m["n"], m["cfg"]
    X, Ws, labels = cfg.features(n), cfg.weights(), cfg.labels(n)
    model = mg.Model(m["graph"], cfg.dims, flags=mg.MODEL_GATHER_BF16)
    Xd, Wd, ld = torch.from_numpy(X).to(dev), [torch.from_numpy(w).to(dev) for w in Ws], torch.from_numpy(labels).to(dev)
    loss, WG = mg.mggcn_epoch(model, Xd, ld, Wd)
    mloss, mWG, masks, fwd, bwd = manual_epoch(mg, model, Xd, ld, Wd)
    assert loss.item() == mloss.item()
    for a, b in zip(WG, mWG):
        assert torch.equal(a, b), "layer-by-layer epoch differs from mggcn_epoch"
    say(f"[medium epoch bf16] gpu loss {loss.item():.7f}; running the fp64 oracle epoch on the host ...")
    v64 = m["rv"].astype(np.float32).astype(np.float64)
    flips = assert_bf16_relu_decisions_agree(ref, n, m["rp"], m["ci"], v64, [w.astype(np.float64) for w in Ws],
                                             [ref.GEMM_FIRST, ref.GEMM_FIRST], fwd, masks, "medium epoch bf16")
    say(f"[medium epoch bf16] ReLU' decisions that differ from the oracle's on the same operand: {flips}")
    t0 = time.time()
    rl, rWG, own_f, own_b = ref.epoch_bf16(n, m["rp"], m["ci"], m["rv"].astype(np.float32).astype(np.float64),
                                           X.astype(np.float64), labels, [w.astype(np.float64) for w in Ws],
                                           relu_masks=masks, fwd_codes=fwd, bwd_codes=bwd)
    say(f"[medium epoch bf16] oracle {time.time() - t0:.1f}s loss {rl:.7f}")
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    for l, (a, b) in enumerate(zip(WG, rWG)):
        e = row_err(a.cpu().numpy(), b)
        say(f"[medium epoch bf16] W_G[{l}] max row rel err {e.max():.3e}")
        assert e.max() <= 1e-4
        f1 = assert_operands_are_roundings(fwd[l], own_f[l], f"fwd operand {l}")
        f2 = assert_operands_are_roundings(bwd[l], own_b[l], f"bwd operand {l}")
        say(f"[medium epoch bf16] layer {l}: operand entries rounded to the other neighbour: fwd {f1:.2e}, bwd {f2:.2e}")


# ----------------------------------------------------------------------------------------------
# Products-shaped "large" configuration: 2,449,029 vertices, ~126M entries, 100 -> 256 -> 256 -> 47
# (first layer runs SpMM first, the other two GeMM first)
# ----------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def large(ref):
    import torch

    import paper_2110_08688_amd as mg

    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS["large"]
    t0 = time.time()
    g = cfg.graph()
    n = g.n_rows
    say(f"[large] generated n={n} nnz={g.nnz} in {time.time() - t0:.1f}s")
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev))
    rp, ci, rv = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(colidx.cpu().numpy(), ci)
    assert np.array_equal(val.cpu().numpy().view(np.int32), rv.astype(np.float32).view(np.int32))
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=256)
    return dict(mg=mg, dev=dev, cfg=cfg, n=n, rp=rp, ci=ci, v64=rv.astype(np.float32).astype(np.float64),
                graph=graph)


@pytest.mark.parametrize("F,ld", [(100, 112), (256, 256), (47, 48)])
def test_large_spmm_all_rows(large, ref, F, ld):
    import torch

    m = large
    mg, dev, n = m["mg"], m["dev"], m["n"]
    say(f"[large spmm] F={F} ld={ld}")
    Xp = wl.normal_f32(777, F, (n, ld))
    Xd = torch.from_numpy(Xp).to(dev)
    Yd = torch.zeros((n, ld), device=dev)
    mg.mggcn_spmm(m["graph"], mg.OP_N, Xd[:, :F], Y=Yd[:, :F])
    got = Yd.cpu().numpy()
    t0 = time.time()
    want = ref.spmm(ref.OP_N, n, n, m["rp"], m["ci"], m["v64"], Xp[:, :F].astype(np.float64))
    e = row_err(got[:, :F], want)
    say(f"[large spmm] oracle {time.time() - t0:.1f}s, max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    assert np.all(got[:, F:] == 0)


def test_large_epoch(large, ref):
    import torch

    m = large
    mg, dev, n, cfg = m["mg"], m["dev"], m["n"], m["cfg"]
    X, Ws, labels = cfg.features(n), cfg.weights(), cfg.labels(n)
    model = mg.Model(m["graph"], cfg.dims)
    assert [model.order(l) for l in range(3)] == [mg.ORDER_SPMM_FIRST, mg.ORDER_GEMM_FIRST, mg.ORDER_GEMM_FIRST]
    Xd, Wd = torch.from_numpy(X).to(dev), [torch.from_numpy(w).to(dev) for w in Ws]
    loss, WG = mg.mggcn_epoch(model, Xd, torch.from_numpy(labels).to(dev), Wd)
    torch.cuda.synchronize()
    say(f"[large epoch] gpu loss {loss.item():.7f}")
    masks, H = [], Xd
    for l in range(2):  # the device's own ReLU' decisions, same forward calls as inside the epoch
        out = torch.empty((n, 256), device=dev)
        mg.mggcn_layer_fwd(model, l, H, Wd[l], relu=True, H_out=out)
        masks.append((out > 0).cpu().numpy().astype(np.uint8))
        H = out
    del H, out
    t0 = time.time()
    Zs = oracle_preactivations(ref, n, m["rp"], m["ci"], m["v64"], X.astype(np.float64), [w.astype(np.float64) for w in Ws],
                               [ref.SPMM_FIRST, ref.GEMM_FIRST, ref.GEMM_FIRST])
    flips = assert_relu_decisions_agree(masks, Zs, "large epoch")
    del Zs
    say(f"[large epoch] oracle forward chain {time.time() - t0:.1f}s; ReLU' decisions that differ from the oracle's: "
        f"{flips} of {sum(k.size for k in masks)}")
    t0 = time.time()
    rl, rWG, _ = ref.epoch(n, m["rp"], m["ci"], m["v64"], X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws], relu_masks=masks)
    say(f"[large epoch] oracle {time.time() - t0:.1f}s loss {rl:.7f}")
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    for l, (a, b) in enumerate(zip(WG, rWG)):
        e = row_err(a.cpu().numpy(), b)
        say(f"[large epoch] W_G[{l}] max row rel err {e.max():.3e}")
        assert e.max() <= 1e-4


# ----------------------------------------------------------------------------------------------
# skewed R-MAT graph (2^22 vertices, ~62M entries, 2.2M isolated vertices, hubs of ~94K entries)
# ----------------------------------------------------------------------------------------------

def test_rmat_spmm_all_rows(ref):
    import torch

    import paper_2110_08688_amd as mg

    dev = torch.device("cuda:0")
    g = wl.CONFIGS["rmat"].graph()
    n = g.n_rows
    say(f"[rmat] n={n} nnz={g.nnz} max degree {int(np.diff(g.rowptr).max())}")
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev))
    rp, ci, rv = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(colidx.cpu().numpy(), ci)
    assert np.array_equal(val.cpu().numpy().view(np.int32), rv.astype(np.float32).view(np.int32))
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=128)
    X = wl.normal_f32(99, 128, (n, 128))
    got = mg.mggcn_spmm(graph, mg.OP_N, torch.from_numpy(X).to(dev)).cpu().numpy()
    want = ref.spmm(ref.OP_N, n, n, rp, ci, rv.astype(np.float32).astype(np.float64), X.astype(np.float64))
    e = row_err(got, want)
    say(f"[rmat] max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4


# ----------------------------------------------------------------------------------------------
# one GPU's row block of a 1-D partition: 13.9M x 111M, ~200M entries, X 111M x 128 (56.8 GB on the
# device).  The fp64 copy of X does not fit the host, so parity is on sampled output rows (4,096
# random + the 64 longest), recomputed by the oracle from regenerated inputs.
# ----------------------------------------------------------------------------------------------

@pytest.fixture(scope="module")
def block(ref):
    """The row block, its transpose, X on the device and the five products bench.py times on it
    (SpMM-first 128 -> 256 layer, forward and backward), each run once."""
    import torch

    import paper_2110_08688_amd as mg

    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS["block"]
    t0 = time.time()
    g = cfg.graph()
    nr, nc = g.n_rows, g.n_cols
    say(f"[block] generated {nr} x {nc}, nnz={g.nnz} in {time.time() - t0:.1f}s")
    # stand-in global degrees: row degree = local count + 1, column degree = 1 + 8 * (count in block)
    deg_row = (np.diff(g.rowptr) + 1).astype(np.int32)
    deg_col = (1 + 8 * np.bincount(g.colidx, minlength=nc)).astype(np.int32)
    rowptr, colidx, val = mg.mggcn_csr_normalize(nr, nc, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev),
                                                 deg_row=torch.from_numpy(deg_row).to(dev),
                                                 deg_col=torch.from_numpy(deg_col).to(dev))
    rp, ci, rv = ref.csr_normalize(nr, nc, g.rowptr, g.colidx, deg_row=deg_row, deg_col=deg_col)
    del g, deg_row, deg_col
    assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(colidx.cpu().numpy(), ci)
    v32f = rv.astype(np.float32)
    assert np.array_equal(val.cpu().numpy().view(np.int32), v32f.view(np.int32))
    v32 = v32f.astype(np.float64)
    del rv, v32f
    say(f"[block] normalised, nnz with diagonal {len(ci)}")
    t = mg.mggcn_csr_transpose(nr, nc, rowptr, colidx, val)
    graph = mg.Graph(nr, nc, rowptr, colidx, val, transpose=t, F_max=128)
    d_in, d_out = cfg.dims
    F = d_in
    Xd = torch.empty((nc, F), dtype=torch.float32, device=dev)
    t0 = time.time()
    fill_x(Xd, cfg, nc, F)
    say(f"[block] X {nc} x {F} on the device in {time.time() - t0:.1f}s")
    return dict(mg=mg, dev=dev, cfg=cfg, nr=nr, nc=nc, rp=rp, ci=ci, v32=v32, t=t, graph=graph, Xd=Xd, F=F,
                d_in=d_in, d_out=d_out)


def fill_x(Xd, cfg, nc, F, chunk=2_000_000):
    """counter-based generator: row r of X is elements [r*F, (r+1)*F) of the stream"""
    import torch

    for r0 in range(0, nc, chunk):
        r1 = min(nc, r0 + chunk)
        Xd[r0:r1].copy_(torch.from_numpy(wl.normal_f32(cfg.seed + 0x100, 0, (r1 - r0, F), first=r0 * F)))


def test_row_block_spmm_sampled_rows(block, ref):
    import torch

    b = block
    mg, dev, cfg, nr, nc, rp, ci, v32, graph, Xd, F = (b[k] for k in ("mg", "dev", "cfg", "nr", "nc", "rp", "ci", "v32",
                                                                       "graph", "Xd", "F"))
    Yd = mg.mggcn_spmm(graph, mg.OP_N, Xd)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    deg = np.diff(rp)
    rows = np.unique(np.concatenate([rng.integers(0, nr, 4096), np.argsort(deg)[-64:]]))
    got = Yd[torch.from_numpy(rows).to(dev)].cpu().numpy()
    worst = 0.0
    for j, i in enumerate(rows):  # the definition, one sampled row at a time
        cols = ci[rp[i]:rp[i + 1]]
        acc = np.zeros(F)
        for k, c in enumerate(cols):
            x = wl.normal_f32(cfg.seed + 0x100, 0, (F,), first=int(c) * F).astype(np.float64)
            acc += v32[rp[i] + k] * x
        err = np.abs(got[j] - acc).max() / max(np.abs(acc).max(), 1e-300)
        worst = max(worst, err)
    say(f"[block] {len(rows)} sampled rows, max row rel err {worst:.3e}")
    assert worst <= 1e-4
    # the same product with a bfloat16 copy of X: it differs from the fp32 one by the rounding of X
    # only (at most 2^-8 of |A^||X| per row); both are timed here because this is the configuration
    # whose 111 M gathered rows no cache holds
    Xb = torch.empty((nc, F), dtype=torch.int16, device=dev)
    mg.mggcn_f32_to_bf16(Xd, dst=Xb)
    Yb = torch.empty_like(Yd)
    t32, t16 = [], []
    for _ in range(3):
        a, bb, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        a.record()
        mg.mggcn_spmm(graph, mg.OP_N, Xd, Y=Yd)
        bb.record()
        mg.mggcn_spmm_bf16(graph, mg.OP_N, Xb, Y=Yb)
        c.record()
        torch.cuda.synchronize()
        t32.append(a.elapsed_time(bb))
        t16.append(bb.elapsed_time(c))
    nnz = len(ci)
    beff = 8 * nnz + 4 * (nr + 1) + 4 * F * nnz + 4 * F * nr
    say(f"[block] spmm F={F}: fp32 operand {min(t32):.2f} ms = {beff / min(t32) / 1e6:.0f} GB/s by no-reuse bytes; "
        f"bfloat16 operand {min(t16):.2f} ms")
    Ab = mg.mggcn_spmm(graph, mg.OP_N, Xd.abs_())     # |A^||X| (values of A^ are positive); Xd is regenerated below
    diff = (Yb - Yd).abs().max(dim=1).values
    assert bool((diff <= (2.0 ** -8 + 1e-5) * Ab.max(dim=1).values.clamp_min(1e-30)).all())
    del Xb, Yb, Ab
    fill_x(Xd, cfg, nc, F)
    # transposed product on the same block: adjoint identity on a sampled pair, <A X, G> = <X, A^T G>,
    # with G supported on the sampled rows only (the element-wise check of op T is the next test)
    Gd = torch.zeros((nr, F), dtype=torch.float32, device=dev)
    Gs = wl.normal_f32(cfg.seed + 0x400, 0, (len(rows), F))
    Gd[torch.from_numpy(rows).to(dev)] = torch.from_numpy(Gs).to(dev)
    Td = mg.mggcn_spmm(graph, mg.OP_T, Gd)
    lhs = float((Yd.double() * Gd.double()).sum().item())
    rhs = 0.0
    for r0 in range(0, nc, 4_000_000):  # fp64 dot product in slices: the operands are 57 GB each
        r1 = min(nc, r0 + 4_000_000)
        rhs += float((Xd[r0:r1].double() * Td[r0:r1].double()).sum().item())
    say(f"[block] adjoint identity {lhs:.9e} vs {rhs:.9e}")
    assert abs(lhs - rhs) <= 1e-5 * abs(lhs)


def test_row_block_layer_all_five_products(block, ref):
    """The SpMM-first 128 -> 256 layer on the row block, forward and backward, as the five calls bench.py
    times: P = A^ X, H = relu(P W), W_G = P^T G, U = G W^T, X_G = A^^T U.  Every product is compared with
    the oracle's on sampled outputs, each from the device's own input of that product (the identical
    fp32 operand widened to fp64): the three GeMMs on sampled rows (the weight gradient, whose every
    element sums over all 13.9 M rows, on a sampled sub-block of its elements) and the transposed SpMM
    over 111 M output rows on 4,096 random rows plus the 64 heaviest columns of the block, from the
    oracle's own transpose of the block."""
    import torch

    b = block
    mg, dev, cfg, nr, nc, rp, ci, v32, graph, Xd, F, d_out = (b[k] for k in ("mg", "dev", "cfg", "nr", "nc", "rp", "ci",
                                                                             "v32", "graph", "Xd", "F", "d_out"))
    W = cfg.weights()[0]
    Wd = torch.from_numpy(W).to(dev)
    W64 = W.astype(np.float64)
    t0 = time.time()
    G = wl.normal_f32(cfg.seed + 0x500, 0, (nr, d_out))  # seeded stand-in for the gradient arriving from the loss
    Gd = torch.from_numpy(G).to(dev)
    say(f"[block layer] gradient operand {nr} x {d_out} in {time.time() - t0:.1f}s")
    P = mg.mggcn_spmm(graph, mg.OP_N, Xd)
    H = mg.mggcn_gemm(mg.OP_N, mg.OP_N, P, Wd, epilogue=mg.EPI_RELU)
    WG = mg.mggcn_gemm(mg.OP_T, mg.OP_N, P, Gd)
    U = mg.mggcn_gemm(mg.OP_N, mg.OP_T, Gd, Wd)
    XG = mg.mggcn_spmm(graph, mg.OP_T, U)
    torch.cuda.synchronize()
    rng = np.random.default_rng(6)
    rows = np.unique(np.concatenate([rng.integers(0, nr, 8192), [0, 127, 128, nr - 129, nr - 1]]))
    rows_d = torch.from_numpy(rows).to(dev)

    # Eq. 5 + 7 on sampled rows, from the device's own P
    P_rows = P[rows_d].cpu().numpy().astype(np.float64)
    pre = ref.gemm(ref.OP_N, ref.OP_N, P_rows, W64)
    num = np.abs(H[rows_d].cpu().numpy().astype(np.float64) - np.maximum(pre, 0.0)).max(axis=1)
    e = num / np.maximum(np.abs(pre).max(axis=1), 1e-300)
    say(f"[block layer] H = relu(P W): {len(rows)} sampled rows, max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    del H

    # Eq. 11 on sampled rows
    want = ref.gemm(ref.OP_N, ref.OP_T, G[rows].astype(np.float64), W64)
    e = row_err(U[rows_d].cpu().numpy(), want)
    say(f"[block layer] U = G W^T: {len(rows)} sampled rows, max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4

    # Eq. 10: a sampled 24 x 48 sub-block of W_G (rows and columns straddling the kernel's 128 x 64 tiles), each
    # element the full sum over all rows of the block, from the device's own P
    Ph = P.cpu().numpy()
    ra = np.unique(np.concatenate([rng.integers(0, F, 16), [0, 31, 32, 63, 64, 95, 96, 127]]))
    cb = np.unique(np.concatenate([rng.integers(0, d_out, 32), [0, 63, 64, 127, 128, 191, 192, 255]]))
    t0 = time.time()
    want = ref.gemm(ref.OP_T, ref.OP_N, np.ascontiguousarray(Ph[:, ra], dtype=np.float64),
                    np.ascontiguousarray(G[:, cb], dtype=np.float64))
    got = WG.cpu().numpy()[np.ix_(ra, cb)]
    e = row_err(got, want)
    say(f"[block layer] W_G = P^T G: {len(ra)} x {len(cb)} sampled elements (K = {nr}), oracle {time.time() - t0:.1f}s, "
        f"max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    del Ph, P, G, Gd

    # Eq. 9 on the rectangular operator: X_G = A^^T U over 111 M output rows, element-wise on sampled rows
    t0 = time.time()
    rpt, cit, vt = ref.csr_transpose(nr, nc, rp, ci, v32)
    say(f"[block layer] oracle transpose of the block in {time.time() - t0:.1f}s")
    tdev = b["t"]
    assert np.array_equal(tdev[0].cpu().numpy(), rpt) and np.array_equal(tdev[1].cpu().numpy(), cit)
    assert np.array_equal(tdev[2].cpu().numpy(), vt.astype(np.float32))
    cnt = np.diff(rpt)
    out_rows = np.unique(np.concatenate([rng.integers(0, nc, 4096), np.argsort(cnt)[-64:], [0, nc - 1]]))
    Uh = U.cpu().numpy()
    got = XG[torch.from_numpy(out_rows).to(dev)].cpu().numpy()
    worst, heaviest = 0.0, 0
    for j, c in enumerate(out_rows):  # the definition, one sampled output row at a time
        k0, k1 = rpt[c], rpt[c + 1]
        acc = vt[k0:k1] @ Uh[cit[k0:k1]].astype(np.float64) if k1 > k0 else np.zeros(F)
        den = np.abs(acc).max()
        if den == 0:
            assert np.all(got[j] == 0)
            continue
        worst = max(worst, np.abs(got[j] - acc).max() / den)
        heaviest = max(heaviest, int(k1 - k0))
    say(f"[block layer] X_G = A^^T U: {len(out_rows)} sampled rows of {nc} (longest {heaviest} entries), "
        f"max row rel err {worst:.3e}")
    assert worst <= 1e-4


# ----------------------------------------------------------------------------------------------
# Proteins-shaped graph (Table 1 of the paper: 8.74M vertices, 1.3B entries, 128 -> 256 -> 256 -> 256),
# the largest graph the paper trains on a single GPU.  The oracle is still affordable for one
# product over all rows; the first layer is checked on a row sample; the whole epoch is only run.
# ----------------------------------------------------------------------------------------------

def test_proteins_shaped_spmm_and_first_layer(ref):
    import torch

    import paper_2110_08688_amd as mg

    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS["proteins"]
    t0 = time.time()
    g = cfg.graph()
    n = g.n_rows
    say(f"[proteins] generated n={n} nnz={g.nnz} max degree {int(np.diff(g.rowptr).max())} in {time.time() - t0:.1f}s")
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev))
    t0 = time.time()
    rp, ci, rv = ref.csr_normalize(n, n, g.rowptr, g.colidx)
    del g
    say(f"[proteins] oracle normalise {time.time() - t0:.1f}s, entries with self-loops {len(ci)}")
    assert np.array_equal(rowptr.cpu().numpy(), rp) and np.array_equal(colidx.cpu().numpy(), ci)
    v32 = rv.astype(np.float32)
    assert np.array_equal(val.cpu().numpy().view(np.int32), v32.view(np.int32))
    rv = v32.astype(np.float64)
    del v32
    t0 = time.time()
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=256)
    say(f"[proteins] task tables in {time.time() - t0:.1f}s, panels at F=128/256: {graph.panels(128)}/{graph.panels(256)}")
    F = cfg.dims[0]
    X = cfg.features(n)
    Xd = torch.from_numpy(X).to(dev)
    Yd = mg.mggcn_spmm(graph, mg.OP_N, Xd)
    t0 = time.time()
    want = ref.spmm(ref.OP_N, n, n, rp, ci, rv, X.astype(np.float64))
    e = row_err(Yd.cpu().numpy(), want)
    say(f"[proteins] spmm F={F} over all rows: oracle {time.time() - t0:.1f}s, max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    # timing, fp32 and bfloat16 operand
    Xb = mg.mggcn_f32_to_bf16(Xd)
    Yb = torch.empty_like(Yd)
    t32, t16 = [], []
    for _ in range(3):
        a, b, c = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        a.record()
        mg.mggcn_spmm(graph, mg.OP_N, Xd, Y=Yd)
        b.record()
        mg.mggcn_spmm_bf16(graph, mg.OP_N, Xb, Y=Yb)
        c.record()
        torch.cuda.synchronize()
        t32.append(a.elapsed_time(b))
        t16.append(b.elapsed_time(c))
    nnz = len(ci)
    beff = 8 * nnz + 4 * (n + 1) + 4 * F * nnz + 4 * F * n
    say(f"[proteins] spmm F={F}: fp32 operand {min(t32):.2f} ms = {beff / min(t32) / 1e6:.0f} GB/s effective "
        f"({100 * beff / min(t32) / 1e6 / 8000:.1f} % of 8 TB/s); bfloat16 operand {min(t16):.2f} ms")
    _, Xq = ref.bf16_round(X)
    del X
    rows = np.unique(np.random.default_rng(9).integers(0, n, 2048))
    gotb = Yb[torch.from_numpy(rows).to(dev)].cpu().numpy()
    for j, i in enumerate(rows):  # bfloat16 product on sampled rows, by the definition
        k0, k1 = rp[i], rp[i + 1]
        acc = rv[k0:k1] @ Xq[ci[k0:k1]].astype(np.float64)
        assert np.abs(gotb[j] - acc).max() <= 1e-4 * np.abs(acc).max()
    del Xq, Xb, Yb
    # first layer (SpMM first: 128 < 256) on a row sample: relu((A^ X) W), with A^ X from the oracle
    Ws = cfg.weights()
    model = mg.Model(graph, cfg.dims)
    assert model.order(0) == mg.ORDER_SPMM_FIRST and model.order(1) == mg.ORDER_GEMM_FIRST
    Wd = [torch.from_numpy(w).to(dev) for w in Ws]
    H1 = mg.mggcn_layer_fwd(model, 0, Xd, Wd[0], relu=True)
    rows = np.unique(np.random.default_rng(10).integers(0, n, 100_000))
    pre_rows = want[rows] @ Ws[0].astype(np.float64)
    # the error of relu(z) is that of the product z (ReLU is exact and 1-Lipschitz), measured against the row of z
    num = np.abs(H1[torch.from_numpy(rows).to(dev)].cpu().numpy().astype(np.float64) - np.maximum(pre_rows, 0.0)).max(axis=1)
    e = num / np.abs(pre_rows).max(axis=1)
    say(f"[proteins] layer 0 forward on {len(rows)} sampled rows: max row rel err {e.max():.3e}")
    assert e.max() <= 1e-4
    del want, H1
    # the whole epoch at this size: run and timed; its loss must sit just above ln(256) (small random
    # weights, uniform labels) and repeat bit for bit.  No oracle epoch at this size (~10 TFLOP of fp64 GeMM).
    labels = torch.from_numpy(cfg.labels(n)).to(dev)
    loss, WG = mg.mggcn_epoch(model, Xd, labels, Wd)
    torch.cuda.synchronize()
    t0 = time.time()
    loss2, WG2 = mg.mggcn_epoch(model, Xd, labels, Wd)
    torch.cuda.synchronize()
    say(f"[proteins] epoch {1e3 * (time.time() - t0):.1f} ms, loss {loss.item():.6f} (ln 256 = {np.log(256.0):.6f})")
    assert loss.item() == loss2.item() and all(torch.equal(a, b) for a, b in zip(WG, WG2))
    assert np.log(256.0) <= loss.item() <= np.log(256.0) + 0.05
    assert all(bool(torch.isfinite(w).all()) for w in WG)
