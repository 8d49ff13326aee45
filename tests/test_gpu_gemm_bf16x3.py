"""GPU parity of the GeMM on the bfloat16 matrix instructions (mggcn_gemm_bf16x3, model flag
MGGCN_MODEL_GEMM_BF16X3) against the same fp64 oracle as the fp32 GeMM, at the same tolerance and --
because the point of the three-piece split is that nothing is rounded to bfloat16 -- at a far tighter
one where the arithmetic allows it: a reading that rounded an operand to bfloat16 would be wrong by
2^-9 = 2e-3 of a row, four orders of magnitude above what is asserted here."""
import numpy as np
import pytest

import workloads as wl
from test_gpu_parity import (TOL, _model_inputs, assert_relu_decisions_agree, assert_rows_close, dev, gpu_relu_decisions, mg,  # noqa: F401
                             normalized, oracle_preactivations,
                             row_err, say, to_dev)

pytestmark = pytest.mark.gpu

# measured 1.5e-7 - 5e-7 of a row's largest entry for K up to 602 (fp32 rounding of K additions);
# one operand rounded to bfloat16 would give 2e-3
TIGHT = 4e-6


@pytest.mark.parametrize("M,N,K", [(1, 1, 64), (200, 16, 64), (4097, 8, 65), (1000, 41, 128), (777, 128, 602),
                                   (513, 256, 100), (300, 47, 256), (129, 130, 97), (128, 128, 4096),
                                   (257, 64, 95), (50, 7, 16)])
def test_gemm_bf16x3_all_ops(mg, dev, ref, M, N, K):
    """NN, NT, TN, TT on whole and ragged tiles, inner dimensions that are not multiples of the
    k-step, odd leading dimensions (scalar loads) and the short inner dimension that stays on the fp32 kernel"""
    say(f"[gemm bf16x3] {M}x{N}x{K}")
    A = wl.normal_f32(M + N, 21, (M, K))
    Bm = wl.normal_f32(M + K, 22, (K, N))
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    At, Bt = np.ascontiguousarray(A.T), np.ascontiguousarray(Bm.T)
    for name, opA, opB, a, b in (("NN", mg.OP_N, mg.OP_N, A, Bm), ("NT", mg.OP_N, mg.OP_T, A, Bt),
                                 ("TN", mg.OP_T, mg.OP_N, At, Bm), ("TT", mg.OP_T, mg.OP_T, At, Bt)):
        got = mg.mggcn_gemm_bf16x3(opA, opB, to_dev(a, dev), to_dev(b, dev)).cpu().numpy()
        assert_rows_close(got, want, tol=TIGHT, what=f"{name} {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", [(602, 128, 30001), (128, 41, 9999), (16, 8, 4097), (100, 256, 20000)])
def test_gemm_bf16x3_tn_split_k(mg, dev, ref, M, N, K):
    say(f"[gemm bf16x3 TN split-K] {M}x{N}x{K}")
    H = wl.normal_f32(K, 23, (K, M))
    T = wl.normal_f32(K, 24, (K, N))
    want = ref.gemm(ref.OP_T, ref.OP_N, H.astype(np.float64), T.astype(np.float64))
    a = mg.mggcn_gemm_bf16x3(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    # a row of this product is a sum of K signed terms that largely cancel: compare with the matrix's scale
    assert np.abs(a - want).max() <= 2e-6 * np.abs(want).max()
    b = mg.mggcn_gemm_bf16x3(mg.OP_T, mg.OP_N, to_dev(H, dev), to_dev(T, dev)).cpu().numpy()
    assert np.array_equal(a, b), "split-K reduction must be reproducible"


def test_gemm_bf16x3_is_not_a_bfloat16_product_and_has_no_drift(mg, dev, ref):
    """Operands with all 24 significand bits in use, all of one sign, long inner dimension: the
    running sum grows to 2^14 times a term, where an addend cut off instead of rounded, or a dropped
    piece, shows as a one-sided error.  Asserted: the mean signed error stays below 5e-7 (a single
    accumulator for all six piece products measured -2e-5 here, an operand rounded to bfloat16
    about 1e-3)."""
    K = 16384
    A = np.abs(wl.normal_f32(3, 25, (256, K))) + np.float32(1.0)
    Bm = np.abs(wl.normal_f32(3, 26, (K, 128))) + np.float32(1.0)
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    got = mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, to_dev(A, dev), to_dev(Bm, dev)).cpu().numpy().astype(np.float64)
    rel = (got - want) / want
    assert np.abs(rel).max() <= 4e-6
    assert abs(rel.mean()) <= 5e-7, rel.mean()


def test_gemm_bf16x3_pieces_are_exact(mg, dev, ref):
    """One non-zero per row of A, a number that needs all three pieces (1 + 2^-9 + 2^-18 has
    significand bits 0, 9 and 18) times a small integer, against powers of two: every entry of the
    product is a single exact fp32 number, so the result must equal the fp64 one bit for bit --
    and the same with the roles of A and B exchanged."""
    rng = np.random.default_rng(4)
    M, K, N = 130, 128, 70
    base = np.float32(1.0) + np.float32(2.0 ** -9) + np.float32(2.0 ** -18)
    A = np.zeros((M, K), dtype=np.float32)
    A[np.arange(M), np.arange(M) % K] = rng.choice([-3, -2, -1, 1, 2, 3], size=M).astype(np.float32) * base
    Bm = np.ldexp(np.ones((K, N), dtype=np.float32), rng.integers(-3, 4, size=(K, N))).astype(np.float32)
    want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
    assert np.array_equal(want.astype(np.float32).astype(np.float64), want), "case must be exact in fp32"
    got = mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, to_dev(A, dev), to_dev(Bm, dev)).cpu().numpy()
    assert np.array_equal(got.astype(np.float64), want)
    got = mg.mggcn_gemm_bf16x3(mg.OP_T, mg.OP_T, to_dev(Bm, dev), to_dev(A, dev)).cpu().numpy()  # (A Bm)^T = Bm^T A^T
    assert np.array_equal(got.astype(np.float64), want.T)


def test_gemm_bf16x3_epilogues_beta_and_strides(mg, dev, ref):
    M, N, K = 333, 41, 100
    A = wl.normal_f32(1, 27, (M, 112))      # ld 112 > K
    Bm = wl.normal_f32(1, 28, (K, N))       # ld 41: unaligned rows
    C0 = wl.normal_f32(1, 29, (M, 48))
    Ad, Bd = to_dev(A, dev), to_dev(Bm, dev)
    want = ref.gemm(ref.OP_N, ref.OP_N, A[:, :K].astype(np.float64), Bm.astype(np.float64))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, Cm=Cd[:, :N])
    C = Cd.cpu().numpy()
    assert_rows_close(C[:, :N], want, tol=TIGHT, what="strided")
    assert np.array_equal(C[:, N:], C0[:, N:]), "padding columns must not be written"
    plain = C[:, :N].copy()
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, beta=1.0, Cm=Cd[:, :N])
    assert_rows_close(Cd.cpu().numpy()[:, :N], want + C0[:, :N].astype(np.float64), tol=TIGHT, what="beta")
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, epilogue=mg.EPI_RELU, Cm=Cd[:, :N])
    assert np.array_equal(Cd.cpu().numpy()[:, :N], np.maximum(plain, 0))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, Ad[:, :K], Bd, epilogue=mg.EPI_RELU_MASK, Cm=Cd[:, :N])
    assert np.array_equal(Cd.cpu().numpy()[:, :N], np.where(C0[:, :N] > 0, plain, 0).astype(np.float32))


def test_gemm_bf16x3_degenerate_shapes(mg, dev):
    import torch

    assert mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, torch.ones((0, 70), device=dev), torch.ones((70, 7), device=dev)).shape == (0, 7)
    C0 = wl.normal_f32(9, 4, (37, 11))
    Cd = to_dev(C0, dev)
    mg.mggcn_gemm_bf16x3(mg.OP_N, mg.OP_N, torch.ones((37, 0), device=dev), torch.ones((0, 11), device=dev), beta=1.0,
                         epilogue=mg.EPI_RELU, Cm=Cd)
    assert np.array_equal(Cd.cpu().numpy(), np.maximum(C0, 0.0))
    L = mg.binding.lib()
    assert L.mggcn_gemm_bf16x3(5, 0, 1, 2, 3, None, 3, None, 2, 0.0, 0, None, 2, None, 0, None) == mg.binding.E_INVALID_ARG
    # rejected on the host, before anything is launched: the pointers are not real
    need = L.mggcn_gemm_workspace_bytes(1, 0, 602, 128, 232965)
    assert need > 0
    assert L.mggcn_gemm_bf16x3(1, 0, 602, 128, 232965, 256, 602, 256, 128, 0.0, 0, 256, 128, 256, need - 1,
                               None) == mg.binding.E_WORKSPACE


@pytest.mark.parametrize("cfg_name,dims,flags", [
    ("tiny", (64, 100, 32, 8), "x3"),
    ("small_powerlaw", (70, 128, 41), "x3"),
    ("small_powerlaw", (602, 128, 41), "x3+cache"),
])
def test_epoch_with_gemm_bf16x3(mg, dev, ref, cfg_name, dims, flags):
    """whole epochs with every GeMM on the bfloat16 matrix instructions: the same oracle, the same
    tolerance, the same order rule and buffer plan"""
    say(f"[epoch gemm bf16x3] {cfg_name} dims={dims} {flags}")
    g = wl.CONFIGS["tiny"].graph() if cfg_name == "tiny" else wl.chung_lu(5000, 300e3, 2.1, 2500.0, 8)
    n = g.n_rows
    rp, ci, val, X, Ws, labels = _model_inputs(ref, g, dims, 17)
    L = len(dims) - 1
    f = mg.MODEL_GEMM_BF16X3 | (mg.MODEL_CACHE_INPUT if "cache" in flags else 0)
    G = mg.Graph(n, n, to_dev(rp, dev), to_dev(ci, dev), to_dev(val, dev), F_max=max(dims))
    model = mg.Model(G, dims, flags=f)
    Xd, Wd, ld = to_dev(X, dev), [to_dev(w, dev) for w in Ws], to_dev(labels, dev)
    if "cache" in flags:
        model.cache_input(Xd)
    loss, WG = mg.mggcn_epoch(model, Xd, ld, Wd)
    loss2, WG2 = mg.mggcn_epoch(model, Xd, ld, Wd)
    masks = gpu_relu_decisions(mg, model, Xd, Wd)
    r_ords = [ref.SPMM_FIRST if model.order(l) == mg.ORDER_SPMM_FIRST else ref.GEMM_FIRST for l in range(L)]
    assert_relu_decisions_agree(masks, oracle_preactivations(ref, n, rp, ci, val.astype(np.float64), X.astype(np.float64),
                                                             [w.astype(np.float64) for w in Ws], r_ords), "gemm bf16x3")
    rl, rWG, _ = ref.epoch(n, rp, ci, val.astype(np.float64), X.astype(np.float64), labels,
                           [w.astype(np.float64) for w in Ws], orders=r_ords, relu_masks=masks)
    assert abs(loss.item() - rl) <= 1e-5 * abs(rl)
    assert loss.item() == loss2.item()
    for l in range(L):
        a = WG[l].cpu().numpy()
        assert np.array_equal(a, WG2[l].cpu().numpy()), "epoch must be reproducible bit for bit"
        assert_rows_close(a, rWG[l], what=f"W_G[{l}]")


def test_gemm_random_cases_both_entry_points(mg, dev, ref):
    """Seeded random shapes, op combinations, leading dimensions and base-pointer offsets (4-, 8- and
    16-byte aligned operands take different loaders), β and epilogues, through mggcn_gemm and
    mggcn_gemm_bf16x3 alike."""
    import torch

    rng = np.random.default_rng(2024)

    def view(a, ld, off):
        r, c = a.shape
        buf = torch.zeros(off + max(r, 1) * ld + 8, dtype=torch.float32, device=dev)
        v = buf[off: off + r * ld].view(r, ld)[:, :c]
        v.copy_(to_dev(a, dev))
        return v

    for case in range(48):
        M = int(rng.choice([1, 5, 63, 64, 127, 128, 129, 300, 1000]))
        N = int(rng.choice([1, 7, 16, 41, 47, 64, 65, 100, 128, 130, 256]))
        K = int(rng.choice([1, 15, 16, 63, 64, 65, 96, 100, 128, 257, 602, 5000]))
        opA, opB = int(rng.integers(0, 2)), int(rng.integers(0, 2))
        A = wl.normal_f32(case, 61, (M, K))
        Bm = wl.normal_f32(case, 62, (K, N))
        a = A if opA == 0 else np.ascontiguousarray(A.T)
        b = Bm if opB == 0 else np.ascontiguousarray(Bm.T)
        lda = a.shape[1] + int(rng.choice([0, 1, 2, 3, 4, 6]))
        ldb = b.shape[1] + int(rng.choice([0, 1, 2, 4]))
        ldc = N + int(rng.choice([0, 1, 3]))
        offs = [int(rng.choice([0, 1, 2, 4])) for _ in range(3)]
        beta = float(rng.integers(0, 2))
        epi = int(rng.choice([mg.EPI_NONE, mg.EPI_RELU, mg.EPI_RELU_MASK])) if beta == 0 else int(rng.choice([mg.EPI_NONE, mg.EPI_RELU]))
        C0 = wl.normal_f32(case, 63, (M, N))
        want = ref.gemm(ref.OP_N, ref.OP_N, A.astype(np.float64), Bm.astype(np.float64))
        if beta:
            want = want + C0
        if epi == mg.EPI_RELU:
            want = np.maximum(want, 0)
        if epi == mg.EPI_RELU_MASK:
            want = np.where(C0 > 0, want, 0)
        for name, fn in (("fp32", mg.mggcn_gemm), ("bf16x3", mg.mggcn_gemm_bf16x3)):
            say(f"[gemm random {case} {name}] {M}x{N}x{K} op=({opA},{opB}) ld=({lda},{ldb},{ldc}) off={offs} beta={beta} epi={epi}")
            Cd = view(C0, ldc, offs[2])
            fn(opA, opB, view(a, lda, offs[0]), view(b, ldb, offs[1]), beta=beta, epilogue=epi, Cm=Cd)
            got = Cd.cpu().numpy().astype(np.float64)
            # forward error bound of a dot product: a small multiple of the unit roundoff times |A||B|
            bound = 2e-5 * (np.abs(A).astype(np.float64) @ np.abs(Bm).astype(np.float64) + beta * np.abs(C0)) + 1e-30
            assert np.all(np.abs(got - want) <= bound), (name, case, float(np.abs(got - want).max()))
