#!/usr/bin/env python3
"""Benchmark of the GCN hot path on one MI355X.

Default workload: the largest single-GPU configuration, one GPU's 1/8 row block of a Papers-shaped
graph (13.9 M x 111 M, ~200 M entries, X 111 M x 128 = 56.8 GB resident in HBM) -- the regime in which
the paper finds the SpMM to take 60-94 % of the time.  A step is the 128 -> 256 layer forward and
backward in SpMM-first order, the five calls mggcn_layer_fwd / mggcn_layer_bwd make:
P = A^ X, H = relu(P W), W_G = P^T G, U = G W^T, X_G = A^^T U.  `--config medium|large|...` times a whole
epoch (forward, softmax-CE, backward) of a square configuration instead; with the default workload
the medium and large epochs are also run briefly and reported under `other_configs`.

All inputs are seeded, synthetic and resident in HBM before the timed region.  Prints ONE JSON line.

Byte accounting of an SpMM with nnz entries, n_r output rows, F columns (fp32, int32):
  no-reuse (`B_eff`)  8 nnz + 4 (n_r + 1) + 4F nnz + 4F n_r   every gathered row counted as memory traffic
  compulsory (`B_min`) 8 nnz + 4 (n_r + 1) + 4F touched + 4F n_r   every touched row of X fetched once
  measured             L2 <-> fabric bytes from rocprofv3 counters (FETCH_SIZE, WRITE_SIZE), profile named
`value` and `roofline.achieved` use the measured bytes (they cannot exceed what the memory system moved);
the other two are printed beside them under explicit names.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
FP32_MFMA_PEAK_TFLOPS = 157.3

# L2 <-> fabric bytes per call of the SpMM launches named, measured with rocprofv3 --pmc FETCH_SIZE and
# --pmc WRITE_SIZE on this build and configuration (`bench.py --config C --profile-spmm N`), scaled by
# what the same counters read for a 1 GiB copy; each entry names the summary it comes from.  These
# counters sit between L2 and the fabric: fills served by the 256 MB Infinity Cache are included, so
# the figure is an upper bound of the HBM traffic.
MEASURED_TRAFFIC = {
    "block": {"profile": "profiles/spmm_block_F128_pmc.md", "spmm_fwd": 97_286_051_699, "spmm_bwd": 164_695_447_106},
    "large": {"profile": "profiles/spmm_large_pmc.md", "spmm_fwd_F256": 129_270_000_000, "spmm_fwd_F100": 63_700_000_000,
              "spmm_fwd_F47": 31_500_000_000},
    "medium": {"profile": "profiles/spmm_medium_F128_pmc.md", "spmm_fwd_F128": 17_018_680_064},
}

NOMINAL_NNZ = {"tiny": 65_536 + 4096, "medium": 114_600_000 + 232_965, "large": 123_700_000 + 2_449_029,
               "block": 200_000_000, "rmat": 64_000_000 + (1 << 22), "proteins": 1_300_000_000 + 8_740_000}


def log(msg: str) -> None:
    """progress lines on stderr (stdout carries the one JSON line)"""
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


def spmm_bytes(nnz: int, n_rows: int, F: int) -> int:
    """no-reuse algorithmic bytes of one SpMM"""
    return 8 * nnz + 4 * (n_rows + 1) + 4 * F * nnz + 4 * F * n_rows


def spmm_bytes_min(nnz: int, n_rows: int, touched_cols: int, F: int) -> int:
    """compulsory bytes of one SpMM: every touched row of the dense operand fetched exactly once"""
    return 8 * nnz + 4 * (n_rows + 1) + 4 * F * touched_cols + 4 * F * n_rows


def stats(ts):
    ts = sorted(ts)
    k = len(ts)
    med = ts[k // 2] if k % 2 else 0.5 * (ts[k // 2 - 1] + ts[k // 2])
    return {"mean": sum(ts) / k, "median": med, "min": ts[0]}


def timed(torch, fn, reps, warm=2):
    """HIP events on the launch stream (the binding launches on torch's current stream) around each call"""
    for _ in range(warm):
        fn()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    for a, b in evs:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return stats([a.elapsed_time(b) for a, b in evs])


def r4(st):
    return {k: round(v, 4) for k, v in st.items()}


def sha256_arrays(*arrays) -> str:
    h = hashlib.sha256()
    for a in arrays:
        h.update(memoryview(a).cast("B"))
    return h.hexdigest()


def calibrate(mg, torch, dev, gib=8, reps=5):
    """What this machine delivers for the access patterns of the SpMM, measured in this run: a plain device
    copy, a read-only and a write-only stream, and random row gathers (512-byte and 1-KiB rows, uniform over a buffer
    no cache holds)."""
    n = gib << 28  # floats
    buf = torch.empty(n, dtype=torch.float32, device=dev).fill_(1.0)
    out = {"buffer_GiB": gib}
    half = n // 2
    ms = timed(torch, lambda: buf[:half].copy_(buf[half:]), reps)["min"]
    out["device_copy_GBps"] = round(2.0 * half * 4 / (ms * 1e-3) / 1e9, 1)
    ms = timed(torch, lambda: mg.mggcn_probe_read(buf), reps)["min"]
    out["read_stream_GBps"] = round(n * 4 / (ms * 1e-3) / 1e9, 1)
    ms = timed(torch, lambda: mg.mggcn_probe_write(buf, 1.0), reps)["min"]
    out["write_stream_GBps"] = round(n * 4 / (ms * 1e-3) / 1e9, 1)
    gen = torch.Generator(device=dev).manual_seed(12345)
    for row_bytes in (512, 1024):
        X = buf.view(-1, row_bytes // 4)
        n_idx = (16 << 30) // row_bytes  # 16 GiB gathered
        idx = torch.randint(0, X.shape[0], (n_idx,), device=dev, dtype=torch.int32, generator=gen)
        ms = timed(torch, lambda: mg.mggcn_probe_gather(X, idx), reps)["min"]
        out[f"random_gather_{row_bytes}B_GBps"] = round(n_idx * row_bytes / (ms * 1e-3) / 1e9, 1)
        del idx
    # the same gather over 128 MiB: beyond the 8 x 4 MB of L2, inside the 256 MB Infinity Cache -- what L2 misses
    # cost when the fabric-side cache serves them (the traffic counters cannot tell these from HBM reads)
    small = buf[: 128 << 18].view(-1, 128)
    idx = torch.randint(0, small.shape[0], ((8 << 30) // 512,), device=dev, dtype=torch.int32, generator=gen)
    ms = timed(torch, lambda: mg.mggcn_probe_gather(small, idx), reps)["min"]
    out["random_gather_512B_over_128MiB_GBps"] = round(idx.numel() * 512 / (ms * 1e-3) / 1e9, 1)
    del idx, small
    # the fp32 matrix instruction on register operands: what the matrix pipes sustain with nothing else going on
    sink = torch.empty(4096, dtype=torch.float32, device=dev)
    flop = mg.mggcn_probe_mfma(20000, sink)
    ms = timed(torch, lambda: mg.mggcn_probe_mfma(20000, sink), 3, warm=1)["min"]
    out["mfma_f32_registers_only_TFLOPs"] = round(flop / (ms * 1e-3) / 1e12, 1)
    # the library's own GeMM on N(0,1) and on all-zero operands: the same instruction stream, and the chip runs it
    # faster when the data do not switch (it lowers its clock under the load of LDS, load path and matrix pipes)
    M, N, K = 2_449_029, 256, 256
    A, B, C = buf[: M * K].view(M, K), buf[M * K: M * K + K * N].view(K, N), buf[n // 2: n // 2 + M * N].view(M, N)
    for name, fill in (("normal", lambda t: t.normal_(generator=gen)), ("zero", lambda t: t.zero_())):
        fill(A), fill(B)
        ms = timed(torch, lambda: mg.mggcn_gemm(mg.OP_N, mg.OP_N, A, B, Cm=C), reps)["median"]
        out[f"gemm_f32_{M}x{N}x{K}_{name}_operands_TFLOPs"] = round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1)
        if name == "normal":  # for scale: the vendor library's fp32 product behind torch.matmul, same operands
            ms = timed(torch, lambda: torch.matmul(A, B, out=C), reps)["median"]
            out[f"vendor_matmul_f32_{M}x{N}x{K}_TFLOPs"] = round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1)
    log(f"calibration {out}")
    del buf, A, B, C
    torch.cuda.empty_cache()
    return out


def roofline_object(kernel, ms, bytes_measured, bytes_eff, bytes_min, flops, calib, profile, launches=1):
    """`achieved` from measured traffic where a profile of this configuration exists, else from the
    compulsory bytes; either way a figure the memory system really had to move, never above the peak
    by construction of the byte count."""
    by = bytes_measured if bytes_measured else bytes_min
    ach = by / (ms * 1e-3) / 1e9
    t_min_ms = max(bytes_min / (HBM_PEAK_GBPS * 1e9), flops / (FP32_MFMA_PEAK_TFLOPS * 1e12)) * 1e3
    o = {
        "kernel": kernel, "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": round(ach / HBM_PEAK_GBPS, 4),
        "traffic": bytes_measured, "traffic_profile": profile,
        "bytes_used_for_achieved": "measured L2<->fabric traffic (FETCH_SIZE + WRITE_SIZE, calibrated)" if bytes_measured
                                   else "compulsory bytes (no measured traffic for this configuration)",
        "launches_per_call": launches, "avg_launch_ms": round(ms / launches, 4),
        "compulsory_bytes": bytes_min, "compulsory_GBps": round(bytes_min / (ms * 1e-3) / 1e9, 1),
        "frac_by_compulsory_bytes": round(bytes_min / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "no_reuse_bytes": bytes_eff, "no_reuse_GBps": round(bytes_eff / (ms * 1e-3) / 1e9, 1),
        "gflops": round(flops / (ms * 1e-3) / 1e9, 1), "t_min_ms": round(t_min_ms, 4), "t_min_over_t": round(t_min_ms / ms, 4),
    }
    if calib:
        o["achieved_over_read_stream"] = round(ach / calib["read_stream_GBps"], 4)
        o["no_reuse_over_random_gather_512B"] = round(o["no_reuse_GBps"] / calib["random_gather_512B_GBps"], 4)
    return o


# ------------------------------------------------------------------------------------------------
# the row block: one layer forward + backward
# ------------------------------------------------------------------------------------------------

def run_block(args, cfg, mg, wl, torch, dev, calib):
    import numpy as np

    t0 = time.time()
    g = cfg.graph()
    nr, nc = g.n_rows, g.n_cols
    col_count = np.bincount(g.colidx, minlength=nc)
    deg_row = (np.diff(g.rowptr) + 1).astype(np.int32)          # stand-in global degrees
    deg_col = (1 + 8 * col_count).astype(np.int32)
    gen_s = time.time() - t0
    log(f"block: generated {nr} x {nc}, {g.nnz} entries in {gen_s:.1f}s")
    setup = {}
    torch.cuda.synchronize()
    t0 = time.time()
    rowptr, colidx, val = mg.mggcn_csr_normalize(nr, nc, torch.from_numpy(g.rowptr).to(dev), torch.from_numpy(g.colidx).to(dev),
                                                 deg_row=torch.from_numpy(deg_row).to(dev), deg_col=torch.from_numpy(deg_col).to(dev))
    torch.cuda.synchronize()
    setup["normalize_s"] = round(time.time() - t0, 3)
    nnz = int(colidx.numel())
    t0 = time.time()
    t = mg.mggcn_csr_transpose(nr, nc, rowptr, colidx, val)
    torch.cuda.synchronize()
    setup["transpose_s"] = round(time.time() - t0, 3)
    d_in, d_out = cfg.dims
    t0 = time.time()
    graph = mg.Graph(nr, nc, rowptr, colidx, val, transpose=t, F_max=d_in, seg_len=args.seg_len)
    torch.cuda.synchronize()
    setup["task_tables_s"] = round(time.time() - t0, 3)
    # touched rows of the dense operand: columns of the block with at least one entry (the diagonal included)
    touched_fwd = nr + int(np.count_nonzero(col_count[nr:] > 0))  # columns below nr hold a diagonal entry
    touched_bwd = nr  # every row of the block holds its diagonal entry
    sha = sha256_arrays(rowptr.cpu().numpy(), colidx.cpu().numpy(), val.cpu().numpy())
    log(f"block: setup {setup}, nnz {nnz}")

    gen = torch.Generator(device=dev).manual_seed(cfg.seed + 0x100)
    X = torch.randn((nc, d_in), device=dev, generator=gen)
    W = torch.from_numpy(cfg.weights()[0]).to(dev)
    G = torch.randn((nr, d_out), device=dev, generator=gen)
    P = torch.empty((nr, d_in), device=dev)
    H = torch.empty((nr, d_out), device=dev)
    U = torch.empty((nr, d_in), device=dev)
    XG = torch.empty((nc, d_in), device=dev)
    WG = torch.empty_like(W)
    ws = mg.gemm_workspace(mg.OP_T, mg.OP_N, d_in, d_out, nr, dev)

    calls = {
        f"spmm_fwd_F{d_in}": lambda: mg.mggcn_spmm(graph, mg.OP_N, X, Y=P),
        f"gemm_fwd_{d_in}x{d_out}": lambda: mg.mggcn_gemm(mg.OP_N, mg.OP_N, P, W, epilogue=mg.EPI_RELU, Cm=H),
        "gemm_wgrad": lambda: mg.mggcn_gemm(mg.OP_T, mg.OP_N, P, G, Cm=WG, ws=ws),
        "gemm_hgrad": lambda: mg.mggcn_gemm(mg.OP_N, mg.OP_T, G, W, Cm=U),
        f"spmm_bwd_F{d_in}": lambda: mg.mggcn_spmm(graph, mg.OP_T, U, Y=XG),
    }

    def step():
        for fn in calls.values():
            fn()

    if args.profile_spmm > 0:
        step()
        for _ in range(args.profile_spmm):
            calls[f"spmm_fwd_F{d_in}"]()
        for _ in range(args.profile_spmm):
            calls[f"spmm_bwd_F{d_in}"]()
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)  # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a)  # reads 1 GiB, writes 1 GiB: the calibration of the counters
        torch.cuda.synchronize()
        return {"mode": "profile-spmm", "config": "block", "calls": args.profile_spmm, "F": d_in, "nnz": nnz,
                "no_reuse_bytes_fwd": spmm_bytes(nnz, nr, d_in), "no_reuse_bytes_bwd": spmm_bytes(nnz, nc, d_in),
                "copy_bytes_each_way": 4 << 28}

    if args.profile_gemm > 0:
        step()
        if args.zero_operands:  # the same launches on data that do not switch
            for t_ in (P, W, G):
                t_.zero_()
        for k in (f"gemm_fwd_{d_in}x{d_out}", "gemm_wgrad", "gemm_hgrad"):
            for _ in range(args.profile_gemm):
                calls[k]()
        torch.cuda.synchronize()
        return {"mode": "profile-gemm", "config": "block", "calls": args.profile_gemm, "M": nr, "d_in": d_in, "d_out": d_out,
                "operands": "zero" if args.zero_operands else "as in a step", "flop_per_call": 2 * nr * d_in * d_out}

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    step_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    log(f"block: {args.steps} steps, {step_ms:.3f} ms per step")

    reps = max(5, args.steps)
    ops = {k: timed(torch, fn, reps) for k, fn in calls.items()}
    log(f"block: per-call medians {({k: round(v['median'], 3) for k, v in ops.items()})}")
    fwd_ms, bwd_ms = ops[f"spmm_fwd_F{d_in}"]["median"], ops[f"spmm_bwd_F{d_in}"]["median"]
    gemm_ms = sum(v["median"] for k, v in ops.items() if k.startswith("gemm"))
    eff_f, eff_b = spmm_bytes(nnz, nr, d_in), spmm_bytes(nnz, nc, d_in)
    min_f, min_b = spmm_bytes_min(nnz, nr, touched_fwd, d_in), spmm_bytes_min(nnz, nc, touched_bwd, d_in)
    mt = MEASURED_TRAFFIC["block"]
    tr_f, tr_b = mt["spmm_fwd"], mt["spmm_bwd"]
    by_f, by_b = (tr_f or min_f), (tr_b or min_b)
    value = (by_f + by_b) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9
    flops = 2.0 * nnz * d_in
    lanes = min(64, 1 << max(0, (d_in + 3) // 4 - 1).bit_length())
    roof = roofline_object(f"spmm_tasks<float,VW=4,LPR={lanes},U=4>: forward product A^ X at F={d_in}, one launch per call",
                           fwd_ms, tr_f, eff_f, min_f, flops, calib, mt["profile"], graph.panels(d_in))
    roof_b = roofline_object(f"spmm_tasks<float,VW=4,LPR={lanes},U=4> + spmm_zero_rows<4>: transposed product A^^T U at F={d_in} ({nc} output rows: "
                             f"the gather launch over the rows that hold entries, the fill launch over the others, the small fix-up launch)",
                             bwd_ms, tr_b, eff_b, min_b, flops, calib, mt["profile"], graph.panels(d_in, mg.OP_T))

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline_block(np, torch, dev, rowptr, colidx, val, X, nr, nc, nnz, d_in)
        log(f"block: cpu baseline {cpu['value']} GB/s")

    out = {
        "metric": "spmm_hbm_bandwidth", "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(step_ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"block: one GPU's 1/8 row block of a Papers-shaped graph, {nr} x {nc}, nnz={nnz} realised with "
                               f"the diagonal ({NOMINAL_NNZ['block']} nominal), X {nc} x {d_in} fp32 in HBM, layer {d_in}->{d_out} "
                               f"forward + backward (SpMM first): A^X, relu(PW), P^T G, G W^T, A^^T U",
                   "nnz_realised": nnz, "nnz_nominal": NOMINAL_NNZ["block"], "csr_sha256": sha,
                   "touched_columns": touched_fwd},
        "value_is": "bytes moved between L2 and the fabric by the two SpMM launches of a step (measured; compulsory bytes "
                    "where no measurement exists) / their time",
        "spmm_pct_hbm_roofline": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "spmm_no_reuse_GBps": round((eff_f + eff_b) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9, 1),
        "spmm_compulsory_GBps": round((min_f + min_b) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9, 1),
        "spmm_gflops": round(2 * flops / ((fwd_ms + bwd_ms) * 1e-3) / 1e9, 1),
        "spmm_share_of_step": round((fwd_ms + bwd_ms) / sum(v["median"] for v in ops.values()), 4),
        "gemm_tflops": round(3 * 2.0 * nr * d_in * d_out / (gemm_ms * 1e-3) / 1e12, 2),
        "gemm_mfma_utilisation": round(3 * 2.0 * nr * d_in * d_out / (gemm_ms * 1e-3) / 1e12 / FP32_MFMA_PEAK_TFLOPS, 4),
        "ops_ms": {k: r4(v) for k, v in ops.items()},
        # Under the paper's 1-D row distribution (broadcast stages, Section "partitioning") a GPU's backward product is
        # its row block of A^^T times the whole gradient matrix: the same launch shape as the forward product (for the
        # symmetric A^ the same block).  The transposed product timed here, over all 111 M columns of the block, is what
        # the reduction-based alternative needs and the more expensive of the two.
        "step_ms_with_a_forward_shaped_backward_product": round(2 * fwd_ms + gemm_ms, 4),
        "generate_s": round(gen_s, 3), "setup_s": setup,
        "box_calibration": calib,
        "roofline": roof, "roofline_transposed_launch": roof_b, "cpu_baseline": cpu,
    }
    return out


def cpu_baseline_block(np, torch, dev, rowptr, colidx, val, X, nr, nc, nnz, F):
    """The oracle's SpMM on a bounded sample of the block: its first rows (vertices are relabelled at
    random, so a prefix is a fair sample) with the columns renumbered to the ones they touch, so that
    the fp64 operand fits the host; N and T form, median of three."""
    from oracle import ref

    rp = rowptr.cpu().numpy()
    R = int(np.searchsorted(rp, nnz // 8))  # about an eighth of the entries
    rp_s = rp[: R + 1].astype(np.int32)
    n_s = int(rp_s[-1])
    ci_s = colidx[:n_s].cpu().numpy()
    cols, inv = np.unique(ci_s, return_inverse=True)
    v_s = val[:n_s].cpu().numpy().astype(np.float64)
    Xs = X[torch.from_numpy(cols.astype(np.int64)).to(dev)].cpu().numpy().astype(np.float64)
    Gs = np.ascontiguousarray(Xs[: R] if len(cols) >= R else np.resize(Xs, (R, F)))
    inv = inv.astype(np.int32)
    tn, tt = [], []
    for _ in range(3):
        t0 = time.perf_counter()
        ref.spmm(ref.OP_N, R, len(cols), rp_s, inv, v_s, Xs)
        tn.append(time.perf_counter() - t0)
        t0 = time.perf_counter()
        ref.spmm(ref.OP_T, R, len(cols), rp_s, inv, v_s, Gs)
        tt.append(time.perf_counter() - t0)
    sn, st = stats(tn)["median"], stats(tt)["median"]
    b = spmm_bytes(n_s, R, F) + spmm_bytes(n_s, len(cols), F)
    return {
        "value": round(b / (sn + st) / 1e9, 3), "unit": "GB/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)),
        "kind": "oracle",
        "sample": f"fp64 oracle SpMM, N and T form, on the first {R} rows of the block ({n_s} entries, {len(cols)} touched "
                  f"columns renumbered, F={F}); median of 3; bytes by the no-reuse count (compare spmm_no_reuse_GBps)",
        "seconds_N": round(sn, 3), "seconds_T": round(st, 3),
        "ns_per_nnz_N": round(sn / n_s * 1e9, 3), "ns_per_nnz_T": round(st / n_s * 1e9, 3),
    }


# ------------------------------------------------------------------------------------------------
# square configurations: one whole epoch
# ------------------------------------------------------------------------------------------------

def run_epoch_config(args, name, cfg, mg, wl, torch, dev, calib, brief=False):
    import numpy as np

    dims = cfg.dims
    L = len(dims) - 1
    steps, warmup = (min(args.steps, 5), min(args.warmup, 2)) if brief else (args.steps, args.warmup)
    t0 = time.time()
    g = cfg.graph()
    n = g.n_rows
    # X is stored with its rows padded to a multiple of 16 floats (602 -> 608): the layout any
    # caller should pick, it keeps every row 64-byte aligned for the 16-byte load paths
    d0p = (dims[0] + 15) // 16 * 16
    Xbuf = torch.zeros((n, d0p), dtype=torch.float32, device=dev)
    Xbuf[:, :dims[0]] = torch.from_numpy(cfg.features(n)).to(dev)
    X = Xbuf[:, :dims[0]]
    Ws = [torch.from_numpy(w).to(dev) for w in cfg.weights()]
    labels = torch.from_numpy(cfg.labels(n)).to(dev)
    gen_s = time.time() - t0
    log(f"{name}: generated n={n}, {g.nnz} entries in {gen_s:.1f}s")

    setup = {}
    torch.cuda.synchronize()
    t0 = time.time()
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev), torch.from_numpy(g.colidx).to(dev))
    torch.cuda.synchronize()
    setup["normalize_s"] = round(time.time() - t0, 3)
    nnz = int(colidx.numel())
    t0 = time.time()
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=max(dims), seg_len=args.seg_len)
    torch.cuda.synchronize()
    setup["task_tables_s"] = round(time.time() - t0, 3)
    model = mg.Model(graph, dims)
    sha = sha256_arrays(rowptr.cpu().numpy(), colidx.cpu().numpy(), val.cpu().numpy())

    if args.profile_spmm > 0 and not brief:
        F = args.profile_width or max(dims[l] if model.order(l) == mg.ORDER_SPMM_FIRST else dims[l + 1] for l in range(L))
        ld = (F + 15) // 16 * 16
        src = torch.randn((n, ld), device=dev)[:, :F]
        dst = torch.empty((n, ld), device=dev)[:, :F]
        for _ in range(args.profile_spmm):
            mg.mggcn_spmm(graph, mg.OP_N, src, epilogue=mg.EPI_RELU, Y=dst)
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)  # 1 GiB
        b = torch.empty_like(a)
        b.copy_(a)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        return {"mode": "profile-spmm", "config": name, "calls": args.profile_spmm, "F": F, "n": n, "nnz": nnz,
                "passes": graph.panels(F), "no_reuse_bytes_per_call": spmm_bytes(nnz, n, F), "copy_bytes_each_way": 4 << 28}

    if args.profile_gemm > 0 and not brief:
        out = torch.empty((n, (dims[1] + 15) // 16 * 16), device=dev)[:, :dims[1]]
        wg = torch.empty_like(Ws[0])
        ws = mg.gemm_workspace(mg.OP_T, mg.OP_N, dims[0], dims[1], n, dev)
        for _ in range(args.profile_gemm):
            mg.mggcn_gemm(mg.OP_N, mg.OP_N, X, Ws[0], Cm=out)
        for _ in range(args.profile_gemm):  # the same layer's weight gradient: inner dimension = vertex count, split
            mg.mggcn_gemm(mg.OP_T, mg.OP_N, X, out, Cm=wg, ws=ws)
        torch.cuda.synchronize()
        return {"mode": "profile-gemm", "config": name, "calls": args.profile_gemm, "M": n, "N": dims[1], "K": dims[0],
                "lda": int(X.stride(0)), "flop_per_call": 2 * n * dims[0] * dims[1]}

    WG = [torch.empty_like(w) for w in Ws]
    loss = torch.empty(1, dtype=torch.float32, device=dev)

    def epoch_ms_of(m, Xarg):
        for _ in range(warmup):
            mg.mggcn_epoch(m, Xarg, labels, Ws, W_Gs=WG, loss=loss)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            mg.mggcn_epoch(m, Xarg, labels, Ws, W_Gs=WG, loss=loss)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps, float(loss.item())

    epoch_ms, loss_value = epoch_ms_of(model, X)
    log(f"{name}: setup {setup}; epoch {epoch_ms:.3f} ms, loss {loss_value:.6f}")

    # ---- the same epoch with A^ X formed once outside it (X is constant across epochs)
    model_c = mg.Model(graph, dims, flags=mg.MODEL_CACHE_INPUT)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    model_c.cache_input(X)
    torch.cuda.synchronize()
    cache_fill_ms = (time.perf_counter() - t0) * 1e3
    epoch_cached_ms, _ = epoch_ms_of(model_c, None)
    del model_c

    # ---- extensions beyond the paper's fp32 (reported beside the fp32 figures, never in their place)
    ext = {}
    if not brief:
        for key, flags in (("bf16_gather", mg.MODEL_GATHER_BF16), ("gemm_bf16x3", mg.MODEL_GEMM_BF16X3),
                           ("gemm_bf16x3+bf16_gather", mg.MODEL_GEMM_BF16X3 | mg.MODEL_GATHER_BF16)):
            model_x = mg.Model(graph, dims, flags=flags)
            ms, lv = epoch_ms_of(model_x, X)
            ext[key] = {"epoch_ms": round(ms, 4), "loss": lv}
            del model_x

    # ---- per-operation timing with HIP events on the launch stream: the same calls an epoch makes
    reps = max(5, steps)
    ops = {}
    spmm_widths = []
    for l in range(L):
        order = model.order(l)
        F = dims[l] if order == mg.ORDER_SPMM_FIRST else dims[l + 1]
        spmm_widths.append(F)
        ld = (F + 15) // 16 * 16
        src = torch.randn((n, ld), device=dev)
        dst = torch.empty((n, ld), device=dev)
        epi = mg.EPI_RELU if (l + 1 < L and order == mg.ORDER_GEMM_FIRST) else mg.EPI_NONE
        ops[f"spmm_fwd_l{l}_F{F}"] = timed(torch, lambda: mg.mggcn_spmm(graph, mg.OP_N, src[:, :F], epilogue=epi, Y=dst[:, :F]), reps)
        # backward: the ReLU' mask of the layer below rides on whichever product writes H_G (in place over the activation)
        bepi = mg.EPI_RELU_MASK if (l > 0 and order == mg.ORDER_SPMM_FIRST) else mg.EPI_NONE
        if l > 0 or order == mg.ORDER_GEMM_FIRST:
            ops[f"spmm_bwd_l{l}_F{F}"] = timed(torch, lambda: mg.mggcn_spmm(graph, mg.OP_T, src[:, :F], epilogue=bepi, Y=dst[:, :F]), reps)
        H = X if l == 0 else torch.randn((n, (dims[l] + 15) // 16 * 16), device=dev)[:, :dims[l]]
        out = torch.empty((n, (dims[l + 1] + 15) // 16 * 16), device=dev)[:, :dims[l + 1]]
        wg = torch.empty_like(Ws[l])
        hg = torch.randn((n, (dims[l] + 15) // 16 * 16), device=dev)[:, :dims[l]] if l > 0 else None
        ws = mg.gemm_workspace(mg.OP_T, mg.OP_N, dims[l], dims[l + 1], n, dev)
        fepi = mg.EPI_RELU if (l + 1 < L and order == mg.ORDER_SPMM_FIRST) else mg.EPI_NONE
        ops[f"gemm_fwd_l{l}_{dims[l]}x{dims[l + 1]}"] = timed(torch, lambda: mg.mggcn_gemm(mg.OP_N, mg.OP_N, H, Ws[l], epilogue=fepi, Cm=out), reps)
        ops[f"gemm_wgrad_l{l}"] = timed(torch, lambda: mg.mggcn_gemm(mg.OP_T, mg.OP_N, H, out, Cm=wg, ws=ws), reps)
        if l > 0:
            hepi = mg.EPI_RELU_MASK if order == mg.ORDER_GEMM_FIRST else mg.EPI_NONE
            ops[f"gemm_hgrad_l{l}"] = timed(torch, lambda: mg.mggcn_gemm(mg.OP_N, mg.OP_T, out, Ws[l], epilogue=hepi, Cm=hg), reps)
        del src, dst
    logits = torch.randn((n, (dims[L] + 15) // 16 * 16), device=dev)[:, :dims[L]]
    ops["softmax_ce"] = timed(torch, lambda: mg.mggcn_softmax_ce(logits, labels), reps)

    touched = n  # every vertex has its self-loop: every row of the operand is touched
    spmm_keys = [k for k in ops if k.startswith("spmm")]
    spmm_ms = sum(ops[k]["median"] for k in spmm_keys)
    width_of = lambda k: int(k.rsplit("F", 1)[1])
    spmm_eff = sum(spmm_bytes(nnz, n, width_of(k)) for k in spmm_keys)
    spmm_min = sum(spmm_bytes_min(nnz, n, touched, width_of(k)) for k in spmm_keys)
    mt = MEASURED_TRAFFIC.get(name, {})
    spmm_meas = [mt.get(f"spmm_fwd_F{width_of(k)}") for k in spmm_keys]  # T on a symmetric operator = the same launches
    spmm_by = sum(spmm_meas) if all(spmm_meas) else spmm_min
    gemm_ms = sum(v["median"] for k, v in ops.items() if k.startswith("gemm"))
    gemm_flops = sum(2.0 * n * dims[l] * dims[l + 1] * (2 if l == 0 else 3) for l in range(L))
    gemm_tflops = gemm_flops / (gemm_ms * 1e-3) / 1e12

    # dominant kernel: the widest SpMM of the epoch
    Fdom = max(spmm_widths)
    ldom = spmm_widths.index(Fdom)
    dom_ms = ops[f"spmm_fwd_l{ldom}_F{Fdom}"]["median"]
    P = graph.panels(Fdom)
    lanes = min(64, 1 << max(0, (Fdom + 3) // 4 - 1).bit_length())
    roofline = roofline_object(
        f"spmm_tasks<float,VW=4,LPR={lanes},U=4>: one mggcn_spmm call at F={Fdom} = {P} launches of it, one per pass over the "
        f"entries (column panels x feature slices; + the small row fix-up launches)",
        dom_ms, mt.get(f"spmm_fwd_F{Fdom}"), spmm_bytes(nnz, n, Fdom), spmm_bytes_min(nnz, n, touched, Fdom), 2.0 * nnz * Fdom,
        calib, mt.get("profile"), P)

    log(f"{name}: per-call timings done; oracle baseline next")
    cpu = None
    if not args.no_cpu_baseline and not brief:
        cpu = cpu_baseline_epoch(args, name, np, wl, X, rowptr, colidx, val, n, nnz, spmm_keys, cfg, labels, Ws)
    elif not args.no_cpu_baseline and brief and name in args.oracle_epoch.split(","):
        cpu = {"oracle_epoch_s": oracle_epoch_seconds(np, cfg, n, rowptr, colidx, val, X, labels, Ws)}

    value = spmm_by / (spmm_ms * 1e-3) / 1e9
    return {
        "metric": "spmm_hbm_bandwidth", "value": round(value, 1), "unit": "GB/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(epoch_ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{name}: Chung-Lu power-law graph, n={n}, nnz={nnz} realised with self-loops "
                               f"({NOMINAL_NNZ.get(name)} nominal), GCN {'-'.join(map(str, dims))}, one epoch = fwd+loss+bwd, no optimiser",
                   "spmm_widths": spmm_widths, "orders": [model.order(l) for l in range(L)],
                   "nnz_realised": nnz, "nnz_nominal": NOMINAL_NNZ.get(name), "csr_sha256": sha},
        "value_is": "bytes moved between L2 and the fabric by the SpMM launches of an epoch (measured where a profile of this "
                    "configuration exists, else compulsory bytes) / their time",
        "epoch_ms": round(epoch_ms, 4),
        "epoch_ms_cached_input": round(epoch_cached_ms, 4), "cache_input_fill_ms": round(cache_fill_ms, 3),
        "spmm_pct_hbm_roofline": round(100.0 * value / HBM_PEAK_GBPS, 2),
        "spmm_no_reuse_GBps": round(spmm_eff / (spmm_ms * 1e-3) / 1e9, 1),
        "spmm_compulsory_GBps": round(spmm_min / (spmm_ms * 1e-3) / 1e9, 1),
        "spmm_ms_per_epoch": round(spmm_ms, 4), "gemm_ms_per_epoch": round(gemm_ms, 4),
        "gemm_tflops": round(gemm_tflops, 2),
        "gemm_mfma_utilisation": round(gemm_tflops / FP32_MFMA_PEAK_TFLOPS, 4),
        "ops_ms": {k: r4(v) for k, v in ops.items()},
        "extensions_beyond_fp32": ext,
        "loss": loss_value, "setup_s": setup, "generate_s": round(gen_s, 3),
        "box_calibration": calib, "roofline": roofline, "cpu_baseline": cpu,
    }


def oracle_epoch_seconds(np, cfg, n, rowptr, colidx, val, X, labels, Ws):
    from oracle import ref

    t0 = time.perf_counter()
    ref.epoch(n, rowptr.cpu().numpy(), colidx.cpu().numpy(), val.cpu().numpy().astype(np.float64),
              X.cpu().numpy().astype(np.float64), labels.cpu().numpy(), [w.cpu().numpy().astype(np.float64) for w in Ws])
    return round(time.perf_counter() - t0, 3)


def cpu_baseline_epoch(args, name, np, wl, X, rowptr, colidx, val, n, nnz, spmm_keys, cfg, labels, Ws):
    from oracle import ref

    rp, ci = rowptr.cpu().numpy(), colidx.cpu().numpy()
    v64 = val.cpu().numpy().astype(np.float64)
    cpu_s, cpu_b, what = 0.0, 0, []
    for k in spmm_keys:  # the same SpMM products an epoch makes, forward (N) and backward (T) forms
        if nnz > 500_000_000 and what:  # a billion-entry graph: one product keeps the sample bounded
            break
        F = int(k.rsplit("F", 1)[1])
        Xs = (X[:, :F].cpu().numpy() if F <= X.shape[1] else wl.normal_f32(1, F, (n, F))).astype(np.float64)
        t0 = time.perf_counter()
        ref.spmm(ref.OP_T if "bwd" in k else ref.OP_N, n, n, rp, ci, v64, Xs)
        cpu_s += time.perf_counter() - t0
        cpu_b += spmm_bytes(nnz, n, F)
        what.append(k)
    cpu = {
        "value": round(cpu_b / cpu_s / 1e9, 3), "unit": "GB/s",
        "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), "kind": "oracle",
        "sample": f"the {len(what)} SpMM products of one epoch on the full {name} graph ({', '.join(what)}), fp64 oracle, "
                  f"{cpu_s:.2f} s; bytes by the no-reuse count (compare spmm_no_reuse_GBps)",
        "seconds": round(cpu_s, 3),
    }
    if name in args.oracle_epoch.split(","):
        cpu["oracle_epoch_s"] = oracle_epoch_seconds(np, cfg, n, rowptr, colidx, val, X, labels, Ws)
    return cpu


def spmm_sweep(args, cfg, mg, torch, dev) -> int:
    """SpMM-only feature-width sweep (the density / width study of the paper's evaluation, on the
    synthetic stand-in graphs)."""
    widths = [int(x) for x in args.spmm_sweep.split(",")]
    g = cfg.graph()
    n = g.n_rows
    rowptr, colidx, val = mg.mggcn_csr_normalize(n, n, torch.from_numpy(g.rowptr).to(dev),
                                                 torch.from_numpy(g.colidx).to(dev))
    nnz = int(colidx.numel())
    graph = mg.Graph(n, n, rowptr, colidx, val, F_max=max(widths), seg_len=args.seg_len)
    rows = []
    for F in widths:
        ld = (F + 15) // 16 * 16
        src = torch.randn((n, ld), device=dev)
        dst = torch.empty((n, ld), device=dev)
        ms = timed(torch, lambda: mg.mggcn_spmm(graph, mg.OP_N, src[:, :F], Y=dst[:, :F]), 10)["min"]
        beff = spmm_bytes(nnz, n, F)
        rows.append({"F": F, "ms": round(ms, 4), "passes": graph.panels(F), "no_reuse_GB": round(beff / 1e9, 2),
                     "no_reuse_GBps": round(beff / ms / 1e6, 1),
                     "compulsory_GBps": round(spmm_bytes_min(nnz, n, n, F) / ms / 1e6, 1),
                     "gflops": round(2.0 * nnz * F / ms / 1e6, 1)})
        del src, dst
    print(json.dumps({"mode": "spmm-sweep", "config": args.config, "n": n, "nnz": nnz, "rows": rows}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="block", choices=["tiny", "medium", "large", "rmat", "proteins", "block"])
    ap.add_argument("--also", default="medium,large", metavar="C1,C2",
                    help="with the default block workload: square configurations whose epoch is also run briefly and "
                         "reported under other_configs ('' = none)")
    ap.add_argument("--oracle-epoch", default="tiny,medium", metavar="C1,C2",
                    help="configurations on which the fp64 oracle's whole epoch is timed on the host as well")
    ap.add_argument("--spmm-sweep", default="", metavar="F1,F2,...",
                    help="feature-width sweep mode: time the forward SpMM of the chosen configuration's graph at "
                         "each width (HIP events, min of 10), print one JSON object, then exit")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-calibration", action="store_true")
    ap.add_argument("--seg-len", type=int, default=0)
    ap.add_argument("--profile-spmm", type=int, default=0, metavar="N",
                    help="counter-collection mode: N SpMM calls at the widest width (block: N forward, then N transposed) "
                         "plus one 1 GiB device copy of known size (calibration), then exit")
    ap.add_argument("--profile-width", type=int, default=0, metavar="F",
                    help="with --profile-spmm: the feature width to run at (default: the epoch's widest SpMM)")
    ap.add_argument("--profile-gemm", type=int, default=0, metavar="N",
                    help="counter-collection mode: N calls of the first layer's forward GeMM (H W with the padded "
                         "leading dimension the epoch uses) and N of its weight-gradient GeMM, then exit; block: N calls "
                         "of each of the layer's three GeMMs")
    ap.add_argument("--zero-operands", action="store_true",
                    help="with --config block --profile-gemm: all-zero operands (the same launches on data that do not switch)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_2110_08688_amd as mg
    import workloads as wl

    mg.binding.lib()  # fail loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    cfg = wl.CONFIGS[args.config]

    if args.spmm_sweep:
        return spmm_sweep(args, cfg, mg, torch, dev)
    profiling = args.profile_spmm > 0 or args.profile_gemm > 0
    calib = None if (args.no_calibration or profiling) else calibrate(mg, torch, dev)

    if args.config == "block":
        out = run_block(args, cfg, mg, wl, torch, dev, calib)
        if not profiling and args.also:
            torch.cuda.empty_cache()
            others = {}
            for name in args.also.split(","):
                o = run_epoch_config(args, name, wl.CONFIGS[name], mg, wl, torch, dev, calib, brief=True)
                for drop in ("box_calibration", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "dtype", "data", "metric",
                             "unit"):
                    o.pop(drop, None)
                others[name] = o
                torch.cuda.empty_cache()
            out["other_configs"] = others
    else:
        out = run_epoch_config(args, args.config, cfg, mg, wl, torch, dev, calib)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
