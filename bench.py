#!/usr/bin/env python3
"""Benchmark of libtng on one MI355X.

Workload (the one the headline metric is quoted on): the encode/decode microbenchmark --
M = 8 worker gradients of d = 2^27 fp32, g_m = g~ + N(0, 0.1) |g~|, g~ ~ N(0, 1), seed 1.
One step = tng_normalize_encode + tng_decode_aggregate over all 8 gradients (iteration number =
step number), inputs resident in HBM.  The headline value is ternary codes with subtraction
normalisation; the other three variants (4-bit, quotient) are timed the same way and reported
under "variants".  Per-kernel durations come from HIP events recorded by the library on its
stream inside the timed region; the oracle is timed on the host on a bounded sample.

Prints one JSON line on stdout (progress goes to stderr).
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0  # MI355X HBM3E, published peak


def log(msg):
    print(msg, file=sys.stderr, flush=True)


class HipEvents:
    """hipEvent_t handles created through the HIP runtime (the library records them itself)."""

    def __init__(self, n):
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.ev = []
        for _ in range(n):
            e = ctypes.c_void_p()
            rc = self.hip.hipEventCreate(ctypes.byref(e))
            if rc != 0:
                raise RuntimeError(f"hipEventCreate failed: {rc}")
            self.ev.append(e.value)

    def elapsed_ms(self, a, b):
        out = ctypes.c_float()
        rc = self.hip.hipEventElapsedTime(ctypes.byref(out), ctypes.c_void_p(self.ev[a]), ctypes.c_void_p(self.ev[b]))
        if rc != 0:
            raise RuntimeError(f"hipEventElapsedTime failed: {rc}")
        return float(out.value)

    def destroy(self):
        for e in self.ev:
            self.hip.hipEventDestroy(ctypes.c_void_p(e))
        self.ev = []


def time_codec(torch, B, g, gref, bits, norm, steps, warmup, seed, scale=0):
    """Times `steps` encode+decode passes; returns whole-loop ms/step and per-kernel mean ms."""
    M, d = g.shape
    ctx = B.Context(d=d, M=M, bits=bits, norm=norm, seed=seed, scale=scale, device=g.device)
    if norm == B.NORM_MEAN:
        ctx.set_worker_means(torch.empty(M, device=g.device))
    codes = torch.empty((M, ctx.words), dtype=torch.int32, device=g.device)
    scales = torch.empty(M, device=g.device)
    vbar = torch.empty(d, device=g.device)
    for it in range(warmup):
        ctx.normalize_encode(it, g, gref, codes, scales)
        ctx.decode_aggregate(codes, scales, gref, vbar)
    ev = HipEvents(5 * steps)
    ctx.set_profile_events(ev.ev, steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(steps):
        ctx.normalize_encode(warmup + it, g, gref, codes, scales)
        ctx.decode_aggregate(codes, scales, gref, vbar)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    t_scale = [ev.elapsed_ms(5 * i + 0, 5 * i + 1) for i in range(steps)]
    t_quant = [ev.elapsed_ms(5 * i + 1, 5 * i + 2) for i in range(steps)]
    t_dec = [ev.elapsed_ms(5 * i + 3, 5 * i + 4) for i in range(steps)]
    k_scale, k_quant, k_dec = sum(t_scale) / steps, sum(t_quant) / steps, sum(t_dec) / steps

    def spread(ts):
        ts = sorted(ts)
        return {"min": round(ts[0], 4), "median": round(ts[len(ts) // 2], 4)}
    ctx.set_profile_events(None, 0)
    ev.destroy()
    words = ctx.words
    ctx.close()
    del codes, scales, vbar
    ms = (t1 - t0) * 1e3 / steps
    # algorithmic bytes per launch: each operand once per kernel (the mean reference reads no shared
    # reference; its mean and its scale come out of one pass)
    b_ref = {B.NORM_NONE: 0, B.NORM_MEAN: 0, B.NORM_COMB: 8 * d}.get(norm, 4 * d)
    b_scale = (2 if norm == B.NORM_MEAN and scale == B.SCALE_L2 else 1) * 4 * M * d + b_ref
    b_quant = 4 * M * d + b_ref + 4 * M * words
    b_dec = 4 * M * words + b_ref + 4 * d
    two_pass = b_scale + b_quant + b_dec
    # long rows of ternary codes (Eq. 1 or no normalisation, largest-magnitude scale): the scale pass keeps the
    # elements that can code non-zero and the quantise pass codes those, so g is read once; what the quantise
    # pass must move is then the packed codes (the candidate words, a few percent of the elements, are the
    # method's own overhead and are not counted as algorithmic bytes)
    single_read = (bits == 2 and scale == B.SCALE_MAX and norm in (B.NORM_NONE, B.NORM_SUB)
                   and d % 1024 == 0 and M * d >= 1 << 26 and d // 1024 >= 512)
    if single_read:
        b_quant = 4 * M * words
    return {
        "ms_per_step": ms,
        "path": "g read once (candidate slots)" if single_read else "two passes over g",
        "compulsory_bytes": 4 * M * d + b_ref + 4 * M * words + b_dec,
        "compulsory_GBps": (4 * M * d + b_ref + 4 * M * words + b_dec) / (ms * 1e-3) / 1e9,
        "fp32_in_GBps": 4.0 * M * d / (ms * 1e-3) / 1e9,
        "kernels": {
            "absmax": {"ms": k_scale, "bytes": b_scale, "GBps": b_scale / (k_scale * 1e-3) / 1e9, **spread(t_scale)},
            "quantize_pack": {"ms": k_quant, "bytes": b_quant, "GBps": b_quant / (k_quant * 1e-3) / 1e9,
                              **spread(t_quant)},
            "decode": {"ms": k_dec, "bytes": b_dec, "GBps": b_dec / (k_dec * 1e-3) / 1e9, **spread(t_dec)},
        },
        "bits_per_element": (32.0 * words * M + 32.0 * M * (2 if norm == B.NORM_MEAN else 1)) / (M * d),
        "two_pass_bytes": two_pass,
        "two_pass_GBps": two_pass / (ms * 1e-3) / 1e9,
    }


def cpu_baseline(g, gref, seed, sample_d):
    """The oracle as it stands, on a bounded sample (first sample_d coordinates of every worker)."""
    import numpy as np

    from oracle import tng_oracle as O

    M = g.shape[0]
    gh = g[:, :sample_d].cpu().numpy()
    rh = gref[:sample_d].cpu().numpy()
    cfg = O.Config(d=sample_d, M=M, bits=2, norm=O.NORM_SUB, seed=seed)
    t0 = time.perf_counter()
    codes, scales = O.normalize_encode(cfg, 0, gh, rh)
    vbar = O.decode_aggregate(cfg, codes, scales, rh, sample_d)
    t1 = time.perf_counter()
    assert np.isfinite(vbar).all()
    return {
        "value": 4.0 * M * sample_d / (t1 - t0) / 1e9,
        "unit": "GB/s",
        "cores": 1,
        "kind": "oracle",
        "sample": f"numpy oracle, one encode+decode pass (ternary, subtraction) over M={M} x the first "
                  f"2^{sample_d.bit_length() - 1} of 2^{g.shape[1].bit_length() - 1} coordinates, "
                  f"{t1 - t0:.1f} s, single thread; host has {os.cpu_count()} logical CPUs",
    }


def time_steps(torch, ctx, state, steps, warmup, per_step=None):
    """Times `steps` calls of tng_step (whole iteration); returns ms per step."""
    w, gref, g, codes, scales, vbar = state
    for it in range(warmup):
        if per_step:
            per_step(it)
        ctx.step(it, w, gref, g, codes, scales, vbar)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(warmup, warmup + steps):
        if per_step:
            per_step(it)
        ctx.step(it, w, gref, g, codes, scales, vbar)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e3 / steps


def step_state(torch, ctx, w0):
    dev = w0.device
    return (w0.clone(), torch.zeros(ctx.d, device=dev), torch.empty((ctx.M, ctx.d), device=dev),
            torch.empty((ctx.M, ctx.words), dtype=torch.int32, device=dev), torch.empty(ctx.M, device=dev),
            torch.empty(ctx.d, device=dev))


def oracle_step_seconds(ctx, grads, w0):
    """One whole iteration of the oracle on the host: `grads()` returns the M local gradients (timed),
    then normalise/encode/decode/update/refresh.  Returns seconds."""
    import numpy as np

    from oracle import tng_oracle as O

    c = ctx.cfg
    cfg = O.Config(d=int(c.d), M=int(c.M), bits=int(c.bits), norm=int(c.norm), quot_eps=float(c.quot_eps),
                   ref_policy=int(c.ref_policy), ref_period=int(c.ref_period), seed=int(c.seed), lr=float(c.lr),
                   l2=float(c.l2), batch=int(c.batch))
    t0 = time.perf_counter()
    g = np.stack(grads(O)).astype(np.float32)
    O.step(cfg, 0, w0, np.zeros(cfg.d, np.float32), g)
    return time.perf_counter() - t0


def step_bytes(kind, M, d, words, batch=0, nnz=0, ntiles=0, noise_tensor=False, row_splits=0):
    """HBM bytes of one tng_step, two ways.  `moved`: what the path as built transfers (every kernel's
    operands once per kernel; the scale pass rides along with the gradient kernel, so g is written once and
    read once).  `compulsory`: every operand of the iteration once (minibatch data once, g written and read
    once, codes written and read once, the d-vectors w, g~, v once each way)."""
    codes = 4 * M * words
    vectors = 4 * d * 6                      # decode: g~ read, v written, w read + written, g~ refreshed; gradient: w read
    codec = 4 * M * d + 4 * d + codes + codes   # quantise: g + g~ read, codes written; decode: codes read
    if kind == "dense":
        x = 4 * M * batch * d
        # rows kept on chip (row_splits workgroups per worker): the minibatch rows once, and the workgroups'
        # partial gradients written and read; otherwise the rows twice (residual pass, accumulation pass)
        grad = x + 2 * 4 * M * row_splits * d if row_splits else 2 * x
        return {"moved": grad + 4 * M * d + codec + vectors, "compulsory": x + 4 * M * d + codec + vectors}
    if kind == "csr":
        entries = 8 * nnz
        bounds = 4 * M * batch * (ntiles + 1)
        # gather reads the index rows and writes the bounds; both passes read the bounds; partial dot products
        # written and read once
        side = 4 * bounds + 2 * 4 * M * batch * ((ntiles + 1) // 2)
        return {"moved": 2 * entries + side + 4 * M * d + codec + vectors,
                "compulsory": entries + 4 * M * d + codec + vectors}
    if kind == "rosenbrock":
        noise = 4 * M * d if noise_tensor else 0
        both = noise + 4 * M * d + codec + vectors
        return {"moved": both, "compulsory": both}
    raise ValueError(kind)


def whole_iteration_benchmarks(torch, B, synth, dev, steps, warmup, with_oracle=False, csr_rows=16384, dense_rows=0):
    """tng_step (local gradient + encode + decode + update + reference refresh) on the four training
    workloads.  The sparse workload holds its full shards (64 workers x 16384 rows x 16777 entries, 141 GB)
    when they fit; the wide dense workload holds the largest power-of-two number of rows per worker that
    fits next to the other buffers (the full 65536 rows per worker are 256 GiB)."""
    out = []

    def record(name, ms, nbytes, note, oracle=None, bound="hbm"):
        rec = {"workload": name, "ms_per_step": round(ms, 4), "steps_per_s": round(1e3 / ms, 1),
               "bytes_moved": nbytes["moved"], "bytes_compulsory": nbytes["compulsory"], "bound": bound}
        if bound == "hbm":
            rec["pct_hbm_peak_moved"] = round(100 * nbytes["moved"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)
            rec["pct_hbm_peak_compulsory"] = round(100 * nbytes["compulsory"] / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2)
        else:       # no HBM percentage: the time is not set by HBM traffic
            rec["pct_hbm_peak_moved"] = rec["pct_hbm_peak_compulsory"] = None
        rec["note"] = note
        if oracle is not None:      # (seconds, what was timed): the numpy oracle, one iteration, single thread
            rec["oracle_ms_per_step"] = round(oracle[0] * 1e3, 2)
            rec["oracle_sample"] = oracle[1]
        out.append(rec)

    def logistic_oracle(ctx, Xs, ys, n, d, dense=True, shards=None):
        """Times the oracle on the rows the first minibatch touches (copied to the host beforehand)."""
        import numpy as np

        from oracle import tng_oracle as O

        M, batch, seed = ctx.M, int(ctx.cfg.batch), int(ctx.cfg.seed)
        ids = [O.minibatch_indices(seed, 0, m, batch, n) for m in range(M)]
        w0 = np.zeros(d, np.float32)
        if dense:
            rows = [(Xs[m][torch.from_numpy(ids[m].astype(np.int64)).to(dev)].cpu().numpy(),
                     ys[m].cpu().numpy()[ids[m]]) for m in range(M)]
            return oracle_step_seconds(ctx, lambda O: [O.grad_logreg_dense(rows[m][0], rows[m][1], w0, np.arange(batch))
                                                       for m in range(M)], w0)
        host = [tuple(t.cpu().numpy() for t in sh) for sh in shards]
        return oracle_step_seconds(ctx, lambda O: [O.grad_logreg_csr(*host[m], w0, ids[m], d) for m in range(M)], w0)

    def free_bytes():
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        return torch.cuda.mem_get_info(dev)[0]

    # small dense logistic regression: latency bound
    M, n, d, batch = 4, 2000, 1000, 64
    X, y, _ = synth.logreg_dense(M, n, d, seed=0, device=dev)
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, seed=0, lr=0.1, batch=batch, problem=B.PROB_LOGREG_DENSE, device=dev)
    ctx.set_logreg_dense([X[m] for m in range(M)], [y[m] for m in range(M)])
    ms = time_steps(torch, ctx, step_state(torch, ctx, torch.zeros(d, device=dev)), steps * 4, warmup)
    orc = (logistic_oracle(ctx, X, y, n, d), "same shape") if with_oracle else None
    record("dense logistic d=1000 M=4 B=64 ternary sub", ms, step_bytes("dense", M, d, ctx.words, batch),
           "3 kernel launches per iteration, 1 MB of minibatch rows: bound by launch latency, not by memory", orc,
           bound="launch latency")
    ctx.close()
    del X, y

    # Rosenbrock chain
    M, d = 8, 1 << 20
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, seed=1, lr=1e-5, problem=B.PROB_ROSENBROCK, device=dev)
    noises = [synth.gradient_noise(M, d, 1, it, variance=0.01, device=dev) for it in range(8)]
    ms = time_steps(torch, ctx, step_state(torch, ctx, synth.rosenbrock_start(d, 1, device=dev)), steps, warmup,
                    per_step=lambda it: ctx.set_noise(noises[it % 8]))
    orc = None
    if with_oracle:
        x0, nz = synth.rosenbrock_start(d, 1, device=dev).cpu().numpy(), noises[0].cpu().numpy()
        orc = (oracle_step_seconds(ctx, lambda O: [O.grad_rosenbrock(x0, nz[m]) for m in range(M)], x0), "same shape")
    cache_note = ("3 launches; the 32 MiB of gradients written by one kernel are read by the next out of the 256 MB "
                  "last-level cache: bound by launches and cache, not an HBM figure")
    record("Rosenbrock chain d=2^20 M=8 ternary sub", ms, step_bytes("rosenbrock", M, d, ctx.words, noise_tensor=True),
           "noise tensors of 8 iterations resident; " + cache_note, orc, bound="launch latency and last-level cache")
    del noises
    ctx.set_noise_variance(0.01)
    ms = time_steps(torch, ctx, step_state(torch, ctx, synth.rosenbrock_start(d, 1, device=dev)), steps, warmup)
    record("Rosenbrock chain d=2^20 M=8 ternary sub, noise generated on the device", ms,
           step_bytes("rosenbrock", M, d, ctx.words),
           "Box-Muller on Philox draws inside the gradient kernel; " + cache_note,
           bound="launch latency and last-level cache")
    ctx.close()

    # wide dense logistic regression, quotient normalisation
    M, d, batch = 16, 1 << 16, 256
    n = dense_rows
    if n == 0:      # the largest power of two that fits, up to the 65536 rows of the workload
        n = 65536
        while n > 256 and M * n * d * 4 > free_bytes() - (12 << 30):
            n //= 2
    X = [torch.randn((n, d), device=dev, generator=torch.Generator(device=dev).manual_seed(m)) for m in range(M)]
    y = [(torch.rand(n, device=dev) < 0.5).float() for _ in range(M)]
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_QUOT, seed=2, lr=0.1, batch=batch, problem=B.PROB_LOGREG_DENSE, device=dev)
    ctx.set_logreg_dense(X, y)
    ms = time_steps(torch, ctx, step_state(torch, ctx, torch.zeros(d, device=dev)), steps, warmup)
    orc = (logistic_oracle(ctx, X, y, n, d), "same shape, minibatch rows already on the host") if with_oracle else None
    record("dense logistic d=2^16 M=16 B=256 2-bit quot", ms, step_bytes("dense", M, d, ctx.words, batch, row_splits=256 // M),
           f"{n} of 65536 rows per worker resident ({M * n * d * 4 / 2**30:.0f} GiB: the largest power of two that fits); "
           "every minibatch row is read once and kept on chip (LDS + registers) between the dot product and the "
           f"accumulation, {256 // M} workgroups per worker whose partial gradients are then added", orc)
    ctx.close()
    del X, y, ctx

    # sparse logistic regression at d = 2^24
    M, d, batch = 64, 1 << 24, 512
    nnz_row = round(1e-3 * d)
    n = csr_rows
    per_row = nnz_row * 8 + 8 + 4 * (d // 16384 + 1)        # entries + row pointer + tile index
    while n > 512 and M * n * per_row + 3 * n * nnz_row * 8 > free_bytes() - (16 << 30):
        n //= 2
    log(f"  sparse shards: {M} workers x {n} rows x {nnz_row} entries ({M * n * nnz_row * 8 / 1e9:.0f} GB), (column, value) pairs")
    rowptrs, pairs, ys = [], [], []
    for m in range(M):       # one worker at a time: the generator's temporaries are three times a shard
        (rp, col, val, yy), = synth.logreg_csr(1, n, d, nnz_row, seed=3 + m, device=dev)[0]
        rowptrs.append(rp)
        pairs.append(B.csr_pairs(col, val))
        ys.append(yy)
        del col, val
    ctx = B.Context(d=d, M=M, bits=4, norm=B.NORM_SUB, seed=3, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR, device=dev)
    ctx.set_logreg_csr_pairs(rowptrs, pairs, ys)
    ctx.build_csr_index()          # one-off, depends on the shards only
    ms = time_steps(torch, ctx, step_state(torch, ctx, torch.zeros(d, device=dev)), max(steps // 2, 5), max(warmup // 2, 2))
    nnz = M * batch * nnz_row
    words = ctx.words
    ctx.close()
    del rowptrs, pairs, ys, ctx
    orc = None
    if with_oracle:     # the oracle on the scaled shape the parity tests use: d = 2^16, 8 workers, same density
        torch.cuda.empty_cache()
        Ms, ns, ds = 8, 2048, 1 << 16
        small, _ = synth.logreg_csr(Ms, ns, ds, round(1e-3 * ds), seed=3, device=dev)
        sctx = B.Context(d=ds, M=Ms, bits=4, norm=B.NORM_SUB, seed=3, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR, device=dev)
        orc = (logistic_oracle(sctx, None, None, ns, ds, dense=False, shards=small),
               "scaled to d=2^16, M=8, B=512, nnz/row=66 (1/2048 of the entries of the timed shape)")
        sctx.close()
    record("sparse logistic d=2^24 M=64 B=512 nnz/row=16777 4-bit sub", ms,
           step_bytes("csr", M, d, words, batch, nnz=nnz, ntiles=d // 16384),
           f"{n} of 16384 rows per worker resident ({M * n * nnz_row * 8 / 1e9:.0f} GB of entries as (column, value) pairs), "
           "per-row tile index prebuilt; the minibatch rows' entries are read by the dot-product pass and again by "
           "the gradient pass", orc)
    return out


def measured_traffic(kernel, M, d, bits, norm_name):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 counter summary, or None when
    the summary is for another workload or the kernel sources have changed since it was taken."""
    import glob
    import hashlib

    path = os.path.join(ROOT, "profiles", "codec_M8_d2p27_ternary_sub_hbm_traffic.json")
    try:
        rec = json.load(open(path))
    except OSError:
        return None
    if rec.get("workload") != f"M={M} d=2^{d.bit_length() - 1} bits={bits} norm={norm_name}":
        return None
    h = hashlib.sha256()
    # the file that holds the three codec kernels and the device helpers they are built from
    for fn in [os.path.join(ROOT, "paper_1901_08227_amd", "csrc", n) for n in ("tng_codec.hip", "tng_device.hpp")]:
        h.update(open(fn, "rb").read())
    if h.hexdigest() != rec.get("kernel_source_sha256"):
        return None
    return rec["traffic_bytes_per_launch"].get(kernel)


TRAFFIC_SOURCE = ("not measured in this run: from the committed rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE summary "
                  "profiles/codec_M8_d2p27_ternary_sub_hbm_traffic.md, valid while the kernel sources hash to the value "
                  "recorded there (null otherwise)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--log2d", type=int, default=27, help="log2 of the gradient dimension (27 = the headline workload)")
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--cpu-log2d", type=int, default=25, help="log2 of the oracle's sample size per worker")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--no-variants", action="store_true", help="time only the headline variant")
    ap.add_argument("--no-codec", action="store_true", help="skip the encode/decode microbenchmark (development aid)")
    ap.add_argument("--no-steps", action="store_true", help="skip the whole-iteration (tng_step) workloads")
    ap.add_argument("--csr-rows", type=int, default=16384, help="rows per worker of the sparse workload's shards "
                    "(halved until they fit)")
    ap.add_argument("--dense-rows", type=int, default=0, help="rows per worker of the wide dense workload "
                    "(0 = the largest power of two that fits)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain copy kernel of known size (d floats read, d floats written) three "
                         "times, as the reference for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (the workers are simulated on it); --gpus above 1 is not supported")
        sys.exit(2)

    import torch

    from paper_1901_08227_amd import binding as B
    from paper_1901_08227_amd import synth

    B.lib()  # fail loudly if the HIP library is not built
    dev = torch.device("cuda:0")
    if args.no_codec:
        if args.copy_calibration:      # reference for scaling the counters of a profiler run over this mode
            cal = torch.randn(1 << 27, device=dev)
            cctx = B.Context(d=1 << 27, M=1, bits=2, norm=B.NORM_SUB, ref_policy=B.REF_LAST_AVG, ref_period=1, device=dev)
            dst = torch.empty(1 << 27, device=dev)
            for _ in range(3):
                cctx.update_reference(0, cal, dst)   # copy_f32x4_kernel: reads 2^29 bytes, writes 2^29 bytes
            torch.cuda.synchronize()
            cctx.close()
            del cal, dst
        for r in whole_iteration_benchmarks(torch, B, synth, dev, args.steps, args.warmup, csr_rows=args.csr_rows,
                                            dense_rows=args.dense_rows):
            print(json.dumps(r), flush=True)
        return
    M, d, seed = args.workers, 1 << args.log2d, 1
    log(f"generating g[{M}][2^{args.log2d}] and the reference on {torch.cuda.get_device_name(0)}")
    g, gref = synth.codec_inputs(M, d, seed, rel_variance=0.1, device=dev)
    torch.cuda.synchronize()

    log("timing ternary / subtraction (headline)")
    head = time_codec(torch, B, g, gref, 2, B.NORM_SUB, args.steps, args.warmup, seed)
    variants = []
    if not args.no_variants:
        for bits, norm, scale, name in [(4, B.NORM_SUB, B.SCALE_MAX, "4bit/sub"),
                                        (2, B.NORM_QUOT, B.SCALE_MAX, "ternary/quot"),
                                        (4, B.NORM_QUOT, B.SCALE_MAX, "4bit/quot"),
                                        (2, B.NORM_MEAN, B.SCALE_MAX, "ternary/mean"),
                                        (2, B.NORM_SUB, B.SCALE_L2, "ternary/sub/l2")]:
            log(f"timing {name}")
            r = time_codec(torch, B, g, gref, bits, norm, args.steps, args.warmup, seed, scale)
            variants.append({"variant": name, "path": r["path"], "ms_per_step": round(r["ms_per_step"], 4),
                             "fp32_in_GBps": round(r["fp32_in_GBps"], 1),
                             "two_pass_GBps": round(r["two_pass_GBps"], 1),
                             "kernel_ms": {k: round(v["ms"], 4) for k, v in r["kernels"].items()}})

    if args.copy_calibration:
        ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, ref_policy=B.REF_LAST_AVG, ref_period=1, device=dev)
        dst = torch.empty(d, device=dev)
        for _ in range(3):
            ctx.update_reference(0, gref, dst)   # copy_f32x4_kernel: reads 4 d bytes, writes 4 d bytes
        torch.cuda.synchronize()
        ctx.close()
        log(f"copy calibration: 3 launches of the plain copy kernel, {4 * d} bytes read and written each")

    # practical ceiling: the library's plain float4 copy kernel on the same buffers (reads 4d, writes 4d bytes)
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, ref_policy=B.REF_LAST_AVG, ref_period=1, device=dev)
    dst = torch.empty(d, device=dev)
    for _ in range(3):
        ctx.update_reference(0, gref, dst)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(20):
        ctx.update_reference(0, gref, dst)
    torch.cuda.synchronize()
    copy_gbps = 8.0 * d * 20 / (time.perf_counter() - t0) / 1e9
    ctx.close()
    del dst

    cpu = None
    if not args.no_cpu:
        log("timing the oracle on the host")
        cpu = cpu_baseline(g, gref, seed, min(1 << args.cpu_log2d, d))
    iteration_results = []
    if not args.no_steps:
        del g, gref
        torch.cuda.empty_cache()
        log("timing whole iterations (tng_step) on the training workloads")
        iteration_results = whole_iteration_benchmarks(torch, B, synth, dev, 20, 5, with_oracle=not args.no_cpu,
                                                       csr_rows=args.csr_rows, dense_rows=args.dense_rows)
        g = gref = None

    dom_name = max(head["kernels"], key=lambda k: head["kernels"][k]["ms"])
    dom = head["kernels"][dom_name]
    out = {
        "metric": "tng_encode_decode_fp32_in_throughput",
        "value": round(head["fp32_in_GBps"], 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(head["ms_per_step"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"encode+decode microbenchmark: M={M} workers x d=2^{args.log2d} fp32, "
                               "g = ref + N(0,0.1)|ref|, ref ~ N(0,1), ternary codes, subtraction normalisation, seed 1",
                   "M": M, "d": d, "bits": 2, "norm": "sub"},
        "path": head["path"],
        "pct_hbm_peak_compulsory": round(100.0 * head["compulsory_GBps"] / HBM_PEAK_GBPS, 2),
        "compulsory_algorithmic_GBps": round(head["compulsory_GBps"], 1),
        "pct_hbm_peak_two_pass": round(100.0 * head["two_pass_GBps"] / HBM_PEAK_GBPS, 2),
        "two_pass_algorithmic_GBps": round(head["two_pass_GBps"], 1),
        "note_two_pass": "bytes a coder with two passes over g would move, divided by this run's time: a yardstick "
                         "kept for comparison (the headline path reads g once, so it moves fewer)",
        "kernel_ms": {k: round(v["ms"], 4) for k, v in head["kernels"].items()},
        "kernel_GBps": {k: round(v["GBps"], 1) for k, v in head["kernels"].items()},
        "kernel_ms_min_median": {k: [v["min"], v["median"]] for k, v in head["kernels"].items()},
        "bits_per_element_on_the_wire": round(head["bits_per_element"], 6),
        "copy_kernel_GBps": round(copy_gbps, 1),
        "pct_of_copy_kernel_two_pass": round(100.0 * head["two_pass_GBps"] / copy_gbps, 2),
        "variants": variants,
        "iterations": iteration_results,
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(dom["GBps"], 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(dom["GBps"] / HBM_PEAK_GBPS, 4),
                     "algorithmic_bytes_per_launch": dom["bytes"],
                     "traffic": measured_traffic(dom_name, M, d, 2, "sub"), "traffic_source": TRAFFIC_SOURCE},
    }
    if cpu is not None:
        out["cpu_baseline"] = cpu
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
