"""GPU parity of the CSR logistic iteration in the launch shapes of the sparse workload at its full
dimension: d = 2^24, 0.1 % density, minibatch 512, 4-bit codes, subtraction normalisation, with the
per-row tile index and the entries stored as (column, value) pairs (what bench.py times), and with
separate column and value arrays.  At this dimension the dot-product pass hands a pair of
column tiles to a workgroup that serves 2, 4 or 8 workers in turn (1 in every small test): 64
workers as in the workload (8 per workgroup), 8 and 16 workers (2 and 4), worker counts that the
group size does not divide, and a minibatch longer than one staging trip together with a group of
workers.  Shards hold 512 rows (a step only touches minibatch rows).

Teacher-forced: gradients within 1e-5 of the float64 oracle (2-norm, max-norm and elementwise with
the cancellation term, see gpu_util.grad_close), then codes, scales, decoded average, iterate and
reference bit for bit from the library's own gradients.  The oracle's work is shared between host
processes (gradients) and threads (codec); every value compared comes out of an oracle function."""
import os

import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, buffers, make_ctx, oracle_cfg, oracle_step_threaded, say, set_csr, u32
from oracle_pool import CsrGradientChecker
from paper_1901_08227_amd import binding as B
from paper_1901_08227_amd import synth

pytestmark = pytest.mark.gpu

D = 1 << 24
HOST_WORKERS = max(2, min(16, os.cpu_count() or 2))


@pytest.mark.parametrize("M,batch,nnz_row,steps,pairs", [
    (64, 512, 16777, 2, True),    # the sparse workload itself: 8 workers per workgroup in the dot-product pass
    (64, 512, 16777, 1, False),   # the same with separate column and value arrays
    (8, 512, 16777, 2, True),     # 2 workers per workgroup
    (16, 512, 16777, 2, False),   # 4 workers per workgroup
    (9, 600, 4000, 2, True),      # 2 per workgroup, the last group short, two staging trips per worker
    (9, 600, 4000, 1, False),
    (18, 512, 4000, 1, True),     # 4 per workgroup, the last group holds 2
    (36, 100, 2000, 1, False),    # 8 per workgroup, the last group holds 4, a short minibatch
])
def test_csr_logistic_full_dimension_worker_groups(M, batch, nnz_row, steps, pairs):
    n, seed = 512, 6 + M
    say(f"csr logistic d=2^24 M={M} B={batch} nnz/row={nnz_row} pairs={pairs}: generating shards")
    shards, _ = synth.logreg_csr(M, n, D, nnz_row, seed, device=DEV)
    ctx = make_ctx(D, M, 4, B.NORM_SUB, seed=seed, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR)
    set_csr(ctx, shards, pairs)
    ctx.build_csr_index()
    cfg = oracle_cfg(ctx)
    host = [tuple(t.cpu().numpy() for t in s) for s in shards]
    checker = CsrGradientChecker(host, D, processes=HOST_WORKERS)
    try:
        w = 0.01 * torch.randn(D, device=DEV, generator=torch.Generator(device=DEV).manual_seed(1))
        gref = torch.zeros(D, device=DEV)
        buf = buffers(ctx)
        for it in range(steps):
            w0, r0 = w.cpu().numpy(), gref.cpu().numpy()
            say(f"  it={it}: tng_step")
            ctx.step(it, w, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
            torch.cuda.synchronize()
            gh = buf["g"].cpu().numpy()
            say(f"  it={it}: oracle gradients of {M} workers in {min(HOST_WORKERS, M)} host processes")
            ids = [O.minibatch_indices(seed, it, m, batch, n) for m in range(M)]
            for rec in checker.check(w0, gh, ids):
                assert rec["norm2_ok"] and rec["max_ok"] and rec["elementwise_ok"], f"it={it}: local gradient {rec}"
                assert rec["nonzero"] > 0
            say(f"  it={it}: oracle codec over {M} x 2^24 elements")
            w1, r1, c1, s1, v1 = oracle_step_threaded(cfg, it, w0, r0, gh, threads=HOST_WORKERS)
            assert np.array_equal(buf["scales"].cpu().numpy(), s1), f"it={it}: scales"
            assert np.array_equal(u32(buf["codes"]), c1), f"it={it}: packed codes"
            del c1
            assert np.array_equal(buf["vbar"].cpu().numpy(), v1), f"it={it}: decoded average"
            assert np.array_equal(w.cpu().numpy(), w1), f"it={it}: iterate"
            assert np.array_equal(gref.cpu().numpy(), r1), f"it={it}: reference"
    finally:
        checker.close()
        ctx.close()
