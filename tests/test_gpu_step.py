"""GPU parity of tng_local_grad and of whole iterations (tng_step), teacher-forced: at every
iteration the oracle restarts from the library's own (w, g~) and is fed the library's own local
gradients, so that last-bit differences in the gradients (exp, summation order, atomics) cannot
flip a rounding decision downstream.  Gradients: Rosenbrock bit-exact; logistic within 1e-5
relative: ||a-b||_2 <= 1e-5 ||b||_2, max|a-b| <= 1e-5 ||b||_inf, and elementwise
|a-b| <= 1e-5 |b| + 4 eps32 cond (cond = size of the summed terms).  Codes, scales bit-exact;
decoded average, iterate and reference bit-exact (contract: 1e-5 relative)."""
import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import (DEV, assert_row_sums_are_the_exact_ones, buffers, set_csr, grad_close, logistic_condition, logistic_condition_csr, make_ctx, oracle_cfg,
                      say, u32)
from paper_1901_08227_amd import binding as B
from paper_1901_08227_amd import synth

pytestmark = pytest.mark.gpu


def _teacher_forced_step(ctx, cfg, it, w, gref, buf, grad_ref, grad_exact=False):
    w0, r0 = w.cpu().numpy(), gref.cpu().numpy()
    ctx.step(it, w, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
    torch.cuda.synchronize()
    gh = buf["g"].cpu().numpy()
    if grad_ref is not None:
        if grad_exact:
            assert np.array_equal(gh, grad_ref(w0)), f"it={it}: local gradient not bit-exact"
        else:
            ref, cond = grad_ref(w0)
            for m in range(ctx.M):
                assert grad_close(gh[m], ref[m], cond[m]), f"it={it} m={m}: local gradient out of tolerance"
    w1, r1, c1, s1, v1 = O.step(cfg, it, w0, r0, gh)
    assert np.array_equal(buf["scales"].cpu().numpy(), s1), f"it={it}: scales"
    assert np.array_equal(u32(buf["codes"]), c1), f"it={it}: packed codes"
    assert np.array_equal(buf["vbar"].cpu().numpy(), v1), f"it={it}: decoded average"
    assert np.array_equal(w.cpu().numpy(), w1), f"it={it}: iterate"
    assert np.array_equal(gref.cpu().numpy(), r1), f"it={it}: reference"


def _dense_case(M, n, d, batch, bits, norm, T, seed, lr=0.1, l2=0.0, ref_period=1, data=None,
                full_gradient_reference=False):
    X, y = data if data is not None else synth.logreg_dense(M, n, d, seed=seed, device=DEV)[:2]
    ctx = make_ctx(d, M, bits, norm, seed=seed, lr=lr, l2=l2, batch=batch, ref_period=ref_period,
                   problem=B.PROB_LOGREG_DENSE)
    ctx.set_logreg_dense([X[m] for m in range(M)], [y[m] for m in range(M)])
    cfg = oracle_cfg(ctx)
    Xh, yh = X.cpu().numpy(), y.cpu().numpy()
    w = torch.zeros(d, device=DEV)
    gref = torch.zeros(d, device=DEV)
    if full_gradient_reference:      # the convex experiments start the reference from a full gradient
        full = np.mean([O.grad_logreg_dense(Xh[m], yh[m], np.zeros(d, np.float32), np.arange(n), l2)
                        for m in range(M)], axis=0)
        gref = torch.from_numpy(full.astype(np.float32)).to(DEV)
    buf = buffers(ctx)

    def loss(wv):
        z = Xh.reshape(-1, d).astype(np.float64) @ wv.astype(np.float64)
        return float(np.mean(np.logaddexp(0, z) - yh.reshape(-1) * z))

    first = loss(w.cpu().numpy())
    for it in range(T):
        def grad_ref(w0, it=it):
            ids = [O.minibatch_indices(seed, it, m, batch, n) for m in range(M)]
            ref = np.stack([O.grad_logreg_dense(Xh[m], yh[m], w0, ids[m], l2) for m in range(M)])
            cond = np.stack([logistic_condition(Xh[m][ids[m]], yh[m][ids[m]], w0, l2) for m in range(M)])
            return ref, cond
        _teacher_forced_step(ctx, cfg, it, w, gref, buf, grad_ref)
        if it % 50 == 49:
            say(f"  it={it} done")
    last = loss(w.cpu().numpy())
    ctx.close()
    return first, last


def test_dense_logistic_small_config_all_iterations():
    # d=1000, 4 workers x 2000 samples, minibatch 64, lr 0.1, ternary, subtraction, 100 iterations, seed 0
    say("dense logistic d=1000 M=4 n=2000 B=64 T=100")
    first, last = _dense_case(M=4, n=2000, d=1000, batch=64, bits=2, norm=B.NORM_SUB, T=100, seed=0)
    assert abs(first - np.log(2)) < 1e-6 and last < first - 0.02


def test_dense_logistic_skewed_features_at_the_experiments_shape():
    # D = 512, N = 2048 over M = 4 workers, batch 8, c_th = 0.6, c_sk = 1/16, l2 > 0, reference started
    # from the full gradient and refreshed from the last decoded average (section "Convex Problems")
    for bits, norm in [(2, B.NORM_SUB), (4, B.NORM_SUB), (2, B.NORM_MEAN)]:
        say(f"skewed logistic d=512 M=4 n=512 B=8 bits={bits} norm={norm}")
        X, y, mag = synth.logreg_skewed(4, 512, 512, c_sk=1.0 / 16, c_th=0.6, seed=11, device=DEV)
        assert 0.5 < float((mag < 0.6 / 16 + 1e-6).float().mean()) < 0.7          # about c_th of the columns shrunk
        if norm == B.NORM_MEAN:
            continue                                                               # covered by the codec tests
        first, last = _dense_case(M=4, n=512, d=512, batch=8, bits=bits, norm=norm, T=60, seed=11, lr=0.1,
                                  l2=0.01, data=(X, y), full_gradient_reference=True)
        assert last < first - 0.02


def test_free_running_trajectories_decrease_the_loss_alike():
    # no teacher forcing: the library and the oracle each run 100 iterations on their own iterates; the
    # trajectories may part after the first rounding decision that flips, the loss curves may not
    M, n, d, batch, seed, T = 4, 2000, 1000, 64, 0, 100
    say("free-running dense logistic d=1000 M=4 B=64 T=100")
    X, y, _ = synth.logreg_dense(M, n, d, seed=seed, device=DEV)
    ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=seed, lr=0.1, batch=batch, problem=B.PROB_LOGREG_DENSE)
    ctx.set_logreg_dense([X[m] for m in range(M)], [y[m] for m in range(M)])
    cfg = oracle_cfg(ctx)
    Xh, yh = X.cpu().numpy(), y.cpu().numpy()

    def loss(wv):
        z = Xh.reshape(-1, d).astype(np.float64) @ np.asarray(wv, dtype=np.float64)
        return float(np.mean(np.logaddexp(0, z) - yh.reshape(-1) * z))

    w = torch.zeros(d, device=DEV)
    gref = torch.zeros(d, device=DEV)
    buf = buffers(ctx)
    wo, ro = np.zeros(d, np.float32), np.zeros(d, np.float32)
    curve_gpu, curve_cpu = [], []
    for it in range(T):
        ctx.step(it, w, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
        ids = [O.minibatch_indices(seed, it, m, batch, n) for m in range(M)]
        go = np.stack([O.grad_logreg_dense(Xh[m], yh[m], wo, ids[m]) for m in range(M)]).astype(np.float32)
        wo, ro, _, _, _ = O.step(cfg, it, wo, ro, go)
        if it % 10 == 9:
            torch.cuda.synchronize()
            curve_gpu.append(loss(w.cpu().numpy()))
            curve_cpu.append(loss(wo))
    ctx.close()
    assert curve_gpu[-1] < np.log(2) - 0.02 and curve_cpu[-1] < np.log(2) - 0.02
    assert max(abs(a - b) for a, b in zip(curve_gpu, curve_cpu)) < 5e-3, (curve_gpu, curve_cpu)


def test_dense_logistic_quotient_two_bit_scaled():
    # shape of the 16-worker quotient configuration, scaled to d=2^10, 2^12 rows per worker
    # all 200 iterations
    say("dense logistic quotient d=1024 M=16 n=4096 B=256 T=200")
    _dense_case(M=16, n=4096, d=1024, batch=256, bits=2, norm=B.NORM_QUOT, T=200, seed=3)


def test_dense_logistic_odd_dimension_four_bit_l2_period():
    say("dense logistic d=1003 (scalar path) M=3 B=300 4-bit l2 K=4")
    _dense_case(M=3, n=500, d=1003, batch=300, bits=4, norm=B.NORM_SUB, T=9, seed=5, l2=0.01, ref_period=4)


def test_dense_logistic_few_columns_ragged_minibatch_over_one_staging_chunk():
    # few columns (the gradient kernel deals the minibatch rows to row groups), minibatch 301: more than
    # one staging chunk of 256 rows and not a multiple of the number of row groups
    say("dense logistic d=1000 M=2 n=400 B=301 T=6")
    _dense_case(M=2, n=400, d=1000, batch=301, bits=2, norm=B.NORM_SUB, T=6, seed=9, l2=0.001)


def test_dense_logistic_wide_rows_first_iterations():
    # d = 2^16, 16 workers, minibatch 256 as in the large dense configuration (rows of 256 KiB), shards of
    # 512 rows (a step only touches minibatch rows): first 3 iterations
    say("dense logistic d=65536 M=16 n=512 B=256 T=3")
    _dense_case(M=16, n=512, d=65536, batch=256, bits=2, norm=B.NORM_QUOT, T=3, seed=7)


@pytest.mark.parametrize("d,M,batch", [(16384, 8, 64), (16388, 4, 130), (32768, 3, 200), (20000, 16, 33), (32764, 2, 256)])
def test_dense_logistic_rows_kept_on_chip(d, M, batch):
    # 16 K to 64 K columns and at least 512 minibatch rows in all: the gradient kernel that reads every
    # minibatch row once and keeps it in LDS and registers between the dot product and the accumulation;
    # full and ragged widths of both narrower variants (the widest, d = 2^16, is the test above), worker
    # counts that give 32 to 128 workgroups per worker, row counts the workgroups do not divide
    say(f"dense logistic, rows kept on chip: d={d} M={M} B={batch}")
    _dense_case(M=M, n=300, d=d, batch=batch, bits=4, norm=B.NORM_SUB, T=3, seed=d % 97 + M, l2=0.001)


def test_rosenbrock_chain_first_iterations_at_full_shape():
    # d = 2^20, M = 8, noise N(0, 0.01), ternary, subtraction; reference refreshed every 16 iterations
    # ("Nonconvex Problems"): the first 48 of the 500 iterations, three refreshes
    d, M, seed = 1 << 20, 8, 1
    say(f"rosenbrock d={d} M={M} K=16, 48 iterations")
    ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=seed, lr=1e-5, ref_period=16, problem=B.PROB_ROSENBROCK)
    cfg = oracle_cfg(ctx)
    x = synth.rosenbrock_start(d, seed, device=DEV)
    gref = torch.zeros(d, device=DEV)
    buf = buffers(ctx)
    refreshes = 0
    for it in range(48):
        noise = synth.gradient_noise(M, d, seed, it, variance=0.01, device=DEV)
        ctx.set_noise(noise)
        nh = noise.cpu().numpy()
        before = gref.clone()
        _teacher_forced_step(ctx, cfg, it, x, gref, buf,
                             lambda w0: np.stack([O.grad_rosenbrock(w0, nh[m]) for m in range(M)]), grad_exact=True)
        changed = not torch.equal(before, gref)
        assert changed == ((it + 1) % 16 == 0), f"it={it}: the reference changes on refresh iterations only"
        refreshes += changed
        if it % 8 == 7:
            say(f"  it={it} done")
    assert refreshes == 3
    ctx.close()


def test_rosenbrock_noise_generated_on_the_device():
    # N(0, 0.01) noise from the library's own Box-Muller (binary32) against the float64 oracle: the
    # gradient within a few units in the last place of the noise, everything downstream bit for bit
    for d, M, bits in [(1 << 16, 8, 2), (4099, 3, 4), (6, 2, 2)]:
        say(f"rosenbrock with device noise d={d} M={M}")
        seed, variance = (5 << 32) | 77, 0.01
        ctx = make_ctx(d, M, bits, B.NORM_SUB, seed=seed, lr=1e-5, ref_period=2, problem=B.PROB_ROSENBROCK)
        ctx.set_noise(torch.ones((M, d), device=DEV))       # replaced by the generator below
        ctx.set_noise_variance(variance)
        cfg = oracle_cfg(ctx)
        x = synth.rosenbrock_start(d, 4, device=DEV)
        gref = torch.zeros(d, device=DEV)
        buf = buffers(ctx)
        for it in range(3):
            w0, r0 = x.cpu().numpy(), gref.cpu().numpy()
            ctx.step(it, x, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
            torch.cuda.synchronize()
            gh = buf["g"].cpu().numpy()
            base = O.grad_rosenbrock(w0).astype(np.float64)
            for m in range(M):
                noise = O.gaussian_noise(seed, it, m, d, variance)
                want = base + noise
                err = np.abs(gh[m] - want)
                assert np.all(err <= 2.0 ** -24 * np.abs(want) + 8 * 2.0 ** -24 * np.abs(noise) + 1e-30), \
                    f"it={it} m={m}: worst {err.max()}"
            w1, r1, c1, s1, v1 = O.step(cfg, it, w0, r0, gh)
            assert np.array_equal(buf["scales"].cpu().numpy(), s1) and np.array_equal(u32(buf["codes"]), c1)
            assert np.array_equal(buf["vbar"].cpu().numpy(), v1) and np.array_equal(x.cpu().numpy(), w1)
            assert np.array_equal(gref.cpu().numpy(), r1)
        # local_grad alone gives the same gradient as the fused step did (same iteration, same iterate)
        g2 = torch.empty_like(buf["g"])
        xs = torch.from_numpy(w0).to(DEV)
        ctx.local_grad(2, xs, g2)
        torch.cuda.synchronize()
        assert torch.equal(g2, buf["g"])
        # switching the generator off gives the noiseless gradient
        ctx.set_noise_variance(0.0)
        ctx.local_grad(2, xs, g2)
        torch.cuda.synchronize()
        assert np.array_equal(g2[0].cpu().numpy(), O.grad_rosenbrock(w0))
        ctx.close()


def test_rosenbrock_small_and_ragged():
    for d, M in [(1, 2), (2, 1), (3, 3), (1001, 2), (4097, 2)]:
        say(f"rosenbrock d={d} M={M}")
        ctx = make_ctx(d, M, 4, B.NORM_SUB, seed=2, lr=1e-5, problem=B.PROB_ROSENBROCK)
        cfg = oracle_cfg(ctx)
        x = synth.rosenbrock_start(d, 3, device=DEV)
        gref = torch.zeros(d, device=DEV)
        buf = buffers(ctx)
        for it in range(3):
            if it == 2:
                nh = np.zeros((M, d), dtype=np.float32)
                ctx.set_noise(None)
            else:
                noise = synth.gradient_noise(M, d, 2, it, device=DEV)
                ctx.set_noise(noise)
                nh = noise.cpu().numpy()
            _teacher_forced_step(ctx, cfg, it, x, gref, buf,
                                 lambda w0: np.stack([O.grad_rosenbrock(w0, nh[m]) for m in range(M)]),
                                 grad_exact=True)
        ctx.close()


def test_every_normalisation_through_the_fused_step():
    # tng_step takes the scale from the gradient kernel's own partial maxima where it can: every
    # normalisation and both scales, vector (d = 8192) and scalar (d = 8191) paths, against the oracle
    M, seed = 3, 21
    cases = [(n, B.SCALE_MAX) for n in (B.NORM_NONE, B.NORM_SUB, B.NORM_QUOT, B.NORM_COMB, B.NORM_MEAN)]
    cases += [(B.NORM_SUB, B.SCALE_L2), (B.NORM_MEAN, B.SCALE_L2)]
    for d in (8192, 8191):
        for norm, scale in cases:
            say(f"fused step d={d} norm={norm} scale={scale}")
            ctx = make_ctx(d, M, 4, norm, seed=seed, lr=1e-5, problem=B.PROB_ROSENBROCK, scale=scale)
            cfg = oracle_cfg(ctx)
            x = synth.rosenbrock_start(d, seed, device=DEV)
            gref = synth.rosenbrock_start(d, seed + 1, device=DEV) * 100.0
            gref2 = torch.rand(d, device=DEV, generator=torch.Generator(device=DEV).manual_seed(3)) + 0.5
            if norm == B.NORM_COMB:
                ctx.set_second_reference(gref2)
            if norm == B.NORM_MEAN:
                means = torch.zeros(M, device=DEV)
                ctx.set_worker_means(means)
            buf = buffers(ctx)
            for it in range(2):
                noise = synth.gradient_noise(M, d, seed, it, device=DEV)
                ctx.set_noise(noise)
                w0, r0 = x.cpu().numpy(), gref.cpu().numpy()
                ctx.step(it, x, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
                torch.cuda.synchronize()
                gh = buf["g"].cpu().numpy()
                nh = noise.cpu().numpy()
                assert np.array_equal(gh, np.stack([O.grad_rosenbrock(w0, nh[m]) for m in range(M)]))
                w1, r1, c1, s1, v1 = O.step(cfg, it, w0, r0, gh, gref2.cpu().numpy())
                assert np.array_equal(buf["scales"].cpu().numpy(), s1), "scales from the fused partial maxima"
                if norm == B.NORM_MEAN:
                    assert np.array_equal(means.cpu().numpy(), O.worker_means(gh))
                assert_row_sums_are_the_exact_ones(cfg, gh, r0, gref2.cpu().numpy(),
                                                   means.cpu().numpy() if norm == B.NORM_MEAN else None, s1)
                assert np.array_equal(u32(buf["codes"]), c1) and np.array_equal(buf["vbar"].cpu().numpy(), v1)
                assert np.array_equal(x.cpu().numpy(), w1) and np.array_equal(gref.cpu().numpy(), r1)
            ctx.close()


@pytest.mark.parametrize("use_index,bits,norm,T,pairs", [(False, 4, B.NORM_SUB, 6, False), (True, 4, B.NORM_SUB, 100, True),
                                                         (True, 4, B.NORM_SUB, 6, False), (False, 4, B.NORM_SUB, 6, True),
                                                         (True, 2, B.NORM_QUOT, 6, True), (True, 4, B.NORM_NONE, 6, False)])
def test_csr_logistic_scaled(use_index, bits, norm, T, pairs):
    # shape of the sparse configuration scaled to d=2^16, M=8, 0.1% density, 4-bit, subtraction, with the
    # prebuilt per-row tile index: all 100 iterations; without the index, and the other normalisations
    # through the scale pass that rides along with the gradient kernel's write-out: the first 6
    M, n, d, batch, seed = 8, 1024, 1 << 16, 128, 4
    nnz_row = round(1e-3 * d)
    say(f"csr logistic d={d} M={M} nnz/row={nnz_row} index={use_index} bits={bits} norm={norm} pairs={pairs}")
    shards, _ = synth.logreg_csr(M, n, d, nnz_row, seed, device=DEV)
    ctx = make_ctx(d, M, bits, norm, seed=seed, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR)
    set_csr(ctx, shards, pairs)
    if use_index:
        ctx.build_csr_index()
    cfg = oracle_cfg(ctx)
    host = [tuple(t.cpu().numpy() for t in s) for s in shards]
    w = torch.zeros(d, device=DEV)
    gref = torch.zeros(d, device=DEV)
    if norm == B.NORM_QUOT:      # a reference that is not zero everywhere, so that most quotients are finite
        gref = 1e-3 * torch.randn(d, device=DEV, generator=torch.Generator(device=DEV).manual_seed(9))
        gref[::7] = 0.0
    buf = buffers(ctx)
    for it in range(T):
        def grad_ref(w0, it=it):
            ids = [O.minibatch_indices(seed, it, m, batch, n) for m in range(M)]
            ref = np.stack([O.grad_logreg_csr(host[m][0], host[m][1], host[m][2], host[m][3], w0, ids[m], d)
                            for m in range(M)])
            cond = np.stack([logistic_condition_csr(*host[m], w0, ids[m], d) for m in range(M)])
            return ref, cond
        _teacher_forced_step(ctx, cfg, it, w, gref, buf, grad_ref)
        if it % 20 == 19:
            say(f"  it={it} done")
    ctx.close()


def test_csr_logistic_full_dimension_first_step():
    # the sparse configuration's per-worker shape in full: d = 2^24, 16 777 entries per row, minibatch 512,
    # 4-bit codes, subtraction -- with 4 workers and 512-row shards (a step only touches minibatch rows);
    # gradient against the float64 oracle norm-wise, everything downstream bit for bit
    M, n, d, batch, seed = 4, 512, 1 << 24, 512, 6
    nnz_row = round(1e-3 * d)
    say(f"csr logistic full dimension d={d} M={M} nnz/row={nnz_row} B={batch}")
    shards, _ = synth.logreg_csr(M, n, d, nnz_row, seed, device=DEV)
    ctx = make_ctx(d, M, 4, B.NORM_SUB, seed=seed, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR)
    ctx.set_logreg_csr([s[0] for s in shards], [s[1] for s in shards], [s[2] for s in shards], [s[3] for s in shards])
    ctx.build_csr_index()
    cfg = oracle_cfg(ctx)
    host = [tuple(t.cpu().numpy() for t in s) for s in shards]
    w = 0.01 * torch.randn(d, device=DEV, generator=torch.Generator(device=DEV).manual_seed(1))
    gref = torch.zeros(d, device=DEV)
    buf = buffers(ctx)
    w0, r0 = w.cpu().numpy(), gref.cpu().numpy()
    ctx.step(0, w, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
    torch.cuda.synchronize()
    gh = buf["g"].cpu().numpy()
    for m in range(M):
        ids = O.minibatch_indices(seed, 0, m, batch, n)
        ref = O.grad_logreg_csr(host[m][0], host[m][1], host[m][2], host[m][3], w0, ids, d)
        err = gh[m].astype(np.float64) - ref
        assert np.linalg.norm(err) <= 1e-5 * np.linalg.norm(ref), f"worker {m}: gradient (2-norm)"
        assert np.abs(err).max() <= 1e-5 * np.abs(ref).max(), f"worker {m}: gradient (max-norm)"
    w1, r1, c1, s1, v1 = O.step(cfg, 0, w0, r0, gh)
    assert np.array_equal(buf["scales"].cpu().numpy(), s1) and np.array_equal(u32(buf["codes"]), c1)
    assert np.array_equal(buf["vbar"].cpu().numpy(), v1) and np.array_equal(w.cpu().numpy(), w1)
    assert np.array_equal(gref.cpu().numpy(), r1)
    ctx.close()


def _ragged_csr(M, n, d, lengths_fn, seed):
    """CSR shards with a different number of stored entries per row (sorted distinct columns)."""
    gen = torch.Generator(device="cpu").manual_seed(seed)
    shards = []
    for m in range(M):
        lens = [int(lengths_fn(m, i)) for i in range(n)]
        rowptr = torch.zeros(n + 1, dtype=torch.int64)
        rowptr[1:] = torch.cumsum(torch.tensor(lens, dtype=torch.int64), 0)
        cols = [torch.sort(torch.randperm(d, generator=gen)[:k])[0] for k in lens]
        col = torch.cat(cols).to(torch.int32) if sum(lens) else torch.zeros(0, dtype=torch.int32)
        val = torch.randn(int(rowptr[-1]), generator=gen)
        y = (torch.rand(n, generator=gen) < 0.5).float()
        shards.append((rowptr.to(DEV), torch.cat([col, torch.zeros(1, dtype=torch.int32)]).to(DEV)[:max(len(col), 1)],
                       torch.cat([val, torch.zeros(1)]).to(DEV)[:max(len(val), 1)], y.to(DEV)))
    return shards


@pytest.mark.parametrize("pairs", [False, True])
@pytest.mark.parametrize("use_index", [False, True])
@pytest.mark.parametrize("case", ["ragged", "tiny_d", "odd_d_many_rows", "dense_rows", "one_entry"])
def test_csr_logistic_edge_cases(case, use_index, pairs):
    if case == "ragged":        # empty rows, one-entry rows, rows longer than a lane group inside one tile
        M, n, d, batch = 3, 40, (1 << 15) + 24, 33
        lens = lambda m, i: [0, 1, 2, 700, 33, 5000][(i + m) % 6]
    elif case == "tiny_d":      # d smaller than a tile, a single partial tile
        M, n, d, batch = 2, 30, 100, 7
        lens = lambda m, i: (i * 7 + m) % 60
    elif case == "odd_d_many_rows":   # more minibatch rows than one staging trip, d not a multiple of 4 (scalar codec)
        M, n, d, batch = 2, 900, 3 * (1 << 14) + 1, 1100
        lens = lambda m, i: 20 + (i % 50)
    elif case == "one_entry":   # a worker that stores one entry in all; another whose arrays end on an odd segment
        M, n, d, batch = 2, 5, 1 << 15, 9
        lens = lambda m, i: [[0, 0, 1, 0, 0], [3, 0, 5, 0, 7]][m][i]
    else:                       # nearly dense rows: many entries per (row, tile) segment
        M, n, d, batch = 2, 12, 1 << 14, 12
        lens = lambda m, i: (1 << 14) - 1 - i
    say(f"csr edge case {case}: d={d} M={M} n={n} B={batch} index={use_index} pairs={pairs}")
    seed = 11
    shards = _ragged_csr(M, n, d, lens, seed)
    ctx = make_ctx(d, M, 4, B.NORM_SUB, seed=seed, lr=0.1, l2=0.001, batch=batch, problem=B.PROB_LOGREG_CSR)
    set_csr(ctx, shards, pairs)
    if use_index:
        ctx.build_csr_index()
    cfg = oracle_cfg(ctx)
    host = [tuple(t.cpu().numpy() for t in s) for s in shards]
    w = 0.1 * torch.randn(d, device=DEV)
    gref = torch.zeros(d, device=DEV)
    buf = buffers(ctx)
    for it in range(2):
        def grad_ref(w0, it=it):
            ids = [O.minibatch_indices(seed, it, m, batch, n) for m in range(M)]
            ref = np.stack([O.grad_logreg_csr(host[m][0], host[m][1], host[m][2], host[m][3], w0, ids[m], d, 0.001)
                            for m in range(M)])
            cond = np.zeros((M, d))
            for m in range(M):
                Xb = np.zeros((batch, d), dtype=np.float32)
                for j, i in enumerate(ids[m]):
                    a, b = host[m][0][i], host[m][0][i + 1]
                    Xb[j, host[m][1][a:b]] = host[m][2][a:b]
                cond[m] = logistic_condition(Xb, host[m][3][ids[m]], w0, 0.001)
            return ref, cond
        _teacher_forced_step(ctx, cfg, it, w, gref, buf, grad_ref)
    ctx.close()


@pytest.mark.parametrize("pairs", [False, True])
@pytest.mark.parametrize("norm", [B.NORM_SUB, B.NORM_QUOT, B.NORM_NONE, B.NORM_COMB])
def test_csr_logistic_pipelined_gradient_pass(norm, pairs):
    # full tiles, no l2 term, minibatch <= 512: the gradient pass that keeps a workgroup on a run of 16
    # consecutive tiles (next tile's entries requested before this tile is written out), with the scale pass
    # fused for each normalisation.  20 tiles: one full run and one of 4; empty rows, one-entry rows and rows
    # with far more entries per tile than a lane group holds; fewer minibatch rows than staging slots
    M, n, d, batch, seed = 3, 60, 20 << 14, 130, 23
    lens = lambda m, i: [0, 1, 300, 9000, 40, 2500][(i + m) % 6]
    say(f"csr pipelined gradient pass d={d} M={M} B={batch} norm={norm} pairs={pairs}")
    shards = _ragged_csr(M, n, d, lens, seed)
    ctx = make_ctx(d, M, 4, norm, seed=seed, lr=0.1, batch=batch, problem=B.PROB_LOGREG_CSR)
    set_csr(ctx, shards, pairs)
    ctx.build_csr_index()
    cfg = oracle_cfg(ctx)
    host = [tuple(t.cpu().numpy() for t in s) for s in shards]
    gen = torch.Generator(device=DEV).manual_seed(seed)
    w = 0.1 * torch.randn(d, device=DEV, generator=gen)
    gref = 1e-3 * torch.randn(d, device=DEV, generator=gen)
    gref[::5] = 0.0
    gref2 = torch.rand(d, device=DEV, generator=gen) + 0.5
    if norm == B.NORM_COMB:
        ctx.set_second_reference(gref2)
    buf = buffers(ctx)
    for it in range(2):
        w0, r0 = w.cpu().numpy(), gref.cpu().numpy()
        ctx.step(it, w, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
        torch.cuda.synchronize()
        gh = buf["g"].cpu().numpy()
        for m in range(M):
            ids = O.minibatch_indices(seed, it, m, batch, n)
            ref = O.grad_logreg_csr(*host[m], w0, ids, d)
            assert grad_close(gh[m], ref, logistic_condition_csr(*host[m], w0, ids, d)), f"it={it} m={m}: local gradient"
        w1, r1, c1, s1, v1 = O.step(cfg, it, w0, r0, gh, gref2.cpu().numpy())
        assert np.array_equal(buf["scales"].cpu().numpy(), s1), f"it={it}: scales from the fused partial maxima"
        assert np.array_equal(u32(buf["codes"]), c1) and np.array_equal(buf["vbar"].cpu().numpy(), v1)
        assert np.array_equal(w.cpu().numpy(), w1) and np.array_equal(gref.cpu().numpy(), r1)
    ctx.close()


def test_csr_tile_index_changes_nothing_but_the_speed():
    # same shards, same iterate: the gradient with the prebuilt index equals the one without, bit for bit;
    # shards with different row counts; setting new shards drops the index
    M, d, batch, seed = 3, (1 << 16) + 40, 50, 5
    shards = [synth.logreg_csr(1, n, d, 70, seed + n, device=DEV)[0][0] for n in (60, 200, 33)]
    ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=seed, batch=batch, problem=B.PROB_LOGREG_CSR)
    parts = [[s[k] for s in shards] for k in range(4)]
    ctx.set_logreg_csr(*parts)
    w = 0.05 * torch.randn(d, device=DEV)
    g0, g1, g2 = (torch.empty((M, d), device=DEV) for _ in range(3))
    ctx.local_grad(3, w, g0)
    # an index buffer that is too small or misaligned is refused before anything is built
    import ctypes
    rows = (ctypes.c_uint64 * M)(*ctx.n_rows)
    need = B.lib().tng_csr_index_bytes(ctypes.byref(ctx.cfg), rows)
    small = torch.empty(need, dtype=torch.uint8, device=DEV)
    assert B.lib().tng_set_csr_index(ctx.handle, ctypes.c_void_p(small.data_ptr()), need - 1) == B.TNG_ERR_WORKSPACE
    assert B.lib().tng_set_csr_index(ctx.handle, ctypes.c_void_p(small.data_ptr() + 8), need) == B.TNG_ERR_INVALID_ARG
    ctx.build_csr_index()
    ctx.local_grad(3, w, g1)
    ctx.set_logreg_csr(*parts)          # index dropped: back to the pass over the column ids
    ctx.local_grad(3, w, g2)
    torch.cuda.synchronize()
    assert torch.equal(g0, g1) and torch.equal(g0, g2)
    # the same shards as (column, value) pairs: the same gradient, bit for bit, with and without the index
    # (per row and tile the same products are added in the same order)
    g3, g4 = torch.empty((M, d), device=DEV), torch.empty((M, d), device=DEV)
    set_csr(ctx, shards, pairs=True)
    ctx.local_grad(3, w, g3)
    ctx.build_csr_index()
    ctx.local_grad(3, w, g4)
    torch.cuda.synchronize()
    assert torch.equal(g0, g3) and torch.equal(g0, g4)
    ctx.close()


def test_csr_validation_finds_what_the_gradient_kernels_cannot_check():
    # tng_validate_csr: sound shards pass; a column id at d, a negative one, columns out of order, equal
    # neighbours, row pointers that decrease or run past the stored entries are each reported (the pass over
    # the column ids only runs when the row pointers are sound, so it never reads out of range)
    M, n, d, nnz_row, seed = 3, 50, (1 << 15) + 9, 40, 17
    shards, _ = synth.logreg_csr(M, n, d, nnz_row, seed, device=DEV)
    ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=seed, batch=8, problem=B.PROB_LOGREG_CSR)

    def verdict(mutate=None, pairs=False):
        parts = [[s[k].clone() for s in shards] for k in range(4)]
        if mutate is not None:
            mutate(parts)
        set_csr(ctx, list(zip(*parts)), pairs)
        try:
            ctx.validate_csr()
            return B.TNG_OK
        except B.TngError as e:
            return e.status

    def set_col(parts, m, pos, value):
        parts[1][m][pos] = value

    def set_rowptr(parts, m, pos, value):
        parts[0][m][pos] = value

    assert verdict() == B.TNG_OK
    assert verdict(lambda p: set_col(p, 1, 7 * nnz_row + nnz_row - 1, d)) == B.TNG_ERR_INVALID_ARG       # column == d
    assert verdict(lambda p: set_col(p, 0, 0, -1)) == B.TNG_ERR_INVALID_ARG                             # negative column
    first, second = int(shards[2][1][3 * nnz_row + 5]), int(shards[2][1][3 * nnz_row + 6])
    assert verdict(lambda p: (set_col(p, 2, 3 * nnz_row + 5, second), set_col(p, 2, 3 * nnz_row + 6, first))) \
        == B.TNG_ERR_INVALID_ARG                                                                        # out of order
    assert verdict(lambda p: set_col(p, 2, 3 * nnz_row + 6, first)) == B.TNG_ERR_INVALID_ARG             # equal neighbours
    assert verdict(lambda p: set_rowptr(p, 1, 10, int(shards[1][0][9]) - 1)) == B.TNG_ERR_INVALID_ARG    # decreasing
    assert verdict(lambda p: set_rowptr(p, 0, n, n * nnz_row + 1)) == B.TNG_ERR_INVALID_ARG              # past the entries
    assert verdict(lambda p: set_rowptr(p, 0, 0, -3)) == B.TNG_ERR_INVALID_ARG                           # negative start
    assert verdict() == B.TNG_OK
    # the same checks read the (column, value) pair layout
    assert verdict(pairs=True) == B.TNG_OK
    assert verdict(lambda p: set_col(p, 1, 7 * nnz_row + nnz_row - 1, d), pairs=True) == B.TNG_ERR_INVALID_ARG
    assert verdict(lambda p: set_col(p, 2, 3 * nnz_row + 6, first), pairs=True) == B.TNG_ERR_INVALID_ARG
    assert verdict(lambda p: set_rowptr(p, 0, n, n * nnz_row + 1), pairs=True) == B.TNG_ERR_INVALID_ARG
    ctx.close()


def test_external_gradients_and_separate_calls_equal_the_fused_step():
    d, M = 4096 * 3 + 4, 4
    g, gref0 = synth.codec_inputs(M, d, 9, device=DEV)
    for norm in (B.NORM_SUB, B.NORM_QUOT):
        ctx = make_ctx(d, M, 4, norm, seed=6, lr=0.05, ref_period=1, problem=B.PROB_EXTERNAL)
        w = torch.randn(d, device=DEV)
        w_a, w_b = w.clone(), w.clone()
        ref_a, ref_b = gref0.clone(), gref0.clone()
        a, b = buffers(ctx), buffers(ctx)
        a["g"].copy_(g)
        ctx.step(0, w_a, ref_a, a["g"], a["codes"], a["scales"], a["vbar"])
        ctx.normalize_encode(0, g, ref_b, b["codes"], b["scales"])
        ctx.decode_aggregate(b["codes"], b["scales"], ref_b, b["vbar"])
        ctx.update_reference(0, b["vbar"], ref_b)
        torch.cuda.synchronize()
        assert torch.equal(a["codes"], b["codes"]) and torch.equal(a["vbar"], b["vbar"])
        assert torch.equal(ref_a, ref_b) and torch.equal(ref_a, a["vbar"])
        cfg = oracle_cfg(ctx)
        assert np.array_equal(w_a.cpu().numpy(), O.update_iterate(w.cpu().numpy(), a["vbar"].cpu().numpy(), cfg.lr))
        ctx.close()


def test_window_average_reference():
    # reference = mean of the last 3 decoded averages, refreshed every 2 iterations
    for d, M, W, K in [(5000, 3, 3, 2), (4099, 2, 4, 1), (1 << 16, 4, 2, 3), (1000, 4, 3, 2)]:   # the last: single-workgroup path
        say(f"window-average reference d={d} M={M} window={W} period={K}")
        ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=5, lr=1e-5, ref_policy=B.REF_WINDOW_AVG, ref_period=K, ref_window=W,
                       problem=B.PROB_ROSENBROCK)
        cfg = oracle_cfg(ctx)
        history_dev = torch.zeros((W, d), device=DEV)
        ctx.set_reference_history(history_dev)
        x = synth.rosenbrock_start(d, 5, device=DEV)
        gref = torch.zeros(d, device=DEV)
        buf = buffers(ctx)
        past = []
        for it in range(9):
            noise = synth.gradient_noise(M, d, 5, it, device=DEV)
            ctx.set_noise(noise)
            w0, r0 = x.cpu().numpy(), gref.cpu().numpy()
            ctx.step(it, x, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
            torch.cuda.synchronize()
            gh = buf["g"].cpu().numpy()
            w1, r1, c1, s1, v1 = O.step(cfg, it, w0, r0, gh, history=past)
            assert np.array_equal(u32(buf["codes"]), c1) and np.array_equal(buf["vbar"].cpu().numpy(), v1)
            assert np.array_equal(x.cpu().numpy(), w1), f"it={it}: iterate"
            assert np.array_equal(gref.cpu().numpy(), r1), f"it={it}: window-average reference"
            past.append(v1)
            assert np.array_equal(history_dev[it % W].cpu().numpy(), v1)
        # the separate call does the same as the fused step
        gref2 = torch.zeros(d, device=DEV)
        hist2 = torch.zeros((W, d), device=DEV)
        ctx.set_reference_history(hist2)
        for it in range(9):
            ctx.update_reference(it, torch.from_numpy(past[it]).to(DEV), gref2)
        torch.cuda.synchronize()
        assert torch.equal(gref2, gref) and torch.equal(hist2, history_dev)
        ctx.close()


def test_resume_from_saved_state_reproduces_the_run():
    # the RNG is counter based: (w, g~, iteration) is the whole state
    d, M, seed = 4096, 4, 13
    ctxs = [make_ctx(d, M, 2, B.NORM_SUB, seed=seed, lr=1e-5, problem=B.PROB_ROSENBROCK) for _ in range(2)]
    x0 = synth.rosenbrock_start(d, seed, device=DEV)
    runs = []
    for which, ctx in enumerate(ctxs):
        x, gref, buf = x0.clone(), torch.zeros(d, device=DEV), buffers(ctx)
        for it in range(10):
            if which == 1 and it == 5:            # "checkpoint": drop the context, keep (x, gref, it)
                ctx.close()
                ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=seed, lr=1e-5, problem=B.PROB_ROSENBROCK)
                x, gref = x.clone(), gref.clone()
            noise = synth.gradient_noise(M, d, seed, it, device=DEV)
            ctx.set_noise(noise)
            ctx.step(it, x, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
            torch.cuda.synchronize()
        runs.append((x.clone(), gref.clone(), buf["codes"].clone()))
        ctx.close()
    for a, b in zip(runs[0], runs[1]):
        assert torch.equal(a, b)


def test_tiny_problem_one_workgroup_equals_separate_passes():
    # d <= 1024 (a multiple of 4), M <= 16: everything after the gradient is one single-workgroup launch,
    # unless timing events are being recorded -- they mark the separate passes, which then run instead.
    # Both ways give the same bits (each is also compared with the oracle by the other tests).
    import bench
    cases = [(1000, 4, 2, B.NORM_SUB), (1024, 16, 4, B.NORM_QUOT), (36, 3, 2, B.NORM_COMB), (512, 9, 4, B.NORM_NONE),
             (4, 1, 2, B.NORM_SUB)]
    for d, M, bits, norm in cases:
        say(f"one workgroup against separate passes d={d} M={M} bits={bits} norm={norm}")
        outs = []
        for separate in (False, True):
            ctx = make_ctx(d, M, bits, norm, seed=13, lr=1e-5, ref_period=2, problem=B.PROB_ROSENBROCK)
            ev = None
            if separate:
                ev = bench.HipEvents(5)
                ctx.set_profile_events(ev.ev, 1)
            if norm == B.NORM_COMB:
                gref2 = torch.rand(d, generator=torch.Generator(device=DEV).manual_seed(3), device=DEV) + 0.5
                ctx.set_second_reference(gref2)
            x = synth.rosenbrock_start(d, 6, device=DEV)
            gref = 0.1 * synth.rosenbrock_start(d, 7, device=DEV)
            buf = buffers(ctx)
            trace = []
            for it in range(3):
                ctx.set_noise(synth.gradient_noise(M, d, 5, it, device=DEV))
                ctx.step(it, x, gref, buf["g"], buf["codes"], buf["scales"], buf["vbar"])
                torch.cuda.synchronize()
                trace.append([t.clone() for t in (buf["g"], buf["codes"], buf["scales"], buf["vbar"], x, gref)])
            # the encoder on its own takes the same route
            codes2, scales2 = torch.empty_like(buf["codes"]), torch.empty_like(buf["scales"])
            ctx.normalize_encode(7, buf["g"], gref, codes2, scales2)
            torch.cuda.synchronize()
            trace.append([codes2, scales2])
            if ev is not None:
                ctx.set_profile_events(None, 0)
                ev.destroy()
            ctx.close()
            outs.append(trace)
        for a, b in zip(outs[0], outs[1]):
            for ta, tb in zip(a, b):
                assert torch.equal(ta, tb)
