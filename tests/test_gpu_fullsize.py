"""Parity at the full size of the encode/decode benchmark (M = 8, d = 2^27), in the launch
configuration bench.py times.  The four variants of the benchmark (ternary and 4-bit codes, Eq. 1 and
Eq. 2): EVERY packed word, scale and decoded average of one whole repetition against the oracle, which
works through the 2^30 elements in blocks shared between host threads.  The other variants (mean
reference, l2 scale) and large ragged rows: scales exactly (full pass on the host), packed codes and
decoded averages on sampled windows."""
import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, assert_row_sums_are_the_exact_ones, buffers, make_ctx, oracle_cfg, say, u32
from paper_1901_08227_amd import binding as B
from paper_1901_08227_amd import synth

pytestmark = pytest.mark.gpu

D_FULL, M_FULL = 1 << 27, 8


@pytest.fixture(scope="module")
def full_inputs():
    say("generating M=8 x d=2^27 codec inputs on the device")
    g, gref = synth.codec_inputs(M_FULL, D_FULL, seed=1, device=DEV)
    torch.cuda.synchronize()
    return g, gref


@pytest.mark.parametrize("bits,norm", [(2, B.NORM_SUB), (4, B.NORM_SUB), (2, B.NORM_QUOT), (4, B.NORM_QUOT)])
def test_full_size_every_element(full_inputs, bits, norm):
    g, gref = full_inputs
    d, M, it = D_FULL, M_FULL, 2
    ctx = make_ctx(d, M, bits, norm, seed=1)
    cfg = oracle_cfg(ctx)
    buf = buffers(ctx)
    say(f"full size, every element: bits={bits} norm={norm}: encode + decode on the GPU")
    ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
    ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
    torch.cuda.synchronize()
    ctx.close()
    gh, rh = g.cpu().numpy(), gref.cpu().numpy()
    got_codes, got_scales, got_vbar = u32(buf["codes"]), buf["scales"].cpu().numpy(), buf["vbar"].cpu().numpy()
    del buf
    block, per = 1 << 22, 32 // bits
    starts = range(0, d, block)
    threads = max(2, min(16, os.cpu_count() or 2))
    with ThreadPoolExecutor(max_workers=threads) as pool:
        # R_m: the largest magnitude of the normalised row is the largest of its blocks' (a maximum does not
        # depend on how it is split; a block below the smallest normal number reports 0 and cannot win)
        def block_scale(task):
            m, s = task
            return m, O.scale_of(O.normalize(gh[m, s:s + block], rh[s:s + block], norm, cfg.quot_eps))
        scales = np.zeros(M, dtype=np.float32)
        for m, r in pool.map(block_scale, [(m, s) for m in range(M) for s in starts]):
            scales[m] = max(scales[m], r)
        assert np.array_equal(got_scales, scales), "scales"
        say("  scales equal; codes of all 2^30 elements")

        def block_codes(task):
            m, s = task
            v = O.normalize(gh[m, s:s + block], rh[s:s + block], norm, cfg.quot_eps)
            u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, block, first=s))
            level, neg = O.quantize(v, scales[m], bits, u)
            return m, s, np.array_equal(got_codes[m, s // per:(s + block) // per], O.pack(level, neg, bits))
        for m, s, same in pool.map(block_codes, [(m, s) for m in range(M) for s in starts]):
            assert same, f"packed codes of worker {m} in the block at {s}"
        say("  codes equal; decoded average of all 2^27 coordinates")

        def block_decode(s):
            vb = O.decode_aggregate(cfg, got_codes[:, s // per:(s + block) // per], scales, rh[s:s + block], block)
            return s, np.array_equal(got_vbar[s:s + block], vb)
        for s, same in pool.map(block_decode, starts):
            assert same, f"decoded average in the block at {s}"


@pytest.mark.parametrize("bits,norm,scale", [(2, B.NORM_MEAN, B.SCALE_MAX), (4, B.NORM_SUB, B.SCALE_L2)])
def test_full_size_windows(full_inputs, bits, norm, scale):
    g, gref = full_inputs
    d, M = D_FULL, M_FULL
    ctx = make_ctx(d, M, bits, norm, seed=1, scale=scale)
    cfg = oracle_cfg(ctx)
    buf = buffers(ctx)
    means_dev = None
    if norm == B.NORM_MEAN:
        means_dev = torch.zeros(M, device=DEV)
        ctx.set_worker_means(means_dev)
    it = 3
    say(f"full size bits={bits} norm={norm} scale={scale}: encode + decode")
    ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
    ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
    torch.cuda.synchronize()
    scales = buf["scales"].cpu().numpy()
    rh = gref.cpu().numpy()
    say("means and scales on the host")
    means = None
    if means_dev is not None:
        means = np.array([O.worker_mean(g[m].cpu().numpy()) for m in range(M)], dtype=np.float32)
        assert np.array_equal(means_dev.cpu().numpy(), means), "worker means"
    for m in range(M):
        v = O.normalize(g[m].cpu().numpy(), rh, norm, cfg.quot_eps, None, None if means is None else means[m])
        assert O.scale_of(v, scale) == scales[m], f"scale of worker {m}"
        del v
    say("the same sums in exact integer arithmetic (first and last worker)")
    for m in (0, M - 1):
        row = g[m].cpu().numpy()[None, :]
        assert_row_sums_are_the_exact_ones(cfg, row, rh, None, None if means is None else means[m:m + 1], scales[m:m + 1])
    rng = np.random.default_rng(bits * 10 + norm)
    win = 4096
    starts = [0, d - win] + [int(s) * 16 for s in rng.integers(0, (d - win) // 16, 30)]
    per = 32 // bits
    codes_dev, vbar_dev = buf["codes"], buf["vbar"]
    for s in starts:
        gw = g[:, s:s + win].cpu().numpy()
        rw = rh[s:s + win]
        words = np.zeros((M, win // per), dtype=np.uint32)
        for m in range(M):
            v = O.normalize(gw[m], rw, norm, cfg.quot_eps, None, None if means is None else means[m])
            u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, win, first=s))
            level, neg = O.quantize(v, scales[m], bits, u)
            words[m] = O.pack(level, neg, bits)
        got = u32(codes_dev[:, s // per:(s + win) // per])
        assert np.array_equal(got, words), f"codes in window at {s}"
        vb = O.decode_aggregate(cfg, words, scales, rw, win, None, means)
        assert np.array_equal(vbar_dev[s:s + win].cpu().numpy(), vb), f"decoded average in window at {s}"
    # properties that hold at any size: |decoded - mean(g)| is bounded by the mean grid step
    ctx.close()


@pytest.mark.parametrize("bits,norm,scale", [(2, B.NORM_SUB, B.SCALE_MAX), (4, B.NORM_QUOT, B.SCALE_MAX),
                                             (2, B.NORM_MEAN, B.SCALE_L2)])
def test_large_rows_of_odd_length_and_odd_worker_count(bits, norm, scale):
    # d = 2^26 + 3: every row but the first starts off the 16-byte grid (vector kernels over the first
    # d - d % 16 coordinates, element-wise kernels for the rest); M = 5: one short group of workers
    d, M, it = (1 << 26) + 3, 5, 9
    say(f"large ragged rows d=2^26+3 M=5 bits={bits} norm={norm} scale={scale}")
    g, gref = synth.codec_inputs(M, d, seed=4, device=DEV)
    ctx = make_ctx(d, M, bits, norm, seed=8, scale=scale)
    cfg = oracle_cfg(ctx)
    buf = buffers(ctx)
    means_dev = None
    if norm == B.NORM_MEAN:
        means_dev = torch.zeros(M, device=DEV)
        ctx.set_worker_means(means_dev)
    ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
    ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
    torch.cuda.synchronize()
    scales = buf["scales"].cpu().numpy()
    rh = gref.cpu().numpy()
    means = None
    if means_dev is not None:
        means = np.array([O.worker_mean(g[m].cpu().numpy()) for m in range(M)], dtype=np.float32)
        assert np.array_equal(means_dev.cpu().numpy(), means), "worker means"
    for m in range(M):
        v = O.normalize(g[m].cpu().numpy(), rh, norm, cfg.quot_eps, None, None if means is None else means[m])
        assert O.scale_of(v, scale) == scales[m], f"scale of worker {m}"
        del v
    row = g[M - 1].cpu().numpy()[None, :]
    assert_row_sums_are_the_exact_ones(cfg, row, rh, None, None if means is None else means[M - 1:], scales[M - 1:])
    rng = np.random.default_rng(bits + norm)
    win, per = 4096, 32 // bits
    last = (d // 16) * 16 - (win - 16)                       # reaches past the end of the rows
    starts = [0, last] + [int(s) * 16 for s in rng.integers(0, (d - win) // 16, 12)]
    for s in starts:
        n = min(win, d - s)
        gw = g[:, s:s + n].cpu().numpy()
        rw = rh[s:s + n]
        nwords = O.words_per_row(n, bits)
        words = np.zeros((M, nwords), dtype=np.uint32)
        for m in range(M):
            v = O.normalize(gw[m], rw, norm, cfg.quot_eps, None, None if means is None else means[m])
            u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, n, first=s))
            level, neg = O.quantize(v, scales[m], bits, u)
            words[m] = O.pack(level, neg, bits)
        got = u32(buf["codes"][:, s // per:s // per + nwords])
        assert np.array_equal(got, words), f"codes in window at {s}"
        vb = O.decode_aggregate(cfg, words, scales, rw, n, None, means)
        assert np.array_equal(buf["vbar"][s:s + n].cpu().numpy(), vb), f"decoded average in window at {s}"
    assert s // per + nwords <= ctx.words
    ctx.close()
