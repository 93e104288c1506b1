"""GPU parity of the ternary coder that reads the gradients once (section "Gradient Compression").

For long rows of 2-bit codes the scale pass also picks out, per worker and tile of 1024 coordinates, the
elements that can code non-zero whatever the scale turns out to be, and the quantise pass codes those
instead of reading g again; a tile with too many of them goes through the ordinary path.  The path is
taken from 2^26 elements on (d a multiple of 1024), so these cases are that large: packed codes, scales
and decoded averages of every element against the oracle, on ordinary data, on data where every tile
overflows, on mixtures, on degenerate rows, and for worker counts that leave short groups."""
import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, buffers, make_ctx, oracle_cfg, oracle_step_threaded, say, u32
from paper_1901_08227_amd import binding as B
from paper_1901_08227_amd import synth

pytestmark = pytest.mark.gpu


def _check(M, d, norm, g, gref, gref2, it, tag, seed=5):
    say(f"candidates case {tag}: d={d} M={M} norm={norm} it={it}")
    assert M * d >= 1 << 26 and d % 1024 == 0, "the case must be one that takes the path under test"
    ctx = make_ctx(d, M, 2, norm, seed=seed)
    if norm == B.NORM_COMB:
        ctx.set_second_reference(gref2)
    buf = buffers(ctx)
    ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
    ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
    torch.cuda.synchronize()
    cfg = oracle_cfg(ctx)
    ctx.close()
    rh, r2h = gref.cpu().numpy(), gref2.cpu().numpy()
    got_codes, got_scales = u32(buf["codes"]), buf["scales"].cpu().numpy()
    want_codes = np.empty_like(got_codes)
    want_scales = np.empty(M, dtype=np.float32)
    for m in range(M):  # one worker at a time keeps the host's memory small
        want_codes[m], want_scales[m] = _encode_one(cfg, it, m, g[m].cpu().numpy(), rh, r2h)
    assert np.array_equal(got_scales, want_scales), f"{tag}: scales {got_scales} vs {want_scales}"
    if not np.array_equal(got_codes, want_codes):
        bad = np.argwhere(got_codes != want_codes)
        raise AssertionError(f"{tag}: {len(bad)} packed words differ, first at {bad[0]}: "
                             f"{got_codes[tuple(bad[0])]:#x} vs {want_codes[tuple(bad[0])]:#x}")
    vbar = O.decode_aggregate(cfg, want_codes, want_scales, rh, d, r2h, None)
    assert np.array_equal(buf["vbar"].cpu().numpy(), vbar), f"{tag}: decoded average"
    return want_codes, want_scales


def _encode_one(cfg, it, m, row, rh, r2h):
    """Worker m's packed codes and scale from the oracle's own functions (what O.normalize_encode does per worker)."""
    v = O.normalize(row, rh, cfg.norm, cfg.quot_eps, r2h, None)
    R = O.scale_of(v, cfg.scale_kind)
    u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, row.shape[0]))
    level, neg = O.quantize(v, R, cfg.bits, u)
    return O.pack(level, neg, cfg.bits), R


def _inputs(M, d, seed):
    g, gref = synth.codec_inputs(M, d, seed, device=DEV)
    gref2 = torch.randn(d, generator=torch.Generator(device=DEV).manual_seed(seed + 1), device=DEV) + 2.0
    return g, gref, gref2


def test_oracle_per_worker_path_is_the_oracle():
    # the helper above against O.normalize_encode on a small case (every value comes out of oracle functions)
    M, d = 3, 4096
    g, gref, gref2 = _inputs(M, d, seed=2)
    cfg = O.Config(d=d, M=M, bits=2, norm=O.NORM_SUB, seed=9)
    codes, scales = O.normalize_encode(cfg, 4, g.cpu().numpy(), gref.cpu().numpy(), gref2.cpu().numpy(), None)
    for m in range(M):
        c, s = _encode_one(cfg, 4, m, g[m].cpu().numpy(), gref.cpu().numpy(), gref2.cpu().numpy())
        assert np.array_equal(c, codes[m]) and s == scales[m]


@pytest.mark.parametrize("norm", [B.NORM_NONE, B.NORM_SUB, B.NORM_QUOT, B.NORM_COMB])
def test_ordinary_data(norm):
    # (the quotient forms keep the two-pass kernels at any size: their |v| is near 1 everywhere)
    M, d = 8, 1 << 23
    g, gref, gref2 = _inputs(M, d, seed=11 + norm)
    codes, _ = _check(M, d, norm, g, gref, gref2, 3, "ordinary")
    nz = sum(int(np.count_nonzero((codes >> s) & 3)) for s in range(0, 32, 2)) / (M * d)
    say(f"  fraction of non-zero codes: {nz:.4f}")
    if norm == B.NORM_SUB:  # the premise of the path: only a few percent of the codes are non-zero
        assert nz < 0.1


@pytest.mark.parametrize("M,d,norm", [(9, 1 << 23, B.NORM_SUB), (3, 1 << 25, B.NORM_SUB), (64, 1 << 20, B.NORM_SUB),
                                      (5, (1 << 24) + 1024 * 7, B.NORM_NONE),
                                      # one and two workers per workgroup: the scale pass's schedule has idle items then
                                      (1, 1 << 26, B.NORM_SUB), (2, (1 << 25) + 1024 * 3, B.NORM_NONE),
                                      (4, 1 << 24, B.NORM_SUB)])
def test_worker_counts_and_row_lengths(M, d, norm):
    g, gref, gref2 = _inputs(M, d, seed=M)
    _check(M, d, norm, g, gref, gref2, 1, "workers and lengths")


def test_every_tile_overflows():
    # |v| uniform in [0.5, 1]: half of the elements or more code non-zero, no slot can hold its tile
    M, d = 8, 1 << 23
    gen = torch.Generator(device=DEV).manual_seed(3)
    gref = torch.randn(d, generator=gen, device=DEV)
    mag = torch.rand((M, d), generator=gen, device=DEV) * 0.5 + 0.5
    sign = (torch.randint(0, 2, (M, d), generator=gen, device=DEV) * 2 - 1).float()
    g = gref[None, :] + mag * sign
    _check(M, d, B.NORM_SUB, g, gref, gref, 2, "all tiles overflow")


def test_mixture_of_tiles_and_degenerate_rows():
    M, d = 8, 1 << 23
    g, gref, gref2 = _inputs(M, d, seed=21)
    v = g - gref[None, :]
    gen = torch.Generator(device=DEV).manual_seed(4)
    # worker 0: a stretch of large equal magnitudes (those tiles overflow), the rest ordinary
    v[0, 5000:300000] = 0.9 * v[0].abs().max()
    # worker 1: all zero (scale 0); worker 2: nothing but values below the smallest normal number (scale taken as 0)
    v[1] = 0.0
    v[2] = (torch.rand(d, generator=gen, device=DEV) - 0.5) * 1e-39
    # worker 3: tiny values and one ordinary element in a tile the sample does not visit
    v[3] = (torch.rand(d, generator=gen, device=DEV) - 0.5) * 1e-30
    v[3, 1024 * 77 + 5] = 0.25
    # worker 4: the largest element sits in the very first tile (which the sample visits), worker 5: in the last tile
    v[4, 3] = 4.0 * v[4].abs().max()
    v[5, d - 2] = -4.0 * v[5].abs().max()
    # worker 6: exact zeros in most places (a sparse gradient), worker 7 stays ordinary
    keep = torch.rand(d, generator=gen, device=DEV) < 0.01
    v[6] = torch.where(keep, v[6], torch.zeros_like(v[6]))
    g = v + gref[None, :]
    for norm, ref in ((B.NORM_NONE, gref), (B.NORM_SUB, gref)):
        src = v if norm == B.NORM_NONE else g
        _check(M, d, norm, src.contiguous(), ref, gref2, 7, "mixture")


@pytest.mark.parametrize("dense_workers", [(17,), (0, 5, 9, 63), tuple(range(0, 64, 2))])
def test_rows_that_the_sample_finds_too_dense(dense_workers):
    # Gaussian residuals (one element in seven codes non-zero: more than a slot holds) on some workers, the
    # ordinary data on the others.  One dense worker in 64 stays under the limit for unused slots, so its tiles
    # go through the quantise pass's own ordinary path; half of them make the whole call fall back.
    M, d = 64, 1 << 20
    g, gref, gref2 = _inputs(M, d, seed=31)
    gen = torch.Generator(device=DEV).manual_seed(32)
    for m in dense_workers:
        g[m] = gref + torch.randn(d, generator=gen, device=DEV)
    codes, _ = _check(M, d, B.NORM_SUB, g.contiguous(), gref, gref2, 4, f"dense workers {dense_workers[:4]}")
    nz = [np.count_nonzero(np.unpackbits(codes[m].view(np.uint8)).reshape(-1, 2).any(axis=1)) / d for m in (dense_workers[0], 1)]
    assert nz[0] > 0.12 and nz[1] < 0.08, nz


def test_same_codes_as_the_two_pass_coder_on_shorter_rows():
    # the same data cut into rows just below the path's threshold goes through the two-pass kernels: worker 0's
    # codes over the first d/2 coordinates must agree between the two (the draws depend on the element index only)
    M, d = 8, 1 << 23
    g, gref, gref2 = _inputs(M, d, seed=31)
    long_ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=8)
    a = buffers(long_ctx)
    long_ctx.normalize_encode(5, g, gref, a["codes"], a["scales"])
    half = d // 2
    short_ctx = make_ctx(half, M, 2, B.NORM_SUB, seed=8)   # 2^25 elements: below the threshold
    b = buffers(short_ctx)
    gh = g[:, :half].contiguous()
    short_ctx.normalize_encode(5, gh, gref[:half].contiguous(), b["codes"], b["scales"])
    torch.cuda.synchronize()
    # same scale only if the row's maximum lies in the first half; compare the workers for which it does
    same = [m for m in range(M) if float(a["scales"][m]) == float(b["scales"][m])]
    assert same, "no worker has its largest element in the first half: change the seed"
    for m in same:
        assert torch.equal(a["codes"][m, :half // 16], b["codes"][m]), f"worker {m}"
    long_ctx.close()
    short_ctx.close()


def test_whole_iteration_with_gradients_from_the_caller():
    # tng_step on gradients handed in by the caller (no problem attached): its encode part takes the same path,
    # the decode part updates the iterate and refreshes the reference in place; two iterations, the second from
    # the state the first one left
    M, d = 8, 1 << 23
    g, gref, _ = _inputs(M, d, seed=41)
    ctx = B.Context(d=d, M=M, bits=2, norm=B.NORM_SUB, ref_policy=B.REF_LAST_AVG, ref_period=2, seed=12, lr=0.05,
                    problem=B.PROB_EXTERNAL, device=DEV)
    cfg = oracle_cfg(ctx)
    buf = buffers(ctx)
    w = torch.randn(d, generator=torch.Generator(device=DEV).manual_seed(5), device=DEV)
    gref = gref.clone()
    for it in range(2):
        say(f"candidates case whole iteration: it={it}")
        gi = g if it == 0 else (g * 0.5 + torch.roll(g, 1, dims=0) * 0.5).contiguous()
        w0, r0 = w.cpu().numpy(), gref.cpu().numpy()
        ctx.step(it, w, gref, gi, buf["codes"], buf["scales"], buf["vbar"])
        torch.cuda.synchronize()
        w1, r1, codes, scales, vbar = oracle_step_threaded(cfg, it, w0, r0, gi.cpu().numpy())
        assert np.array_equal(buf["scales"].cpu().numpy(), scales), "scales"
        assert np.array_equal(u32(buf["codes"]), codes), "packed codes"
        assert np.array_equal(buf["vbar"].cpu().numpy(), vbar), "decoded average"
        assert np.array_equal(w.cpu().numpy(), w1), "iterate"
        assert np.array_equal(gref.cpu().numpy(), r1), "reference"
    ctx.close()


@pytest.mark.parametrize("case", range(6))
def test_seeded_shapes_and_distributions(case):
    # worker counts, row lengths (whole tiles, 2^26 elements or a little more) and value distributions drawn from a
    # seed: Gaussian, heavy-tailed (Cauchy-like), mostly exact zeros, one dominant element per row, blocks of
    # constant magnitude
    rng = np.random.default_rng(1000 + case)
    M = int(rng.integers(2, 21))
    tiles = -(-(1 << 26) // (M * 1024)) + int(rng.integers(0, 50))
    d = tiles * 1024
    gen = torch.Generator(device=DEV).manual_seed(2000 + case)
    gref = torch.randn(d, generator=gen, device=DEV)
    kind = case % 5
    v = torch.randn((M, d), generator=gen, device=DEV)
    if kind == 1:
        v = v / (torch.randn((M, d), generator=gen, device=DEV).abs() + 1e-3)
    elif kind == 2:
        v = torch.where(torch.rand((M, d), generator=gen, device=DEV) < 0.02, v, torch.zeros_like(v))
    elif kind == 3:
        v = v * 1e-3
        for m in range(M):
            v[m, int(rng.integers(0, d))] = float(rng.choice([-1.0, 1.0])) * 50.0
    elif kind == 4:
        a = int(rng.integers(0, d // 2))
        v[:, a:a + d // 3] = torch.sign(v[:, a:a + d // 3]) * 2.5
    norm = B.NORM_SUB if case % 2 == 0 else B.NORM_NONE
    g = (v + gref[None, :]).contiguous() if norm == B.NORM_SUB else v.contiguous()
    _check(M, d, norm, g, gref, gref, int(rng.integers(0, 1000)), f"seeded {case} (kind {kind})", seed=int(rng.integers(0, 2 ** 40)))
