"""Seeded random configurations of the codec on the GPU against the oracle, bit for bit: dimensions
around the tile and word boundaries, worker counts that do and do not divide into workgroups, every
normalisation, both widths and both scales."""
import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, assert_row_sums_are_the_exact_ones, buffers, make_ctx, oracle_cfg, say, u32
from paper_1901_08227_amd import binding as B

pytestmark = pytest.mark.gpu


def _case(rng):
    kind = rng.integers(0, 5)
    tiles = int(rng.integers(1, 18))
    if kind == 0:
        d = 4096 * tiles                                   # whole tiles
    elif kind == 1:
        d = 4096 * tiles + 64 * int(rng.integers(1, 64))   # 16-byte aligned code rows, ragged last tile
    elif kind == 2:
        d = 4096 * tiles + 4 * int(rng.integers(1, 1024))  # vector path, code rows not 16-byte aligned
    elif kind == 3:
        d = 4096 * tiles + int(rng.integers(1, 4096))      # any d: element-at-a-time kernels when d % 4 != 0
    else:
        d = int(rng.integers(1, 300))
    M = int(rng.choice([1, 2, 3, 4, 5, 8, 12, 16, 17, 24]))
    bits = int(rng.choice([2, 4]))
    norm = int(rng.choice([B.NORM_NONE, B.NORM_SUB, B.NORM_QUOT, B.NORM_COMB, B.NORM_MEAN]))
    scale = int(rng.choice([B.SCALE_MAX, B.SCALE_MAX, B.SCALE_L2]))
    return d, M, bits, norm, scale


@pytest.mark.parametrize("block", range(4))
def test_random_configurations(block):
    rng = np.random.default_rng(1000 + block)
    for n in range(12):
        d, M, bits, norm, scale = _case(rng)
        seed = int(rng.integers(0, 1 << 62))
        it = int(rng.integers(0, 1 << 31))
        say(f"fuzz block {block} case {n}: d={d} M={M} bits={bits} norm={norm} scale={scale} it={it}")
        gen = torch.Generator(device=DEV).manual_seed(seed % (1 << 31))
        gref = torch.randn(d, generator=gen, device=DEV)
        g = gref + 0.3 * torch.randn((M, d), generator=gen, device=DEV) * gref.abs() \
            + torch.randn((M, 1), generator=gen, device=DEV)
        gref2 = torch.rand(d, generator=gen, device=DEV) + 0.5
        ctx = make_ctx(d, M, bits, norm, seed=seed, scale=scale)
        cfg = oracle_cfg(ctx)
        buf = buffers(ctx)
        means_dev = None
        if norm == B.NORM_COMB:
            ctx.set_second_reference(gref2)
        if norm == B.NORM_MEAN:
            means_dev = torch.zeros(M, device=DEV)
            ctx.set_worker_means(means_dev)
        ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
        ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
        torch.cuda.synchronize()
        gh, rh, r2h = g.cpu().numpy(), gref.cpu().numpy(), gref2.cpu().numpy()
        means = O.worker_means(gh) if means_dev is not None else None
        if means is not None:
            assert np.array_equal(means_dev.cpu().numpy(), means)
        codes, scales = O.normalize_encode(cfg, it, gh, rh, r2h, means)
        assert np.array_equal(buf["scales"].cpu().numpy(), scales)
        assert_row_sums_are_the_exact_ones(cfg, gh, rh, r2h, means, scales)
        assert np.array_equal(u32(buf["codes"]), codes)
        vbar = O.decode_aggregate(cfg, codes, scales, rh, d, r2h, means)
        assert np.array_equal(buf["vbar"].cpu().numpy(), vbar)
        ctx.close()
