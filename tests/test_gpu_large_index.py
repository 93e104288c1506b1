"""Element indices beyond 2^32: one encode + decode at d = 2^32 + 12368 with two workers (so that row
offsets, tile numbers and RNG counters all pass 32 bits), checked against the oracle on windows at the
start, across the 2^32 boundary and at the end, with scales that are known in closed form."""
import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, buffers, make_ctx, oracle_cfg, say, u32
from paper_1901_08227_amd import binding as B

pytestmark = pytest.mark.gpu


def test_indices_beyond_32_bits():
    d, M, bits, it = (1 << 32) + 3 * 4096 + 80, 2, 2, 7
    free, _ = torch.cuda.mem_get_info()
    if free < 80 * (1 << 30):
        pytest.skip("needs about 70 GiB of device memory")
    say(f"large index case d={d} M={M}")
    gen = torch.Generator(device=DEV).manual_seed(5)
    gref = torch.empty(d, device=DEV)
    gref.normal_(generator=gen)
    g = torch.empty((M, d), device=DEV)
    for m in range(M):
        g[m].uniform_(-0.5, 0.5, generator=gen)
        g[m] += gref
    # planted maxima: |g - gref| <= 0.5 + rounding everywhere else
    e0, e1 = (1 << 32) + 5, d - 1
    gref[e0] = 0.0
    gref[e1] = 0.0
    g[0, e0] = 3.0
    g[1, e1] = -5.0
    ctx = make_ctx(d, M, bits, B.NORM_SUB, seed=(9 << 32) | 3)
    cfg = oracle_cfg(ctx)
    codes = torch.full((M, ctx.words), -1, dtype=torch.int32, device=DEV)
    scales = torch.full((M,), -1.0, device=DEV)
    vbar = torch.empty(d, device=DEV)
    ctx.normalize_encode(it, g, gref, codes, scales)
    ctx.decode_aggregate(codes, scales, gref, vbar)
    torch.cuda.synchronize()
    sc = scales.cpu().numpy()
    assert sc[0] == np.float32(3.0) and sc[1] == np.float32(5.0)
    per = 32 // bits
    win = 4096
    for s in (0, (1 << 32) - 2048, (1 << 32) + 4096 * 2, d - win):
        assert s % per == 0
        gw = g[:, s:s + win].cpu().numpy()
        rw = gref[s:s + win].cpu().numpy()
        words = np.zeros((M, win // per), dtype=np.uint32)
        for m in range(M):
            v = O.normalize(gw[m], rw, B.NORM_SUB, cfg.quot_eps)
            u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, win, first=s))
            level, neg = O.quantize(v, sc[m], bits, u)
            words[m] = O.pack(level, neg, bits)
        assert np.array_equal(u32(codes[:, s // per:(s + win) // per]), words), f"codes in window at {s}"
        vb = O.decode_aggregate(cfg, words, sc, rw, win)
        assert np.array_equal(vbar[s:s + win].cpu().numpy(), vb), f"decoded average in window at {s}"
    # the planted elements are coded with the top level and their signs
    w0 = int(u32(codes[0, e0 // per:e0 // per + 1])[0])
    w1 = int(u32(codes[1, e1 // per:e1 // per + 1])[0])
    assert (w0 >> ((e0 % per) * bits)) & 3 == 1 and (w1 >> ((e1 % per) * bits)) & 3 == 3
    ctx.close()
