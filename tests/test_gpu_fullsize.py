"""Parity at the full size of the encode/decode benchmark (M = 8, d = 2^27), in the launch
configuration bench.py times: scales exactly (full pass on the host), packed codes and decoded
averages on sampled windows the oracle computes element by element."""
import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, buffers, make_ctx, oracle_cfg, say, u32
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
def test_full_size_windows(full_inputs, bits, norm):
    g, gref = full_inputs
    d, M = D_FULL, M_FULL
    ctx = make_ctx(d, M, bits, norm, seed=1)
    cfg = oracle_cfg(ctx)
    buf = buffers(ctx)
    it = 3
    say(f"full size bits={bits} norm={norm}: encode + decode")
    ctx.normalize_encode(it, g, gref, buf["codes"], buf["scales"])
    ctx.decode_aggregate(buf["codes"], buf["scales"], gref, buf["vbar"])
    torch.cuda.synchronize()
    scales = buf["scales"].cpu().numpy()
    rh = gref.cpu().numpy()
    say("scales on the host")
    for m in range(M):
        v = O.normalize(g[m].cpu().numpy(), rh, norm, cfg.quot_eps)
        assert O.scale_of(v) == scales[m], f"scale of worker {m}"
        del v
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
            v = O.normalize(gw[m], rw, norm, cfg.quot_eps)
            u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, win, first=s))
            level, neg = O.quantize(v, scales[m], bits, u)
            words[m] = O.pack(level, neg, bits)
        got = u32(codes_dev[:, s // per:(s + win) // per])
        assert np.array_equal(got, words), f"codes in window at {s}"
        vb = O.decode_aggregate(cfg, words, scales, rw, win)
        assert np.array_equal(vbar_dev[s:s + win].cpu().numpy(), vb), f"decoded average in window at {s}"
    # properties that hold at any size: |decoded - mean(g)| is bounded by the mean grid step
    ctx.close()
