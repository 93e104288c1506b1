"""The frozen record tests/golden/codec_golden.json (written by tests/golden/make_codec_golden.py
from the oracle alone): the oracle must still reproduce it, and so must the HIP library."""
import json
import os

import numpy as np
import pytest

from oracle import tng_oracle as O

PATH = os.path.join(os.path.dirname(__file__), "golden", "codec_golden.json")


def _cases():
    with open(PATH) as fh:
        return json.load(fh)["cases"]


def _f32(bits, shape=None):
    a = np.array(bits, dtype=np.uint32).view(np.float32)
    return a if shape is None else a.reshape(shape)


def test_oracle_reproduces_the_frozen_record():
    cases = _cases()
    assert len(cases) == 16
    for c in cases:
        d, M = c["d"], c["M"]
        cfg = O.Config(d=d, M=M, bits=c["bits"], norm=c["norm"], seed=c["seed"], lr=c["lr"])
        g, gref, gref2 = _f32(c["g"], (M, d)), _f32(c["gref"]), _f32(c["gref2"])
        codes, scales = O.normalize_encode(cfg, c["iter"], g, gref, gref2)
        assert [int(x) for x in codes.reshape(-1)] == c["codes"]
        assert np.array_equal(scales.view(np.uint32), np.array(c["scales"], dtype=np.uint32))
        vbar = O.decode_aggregate(cfg, codes, scales, gref, d, gref2)
        assert np.array_equal(vbar.view(np.uint32), np.array(c["vbar"], dtype=np.uint32))
        w_next = O.update_iterate(_f32(c["w"]), vbar, cfg.lr)
        assert np.array_equal(w_next.view(np.uint32), np.array(c["w_next"], dtype=np.uint32))


@pytest.mark.gpu
def test_library_reproduces_the_frozen_record():
    import torch

    from gpu_util import DEV, buffers, make_ctx, u32
    from paper_1901_08227_amd import binding as B

    for c in _cases():
        d, M = c["d"], c["M"]
        ctx = make_ctx(d, M, c["bits"], c["norm"], seed=c["seed"], lr=c["lr"], ref_policy=B.REF_ZERO,
                       problem=B.PROB_EXTERNAL)
        g = torch.from_numpy(_f32(c["g"], (M, d)).copy()).to(DEV)
        gref = torch.from_numpy(_f32(c["gref"]).copy()).to(DEV)
        gref2 = torch.from_numpy(_f32(c["gref2"]).copy()).to(DEV)
        w = torch.from_numpy(_f32(c["w"]).copy()).to(DEV)
        if c["norm"] == B.NORM_COMB:
            ctx.set_second_reference(gref2)
        buf = buffers(ctx)
        ctx.step(c["iter"], w, gref, g, buf["codes"], buf["scales"], buf["vbar"])
        torch.cuda.synchronize()
        assert [int(x) for x in u32(buf["codes"]).reshape(-1)] == c["codes"]
        assert np.array_equal(u32(buf["scales"]), np.array(c["scales"], dtype=np.uint32))
        assert np.array_equal(u32(buf["vbar"]), np.array(c["vbar"], dtype=np.uint32))
        assert np.array_equal(u32(w), np.array(c["w_next"], dtype=np.uint32))
        assert np.array_equal(u32(gref), np.array(c["gref"], dtype=np.uint32))      # zero policy: untouched
        ctx.close()
