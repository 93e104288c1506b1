"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import tng_oracle as O
from paper_1901_08227_amd import binding as B

DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)


def make_ctx(d, M, bits, norm, seed=0, **kw):
    return B.Context(d=d, M=M, bits=bits, norm=norm, seed=seed, device=DEV, **kw)


def oracle_cfg(ctx, **kw):
    c = ctx.cfg
    return O.Config(d=int(c.d), M=int(c.M), bits=int(c.bits), norm=int(c.norm), quot_eps=float(c.quot_eps),
                    ref_policy=int(c.ref_policy), ref_period=int(c.ref_period), seed=int(c.seed), lr=float(c.lr),
                    l2=float(c.l2), batch=int(c.batch), **kw)


def buffers(ctx):
    dev = ctx.device
    return dict(
        g=torch.empty((ctx.M, ctx.d), device=dev),
        codes=torch.full((ctx.M, ctx.words), -1, dtype=torch.int32, device=dev),
        scales=torch.full((ctx.M,), -1.0, device=dev),
        vbar=torch.full((ctx.d,), float("nan"), device=dev),
    )


def u32(t):
    return t.cpu().numpy().view(np.uint32)


def within_tolerance(a, b, rel=1e-5):
    """Elementwise |a-b| <= rel*max(|b|, 1e-3*||b||_inf) and ||a-b||_2 <= rel*||b||_2."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    floor = 1e-3 * np.abs(b).max() if b.size else 0.0
    ok_el = np.all(np.abs(a - b) <= rel * np.maximum(np.abs(b), floor))
    ok_l2 = np.linalg.norm(a - b) <= rel * np.linalg.norm(b) + 1e-30
    return bool(ok_el and ok_l2)
