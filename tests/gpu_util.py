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
                    l2=float(c.l2), batch=int(c.batch), ref_window=max(int(c.ref_window), 1),
                    scale_kind=int(c.scale), **kw)


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


EPS32 = 2.0 ** -24


def logistic_condition(Xb, yb, w, l2=0.0):
    """Per-coordinate size of what an fp32 evaluation of the minibatch logistic gradient adds up:
    cond_k = (1/B) sum_i (|r_i| + Z_i / 4) |x_ik| + |l2 w_k|, with r_i = sigma(z_i) - y_i and
    Z_i = sum_k |x_ik w_k| (an error dz in z_i moves r_i by at most dz / 4).  Float64, host."""
    Xb = np.asarray(Xb, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    r = O.sigmoid64(Xb @ w) - np.asarray(yb, dtype=np.float64)
    Z = np.abs(Xb) @ np.abs(w)
    return ((np.abs(r) + 0.25 * Z) @ np.abs(Xb)) / Xb.shape[0] + abs(l2) * np.abs(w)


def grad_close(a, b, cond, rel=1e-5):
    """The 1e-5 relative contract for fp32 gradients against the float64 oracle:
    ||a-b||_2 <= rel ||b||_2, max|a-b| <= rel ||b||_inf, and elementwise
    |a-b| <= rel |b| + 4 eps32 cond  (cond: see logistic_condition; the second term is what
    cancellation in an fp32 sum may cost, far below the worst-case bound B eps32 cond)."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    diff = np.abs(a - b)
    return bool(np.linalg.norm(a - b) <= rel * np.linalg.norm(b) and diff.max() <= rel * np.abs(b).max()
                and np.all(diff <= rel * np.abs(b) + 4 * EPS32 * cond))
