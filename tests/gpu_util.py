"""Helpers shared by the GPU parity tests (not collected by pytest)."""
import numpy as np
import torch

from oracle import tng_oracle as O
from paper_1901_08227_amd import binding as B

DEV = "cuda:0"


from progress import say  # noqa: E402,F401  (one progress line, visible through pytest's capture)


def make_ctx(d, M, bits, norm, seed=0, **kw):
    return B.Context(d=d, M=M, bits=bits, norm=norm, seed=seed, device=DEV, **kw)


def set_csr(ctx, shards, pairs):
    """Hands CSR shards (rowptr, col, val, y per worker) to the library in either entry layout."""
    if pairs:
        ctx.set_logreg_csr_pairs([s[0] for s in shards], [B.csr_pairs(s[1], s[2]) for s in shards], [s[3] for s in shards])
    else:
        ctx.set_logreg_csr([s[0] for s in shards], [s[1] for s in shards], [s[2] for s in shards], [s[3] for s in shards])


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


def logistic_condition_csr(rowptr, col, val, y, w, ids, d, l2=0.0):
    """logistic_condition for minibatch rows stored as CSR, without densifying them.  Float64, host."""
    w64 = np.asarray(w, dtype=np.float64)
    cond = np.zeros(d, dtype=np.float64)
    for i in np.asarray(ids):
        a, b = int(rowptr[i]), int(rowptr[i + 1])
        c = np.asarray(col[a:b], dtype=np.int64)
        x = np.asarray(val[a:b], dtype=np.float64)
        r = O.sigmoid64(np.array([x @ w64[c]]))[0] - float(y[i])
        Z = np.abs(x) @ np.abs(w64[c])
        np.add.at(cond, c, (abs(r) + 0.25 * Z) * np.abs(x))
    return cond / float(len(ids)) + abs(l2) * np.abs(w64)


def oracle_step_threaded(cfg, it, w, gref, g, threads=8, block=1 << 22):
    """The oracle's iteration (what O.step computes for the shared-reference normalisations and the
    largest-magnitude or l2 scale) put together from the oracle's own per-worker and per-coordinate
    functions, so that host threads can share the work at large M * d: the workers' side one worker per
    task, the server's side one block of coordinates per task (block: a multiple of 16 coordinates, whole
    packed words for either width).  numpy releases the interpreter lock inside its loops.  Nothing is
    computed here: every value comes out of an oracle function.  tests/test_oracle_step.py holds it
    against O.step."""
    from concurrent.futures import ThreadPoolExecutor

    assert cfg.norm in (O.NORM_NONE, O.NORM_SUB, O.NORM_QUOT) and block % 16 == 0
    g = np.asarray(g, dtype=np.float32)
    M, d = g.shape
    per = 32 // cfg.bits

    def worker(m):
        v = O.normalize(g[m], gref, cfg.norm, cfg.quot_eps)
        R = O.scale_of(v, cfg.scale_kind)
        u = O.uniform_from_word(O.quant_draw_words(cfg.seed, it, m, d))
        level, neg = O.quantize(v, R, cfg.bits, u)
        return O.pack(level, neg, cfg.bits), R

    def server(a):
        b = min(a + block, d)
        return O.decode_aggregate(cfg, codes[:, a // per:(b + per - 1) // per], scales, gref[a:b], b - a)

    with ThreadPoolExecutor(max_workers=threads) as pool:
        enc = list(pool.map(worker, range(M)))
        codes = np.stack([e[0] for e in enc])
        scales = np.array([e[1] for e in enc], dtype=np.float32)
        vbar = np.concatenate(list(pool.map(server, range(0, d, block))))
    w_next = O.update_iterate(w, vbar, cfg.lr)
    assert cfg.ref_policy in (O.REF_ZERO, O.REF_LAST_AVG)
    gref_next = O.update_reference(cfg, it, vbar, gref)
    return w_next, gref_next, codes, scales, vbar


def assert_row_sums_are_the_exact_ones(cfg, g, gref, gref2, means, scales, rows=None):
    """Holds the library's (= the oracle's pinned-order) per-worker means and l2 scales against the
    values mathematics fixes: float32(exact sum / d) and float32(sqrt(exact sum of squares)), computed
    with integer arithmetic (tests/exact_sums.py).  No-op for configurations with neither."""
    from exact_sums import exact_sum, round_to_f32, sqrt_to_f32

    g = np.asarray(g, dtype=np.float32)
    M, d = g.shape
    for m in (range(M) if rows is None else rows):
        mu = None
        if cfg.norm == O.NORM_MEAN:
            mu = means[m]
            assert mu == round_to_f32(exact_sum(g[m]) / d), f"mean of worker {m} is not the exactly rounded mean"
        if cfg.scale_kind == O.SCALE_L2:
            v = O.normalize(g[m], gref, cfg.norm, cfg.quot_eps, gref2, mu)
            want = sqrt_to_f32(exact_sum(v.astype(np.float64) ** 2))
            want = want if want >= O.FLT_MIN else np.float32(0.0)
            assert scales[m] == want, f"l2 scale of worker {m} is not the exactly rounded norm"
