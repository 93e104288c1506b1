"""Vectorised numpy oracle for one iteration of Trajectory Normalized Gradients (TNG).

TEST INFRASTRUCTURE ONLY -- not a product path, never a fallback.

What it states (paper = arXiv 1901.08227):

* the outer iteration  w_{t+1} = w_t - eta * (1/M) sum_m Q[g^m(w_t)]   (Background, Eq. "qsgd");
* trajectory normalisation against a shared reference g~ (section "Normalized Gradients"):
  subtraction  r = Q[g - g~], v = g~ + r               (Eq. 1)
  quotient     r = Q[g ./ g~], v = g~ (.) r            (Eq. 2)
  combined     r = Q[(g - g~) ./ g~'], v = g~' (.) r + g~ (unnumbered display after Eq. 2);
* the stochastic sign coder  Q[v] = R sign(v) (.) z(v), R = max_d |v_d|,
  P(z_d = 1) = |v_d| / R                                (section "Gradient Compression");
  generalised to s = 2^(bits-1) - 1 magnitude levels (bits = 2 is exactly the ternary coder);
* Algorithm 1: local gradient, scale, sample, transmit, average, refresh the reference;
* the reference rule of the convex experiments: g~ <- the averaged decoded gradient of the
  previous iteration, refreshed every K iterations (sections "Reference Vectors", "Convex
  Problems", and the 16-iteration period of "Nonconvex Problems").

Precision.  The quantiser decides integers from floating point, so its arithmetic is fixed:
IEEE binary32, round-to-nearest-even, one rounding per written operation, no fused
multiply-add, subnormals kept.  numpy float32 ufuncs do exactly that.  Gradients of the
logistic model are the textbook definition evaluated in float64.

Readings of the paper taken here:
  - second line of the probability display is P(z=0) = 1 - |v_d|/R;
  - Algorithm 1 uses |g - g~| (not |g|) for the probabilities and sign(g - g~) for the sign;
  - the server adds the reference back after averaging (Eq. 1), which Algorithm 1 omits;
  - "largest element" means largest magnitude (the display defines R = max_d |v_d|);
  - Eq. 2 divides by the reference; entries with |g~_d| < eps are replaced by +-eps.

Parity pins: see tests/test_oracle_*.py.  The paper prints no worked numeric example, so
optimisation quality against the paper's (missing) figures is "parity unpinned".
"""
from __future__ import annotations

import dataclasses

import numpy as np

F32 = np.float32
U32 = np.uint32
U64 = np.uint64

FLT_MIN = F32(1.17549435e-38)  # smallest normal binary32

NORM_NONE = 0  # v = g                       (reference = zeros: plain compressed SGD)
NORM_SUB = 1   # Eq. 1
NORM_QUOT = 2  # Eq. 2
NORM_COMB = 3  # combined two-reference form
NORM_MEAN = 4  # Eq. 1 with the per-worker reference mean(g_m) * ones(D); mean(g_m) travels as one scalar

SCALE_MAX = 0  # R = max_d |v_d|   (the paper's coder)
SCALE_L2 = 1   # R = ||v||_2       (the scale of the cited multi-level quantiser, QSGD)

REF_ZERO = 0        # g~ stays zeros (Algorithm 1's initial value; the C_nz = 1 case)
REF_LAST_AVG = 1    # g~ <- averaged decoded gradient of the last iteration
REF_WINDOW_AVG = 2  # g~ <- mean of the last tau_max averaged decoded gradients

STREAM_QUANT = 0  # Philox counter word 3: draws for the rounding decision
STREAM_BATCH = 1  # Philox counter word 3: draws for minibatch row ids


@dataclasses.dataclass
class Config:
    d: int
    M: int
    bits: int = 2            # 2 (ternary) or 4 (sign + 3-bit level)
    norm: int = NORM_SUB
    quot_eps: float = 1e-8
    ref_policy: int = REF_LAST_AVG
    ref_period: int = 1      # K
    seed: int = 0
    lr: float = 0.1
    l2: float = 0.0
    batch: int = 0
    ref_window: int = 1      # tau_max for REF_WINDOW_AVG
    scale_kind: int = SCALE_MAX


# --------------------------------------------------------------------------------------
# Counter-based RNG: Philox4x32 with 10 rounds (Salmon, Moraes, Dror, Shaw, SC'11).
# One round maps the counter (c0,c1,c2,c3) under round key (k0,k1) to
#   (hi(M1*c2) ^ c1 ^ k0,  lo(M1*c2),  hi(M0*c0) ^ c3 ^ k1,  lo(M0*c0))
# and the key is advanced by the two Weyl constants between rounds.
# --------------------------------------------------------------------------------------
PHILOX_M0 = 0xD2511F53
PHILOX_M1 = 0xCD9E8D57
PHILOX_W0 = 0x9E3779B9  # floor(2^32 * (golden ratio - 1))
PHILOX_W1 = 0xBB67AE85  # floor(2^32 * (sqrt(3) - 1))
_MASK = 0xFFFFFFFF


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Philox4x32-10 on arrays of counters.  c0..c3 broadcast together; returns 4 uint32 arrays."""
    c0, c1, c2, c3 = np.broadcast_arrays(
        np.asarray(c0, dtype=U64), np.asarray(c1, dtype=U64),
        np.asarray(c2, dtype=U64), np.asarray(c3, dtype=U64))
    k0 &= _MASK
    k1 &= _MASK
    m0, m1, mask, sh = U64(PHILOX_M0), U64(PHILOX_M1), U64(_MASK), U64(32)
    for _ in range(10):
        p0 = c0 * m0            # exact: both factors < 2^32
        p1 = c2 * m1
        c0, c1, c2, c3 = ((p1 >> sh) ^ c1 ^ U64(k0), p1 & mask,
                          (p0 >> sh) ^ c3 ^ U64(k1), p0 & mask)
        k0 = (k0 + PHILOX_W0) & _MASK
        k1 = (k1 + PHILOX_W1) & _MASK
    return c0.astype(U32), c1.astype(U32), c2.astype(U32), c3.astype(U32)


def _draw_words(seed: int, it: int, m: int, stream: int, first: int, count: int):
    """Raw 32-bit draws number first..first+count-1 of the (seed, it, m, stream) sequence.

    Draw j is output lane j & 3 of the Philox block with counter (j >> 2, m, it, stream)
    and key (low 32 bits of seed, high 32 bits of seed).
    """
    if count <= 0:
        return np.zeros(0, dtype=U32)
    b0 = first >> 2
    b1 = (first + count - 1) >> 2
    blocks = np.arange(b0, b1 + 1, dtype=U64)
    out = philox4x32_10(blocks, m, it, stream, seed & _MASK, (seed >> 32) & _MASK)
    x = np.stack(out, axis=1).reshape(-1)
    off = first - 4 * b0
    return x[off:off + count]


def quant_draw_words(seed: int, it: int, m: int, d: int, first: int = 0):
    """32-bit draw for each of the elements first..first+d-1 of worker m at iteration it."""
    return _draw_words(seed, it, m, STREAM_QUANT, first, d)


STREAM_NOISE = 2


def gaussian_noise(seed: int, it: int, m: int, d: int, variance: float):
    """Synthetic gradient noise N(0, variance) of section "Nonconvex Problems" for worker m, float64[d].

    Box-Muller on the counter-based draws of stream 2: the Philox block e >> 2 serves elements
    4(e >> 2) .. +3; its words (0, 1) give the pair (cos branch for e & 3 = 0, sin branch for 1), its
    words (2, 3) the pair for e & 3 = 2, 3.  u1 = ((word >> 8) + 1) 2^-24 lies in (0, 1], u2 =
    (word >> 8) 2^-24 in [0, 1); z = sqrt(-2 ln u1) {cos, sin}(2 pi u2); noise = sigma z with
    sigma = float32(sqrt(float32(variance))).  Evaluated in float64; a binary32 evaluation agrees to a
    few units in the last place, so comparisons against it carry a tolerance.
    """
    nb = (d + 3) >> 2
    words = _draw_words(seed, it, m, STREAM_NOISE, 0, 4 * nb).reshape(nb, 4).astype(np.uint64)
    u1 = ((words[:, 0::2] >> np.uint64(8)) + np.uint64(1)).astype(np.float64) * 2.0 ** -24      # [nb][2]
    u2 = (words[:, 1::2] >> np.uint64(8)).astype(np.float64) * 2.0 ** -24
    r = np.sqrt(-2.0 * np.log(u1))
    z = np.stack([r * np.cos(2.0 * np.pi * u2), r * np.sin(2.0 * np.pi * u2)], axis=2)         # [nb][pair][cos, sin]
    sigma = np.float64(np.sqrt(F32(variance), dtype=F32))
    return (sigma * z.reshape(-1))[:d]


def uniform_from_word(x):
    """u = (x >> 8) * 2^-24: uniform on the 24-bit grid {0, ..., 1 - 2^-24}, exact in binary32."""
    return (np.asarray(x, dtype=U32) >> U32(8)).astype(F32) * F32(2.0 ** -24)


def minibatch_indices(seed: int, it: int, m: int, batch: int, n_rows: int):
    """Row ids of worker m's minibatch at iteration it: uniform on [0, n_rows), with replacement.

    idx_j = (x_j * n_rows) >> 32 in 64-bit integer arithmetic ("uniformly sampled" index,
    Background section).  Requires 0 < n_rows < 2^32.
    """
    x = _draw_words(seed, it, m, STREAM_BATCH, 0, batch).astype(U64)
    return ((x * U64(n_rows)) >> U64(32)).astype(np.int64)


# --------------------------------------------------------------------------------------
# Local gradients g^m(w_t)  (Algorithm 1, "each server calculates local gradient")
# --------------------------------------------------------------------------------------
def sigmoid64(z):
    z = np.asarray(z, dtype=np.float64)
    out = np.empty_like(z)
    pos = z >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-z[pos]))
    ez = np.exp(z[~pos])
    out[~pos] = ez / (1.0 + ez)
    return out


def grad_logreg_dense(X, y, w, idx, l2: float = 0.0):
    """Minibatch gradient of the mean log-loss with labels in {0,1}, in float64.

    g = (1/B) sum_{i in batch} (sigma(x_i . w) - y_i) x_i + l2 * w   (l2-regularised logistic
    regression of section "Convex Problems"; rows repeated in idx count repeatedly).
    """
    Xb = np.asarray(X)[np.asarray(idx)].astype(np.float64)
    w64 = np.asarray(w, dtype=np.float64)
    r = sigmoid64(Xb @ w64) - np.asarray(y)[np.asarray(idx)].astype(np.float64)
    return (r @ Xb) / float(len(idx)) + float(l2) * w64


def grad_logreg_csr(rowptr, col, val, y, w, idx, d: int, l2: float = 0.0):
    """Same gradient for rows stored as CSR (rowptr int64, col int32, val float32), float64."""
    w64 = np.asarray(w, dtype=np.float64)
    g = np.zeros(d, dtype=np.float64)
    for i in np.asarray(idx):
        a, b = int(rowptr[i]), int(rowptr[i + 1])
        c = np.asarray(col[a:b], dtype=np.int64)
        x = np.asarray(val[a:b], dtype=np.float64)
        r = sigmoid64(np.array([x @ w64[c]]))[0] - float(y[i])
        np.add.at(g, c, r * x)
    return g / float(len(idx)) + float(l2) * w64


def grad_rosenbrock(x, noise=None):
    """Gradient of f(x) = sum_i 100 (x_{i+1} - x_i^2)^2 + (1 - x_i)^2, plus additive noise.

    The d-dimensional chain form of the Rosenbrock test function of section "Nonconvex
    Problems" (whose minimum is at all-ones), with the synthetic stochastic gradient made
    the way that section does it: exact gradient + Gaussian noise, the noise being an input.
    Evaluated in binary32 with this fixed expression tree (no fused multiply-add):
        a  = x[i+1] - x[i]*x[i];   t1 = (-400*x[i]) * a;   t2 = -2 * (1 - x[i])     [i < d-1]
        b  = x[i] - x[i-1]*x[i-1]; t3 = 200 * b                                     [i > 0]
        g[i] = ((t1 + t2) + t3) + noise[i]     with absent terms left out.
    Returns float32[d].  For d = 1 the sum is empty and g = noise.
    """
    x = np.asarray(x, dtype=F32)
    d = x.shape[0]
    g = np.zeros(d, dtype=F32)
    if d >= 2:
        xi, xn = x[:-1], x[1:]
        a = xn - xi * xi
        t1 = (F32(-400.0) * xi) * a
        t2 = F32(-2.0) * (F32(1.0) - xi)
        lo = t1 + t2                       # elements 0..d-2
        b = xn - xi * xi                   # for element i+1: x[i+1] - x[i]^2
        t3 = F32(200.0) * b                # elements 1..d-1
        g[0] = lo[0]
        g[1:-1] = lo[1:] + t3[:-1]
        g[-1] = t3[-1]
    if noise is not None:
        g = g + np.asarray(noise, dtype=F32)
    return g


# --------------------------------------------------------------------------------------
# Sums that decide codes (a per-worker mean, an l2 norm) must not depend on who adds in which
# order, so their order is part of the definition: float64 terms, added
#   - within a chunk of 4096 consecutive elements: lane j (0..255) adds elements j, j+256, ...,
#     j+3840 in that order; then the 256 lane sums are added in lane order;
#   - chunk sums are added in order within groups of 256 consecutive chunks;
#   - group sums are added in order.
# Positions past the end count as +0 (adding +0 is exact).
# --------------------------------------------------------------------------------------
TREE_CHUNK = 4096
TREE_LANES = 256
TREE_GROUP = 256


def tree_sum64(x):
    """Sum of a vector of float64 terms in the fixed order described above."""
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    n = x.size
    if n == 0:
        return np.float64(0.0)
    nch = -(-n // TREE_CHUNK)
    xp = np.zeros(nch * TREE_CHUNK, dtype=np.float64)
    xp[:n] = x
    xp = xp.reshape(nch, TREE_CHUNK // TREE_LANES, TREE_LANES)
    lane = np.zeros((nch, TREE_LANES), dtype=np.float64)
    for k in range(TREE_CHUNK // TREE_LANES):
        lane = lane + xp[:, k, :]
    chunk = np.zeros(nch, dtype=np.float64)
    for j in range(TREE_LANES):
        chunk = chunk + lane[:, j]
    ngr = -(-nch // TREE_GROUP)
    cp = np.zeros(ngr * TREE_GROUP, dtype=np.float64)
    cp[:nch] = chunk
    cp = cp.reshape(ngr, TREE_GROUP)
    group = np.zeros(ngr, dtype=np.float64)
    for j in range(TREE_GROUP):
        group = group + cp[:, j]
    total = np.float64(0.0)
    for q in range(ngr):
        total = total + group[q]
    return total


def worker_mean(g_row):
    """mean(g) of section "Reference Vectors" (first option): float32(tree sum of the elements / D)."""
    g_row = np.asarray(g_row, dtype=F32)
    return F32(tree_sum64(g_row.astype(np.float64)) / np.float64(g_row.size))


# --------------------------------------------------------------------------------------
# Normalisation  (section "Normalized Gradients")
# --------------------------------------------------------------------------------------
def clamp_reference(gref, eps):
    """Reference made safe to divide by: |g~_d| < eps  ->  copysign(eps, g~_d)."""
    gref = np.asarray(gref, dtype=F32)
    eps = F32(eps)
    return np.where(np.abs(gref) < eps, np.copysign(eps, gref), gref).astype(F32)


def normalize(g, gref, norm: int, eps=1e-8, gref2=None, mu=None):
    """The vector that is handed to the coder Q: g, g - g~, g ./ g~, (g - g~) ./ g~' or g - mean(g)."""
    g = np.asarray(g, dtype=F32)
    if norm == NORM_NONE:
        return g.copy()
    if norm == NORM_MEAN:
        return g - F32(worker_mean(g) if mu is None else mu)
    if norm == NORM_SUB:
        return g - np.asarray(gref, dtype=F32)
    if norm == NORM_QUOT:
        return g / clamp_reference(gref, eps)
    if norm == NORM_COMB:
        return (g - np.asarray(gref, dtype=F32)) / clamp_reference(gref2, eps)
    raise ValueError("norm")


def denormalize(mean, gref, norm: int, eps=1e-8, gref2=None):
    """v = mean, g~ + mean, g~ (.) mean or g~' (.) mean + g~  (the decode halves of Eqs. 1, 2)."""
    mean = np.asarray(mean, dtype=F32)
    if norm == NORM_NONE or norm == NORM_MEAN:   # NORM_MEAN: each worker's mean is added back before averaging
        return mean.copy()
    if norm == NORM_SUB:
        return np.asarray(gref, dtype=F32) + mean
    if norm == NORM_QUOT:
        return clamp_reference(gref, eps) * mean
    if norm == NORM_COMB:
        return clamp_reference(gref2, eps) * mean + np.asarray(gref, dtype=F32)
    raise ValueError("norm")


# --------------------------------------------------------------------------------------
# The coder Q  (section "Gradient Compression")
# --------------------------------------------------------------------------------------
def levels_of(bits: int) -> int:
    if bits not in (2, 4):
        raise ValueError("bits must be 2 or 4")
    return (1 << (bits - 1)) - 1


def scale_of(v, kind: int = SCALE_MAX):
    """R = max_d |v_d|, or ||v||_2 = float32(sqrt(tree sum of the exact squares)); a scale below
    the smallest normal number is taken as 0."""
    v = np.asarray(v, dtype=F32)
    if kind == SCALE_L2:
        v64 = v.astype(np.float64)
        R = F32(np.sqrt(tree_sum64(v64 * v64)))       # squares of binary32 values are exact in binary64
    else:
        R = F32(np.max(np.abs(v))) if v.size else F32(0.0)
    return F32(0.0) if R < FLT_MIN else R


def quantize(v, R, bits: int, u):
    """Stochastic rounding of |v|/R onto the grid {0, 1/s, ..., 1}; returns (level, neg).

    With x = s |v| / R: level = floor(x) + [u < frac(x)], so E[level] = x.  For s = 1 this is
    P(z = 1) = |v|/R of the ternary coder.  neg is the sign bit, cleared when level = 0.
    """
    v = np.asarray(v, dtype=F32)
    s = levels_of(bits)
    R = F32(R)
    if R == 0:
        z = np.zeros(v.shape, dtype=np.int32)
        return z, z.astype(bool)
    inv_r = F32(1.0) / R
    a = np.abs(v)
    t = np.minimum(a * inv_r, F32(1.0))
    x = t * F32(s)
    lo = x.astype(np.int32)              # truncation; x is in [0, s]
    f = x - lo.astype(F32)               # exact
    level = lo + (np.asarray(u, dtype=F32) < f).astype(np.int32)
    neg = (v < 0) & (level > 0)
    return level, neg


def words_per_row(d: int, bits: int) -> int:
    per = 32 // bits
    return (d + per - 1) // per


def pack(level, neg, bits: int):
    """code = level | neg << (bits-1); element e sits in word e // (32/bits) at bit (e % (32/bits)) * bits."""
    level = np.asarray(level).astype(U32)
    code = level | (np.asarray(neg).astype(U32) << U32(bits - 1))
    per = 32 // bits
    n = code.shape[0]
    nw = words_per_row(n, bits)
    padded = np.zeros(nw * per, dtype=U32)
    padded[:n] = code
    shifts = (np.arange(per, dtype=U32) * U32(bits))[None, :]
    return np.bitwise_or.reduce(padded.reshape(nw, per) << shifts, axis=1).astype(U32)


def unpack(words, d: int, bits: int):
    """Inverse of pack: (level, neg) of the first d elements of a row of packed words."""
    words = np.asarray(words, dtype=U32)
    per = 32 // bits
    shifts = (np.arange(per, dtype=U32) * U32(bits))[None, :]
    code = ((words[:, None] >> shifts) & U32((1 << bits) - 1)).reshape(-1)[:d]
    level = (code & U32((1 << (bits - 1)) - 1)).astype(np.int32)
    neg = ((code >> U32(bits - 1)) & U32(1)).astype(bool) & (level > 0)
    return level, neg


def dequantize(level, neg, R, bits: int):
    """R sign z for the ternary coder; in general +-(R/s) level, with level = s giving R itself."""
    s = levels_of(bits)
    R = F32(R)
    step = R / F32(s)
    mag = np.where(level == s, R, step * level.astype(F32)).astype(F32)
    return np.where(neg, -mag, mag).astype(F32)


# --------------------------------------------------------------------------------------
# The five operations of the iteration
# --------------------------------------------------------------------------------------
def worker_means(g):
    """Per-worker scalars of NORM_MEAN, float32[M]."""
    return np.array([worker_mean(row) for row in np.asarray(g, dtype=F32)], dtype=F32)


def normalize_encode(cfg: Config, it: int, g, gref, gref2=None, means=None):
    """Workers' side of Algorithm 1: for each m, normalise, R_m, sample, pack.

    g float32[M][d] -> (codes uint32[M][words], scales float32[M]).  For NORM_MEAN the per-worker
    means (worker_means(g) unless given) are the third thing a worker transmits.
    """
    g = np.asarray(g, dtype=F32)
    M, d = g.shape
    codes = np.zeros((M, words_per_row(d, cfg.bits)), dtype=U32)
    scales = np.zeros(M, dtype=F32)
    if cfg.norm == NORM_MEAN and means is None:
        means = worker_means(g)
    for m in range(M):
        v = normalize(g[m], gref, cfg.norm, cfg.quot_eps, gref2, None if means is None else means[m])
        R = scale_of(v, cfg.scale_kind)
        u = uniform_from_word(quant_draw_words(cfg.seed, it, m, d))
        level, neg = quantize(v, R, cfg.bits, u)
        codes[m] = pack(level, neg, cfg.bits)
        scales[m] = R
    return codes, scales


def decode_aggregate(cfg: Config, codes, scales, gref, d: int, gref2=None, means=None):
    """Server's side: decode every worker, average in worker order, undo the normalisation.
    NORM_MEAN: worker m's value is mean_m + decoded (one rounding) before it is added."""
    M = codes.shape[0]
    acc = np.zeros(d, dtype=F32)
    for m in range(M):
        level, neg = unpack(codes[m], d, cfg.bits)
        val = dequantize(level, neg, scales[m], cfg.bits)
        if cfg.norm == NORM_MEAN:
            val = F32(means[m]) + val
        acc = acc + val
    mean = acc * (F32(1.0) / F32(M))
    return denormalize(mean, gref, cfg.norm, cfg.quot_eps, gref2)


def update_iterate(w, vbar, lr):
    """w <- w - eta * v  (two roundings)."""
    p = F32(lr) * np.asarray(vbar, dtype=F32)
    return np.asarray(w, dtype=F32) - p


def update_reference(cfg: Config, it: int, vbar, gref, history=None):
    """Reference after iteration it.  Refresh happens when (it + 1) is a multiple of K.

    REF_LAST_AVG: g~ <- v of this iteration.  REF_WINDOW_AVG: g~ <- (sum of the last
    ref_window v's, oldest first) * (1/ref_window); history is the caller-kept list of past
    v's, this iteration's included.  REF_ZERO: unchanged.
    """
    if cfg.ref_policy == REF_ZERO or (it + 1) % cfg.ref_period != 0:
        return np.asarray(gref, dtype=F32).copy()
    if cfg.ref_policy == REF_LAST_AVG:
        return np.asarray(vbar, dtype=F32).copy()
    if cfg.ref_policy == REF_WINDOW_AVG:
        past = history[-cfg.ref_window:]
        acc = np.zeros_like(np.asarray(vbar, dtype=F32))
        for h in past:
            acc = acc + np.asarray(h, dtype=F32)
        return acc * (F32(1.0) / F32(cfg.ref_window))
    raise ValueError("ref_policy")


def step(cfg: Config, it: int, w, gref, g, gref2=None, history=None):
    """One whole iteration from given local gradients g[M][d].

    history: the decoded averages of the earlier iterations, oldest first (only read by the
    window-average reference).  Returns (w_next, gref_next, codes, scales, vbar).
    """
    means = worker_means(g) if cfg.norm == NORM_MEAN else None
    codes, scales = normalize_encode(cfg, it, g, gref, gref2, means)
    vbar = decode_aggregate(cfg, codes, scales, gref, g.shape[1], gref2, means)
    w_next = update_iterate(w, vbar, cfg.lr)
    past = None if history is None else list(history) + [vbar]
    gref_next = update_reference(cfg, it, vbar, gref, past)
    return w_next, gref_next, codes, scales, vbar
