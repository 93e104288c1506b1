"""GPU parity of the counter-based RNG and the minibatch ids (bit-exact), plus an independent
pin of the oracle's Philox4x32-10 against rocRAND's generator of the same name."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import tng_oracle as O
from gpu_util import DEV, make_ctx, say, u32
from paper_1901_08227_amd import binding as B

pytestmark = pytest.mark.gpu


def test_raw_draws_match_the_oracle_bit_for_bit():
    for seed in (0, 1, 0x0123456789ABCDEF, (1 << 64) - 1):
        ctx = make_ctx(64, 1, 2, B.NORM_NONE, seed=seed)
        for it, worker, stream, first, count in [(0, 0, 0, 0, 1), (3, 2, 0, 0, 4099), (7, 65000, 1, 5, 1000),
                                                 ((1 << 32) - 1, 9, 0, 3, 77), (1, 1, 0, (1 << 30) + 1, 513)]:
            say(f"rng seed={seed} it={it} worker={worker} stream={stream} first={first} count={count}")
            out = torch.zeros(count, dtype=torch.int32, device=DEV)
            ctx.rng_draws(it, worker, stream, first, count, out)
            torch.cuda.synchronize()
            ref = O._draw_words(seed, it, worker, stream, first, count)
            assert np.array_equal(u32(out), ref)
        ctx.close()


def test_oracle_philox_agrees_with_rocrand():
    """rocRAND's PHILOX4_32_10 with seed s and offset 0 emits, in order, the outputs of the blocks
    with key (s low, s high) and counter (i, 0, 0, 0): the oracle must reproduce that stream."""
    lib = ctypes.CDLL("librocrand.so")
    gen = ctypes.c_void_p()
    assert lib.rocrand_create_generator(ctypes.byref(gen), 404) == 0          # ROCRAND_RNG_PSEUDO_PHILOX4_32_10
    try:
        for seed in (0, 12345, 0xDEADBEEFCAFEF00D):
            assert lib.rocrand_set_seed(gen, ctypes.c_ulonglong(seed)) == 0
            assert lib.rocrand_set_offset(gen, ctypes.c_ulonglong(0)) == 0
            n = 4096
            out = torch.zeros(n, dtype=torch.int32, device=DEV)
            assert lib.rocrand_generate(gen, ctypes.c_void_p(out.data_ptr()), ctypes.c_size_t(n)) == 0
            torch.cuda.synchronize()
            got = u32(out)
            blocks = np.arange(n // 4, dtype=np.uint64)
            ref = np.stack(O.philox4x32_10(blocks, 0, 0, 0, seed & 0xFFFFFFFF, seed >> 32), axis=1).reshape(-1)
            say(f"rocrand seed={seed}: first words {got[:4]} vs oracle {ref[:4]}")
            assert np.array_equal(got, ref)
    finally:
        lib.rocrand_destroy_generator(gen)


def test_minibatch_indices_match_the_oracle():
    M, d, batch = 5, 16, 37
    n_rows = [1, 2, 2000, 65536, 100000]
    ctx = make_ctx(d, M, 2, B.NORM_SUB, seed=77, batch=batch, problem=B.PROB_LOGREG_DENSE)
    X = [torch.zeros((n, d), device=DEV) for n in n_rows]
    y = [torch.zeros(n, device=DEV) for n in n_rows]
    ctx.set_logreg_dense(X, y)
    idx = torch.zeros((M, batch), dtype=torch.int32, device=DEV)
    for it in (0, 1, 99):
        say(f"minibatch ids it={it}")
        ctx.minibatch_indices(it, idx)
        torch.cuda.synchronize()
        got = u32(idx).astype(np.int64)
        for m in range(M):
            assert np.array_equal(got[m], O.minibatch_indices(77, it, m, batch, n_rows[m]))
    ctx.close()
