"""Host-side checks of the C-ABI boundary that need no GPU: the built library loads, exports
every function include/tng.h declares, sizes and validates configurations, and rejects bad
arguments before anything is enqueued."""
import ctypes
import os
import re

import pytest

from paper_1901_08227_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _cfg(**kw):
    base = dict(d=1000, M=4, bits=2, norm=B.NORM_SUB, quot_eps=1e-8, ref_policy=B.REF_LAST_AVG, ref_period=1,
                seed=0, lr=0.1, l2=0.0, batch=64, problem=B.PROB_LOGREG_DENSE, ref_window=1)
    base.update(kw)
    return B.TngConfig(**base)


def test_library_exports_every_declared_entry_point():
    header = open(os.path.join(ROOT, "include", "tng.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(tng_[a-z0-9_]+)\s*\(", header))
    assert {"tng_local_grad", "tng_normalize_encode", "tng_decode_aggregate", "tng_update_reference",
            "tng_step", "tng_create", "tng_destroy", "tng_workspace_bytes"} <= names
    L = B.lib()
    for n in sorted(names):
        assert hasattr(L, n), f"{n} is declared in include/tng.h but not exported"


def test_config_struct_matches_the_header_layout():
    # d(8) M(4) bits(4) norm(4) eps(4) policy(4) period(4) seed(8) lr(4) l2(4) batch(4) problem(4) window(4) scale(4)
    assert ctypes.sizeof(B.TngConfig) == 64 and B.TngConfig.ref_window.offset == 56 and B.TngConfig.scale.offset == 60
    assert B.TngConfig.seed.offset == 32 and B.TngConfig.problem.offset == 52


def test_binding_constants_match_the_header_enums():
    header = open(os.path.join(ROOT, "include", "tng.h")).read()
    enums = {k: int(v) for k, v in re.findall(r"\b(TNG_[A-Z0-9_]+)\s*=\s*(-?\d+)", header)}
    for name, value in enums.items():
        short = name[len("TNG_"):]
        if short.startswith("ERR_") or short == "OK":
            assert getattr(B, name) == value, name
        else:
            assert getattr(B, short) == value, name
    assert {"TNG_NORM_MEAN", "TNG_SCALE_L2", "TNG_REF_WINDOW_AVG", "TNG_PROB_ROSENBROCK", "TNG_ERR_HIP"} <= set(enums)


def test_words_per_row():
    for d in (1, 15, 16, 17, 1000, 1 << 27):
        assert B.tng_words_per_row(d, 2) == -(-d // 16)
        assert B.tng_words_per_row(d, 4) == -(-d // 8)
    assert B.tng_words_per_row(100, 3) == 0


def test_workspace_size_and_config_validation():
    assert B.tng_workspace_bytes(_cfg()) >= 4 * 64 * 8
    assert B.tng_workspace_bytes(_cfg(problem=B.PROB_EXTERNAL, batch=0)) > 0
    assert B.tng_workspace_bytes(_cfg(problem=B.PROB_LOGREG_CSR, d=65535 << 14, M=1, batch=1)) > 0
    bad = [dict(d=0), dict(M=0), dict(bits=3), dict(bits=8), dict(norm=7), dict(norm=5), dict(norm=-1), dict(scale=2), dict(scale=-1), dict(quot_eps=0.0),
           dict(quot_eps=float("nan")), dict(ref_policy=5), dict(ref_period=0), dict(lr=float("inf")),
           dict(l2=float("nan")), dict(batch=0), dict(problem=9), dict(d=(1 << 34) + 1), dict(M=70000),
           dict(ref_policy=B.REF_WINDOW_AVG, ref_window=0),
           dict(problem=B.PROB_LOGREG_CSR, d=(65535 << 14) + 1)]
    for kw in bad:
        assert B.tng_workspace_bytes(_cfg(**kw)) == 0, kw
        h = ctypes.c_void_p()
        st = B.lib().tng_create(ctypes.byref(_cfg(**kw)), ctypes.c_void_p(0x1000), 1 << 20, None, ctypes.byref(h))
        assert st == B.TNG_ERR_INVALID_ARG and not h


def test_workspace_grows_by_the_row_sum_scratch():
    base = B.tng_workspace_bytes(_cfg(d=1 << 22, problem=B.PROB_EXTERNAL, batch=0))
    for kw in (dict(norm=B.NORM_MEAN), dict(scale=B.SCALE_L2)):
        more = B.tng_workspace_bytes(_cfg(d=1 << 22, problem=B.PROB_EXTERNAL, batch=0, **kw))
        # 1024 chunk sums, 1024 (min, max) pairs and 4 group sums of 8 bytes for each of the 4 workers
        assert more - base >= 4 * (2048 + 4) * 8 and more - base < 4 * (2048 + 4) * 8 + 256


def _fake_ctx(**kw):
    cfg = _cfg(**kw)
    h = ctypes.c_void_p()
    # a fake, never dereferenced, 256-byte aligned "device" address: no call below reaches a launch
    st = B.lib().tng_create(ctypes.byref(cfg), ctypes.c_void_p(0x10000), 1 << 20, None, ctypes.byref(h))
    assert st == B.TNG_OK and h
    return h


def test_create_rejects_bad_workspace():
    cfg = _cfg()
    h = ctypes.c_void_p()
    L = B.lib()
    assert L.tng_create(ctypes.byref(cfg), None, 1 << 20, None, ctypes.byref(h)) == B.TNG_ERR_WORKSPACE
    assert L.tng_create(ctypes.byref(cfg), ctypes.c_void_p(0x10010), 1 << 20, None, ctypes.byref(h)) == B.TNG_ERR_WORKSPACE
    assert L.tng_create(ctypes.byref(cfg), ctypes.c_void_p(0x10000), 16, None, ctypes.byref(h)) == B.TNG_ERR_WORKSPACE
    assert L.tng_create(ctypes.byref(cfg), ctypes.c_void_p(0x10000), 1 << 20, None, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_destroy(None) == B.TNG_ERR_INVALID_ARG


def test_calls_reject_null_and_misaligned_pointers_before_launching():
    L = B.lib()
    h = _fake_ctx()
    p = ctypes.c_void_p(0x20000)
    odd = ctypes.c_void_p(0x20004)
    assert L.tng_normalize_encode(h, 0, None, p, p, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_normalize_encode(h, 0, p, None, p, p) == B.TNG_ERR_INVALID_ARG      # SUB needs a reference
    assert L.tng_normalize_encode(h, 0, odd, p, p, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_normalize_encode(h, 0, p, p, None, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_normalize_encode(None, 0, p, p, p, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_decode_aggregate(h, p, p, p, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_decode_aggregate(h, p, None, p, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_decode_aggregate(h, p, p, p, odd) == B.TNG_ERR_INVALID_ARG
    assert L.tng_update_reference(h, 0, None, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_step(h, 0, None, p, p, p, p, p) == B.TNG_ERR_INVALID_ARG
    assert L.tng_step(h, 0, p, p, p, p, p, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_local_grad(h, 0, p, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_rng_draws(h, 0, 0, 0, 0, 4, None) == B.TNG_ERR_INVALID_ARG
    # problem data missing -> BAD_STATE, still nothing launched
    assert L.tng_local_grad(h, 0, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_minibatch_indices(h, 0, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_step(h, 0, p, p, p, p, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_set_noise(h, p) == B.TNG_ERR_BAD_STATE                                # not a Rosenbrock context
    assert L.tng_set_noise_variance(h, 0.01) == B.TNG_ERR_BAD_STATE
    assert L.tng_destroy(h) == B.TNG_OK
    # the combined normalisation needs its second reference first
    h = _fake_ctx(norm=B.NORM_COMB, problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_normalize_encode(h, 0, p, p, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_set_second_reference(h, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_local_grad(h, 0, p, p) == B.TNG_ERR_BAD_STATE                         # external gradients
    assert L.tng_destroy(h) == B.TNG_OK
    # the per-worker mean reference needs the array its means travel in; it needs no shared reference
    h = _fake_ctx(norm=B.NORM_MEAN, problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_normalize_encode(h, 0, p, None, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_decode_aggregate(h, p, p, None, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_set_worker_means(h, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_set_worker_means(h, ctypes.c_void_p(0x20002)) == B.TNG_ERR_INVALID_ARG
    assert L.tng_destroy(h) == B.TNG_OK
    h = _fake_ctx(problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_set_worker_means(h, p) == B.TNG_ERR_BAD_STATE                         # not a mean-reference context
    assert L.tng_destroy(h) == B.TNG_OK
    h = _fake_ctx(problem=B.PROB_ROSENBROCK, batch=0)
    assert L.tng_set_noise_variance(h, -1.0) == B.TNG_ERR_INVALID_ARG
    assert L.tng_set_noise_variance(h, float("nan")) == B.TNG_ERR_INVALID_ARG
    assert L.tng_set_noise_variance(h, float("inf")) == B.TNG_ERR_INVALID_ARG
    assert L.tng_set_noise_variance(h, 0.01) == B.TNG_OK and L.tng_set_noise_variance(h, 0.0) == B.TNG_OK
    assert L.tng_destroy(h) == B.TNG_OK
    # the optional CSR tile index: sized from the row counts, needs the shards first
    rows = (ctypes.c_uint64 * 4)(100, 200, 300, 400)
    cfg = _cfg(problem=B.PROB_LOGREG_CSR, d=(1 << 15) + 1)
    assert L.tng_csr_index_bytes(ctypes.byref(cfg), rows) >= 1000 * 4 * 4       # 3 tiles + 1 offsets per row
    assert L.tng_csr_index_bytes(ctypes.byref(_cfg()), rows) == 0                # dense problem
    assert L.tng_csr_index_bytes(ctypes.byref(cfg), None) == 0
    h = _fake_ctx(problem=B.PROB_LOGREG_CSR)
    assert L.tng_set_csr_index(h, p, 1 << 20) == B.TNG_ERR_BAD_STATE             # no shards yet
    assert L.tng_set_csr_index(h, None, 1 << 20) == B.TNG_ERR_INVALID_ARG
    assert L.tng_destroy(h) == B.TNG_OK
    # update_reference is a no-op (and OK) when no refresh is due
    h = _fake_ctx(ref_period=16, problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_update_reference(h, 3, p, p) == B.TNG_OK
    assert L.tng_destroy(h) == B.TNG_OK
    h = _fake_ctx(ref_policy=B.REF_ZERO, problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_update_reference(h, 0, p, p) == B.TNG_OK
    assert L.tng_set_reference_history(h, p) == B.TNG_ERR_BAD_STATE                    # not a window-average context
    assert L.tng_destroy(h) == B.TNG_OK
    # the window-average reference needs its history buffer first
    h = _fake_ctx(ref_policy=B.REF_WINDOW_AVG, ref_window=4, problem=B.PROB_EXTERNAL, batch=0)
    assert L.tng_update_reference(h, 0, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_step(h, 0, p, p, p, p, p, p) == B.TNG_ERR_BAD_STATE
    assert L.tng_set_reference_history(h, None) == B.TNG_ERR_INVALID_ARG
    assert L.tng_destroy(h) == B.TNG_OK


def test_status_strings():
    seen = {B.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen


def test_binding_refuses_cpu_tensors():
    import torch
    with pytest.raises(TypeError):
        B._ptr(torch.zeros(4), torch.float32, 4, "g")
