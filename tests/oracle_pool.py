"""Host processes that run the oracle's CSR logistic gradient for many workers side by side.

The oracle's gradient loops over the minibatch rows in the interpreter, so threads do not help it; at
64 workers x 512 rows x 16 777 entries it takes minutes in one process.  The parent (which holds the
GPU) writes the inputs as .npy files under a scratch directory in /dev/shm, fresh interpreters
(start method "spawn": nothing of the parent's GPU state is inherited, and they never touch the GPU)
map them read-only, call the oracle, and send back only the error figures of the comparison.
Imports numpy and the oracle only.
"""
import multiprocessing
import os
import shutil
import tempfile

import numpy as np

EPS32 = 2.0 ** -24


def _task(args):
    import threadpoolctl

    with threadpoolctl.threadpool_limits(1):   # the processes are the parallelism; BLAS threads would only spin
        return _compare(args)


def _compare(args):
    root, m, ids, d, l2, rel = args
    from oracle import tng_oracle as O

    load = lambda name: np.load(os.path.join(root, name), mmap_mode="r")
    rowptr, col, val, y = (load(f"{k}{m}.npy") for k in ("rowptr", "col", "val", "y"))
    w = np.asarray(load("w.npy"))
    got = np.asarray(load("g.npy")[m], dtype=np.float64)
    ref = O.grad_logreg_csr(rowptr, col, val, y, w, ids, d, l2)
    # per-coordinate size of what an fp32 evaluation adds up (see gpu_util.logistic_condition)
    w64 = w.astype(np.float64)
    cond = np.zeros(d, dtype=np.float64)
    for i in ids:
        a, b = int(rowptr[i]), int(rowptr[i + 1])
        c = np.asarray(col[a:b], dtype=np.int64)
        x = np.asarray(val[a:b], dtype=np.float64)
        r = O.sigmoid64(np.array([x @ w64[c]]))[0] - float(y[i])
        np.add.at(cond, c, (abs(r) + 0.25 * (np.abs(x) @ np.abs(w64[c]))) * np.abs(x))
    cond = cond / float(len(ids)) + abs(l2) * np.abs(w64)
    diff = np.abs(got - ref)
    return {
        "m": m,
        "norm2_ok": bool(np.linalg.norm(got - ref) <= rel * np.linalg.norm(ref)),
        "max_ok": bool(diff.max() <= rel * np.abs(ref).max()),
        "elementwise_ok": bool(np.all(diff <= rel * np.abs(ref) + 4 * EPS32 * cond)),
        "rel2": float(np.linalg.norm(got - ref) / max(np.linalg.norm(ref), 1e-300)),
        "nonzero": int(np.count_nonzero(ref)),
    }


class CsrGradientChecker:
    """shards: per worker (rowptr, col, val, y) as numpy arrays.  check(w, g, ids) compares g[m] (the
    library's float32 gradients) with the oracle's float64 gradient of worker m on minibatch ids[m] and
    returns one record per worker."""

    def __init__(self, shards, d, l2=0.0, processes=8):
        self.root = tempfile.mkdtemp(prefix="tng_oracle_", dir="/dev/shm" if os.path.isdir("/dev/shm") else None)
        self.d, self.l2, self.M = d, l2, len(shards)
        for m, sh in enumerate(shards):
            for k, a in zip(("rowptr", "col", "val", "y"), sh):
                np.save(os.path.join(self.root, f"{k}{m}.npy"), np.ascontiguousarray(a))
        self.pool = multiprocessing.get_context("spawn").Pool(min(processes, self.M))

    def check(self, w, g, ids, rel=1e-5):
        np.save(os.path.join(self.root, "w.npy"), np.ascontiguousarray(w, dtype=np.float32))
        np.save(os.path.join(self.root, "g.npy"), np.ascontiguousarray(g, dtype=np.float32))
        tasks = [(self.root, m, np.asarray(ids[m]), self.d, self.l2, rel) for m in range(self.M)]
        return self.pool.map(_task, tasks, chunksize=1)

    def close(self):
        self.pool.close()
        self.pool.join()
        shutil.rmtree(self.root, ignore_errors=True)
