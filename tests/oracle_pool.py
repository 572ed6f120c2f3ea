"""Runs oracle samples in worker processes (test and benchmark infrastructure).

The oracle is plain single-threaded numpy; a full-size parity test wants hundreds of sampled outputs
and the benchmark's CPU baseline is defined on all host cores, so both hand independent samples -
one (sequence, KV head) pair, one window row - to a pool of processes.  Workers are started with the
"spawn" method and import only numpy and the oracle (never torch, never the GPU library): a process
that has initialised the GPU must not be forked.  Every task carries plain numpy arrays and calls
the oracle's own functions unchanged.
"""
from __future__ import annotations

import atexit
import multiprocessing as mp
import os
from concurrent.futures import ProcessPoolExecutor

_POOL = None
_WORKERS = 0


def n_workers() -> int:
    """Worker count: the host cores this process may use, at most 16 (the CPU share of a one-GPU machine)."""
    try:
        n = len(os.sched_getaffinity(0))
    except AttributeError:  # pragma: no cover
        n = os.cpu_count() or 1
    return max(1, min(16, n))


def pool() -> ProcessPoolExecutor:
    global _POOL, _WORKERS
    if _POOL is None:
        _WORKERS = n_workers()
        _POOL = ProcessPoolExecutor(max_workers=_WORKERS, mp_context=mp.get_context("spawn"))
    return _POOL


def shutdown():
    """Stop the workers (idempotent).  Workers that are still busy are killed: nothing here is worth
    waiting for once the caller is done or has failed."""
    global _POOL
    if _POOL is not None:
        procs = list(getattr(_POOL, "_processes", {}).values())
        _POOL.shutdown(wait=False, cancel_futures=True)
        for p in procs:
            if p.is_alive():
                p.kill()
        _POOL = None


atexit.register(shutdown)


def _limit_blas_threads():
    # one oracle sample per process: numpy's BLAS must not start a thread team of its own per worker
    try:
        from threadpoolctl import threadpool_limits
        threadpool_limits(limits=1)
    except Exception:  # pragma: no cover
        pass


def draft_task(task):
    """task: {"q": uint16 [n, 128] query bit patterns of heads that share the KV head, "scale": float,
    "kv": keyword arguments of oracle.draft_keys for sequence 0 / head 0 of a one-pair slice}.
    Returns [(out [128], lse)] per query and the seconds spent in the oracle."""
    import time

    from oracle import vc_oracle as O
    _limit_blas_threads()
    t0 = time.perf_counter()
    k, v = O.draft_keys(0, 0, n_kv_heads=1, **task["kv"])
    res = []
    for q in task["q"]:
        o, lse, _ = O.attend(O.bf16_to_f64(q), k, v, task["scale"])
        res.append((o, lse))
    return res, time.perf_counter() - t0


def verify_task(task):
    """task: one-pair slices (bit patterns) q_win [w, 1, 128], k_full / v_full [n, 1, 128], k_win / v_win
    [w, 1, 128], "rows": window rows to evaluate, "scale".  Returns [(out [128], lse)] per row."""
    import numpy as np

    from oracle import vc_oracle as O
    _limit_blas_threads()
    n, w = task["k_full"].shape[0], task["q_win"].shape[0]
    res = []
    for i in task["rows"]:
        res.append(O.verify_attn_one(task["q_win"], task["k_full"], task["v_full"], task["k_win"], task["v_win"],
                                     np.array([0, n]), np.array([0, w]), 0, int(i), 0, task["scale"],
                                     n_q_heads=1, n_kv_heads=1))
    return res


def run(fn, tasks, timeout: float = 900.0):
    """Map `fn` over `tasks` on the pool, results in task order.  Any failure (a worker that died, a
    task that raised, the time limit) tears the pool down before it propagates, so that no half-dead
    pool is left to block the interpreter's exit."""
    try:
        return list(pool().map(fn, tasks, chunksize=1, timeout=timeout))
    except BaseException:
        shutdown()
        raise
