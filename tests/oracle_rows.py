"""Oracle attention rows in worker PROCESSES (the oracle's row routine holds the interpreter lock most of
the time, so threads do not scale).  The workers are spawned, not forked: they are fresh interpreters that
import numpy, the input generator and the oracle only -- never torch, never the GPU -- and regenerate the
seeded workload themselves, so nothing but row indices, mask rows and results crosses the pipe."""
from __future__ import annotations

import multiprocessing as mp
import os
import sys
from concurrent.futures import ProcessPoolExecutor

import numpy as np

_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
_INPUTS = {}


def _workload_inputs(cfg: str, cut: int):
    key = (cfg, cut)
    if key not in _INPUTS:
        if _ROOT not in sys.path:
            sys.path.insert(0, _ROOT)
        import rr_inputs as ri
        x = ri.generate(ri.get_config(cfg))
        if cut:
            x = {k: np.ascontiguousarray(v[:, :cut]) for k, v in x.items()}
        _INPUTS.clear()                      # one workload at a time per worker
        _INPUTS[key] = x
    return _INPUTS[key]


def _rows_task(task):
    cfg, cut, B, G, items = task
    if _ROOT not in sys.path:
        sys.path.insert(0, _ROOT)
    from oracle import rr_oracle as oracle
    x = _workload_inputs(cfg, cut)
    out = []
    for (h, m, mask_row) in items:
        out.append(oracle.attention_row_block(x["Q"][h], x["K"][h // G], x["V"][h // G], mask_row, m, B))
    return out


_POOL = None


def _ready(_):
    return os.getpid()


def pool(workers: int = 12) -> ProcessPoolExecutor:
    """The workers run one BLAS thread each (the parallelism is across rows): the thread-count variables are
    set only while the workers are being spawned, and put back for this process afterwards."""
    global _POOL
    if _POOL is None:
        names = ("OMP_NUM_THREADS", "OPENBLAS_NUM_THREADS", "MKL_NUM_THREADS")
        saved = {k: os.environ.get(k) for k in names}
        try:
            for k in names:
                os.environ[k] = "1"
            _POOL = ProcessPoolExecutor(max_workers=workers, mp_context=mp.get_context("spawn"))
            list(_POOL.map(_ready, range(4 * workers)))       # all workers exist before the variables go back
        finally:
            for k, v in saved.items():
                if v is None:
                    os.environ.pop(k, None)
                else:
                    os.environ[k] = v
    return _POOL


def attention_rows(cfg: str, cut: int, B: int, G: int, rows, mask_np, workers: int = 12, progress=None):
    """[(O block, lse block)] of oracle.attention_row_block for the (h, m) pairs `rows` of workload `cfg`
    (cut to its first `cut` positions when cut > 0) under the masks mask_np[h, m]."""
    rows = list(rows)
    per = max(1, min(16, -(-len(rows) // (4 * workers))))
    tasks = [(cfg, cut, B, G, [(h, m, np.ascontiguousarray(mask_np[h, m])) for (h, m) in rows[i:i + per]])
             for i in range(0, len(rows), per)]
    out = []
    done = 0
    for res in pool(workers).map(_rows_task, tasks):
        out.extend(res)
        done += len(res)
        if progress and done % (16 * per) < per:
            progress(done, len(rows))
    return out
