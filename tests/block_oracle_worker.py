"""Worker-process side of the full-stack parity test: the float64 oracle step of ONE gradient block (blocks
are independent through accumulate -> roots -> precondition, paper Section 4.1), compared with what the GPU
produced for that block.  Runs in a spawned process that imports numpy and the oracle only (no torch, no GPU);
inputs and GPU outputs arrive as memory-mapped .npy files, the return value is a handful of error figures."""
from __future__ import annotations

import numpy as np


def _errs(x, ref):
    x = np.asarray(x, dtype=np.float64)
    d = x - ref
    return float(np.sqrt((d * d).sum()) / np.sqrt((ref * ref).sum())), float(np.abs(d).max() / np.abs(ref).max())


def check_block(args):
    """args = (directory, j, n_steps, beta, eps, p).  Files in directory: G_<t>.npy (fp32 [n, B, B], the gradients
    of step t for the sampled blocks, the last one is the checked step) and gpu_{L,R,XL,XR,U}.npy (fp32 [n, B, B]).
    Returns (j, {name: (rel. Frobenius error, largest element-wise deviation / max |ref|)})."""
    directory, j, n_steps, beta, eps, p = args
    try:
        from threadpoolctl import threadpool_limits
        limiter = threadpool_limits(limits=1)       # one BLAS thread per worker: the pool is the parallelism
    except Exception:                               # pragma: no cover
        limiter = None
    from oracle import shampoo as oshampoo
    B = np.load(f"{directory}/G_0.npy", mmap_mode="r").shape[1]
    L = np.zeros((1, B, B))
    R = np.zeros((1, B, B))
    for t in range(n_steps - 1):
        G = np.array(np.load(f"{directory}/G_{t}.npy", mmap_mode="r")[j:j + 1])
        L, R = oshampoo.accumulate_factors(G, L, R, beta)
    G = np.array(np.load(f"{directory}/G_{n_steps - 1}.npy", mmap_mode="r")[j:j + 1])
    ref = oshampoo.step(G, L, R, beta=beta, eps=eps, p=p)
    out = {}
    for name, key in (("L", "L"), ("R", "R"), ("XL", "X_L"), ("XR", "X_R"), ("U", "U")):
        gpu = np.load(f"{directory}/gpu_{name}.npy", mmap_mode="r")[j]
        out[name] = _errs(gpu, ref[key][0])
    if limiter is not None:
        limiter.restore_original_limits()
    return j, out
