"""Shared helpers of the GPU parity tests: run the oracle on the same rounded inputs the GPU sees."""
import numpy as np
import torch

import workloads as W
from oracle import isa_oracle as O


def f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def problem_of(wl: W.Workload, **kw):
    import paper_2605_04569_amd as I
    d = dict(H=wl.H, D=wl.D, dtype=wl.dtype, block=wl.block, seg_len=[wl.seg_len(b) for b in range(wl.B)],
             keep_ratio=wl.keep_ratio, full_frac=wl.full_frac, exact_frac=wl.exact_frac, gamma=wl.gamma)
    d.update(kw)
    return I.Problem(**d)


def oracle_plan(wl: W.Workload, Q, K, V, b, h, **kw):
    n = wl.tokens(b)
    args = dict(keep_ratio=wl.keep_ratio, full_frac=wl.full_frac, exact_frac=wl.exact_frac, gamma=wl.gamma)
    args.update(kw)
    return O.isa_plan(f64(Q[b, h, :n]), f64(K[b, h, :n]), f64(V[b, h, :n]), wl.seg_len(b), wl.block, **args)


def selection_is_valid(scores64, chosen, k, rtol):
    """`chosen` (indices into scores64) is an acceptable top-k of scores64 up to relative score noise rtol:
    k distinct entries, none of which is beaten by an unchosen entry by more than the noise."""
    chosen = [int(x) for x in chosen]
    if len(chosen) != k or len(set(chosen)) != k:
        return False
    if k == 0 or k == len(scores64):
        return True
    rest = np.setdiff1d(np.arange(len(scores64)), chosen)
    lo, hi = scores64[chosen].min(), scores64[rest].max()
    return lo >= hi - rtol * max(abs(lo), abs(hi))


def err_stats(got: np.ndarray, want: np.ndarray):
    d = np.abs(got - want)
    return float(d.max()), float(d.mean())
