"""Helpers shared by the GPU parity tests (marshalling between numpy and torch)."""
import numpy as np
import torch

import grid


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a))
    if dtype is not None:
        t = t.view(dtype) if t.element_size() == torch.empty((), dtype=dtype).element_size() else t.to(dtype)
    return t.cuda()


def host_u32(t):
    return t.cpu().numpy().view(np.uint32)


def tree_kw(p):
    return dict(max_depth=p["max_depth"], max_bins=p["max_bins"], lam=p["lam"], gamma=p["gamma"],
                min_child_weight=p["min_child_weight"])


def oracle_prep(oracle, X, B):
    """Oracle-side quantisation and packing of a dense matrix."""
    cuts, nb = oracle.cuts(X, B)
    sym, missing, mx = oracle.bin_matrix(X, cuts, nb)
    bits = oracle.bits_for(mx)
    words = oracle.pack(sym, bits)
    return dict(cuts=cuts, nb=nb, sym=sym, missing=missing, max_value=mx, bits=bits, words=words)


def hist_tolerance(oracle_hist, cnt, scale, rtol=1e-5):
    """|gpu - oracle| allowed per bin: rtol*|oracle| plus the fixed-point rounding
    bound, half a quantum per accumulated row."""
    tol = rtol * np.abs(oracle_hist)
    tol[..., 0] += cnt * (0.5 / scale[0])
    tol[..., 1] += cnt * (0.5 / scale[1])
    return tol + 1e-300


def judge_on_grid(oracle, judge, tree, o, gp, scale, **kw):
    """The tree judged in the GPU library's own precision: on the pairs moved onto its fixed-point grid every
    fp64 sum of the oracle is exact, so totals and weights must agree to rounding of the last operation and
    every decision (valid child? larger gain? above gamma?) must come out the same: the oracle's exhaustive
    best split at every node, no ties to excuse."""
    q, scale_o = grid.fixed_point(gp)
    assert tuple(scale) == scale_o
    rep = judge(tree, o["sym"], o["nb"], o["missing"], grid.on_grid(gp), **kw, sum_rtol=1e-13, tie_rtol=1e-13,
                sum_atol_per_row=0.0)
    assert rep["ok"] and rep["identical"] and not rep["ties"], (rep["errors"][:5], rep["ties"][:3])
    return rep
