"""Optimal pipeline partition by exhaustive enumeration (test infrastructure,
not the product), plus the ctypes front end of the set-by-set evaluation of the
paper's recurrence (Eq. 3) in partition_oracle.c.

Problem (paper sections 3.2-3.3): choose S <= D distinct devices in an order
and cut the L layers into S consecutive non-empty runs, stage k on device u_k.
A stage's period is max(T_comp(layers, u_k), T_comm(u_k, u_{k+1}, P_j)) with
T_comm = P_j / b_{u,v} (Eq. 1, Eq. 2), j the stage's last layer; the last stage
sends nothing.  A strategy is feasible if the memory of each stage's layers
fits its device.  T_opt is the smallest achievable largest period.

Readings taken where the paper leaves a choice: T_comp of a run of layers is
the sum of per-layer times, accumulated first layer to last starting from 0.0;
among all strategies reaching T_opt the canonical answer is the one whose
sequence (u_1, e_1, u_2, e_2, ...) (device id, last layer of the stage) is
lexicographically smallest.

The search space has sum_{k=1}^{min(D,L)} D!/(D-k)! * C(L-1, k-1) strategies
(section 3.3); only small instances are enumerated.
"""
from __future__ import annotations

import ctypes as C
import itertools
import math
import os
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import build as _build

Strategy = List[Tuple[int, int, int]]       # (device, first layer, last layer), 0-based inclusive


def search_space_size(L: int, D: int) -> int:
    return sum(math.perm(D, k) * math.comb(L - 1, k - 1) for k in range(1, min(D, L) + 1))


def all_strategies(L: int, D: int):
    """Every ordered choice of k distinct devices and every composition of L into k parts."""
    for k in range(1, min(D, L) + 1):
        for cuts in itertools.combinations(range(1, L), k - 1):
            ends = list(cuts) + [L]                    # exclusive ends
            starts = [0] + list(cuts)
            for devs in itertools.permutations(range(D), k):
                yield [(devs[s], starts[s], ends[s] - 1) for s in range(k)]


def stage_period(t_comp, xfer_bytes, bw, dev: int, first: int, last: int,
                 next_dev: Optional[int]) -> float:
    comp = 0.0
    for layer in range(first, last + 1):
        comp = comp + float(t_comp[layer][dev])
    if next_dev is None:
        return comp
    comm = float(xfer_bytes[last]) / float(bw[dev][next_dev])
    return comp if comp >= comm else comm


def evaluate(strategy: Strategy, t_comp, layer_mem, dev_mem, xfer_bytes, bw) -> Optional[float]:
    """Largest stage period of a strategy, or None if a stage does not fit in memory."""
    worst = 0.0
    for s, (dev, first, last) in enumerate(strategy):
        need = 0.0
        for layer in range(first, last + 1):
            need = need + float(layer_mem[layer])
        if need > float(dev_mem[dev]):
            return None
        nxt = strategy[s + 1][0] if s + 1 < len(strategy) else None
        per = stage_period(t_comp, xfer_bytes, bw, dev, first, last, nxt)
        if per > worst:
            worst = per
    return worst


def canonical_key(strategy: Strategy) -> Tuple[int, ...]:
    key: List[int] = []
    for dev, _first, last in strategy:
        key += [dev, last]
    return tuple(key)


def brute_force(t_comp, layer_mem, dev_mem, xfer_bytes, bw):
    """(T_opt, canonical strategy, number of strategies visited); (None, None, n) if infeasible."""
    L, D = len(t_comp), len(dev_mem)
    best_t, best_s, visited = None, None, 0
    for strat in all_strategies(L, D):
        visited += 1
        t = evaluate(strat, t_comp, layer_mem, dev_mem, xfer_bytes, bw)
        if t is None:
            continue
        if best_t is None or t < best_t or (t == best_t and canonical_key(strat) < canonical_key(best_s)):
            best_t, best_s = t, strat
    return best_t, best_s, visited


# ---------------------------------------------------------------------------
# the paper's dynamic program, rendered in C (partition_oracle.c)
# ---------------------------------------------------------------------------
_lib = None


def _clib():
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        L = C.CDLL(_build.LIB)
        dp = C.POINTER(C.c_double)
        ip = C.POINTER(C.c_int32)
        L.epo_partition_dp.argtypes = [C.c_int32, C.c_int32, dp, dp, dp, dp, dp, dp, ip, ip, ip, ip]
        L.epo_partition_dp.restype = C.c_int
        _lib = L
    return _lib


def paper_dp(t_comp, layer_mem, dev_mem, xfer_bytes, bw):
    """T_opt and one optimal strategy from the recurrence of Eq. 3 over (layers done,
    device set, device of the last stage), evaluated set by set (partition_oracle.c).
    Returns (None, None) if no strategy fits in memory.  Ties are broken by first
    discovery, so only T_opt and the validity of the strategy are comparable with
    other solvers."""
    t_comp = np.ascontiguousarray(t_comp, dtype=np.float64)
    L, D = t_comp.shape
    arrs = [np.ascontiguousarray(a, dtype=np.float64) for a in (layer_mem, dev_mem, xfer_bytes, bw)]
    t_opt = C.c_double()
    n = C.c_int32()
    dev = np.zeros(D, dtype=np.int32)
    first = np.zeros(D, dtype=np.int32)
    last = np.zeros(D, dtype=np.int32)
    dp = C.POINTER(C.c_double)
    ip = C.POINTER(C.c_int32)
    rc = _clib().epo_partition_dp(L, D, t_comp.ctypes.data_as(dp), *[a.ctypes.data_as(dp) for a in arrs],
                                  C.byref(t_opt), C.byref(n), dev.ctypes.data_as(ip),
                                  first.ctypes.data_as(ip), last.ctypes.data_as(ip))
    if rc == 1:
        return None, None
    if rc:
        raise RuntimeError(f"epo_partition_dp failed: {rc}")
    return t_opt.value, [(int(dev[s]), int(first[s]), int(last[s])) for s in range(n.value)]
