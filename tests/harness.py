"""Oracle-side pipeline helpers for the tests (CPU only).

Chains the per-pair oracle functions in the order of Algorithm 1: digest ->
score -> top-k -> residency split -> partial attention on each side -> merge.
Holds no arithmetic of its own.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

import oracle
from paper_2603_27138_amd import workload as W


@dataclass
class OraclePair:
    dig: np.ndarray            # [nb][2][d] storage
    s: np.ndarray              # float64 [nb] exact scores
    s32: np.ndarray            # float64 [nb] scores as the decision sees them (binary32 values)
    sel: np.ndarray            # int32 [k]
    sel_gpu: np.ndarray
    n_gpu: int
    sel_host: np.ndarray
    n_host: int
    gpu_part: list = field(default_factory=list)   # per head (o, m, l)
    host_part: list = field(default_factory=list)
    out: list = field(default_factory=list)        # per head (out, lse)


def run_pair(wl: W.Workload, b: int, g: int, q=None, table=None, attention: bool = True,
             agg: str = "sum") -> OraclePair:
    cfg = wl.cfg
    q = wl.q if q is None else q
    table = wl.block_table if table is None else table
    K, V = wl.K[(b, g)], wl.V[(b, g)]
    ctx = int(cfg.ctx[b])
    dig = oracle.digest(K, ctx, cfg.S)
    qg = q[b, g * cfg.G:(g + 1) * cfg.G]
    s = oracle.score(qg, dig) if agg == "sum" else oracle.score_max(qg, dig)
    s32 = oracle.decision_scores(s)
    sel = oracle.select(s32, cfg.k)
    sg, ng, sh, nh = oracle.split(sel, table[b, g])
    res = OraclePair(dig, s, s32, sel, sg, ng, sh, nh)
    if attention:
        for h in range(cfg.G):
            pg = oracle.partial_attn(qg[h], K, V, sg, ctx, cfg.S, cfg.sm_scale)
            ph = oracle.partial_attn(qg[h], K, V, sh, ctx, cfg.S, cfg.sm_scale)
            # the host hands its partial over in binary32
            ph32 = (ph[0].astype(np.float32).astype(np.float64), float(np.float32(ph[1])), float(np.float32(ph[2])))
            res.gpu_part.append(pg)
            res.host_part.append(ph32)
            res.out.append(oracle.merge(pg[0], pg[1], pg[2], ph32[0], ph32[1], ph32[2]))
    return res


def run_head(wl: W.Workload, b: int, hq: int, q=None, table=None, attention: bool = True) -> OraclePair:
    """Selection per query head (a variant of Alg. 1's TopK argument: the block importance of one
    head alone decides that head's blocks): the head is a group of one on its KV head's cache."""
    cfg = wl.cfg
    q = wl.q if q is None else q
    table = wl.block_table if table is None else table
    g = hq // cfg.G
    K, V = wl.K[(b, g)], wl.V[(b, g)]
    ctx = int(cfg.ctx[b])
    dig = oracle.digest(K, ctx, cfg.S)
    s = oracle.score(q[b, hq:hq + 1], dig)
    s32 = oracle.decision_scores(s)
    sel = oracle.select(s32, cfg.k)
    sg, ng, sh, nh = oracle.split(sel, table[b, g])
    res = OraclePair(dig, s, s32, sel, sg, ng, sh, nh)
    if not attention:
        return res
    pg = oracle.partial_attn(q[b, hq], K, V, sg, ctx, cfg.S, cfg.sm_scale)
    ph = oracle.partial_attn(q[b, hq], K, V, sh, ctx, cfg.S, cfg.sm_scale)
    ph32 = (ph[0].astype(np.float32).astype(np.float64), float(np.float32(ph[1])), float(np.float32(ph[2])))
    res.gpu_part.append(pg)
    res.host_part.append(ph32)
    res.out.append(oracle.merge(pg[0], pg[1], pg[2], ph32[0], ph32[1], ph32[2]))
    return res


def run_all(wl: W.Workload, **kw) -> Dict[Tuple[int, int], OraclePair]:
    return {p: run_pair(wl, p[0], p[1], **kw) for p in wl.K}


def boundary_gap(op: OraclePair, k: int) -> float:
    """Relative gap between the last kept and first dropped score (binary64 scores)."""
    nb = len(op.s)
    if k >= nb:
        return np.inf
    r = oracle.rank(op.s32)
    a, b = op.s[r[k - 1]], op.s[r[k]]
    return abs(a - b) / max(abs(a), abs(b), 1e-300)


def rel_gap(a: float, b: float) -> float:
    """Relative distance of two scores; infinite when either is not finite (an always-kept block's
    +inf or a padded -inf is never a near-tie)."""
    if not (np.isfinite(a) and np.isfinite(b)):
        return np.inf
    return abs(a - b) / max(abs(a), abs(b), 1e-300)


def selection_gap(s64: np.ndarray, decision: np.ndarray, k: int) -> float:
    """The one gap that decides a top-k selection: between the last kept and the first dropped block in
    the ranking of `decision` (the scores the selection saw), measured on the exact scores `s64`."""
    nb = len(decision)
    if k >= nb:
        return np.inf
    r = oracle.rank(decision)
    return rel_gap(s64[r[k - 1]], s64[r[k]])


def plan_gap(s64: np.ndarray, decision: np.ndarray, k: int, table_row: np.ndarray) -> float:
    """The smallest of the gaps that decide a recall plan (Sec. 3.4) in the oracle's ranking: k-th vs
    (k+1)-th block overall; n-th vs (n+1)-th best of the missing blocks (top-k, not resident) when
    only n of them fit; n-th vs (n+1)-th worst of the spare blocks (resident, not in the top-k) when
    only n of them go.  A device plan that differs from the oracle's is excused only if this is
    below the tolerance: no other pair of scores can change the plan."""
    nb = len(decision)
    ke = min(k, nb)
    r = oracle.rank(decision)
    gaps = [selection_gap(s64, decision, k)]
    top = np.zeros(nb, dtype=bool)
    top[r[:ke]] = True
    res = np.asarray(table_row[:nb]) >= 0
    missing = [j for j in r if top[j] and not res[j]]          # best first
    spare = [j for j in r[::-1] if res[j] and not top[j]]      # worst first
    n = min(len(missing), len(spare))
    if 0 < n < len(missing):
        gaps.append(rel_gap(s64[missing[n - 1]], s64[missing[n]]))
    if 0 < n < len(spare):
        gaps.append(rel_gap(s64[spare[n - 1]], s64[spare[n]]))
    return min(gaps)


def few(excused: int, total: int) -> bool:
    """Excused mismatches must stay rare: at most one, or one in a hundred."""
    return excused <= max(1, total // 100)
