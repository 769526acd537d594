"""CPU oracle for the decoupled, operation-level fault-tolerant attention (Section 3.1 of the paper:
ABFT-GEMM I, DMR row-softmax, ABFT-GEMM II, the comparison system of Section 4.1).

TEST INFRASTRUCTURE ONLY.  Slow, plain, float64; only tests and the benchmark's baseline leg may
import it, the product path never does, and it shares no code with the HIP kernels.

Steps, per (batch, head), in the paper's order:

1. ``S = Q K^T`` protected by ABFT on the GEMM.  The library protects its GEMMs with the strided
   tensor checksum of Section 3.3 (eq. (13)-(16)); this file calls ``ftgemm_oracle.ftgemm`` for that
   step (tokens = queries, weight rows = keys), with injected flips of the fp32 accumulator.
2. Row softmax by dual modular redundancy, eq. (11), (12).  Per row, over the unmasked keys:
   two evaluations ``e_a``, ``e_b`` of ``exp(scale * S - max)``; the row passes eq. (11) when
   ``|e_a - e_b| < eps`` for every element, and then ``DMR(e) = (e_a + e_b) / 2``;
   ``P = DMR(e) / rowsum(DMR(e))`` passes eq. (12) when ``|rowsum(P) - 1| < eps``.  A row that fails
   either test is evaluated again ("iteratively executes ... until the difference ... satisfies a
   predefined error tolerance").  An injected soft error hits one evaluation of the first attempt
   only, so the second attempt is clean.
3. ``O = P V`` protected like step 1 (tokens = queries, weight rows = the features, i.e. rows of V^T).

Readings where the paper is silent: the repeat count is bounded at three attempts; eq. (12)'s c_1 is
the all-ones vector (rows of P sum to one); a causal mask (absent from the paper) restricts the row to
keys <= query; eps is an absolute tolerance on values in [0, 1] (the paper gives no number: which
faults its code would flag at a given eps is "parity unpinned"; the identities and the control flow
are pinned by tests).  Nothing is rounded here; the GPU library stores S in fp32 and P in fp16.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence, Tuple

import numpy as np

from . import ftgemm_oracle as gorc

ST_GEMM1, ST_EXP, ST_PNORM, ST_GEMM2 = 0, 1, 2, 3


@dataclasses.dataclass
class Params:
    scale: float
    causal: bool
    tau_rel: float = 2.0 ** -15     # threshold of the two ABFT GEMMs
    eps_dmr: float = 2.0 ** -12     # tolerance of eq. (11), (12)
    block_n: int = 256              # checksum block of the GEMMs


Fault = Tuple[int, int, int, int]   # (stage, row, col, bit)
Event = Tuple[int, int, int]        # (stage, row, col)


def dmr_softmax_row(s: np.ndarray, scale: float, eps: float, exp_faults=(), p_faults=()):
    """One row of step 2.  s: scores of the unmasked keys.  exp_faults / p_faults: (col, bit) flips
    of evaluation a of the exponentials / of the normalised weights, applied in the first attempt.
    Returns (P row, events as (stage, col), number of attempts, statistics)."""
    events: List[Tuple[int, int]] = []
    stats = {"exp_delta": [], "p_delta": []}
    for attempt in range(3):
        x = scale * s
        e_b = np.exp(x - x.max())
        e_a = e_b.copy()
        if attempt == 0:
            for (col, bit) in exp_faults:
                e_a[col] = gorc.bitflip32(e_a[col], bit)
        with np.errstate(all="ignore"):
            diff = np.abs(e_a - e_b)
        if attempt == 0:
            stats["exp_delta"] += [float(diff[col]) for (col, _) in exp_faults]
        bad = np.flatnonzero(~(diff < eps))
        if bad.size:
            events += [(ST_EXP, int(c)) for c in bad]
            continue
        e = 0.5 * (e_a + e_b)                       # eq. (11)
        P = e / e.sum()
        if attempt == 0:
            for (col, bit) in p_faults:
                before = P[col]
                P[col] = gorc.bitflip32(P[col], bit)
                with np.errstate(all="ignore"):
                    stats["p_delta"].append(float(abs(P[col] - before)))
        with np.errstate(all="ignore"):
            ok = abs(P.sum() - 1.0) < eps           # eq. (12)
        if ok:
            return P, events, attempt + 1, stats
        events.append((ST_PNORM, -1))
    return P, events, 3, stats


def decoupled_attention(Q: np.ndarray, K: np.ndarray, V: np.ndarray, prm: Params, faults: Sequence[Fault] = (),
                        row_idx=None):
    """All three steps for query rows ``row_idx`` (default: all, 0..n-1) of one head; every check of
    the scheme is local to a query row.  Q: [n, d] (the rows row_idx of the head's queries), K, V:
    [N, d].  Fault and event rows are global query indices.  Returns (O [n, d], sorted events
    (stage, row, col), diagnostics)."""
    n, Nk = Q.shape[0], K.shape[0]
    row_idx = np.arange(n) if row_idx is None else np.asarray(row_idx)
    pos = {int(r): i for i, r in enumerate(row_idx)}
    faults = [f for f in faults if int(f[1]) in pos]
    gp = gorc.Params(block_n=prm.block_n, tau_rel=prm.tau_rel)
    f1 = [(pos[r], c, b) for (st, r, c, b) in faults if st == ST_GEMM1]
    f2 = [(pos[r], c, b) for (st, r, c, b) in faults if st == ST_GEMM2]
    S, ev1, dg1 = gorc.ftgemm(Q, K, gp, f1)
    events: List[Event] = [(ST_GEMM1, int(row_idx[r]), c) for (r, c, _) in ev1]
    P = np.zeros((n, Nk))
    exp_delta, p_delta = [], []
    for i in range(n):
        g = int(row_idx[i])
        nv = min(g + 1, Nk) if prm.causal else Nk
        ef = [(c, b) for (st, r, c, b) in faults if st == ST_EXP and r == g]
        pf = [(c, b) for (st, r, c, b) in faults if st == ST_PNORM and r == g]
        P[i, :nv], ev, _, stt = dmr_softmax_row(S[i, :nv], prm.scale, prm.eps_dmr, ef, pf)
        events += [(st, g, c) for (st, c) in ev]
        exp_delta += stt["exp_delta"]; p_delta += stt["p_delta"]
    O, ev2, dg2 = gorc.ftgemm(P, np.ascontiguousarray(V.T), gp, f2)
    events += [(ST_GEMM2, int(row_idx[r]), c) for (r, c, _) in ev2]
    diag = {"gemm1": dg1, "gemm2": dg2, "exp_delta": exp_delta, "p_delta": p_delta}
    return O, sorted(events), diag


def fault_is_robust(diag, prm: Params, band: float = 4.0) -> bool:
    """True when no decision of the run sits within ``band`` of its threshold."""
    if not (gorc.fault_is_robust(diag["gemm1"], band) and gorc.fault_is_robust(diag["gemm2"], band)):
        return False
    for dlt in diag["exp_delta"] + diag["p_delta"]:
        if np.isfinite(dlt) and prm.eps_dmr / band <= dlt <= prm.eps_dmr * band:
            return False
    return True
