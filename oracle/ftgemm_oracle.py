"""CPU oracle for the strided-ABFT linear layer (tensor checksums on a plain 16-bit GEMM).

TEST INFRASTRUCTURE ONLY.  Slow, plain, float64.  Only tests and the smoke check may import
it; the product path never does, and it shares no code with the HIP kernels.

What is computed.  The paper protects the linear modules of the transformer (projections,
feed-forward layers) with the same strided ABFT it builds for Q K^T inside attention
(Section 3.3, last sentence of "Tensor Checksum Design"; Figure 1).  For a linear layer

    Y = X W^T,      X: [M, K] tokens,  W: [N, K] weights  (the operand roles of Q and K),

the output features are cut into blocks of ``block_n`` columns.  For every block the rows of W
are folded at stride s = 8 into two tensor checksums (eq. (13), (14)):

    check1[c, :] = sum_l W[n0 + c + s*l, :],      check2[c, :] = sum_l (l+1) W[n0 + c + s*l, :],

which are multiplied with X like ordinary weight rows (eq. (15), (16)).  In exact arithmetic
X check1^T equals the stride-s fold of Y over the block; a mismatch in class c of row i names
the fold l* = (check2 residual / check1 residual) - 1, i.e. column n0 + c + s*l*, and the
element is restored from the first checksum (text after eq. (16)).

``linear_clean`` is the definition (one matrix product).  ``ftgemm`` takes the steps above in
the paper's order with a list of injected single-bit flips of the fp32 result accumulator
(fault model of Section 2.2).

Readings where the paper is silent:

* Nothing is rounded here: check1, check2 and their products with X are exact float64 sums, so the
  fault-free residual of this file is zero up to float64 rounding.  How an implementation stores
  its checksum rows (the GPU library keeps a high and a low 16-bit word of the input type) is its
  own business and has to fit inside the threshold; the tests keep injected faults a factor 4 away
  from it on either side.
* A class is flagged when |check1 - fold1| exceeds tau_abs + tau_rel * sum_l |Y_l| (a
  threshold relative to the magnitude that was summed; the paper's 0.48 is an absolute value
  tuned to its data), or when that residual is not finite.  Which faults the paper's code
  would flag at a given threshold is therefore "parity unpinned"; the identities, the location
  rule and the repair are pinned by tests against closed forms and brute force.
* Restoring is done by reconstruction (checksum minus the other folds), and a non-finite
  residual ratio names the fold of overwhelming magnitude, as in the attention oracle.
* Output columns beyond N in the last block count as zero weight rows.
* ``fold_tokens`` (the column-checksum counterpart: the paper encodes one operand, K^T in
  attention, and names the other side only to reject its memory cost there, Section 3.3): the
  tensor checksums are taken over the token rows of X instead of the weight rows, in blocks of
  ``block_n`` tokens, so that for every output feature the stride-s fold of Y over the tokens of a
  block equals X_check W^T.  This is the same method applied to Y^T = W X^T, and it is computed
  exactly so: operands swapped, faults and events with rows and columns exchanged.  It repairs
  several errors in one token row (they fall into different columns) and fails on two errors of one
  output feature whose tokens are a multiple of s apart: the mirror image of the default.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Sequence, Tuple

import numpy as np


@dataclasses.dataclass
class Params:
    block_n: int = 256          # output features per checksum block
    stride: int = 8             # s of eq. (13)
    tau_rel: float = 2.0 ** -15
    tau_abs: float = 0.0
    correct: bool = True        # False: detect and locate only
    fold_tokens: bool = False   # checksums over the token rows of X (blocks of block_n tokens) instead of W


Fault = Tuple[int, int, int]    # (row, col, bit) of the fp32 accumulator of Y
Event = Tuple[int, int]         # (row, col); col = -1 when no single element can be named


def bitflip32(x: float, bit: int) -> float:
    """Value of x after rounding to fp32 and inverting one bit of the encoding."""
    u = np.array([x], dtype=np.float64).astype(np.float32).view(np.uint32)
    u ^= np.uint32(1 << bit)
    with np.errstate(all="ignore"):
        return float(u.view(np.float32)[0])


def linear_clean(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y = X W^T by the definition."""
    return X @ W.T


def encode_w(Wb: np.ndarray, s: int) -> Tuple[np.ndarray, np.ndarray]:
    """Tensor checksums of one block of weight rows (eq. (13), (14)): [s, K] each."""
    nb, K = Wb.shape
    W3 = Wb.reshape(nb // s, s, K)
    w = np.arange(1, nb // s + 1, dtype=np.float64)[:, None, None]
    return W3.sum(axis=0), (w * W3).sum(axis=0)


def ftgemm(X: np.ndarray, W: np.ndarray, prm: Params, faults: Sequence[Fault] = ()):
    """Strided-ABFT linear layer.  Returns (Y, events, diagnostics).

    events: list of (row, col, action) in order of (row, block, class); diagnostics hold, for
    the fault selector of the tests, the smallest distance (as a ratio) of any check statistic
    to its threshold and the values that were flipped.
    """
    if prm.fold_tokens:
        # the same method on Y^T = W X^T: W rows take the place of the tokens, X rows that of the weights
        swapped = dataclasses.replace(prm, fold_tokens=False)
        Yt, ev_t, diag = ftgemm(W, X, swapped, [(c, r, b) for (r, c, b) in faults])
        return np.ascontiguousarray(Yt.T), sorted((c, r, a) for (r, c, a) in ev_t), diag
    M, K = X.shape
    N = W.shape[0]
    s, bn = prm.stride, prm.block_n
    nfold = bn // s
    Y = linear_clean(X, W)
    flipped: List[float] = []
    for (row, col, bit) in faults:
        flipped.append(float(Y[row, col]))
        Y[row, col] = bitflip32(Y[row, col], bit)
    events: List[Tuple[int, int, int]] = []
    ratio_near = np.inf
    res_max = 0.0
    for n0 in range(0, N, bn):
        Wb = np.zeros((bn, K))
        nb = min(bn, N - n0)
        Wb[:nb] = W[n0:n0 + nb]
        c1, c2 = encode_w(Wb, s)
        chk1 = X @ c1.T                 # [M, s]   eq. (15)
        chk2 = X @ c2.T                 # [M, s]   eq. (16)
        Yb = np.zeros((M, bn))
        Yb[:, :nb] = Y[:, n0:n0 + nb]
        Y3 = Yb.reshape(M, nfold, s)
        with np.errstate(all="ignore"):
            sum1 = Y3.sum(axis=1)
            mag = np.abs(Y3).sum(axis=1)
            R1 = chk1 - sum1
            thr = prm.tau_abs + prm.tau_rel * mag
            bad = ~(np.abs(R1) <= thr) | ~np.isfinite(R1)
            stat = np.abs(R1) / thr
        ok_stat = stat[~bad]
        if ok_stat.size:
            res_max = max(res_max, float(ok_stat.max()))
        finite = np.isfinite(stat) & (stat > 0)
        if finite.any():
            lr = np.abs(np.log(stat[finite]))
            ratio_near = min(ratio_near, float(np.exp(lr.min())))
        for (i, c) in zip(*np.nonzero(bad)):
            x = Y3[i, :, c].copy()
            with np.errstate(all="ignore"):
                r1 = chk1[i, c] - x.sum()
                r2 = chk2[i, c] - (np.arange(1, nfold + 1) * x).sum()
                ratio = r2 / r1
            lstar = -1
            if np.isfinite(ratio):
                cand = int(np.rint(ratio)) - 1
                if 0 <= cand < nfold:
                    lstar = cand
            else:
                m = np.where(np.isfinite(x), np.abs(x), np.inf)
                top = np.flatnonzero(m == m.max())
                if top.size == 1:
                    lstar = int(top[0])
            col = n0 + c + s * lstar if lstar >= 0 else -1
            if col >= N:
                col, lstar = -1, -1
            fix = prm.correct and lstar >= 0
            events.append((int(i), int(col), 1 if fix else 0))
            if fix:
                rest = np.delete(x, lstar).sum()
                Y[i, col] = chk1[i, c] - rest
    events.sort()
    return Y, events, {"ratio_near": ratio_near, "res_max": res_max, "flipped": flipped}


def fault_is_robust(diag: Dict[str, float], band: float = 4.0) -> bool:
    """True when no check statistic of the run lies within ``band`` of its threshold."""
    return diag["ratio_near"] >= band


def fp32_is_fragile(x: float) -> bool:
    """True when x is so close to a binade edge (or to zero) that an fp32 accumulation in
    another order could land in the neighbouring binade, which would change what a flipped
    bit does to it."""
    if not np.isfinite(x) or x == 0.0:
        return True
    ax = abs(float(x))
    if ax < 2.0 ** -100:
        return True
    mant, ex = np.frexp(ax)
    gap = min(mant - 0.5, 1.0 - mant) * 2.0 ** ex
    return gap < 2.0 ** -14 * max(ax, 1.0)
