"""CPU oracle for end-to-end fault-tolerant attention (EFTA, unified verification).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, float64 statement of what
the GPU library must compute.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import it; the product path never does.  It shares no
code with the HIP kernels.

Two results are defined here.

``attention_clean``
    softmax(scale * Q K^T + mask) V by the definition (two passes, global row
    maximum).  The tiled method reaches exactly this when no fault occurs
    (Section 2.1, eq. (2)-(8)), so this is the reference for fault-free output.

``efta_rows`` (= ``efta_rows_unified`` unless a verification variant is asked for)
    Algorithm 1 ("EFTA with unified verification", Section 3.4) taken step by
    step in float64 for a set of query rows of one (batch, head): tensor-checksum
    encoding (eq. (13), (14)), GEMM I with its two checksum products (eq. (15),
    (16)), running max, exp, the unified product-form check of GEMM I + subtract
    + exp (Section 3.4, case 2), checksum correction / exp recomputation,
    row-sum, GEMM II with rescale and its two checksum products, the range
    check of the row-sum with substitution of the lower bound (case 3 and the
    "optimized" paragraph of Section 3.4), normalisation and the final sum-form
    check of GEMM II + rescale + normalisation.  A list of injected single-bit
    flips (fault model of Section 2.2) is applied to the named fp32 intermediates.

Readings of passages where the paper is silent or inconsistent (each is also
listed in the design notes of the repository):

* The checksum fold of eq. (13)/(14) is taken as a stride-s fold, as the text
  after eq. (16) states: check1[i][c] = sum_l S[i][c + s*l].
* The fold count of the S / P checksums is the number of key columns of the
  tile divided by s (the paper's ceil(d/8) equals it only when the tile width
  equals d); the O checksums fold d/s features.
* With weights l+1 in the second checksum the residual ratio is l+1, so the
  located fold is round(ratio) - 1.
* The product-form comparison of Algorithm 1 is evaluated as a log-ratio
      lambda = ln prod_l P_l - (scale * check1_eff - n_valid * m)
    , the same identity, defined where a product of many small exponentials
  leaves the floating-point range.  It is computed as
      sum_l (ln P_l - x_l) - scale * R1,  R1 = check1 - sum_l S_l,
  and ln P_l - x_l is taken as exactly zero for an element that still holds the
  value the exponential produced.
* A detected class is a linear (GEMM I / subtraction) fault when
  scale*|R1| > eps1/2 and an exponentiation fault otherwise.  After a linear
  correction the row's maximum and exponentials for that tile are recomputed
  ("correct EXP with recomputation").
* Restoring an element is done by reconstruction (checksum minus the other
  folds), which equals "adding the residual" algebraically but never reuses a
  corrupted, possibly infinite, value.  When the residual ratio is not finite
  (an Inf/NaN result, or residuals beyond the floating-point range) the located
  fold is the one of largest magnitude, if it is unique.
* The lower bound of the row-sum uses the *local* maximum of each key tile,
  carried with the same rescale as the row-sum; the upper bound is the number
  of unmasked keys of the row; both get a relative slack delta_l and equality is
  allowed (a single key gives bound = sum = 1).
* A causal mask is not mentioned in the paper.  Masked entries take no part in
  max / exp / sums; the linear residual uses the whole raw tile; the product
  check uses the checksum minus the masked raw scores and the count of unmasked
  folds.  Key tiles with no unmasked entry for a row are skipped for that row.
* The softmax scale is applied inside x = scale*S - m; the S stage is the raw
  accumulator.  Thresholds are in logit units / normalised-output units.

* ``rowsum_fold`` (an extension, off by default; the paper's own row-sum protection is the
  range restriction above).  The row-sum obeys the same recurrence as a column of the output
  accumulator whose V entries are all one.  With this option the value-tile checksums of class 0
  are encoded as if V had such a column at feature index d (fold d/s): check1[:,0] += 1,
  check2[:,0] += d/s + 1 for every real key, so the first checksum of class 0 carries the
  row-sum through GEMM II and the rescale at no extra cost.  After the loop the row-sum that
  the checksum implies, check1[0] - sum of the class-0 output folds, is compared with the
  accumulated one (relative difference against tau_o); on a mismatch the usual location rule is
  applied to the d/s + 1 folds, and if it names the extra fold the row-sum is replaced by the
  implied one (event CHECK_L).  The range restriction is not applied in this mode.  In the final
  sum-form check the normalised extra fold (row-sum / row-sum = 1) is part of class 0.

* ``per_step`` (the paper's EFTA before the unified-verification optimisation of Section 3.4:
  every step is verified where it happens).  In each iteration (a) GEMM I is verified on its own:
  a class whose linear residual exceeds eps1/2 (scale*|R1| > eps1/2) is located and repaired even
  if the product-form statistic stays below eps1, then the product-form check runs as above and
  catches what is left (exponentiation faults); (b) after the reduce-sum the row-sum is checked
  against its range so far (lower bound as above, upper bound the number of unmasked keys seen so
  far) and replaced by the lower bound when outside; (c) after GEMM II the unnormalised output
  accumulator is checked against its checksum, |check1 - fold| <= tau_o * row-sum, and a located
  element is restored.  Events of (b) and (c) carry the key-tile index.  The checks after the loop
  stay as they are (they cover the normalisation).  Not combined with ``rowsum_fold``.
* ``softmax_dmr`` (with ``per_step``; the paper's EFTA protects the softmax by dual modular
  redundancy, Section 3.1 eq. (11), (12), before SNVR replaces it): maximum, subtraction,
  exponential and reduce-sum are evaluated twice and compared exactly; where the two differ the
  step is evaluated again and the value two evaluations agree on is kept.  Under the fault model
  (one upset, in the named intermediate) this means: every exponential whose stored value differs
  from its re-evaluation is reported (CHECK_EXP) and replaced, whatever the size of the difference,
  and a row-sum that differs from its duplicate is reported (CHECK_L, with the key tile) and
  replaced by the duplicate.  The product-form check and the range restriction are not used.

* ``rescale_margin`` (an extension, off by default; Algorithm 1 renews the maximum in every iteration
  and rescales the output with it).  The subtracted value is a *reference* maximum m_ref that is
  replaced by the running maximum only when that exceeds it by more than the margin; in all other
  iterations the rescale factor is exactly one and the rescale of O, of its checksums, of the
  row-sum and of its lower bound falls away.  Exponentials then lie in (0, e^margin] instead of
  (0, 1]; every identity of the method holds with m_ref in place of the maximum (Section 3.4,
  case 1: the subtracted value cancels between numerator and denominator), and the upper bound of
  the row-sum becomes (number of unmasked keys) * exp(running maximum - m_ref).  Not combined with
  the other variants.

Thresholds (eps1, tau_o, delta_l) are this repository's choices: the paper's own
values (0.48 absolute, 7e-6 relative) belong to its one-word fp16 checksums and
carry a 5.9% false-alarm rate.  Which faults the paper's code would flag at a
given threshold is therefore "parity unpinned"; everything else in this file is
pinned by tests against closed forms, invariants and brute force.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

ST_S, ST_EXP, ST_ROWSUM, ST_OACC = 0, 1, 2, 3
CHECK_S, CHECK_EXP, CHECK_L, CHECK_O = 0, 1, 2, 3


@dataclasses.dataclass
class Params:
    scale: float
    causal: bool
    block_n: int                       # key-tile width B_c
    stride: int = 8                    # s of eq. (13)
    eps1: float = 0.03                 # unified product check, log-ratio units
    tau_o: float = 0.75 * 2.0 ** -9    # final sum check, normalised-output units
    delta_l: float = 2.0 ** -10        # relative slack of the row-sum range
    correct: bool = True               # False: detect and locate only
    rowsum_fold: bool = False          # True: the row-sum rides through GEMM II as an extra fold of
                                       # checksum class 0 and is verified / repaired exactly (see below)
    per_step: bool = False             # True: verification after every step instead of unified (see above)
    softmax_dmr: bool = False          # True (needs per_step): softmax protected by duplication, not by SNVR
    rescale_margin: float = 0.0        # > 0 (an extension, see above): the reference maximum is renewed only when the
                                       # running maximum exceeds it by more than this (natural-log units)


def bitflip32(x: float, bit: int) -> float:
    """Value of x after rounding to fp32 and inverting one bit of the encoding."""
    u = np.array([x], dtype=np.float64).astype(np.float32).view(np.uint32)
    u ^= np.uint32(1 << bit)
    with np.errstate(all="ignore"):
        return float(u.view(np.float32)[0])


# ----------------------------------------------------------------------------
# (1) the definition
# ----------------------------------------------------------------------------

def attention_clean(Q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float,
                    causal: bool, row_idx: Optional[np.ndarray] = None) -> np.ndarray:
    """softmax(scale*Q K^T + mask) V for the given query rows (eq. (8), right side).

    Q: [n, d] float64 rows whose global indices are ``row_idx`` (default 0..n-1);
    K, V: [N, d] float64.
    """
    n = Q.shape[0]
    N = K.shape[0]
    if row_idx is None:
        row_idx = np.arange(n)
    out = np.empty((n, V.shape[1]), np.float64)
    step = max(1, (1 << 22) // max(N, 1))
    for a in range(0, n, step):
        z = slice(a, min(n, a + step))
        S = scale * (Q[z] @ K.T)
        if causal:
            S = np.where(np.arange(N)[None, :] <= row_idx[z, None], S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        out[z] = (P / P.sum(axis=1, keepdims=True)) @ V
    return out


# ----------------------------------------------------------------------------
# (2) tensor checksums, eq. (13)-(16)
# ----------------------------------------------------------------------------

def encode_k(Kj: np.ndarray, s: int) -> Tuple[np.ndarray, np.ndarray]:
    """Checksums of a key tile: c1[c,:] = sum_l K[c+s*l,:], c2 with weight l+1."""
    Bc, d = Kj.shape
    K3 = Kj.reshape(Bc // s, s, d)
    w = np.arange(1, Bc // s + 1, dtype=np.float64)[:, None, None]
    return K3.sum(axis=0), (w * K3).sum(axis=0)


def encode_v(Vj: np.ndarray, s: int) -> Tuple[np.ndarray, np.ndarray]:
    """Checksums of a value tile: c1[:,c] = sum_l V[:,c+s*l], c2 with weight l+1."""
    Bc, d = Vj.shape
    V3 = Vj.reshape(Bc, d // s, s)
    w = np.arange(1, d // s + 1, dtype=np.float64)[None, :, None]
    return V3.sum(axis=1), (w * V3).sum(axis=1)


def fold(X: np.ndarray, s: int) -> Tuple[np.ndarray, np.ndarray]:
    """Strided sums of the columns of X: sum_l X[:,c+s*l] and sum_l (l+1) X[:,c+s*l]."""
    n, W = X.shape
    X3 = X.reshape(n, W // s, s)
    w = np.arange(1, W // s + 1, dtype=np.float64)[None, :, None]
    with np.errstate(all="ignore"):
        return X3.sum(axis=1), (w * X3).sum(axis=1)


def locate_and_restore(x: np.ndarray, chk1: float, chk2: float) -> Tuple[int, float]:
    """Strided-ABFT location and repair of one class (text after eq. (16)).

    x: the folds of one class (one row); chk1, chk2: its two checksum values.
    Returns (fold index, restored value); fold index -1 when no single element
    can be named.
    """
    n = x.shape[0]
    with np.errstate(all="ignore"):
        r1 = chk1 - x.sum()
        r2 = chk2 - (np.arange(1, n + 1) * x).sum()
        ratio = r2 / r1
    lstar = -1
    if np.isfinite(ratio):
        cand = int(np.rint(ratio)) - 1
        if 0 <= cand < n:
            lstar = cand
    else:
        # residuals not finite: the fold of overwhelming size (a non-finite value counts as
        # largest); two folds of equal size cannot be told apart
        mag = np.where(np.isfinite(x), np.abs(x), np.inf)
        top = np.flatnonzero(mag == mag.max())
        if top.size == 1:
            lstar = int(top[0])
    if lstar < 0:
        return -1, 0.0
    rest = np.delete(x, lstar).sum()
    return lstar, float(chk1 - rest)


# ----------------------------------------------------------------------------
# (3) Algorithm 1
# ----------------------------------------------------------------------------

Fault = Tuple[int, int, int, int, int]     # (stage, kv_tile, row, col, bit)
Event = Tuple[int, int, int, int]          # (check, kv_tile, row, col)


def _softmax_part(Srows, vrows, m_old, sc):
    """Reduce max and element-wise exp of one key tile (Algorithm 1: m_ij, P_ij) over the unmasked entries."""
    with np.errstate(all="ignore"):
        mh = np.where(vrows, sc * Srows, -np.inf).max(axis=1)
        mn = np.maximum(m_old, mh)
        x = sc * Srows - mn[:, None]
        P = np.where(vrows, np.exp(x), 0.0)
    return mh, mn, x, P


def efta_rows_unified(Q: np.ndarray, row_idx: np.ndarray, K: np.ndarray, V: np.ndarray,
                      prm: Params, faults: Sequence[Fault] = (),
                      max_shift: Optional[Dict[Tuple[int, int], float]] = None
                      ) -> Tuple[np.ndarray, List[Event], Dict[str, float]]:
    """Algorithm 1 ("EFTA with unified verification") for query rows ``row_idx`` of one head, top to
    bottom in the paper's order, with none of the verification variants.

    Q: [n, d] float64 (rows row_idx of the head's query matrix), K, V: [N, d].
    Returns (O [n, d], sorted events, diagnostics).  Diagnostics hold the largest check statistic
    over all evaluated checks relative to its threshold (``lambda_ratio``, ``o_ratio``) and the
    smallest relative distance of a final row-sum to its range boundaries (``l_distance``); the fault
    generator uses them to keep clear of decisions that hinge on rounding.  ``flipped`` lists
    (stage, value before the flip) for every fault that was applied.

    ``max_shift`` maps (kv_tile, row) to an error added to the running maximum the moment it is
    formed (Section 3.4, case 1: such an error needs no protection because it cancels between
    numerator and denominator); tests use it to show exactly that.
    """
    s, Bc, sc = prm.stride, prm.block_n, prm.scale
    n, d = Q.shape
    N = K.shape[0]
    assert Bc % s == 0 and d % s == 0
    assert not (prm.rowsum_fold or prm.per_step or prm.softmax_dmr)
    nK, nV = Bc // s, d // s
    row_idx = np.asarray(row_idx, dtype=np.int64)
    pos = {int(r): i for i, r in enumerate(row_idx)}
    by_tile: Dict[Tuple[int, int], List[Tuple[int, int, int]]] = {}
    for (st, kt, row, col, bit) in faults:
        if int(row) in pos:
            by_tile.setdefault((int(st), int(kt)), []).append((pos[int(row)], int(col), int(bit)))

    m = np.full(n, -np.inf)          # running row maximum
    ell = np.zeros(n)                # running row-sum
    lower = np.zeros(n)              # its lower bound: sum over key tiles of exp(tile maximum - m)
    Ot = np.zeros((n, d))            # un-normalised output and its two checksums
    Oc1 = np.zeros((n, s))
    Oc2 = np.zeros((n, s))
    events: List[Event] = []
    flipped: List[Tuple[int, float]] = []
    lam_ratio = 0.0

    for j in range((N + Bc - 1) // Bc):
        k0 = j * Bc
        act = np.flatnonzero(row_idx >= k0) if prm.causal else np.arange(n)      # rows that see this key tile
        if act.size == 0:
            break
        keys = k0 + np.arange(Bc)
        Kj = np.zeros((Bc, d)); Vj = np.zeros((Bc, d))
        kv = min(N, k0 + Bc) - k0
        Kj[:kv] = K[k0:k0 + kv]; Vj[:kv] = V[k0:k0 + kv]
        valid = np.broadcast_to(keys[None, :] < N, (act.size, Bc)).copy()
        if prm.causal:
            valid &= keys[None, :] <= row_idx[act, None]
        loc = {int(a): i for i, a in enumerate(act)}

        # ---- encode tensor checksums (eq. (13), (14))
        Kc1, Kc2 = encode_k(Kj, s)
        Vc1, Vc2 = encode_v(Vj, s)
        # ---- GEMM I with its checksum products (eq. (15), (16)); injection point S
        Qa = Q[act]
        S = Qa @ Kj.T
        Sc1 = Qa @ Kc1.T
        Sc2 = Qa @ Kc2.T
        for (ri, col, bit) in by_tile.get((ST_S, j), []):
            if ri in loc:
                flipped.append((ST_S, float(S[loc[ri], col - k0])))
                S[loc[ri], col - k0] = bitflip32(S[loc[ri], col - k0], bit)
        # ---- reduce max, element-wise exp; injection point exp
        m_hat, m_new, x, P = _softmax_part(S, valid, m[act], sc)
        for (jt, row), dm in (max_shift or {}).items():
            if jt == j and int(row) in pos and pos[int(row)] in loc:
                i = loc[pos[int(row)]]
                m_new[i] += dm
                x[i] = sc * S[i] - m_new[i]
                P[i] = np.where(valid[i], np.exp(x[i]), 0.0)
        touched = np.zeros_like(valid)
        for (ri, col, bit) in by_tile.get((ST_EXP, j), []):
            if ri in loc and valid[loc[ri], col - k0]:
                flipped.append((ST_EXP, float(P[loc[ri], col - k0])))
                P[loc[ri], col - k0] = bitflip32(P[loc[ri], col - k0], bit)
                touched[loc[ri], col - k0] = True
        # ---- unified verification of GEMM I, subtraction and exp (Section 3.4, case 2):
        # lambda = ln prod P - (scale * check1_eff - n_valid * m) per (row, class)
        with np.errstate(all="ignore"):
            sum1, _ = fold(S, s)
            R1 = Sc1 - sum1
            e = np.where(touched & valid, np.log(P) - x, 0.0)
            E, _ = fold(e, s)
            lam = E - sc * R1
        has_valid = valid.reshape(act.size, nK, s).any(axis=1)
        with np.errstate(invalid="ignore"):
            ok = np.abs(lam) <= prm.eps1
        det = has_valid & ~ok
        fin = has_valid & np.isfinite(lam)
        if fin.any():
            lam_ratio = max(lam_ratio, float(np.abs(lam[fin]).max()) / prm.eps1)
        if (has_valid & ~np.isfinite(lam)).any():
            lam_ratio = np.inf
        redo = []
        for (i, c) in zip(*np.nonzero(det)):
            cols = c + s * np.arange(nK)
            with np.errstate(invalid="ignore"):
                linear = not (sc * abs(R1[i, c]) <= prm.eps1 / 2)
            if linear:
                # a fault of GEMM I: located with the second checksum, restored from the first (text after eq. (16))
                lstar, val = locate_and_restore(S[i, cols], Sc1[i, c], Sc2[i, c])
                col = k0 + int(cols[lstar]) if lstar >= 0 else -1
                events.append((CHECK_S, j, int(row_idx[act[i]]), col))
                if prm.correct and lstar >= 0:
                    S[i, cols[lstar]] = val
                    redo.append(i)
            else:
                # a fault of the exponentiation: recomputed
                with np.errstate(all="ignore"):
                    good = np.exp(x[i, cols])
                for l in range(nK):
                    if valid[i, cols[l]] and touched[i, cols[l]] and P[i, cols[l]] != good[l]:
                        events.append((CHECK_EXP, j, int(row_idx[act[i]]), k0 + int(cols[l])))
                        if prm.correct:
                            P[i, cols[l]] = good[l]
        for i in sorted(set(redo)):      # a repaired score: the row's maximum and exponentials for this tile again
            mh, mn, xx, PP = _softmax_part(S[i:i + 1], valid[i:i + 1], m[act[i]:act[i] + 1], sc)
            m_hat[i], m_new[i], x[i], P[i] = mh[0], mn[0], xx[0], PP[0]
        # ---- reduce sum, GEMM II with rescale and its checksum products; injection points row-sum, output accumulator
        with np.errstate(all="ignore"):
            alpha = np.exp(m[act] - m_new)
            ell[act] = alpha * ell[act] + P.sum(axis=1)
            lower[act] = alpha * lower[act] + np.where(np.isfinite(m_hat), np.exp(m_hat - m_new), 0.0)
            for (ri, col, bit) in by_tile.get((ST_ROWSUM, j), []):
                flipped.append((ST_ROWSUM, float(ell[ri])))
                ell[ri] = bitflip32(ell[ri], bit)
            Ot[act] = alpha[:, None] * Ot[act] + P @ Vj
            Oc1[act] = alpha[:, None] * Oc1[act] + P @ Vc1
            Oc2[act] = alpha[:, None] * Oc2[act] + P @ Vc2
            for (ri, col, bit) in by_tile.get((ST_OACC, j), []):
                flipped.append((ST_OACC, float(Ot[ri, col])))
                Ot[ri, col] = bitflip32(Ot[ri, col], bit)
        m[act] = m_new

    # ---- range restriction of the row-sum with substitution of the lower bound (Section 3.4, case 3; "optimized EFTA")
    U = np.minimum(row_idx + 1, N).astype(np.float64) if prm.causal else np.full(n, float(N))
    with np.errstate(all="ignore"):
        in_range = (lower * (1 - prm.delta_l) <= ell) & (ell <= U * (1 + prm.delta_l))
        dist = np.minimum(np.abs(ell / (lower * (1 - prm.delta_l)) - 1), np.abs(ell / (U * (1 + prm.delta_l)) - 1))
    dist = np.where(np.isfinite(dist), dist, np.inf)
    for i in np.flatnonzero(~in_range):
        events.append((CHECK_L, -1, int(row_idx[i]), 0))
        if prm.correct:
            ell[i] = lower[i]
    # ---- normalisation, then unified verification of GEMM II, rescale and normalisation
    with np.errstate(all="ignore"):
        O = Ot / ell[:, None]
        C1 = Oc1 / ell[:, None]
        C2 = Oc2 / ell[:, None]
        sum1, _ = fold(O, s)
        R = C1 - sum1
        okO = np.abs(R) <= prm.tau_o
    finR = np.isfinite(R)
    o_ratio = float(np.abs(R[finR]).max()) / prm.tau_o if finR.any() else 0.0
    if (~finR).any():
        o_ratio = np.inf
    for (i, c) in zip(*np.nonzero(~okO)):
        cols = c + s * np.arange(nV)
        lstar, val = locate_and_restore(O[i, cols], C1[i, c], C2[i, c])
        events.append((CHECK_O, -1, int(row_idx[i]), int(cols[lstar]) if lstar >= 0 else -1))
        if prm.correct and lstar >= 0:
            O[i, cols[lstar]] = val
    diag = {"lambda_ratio": float(lam_ratio), "o_ratio": float(o_ratio),
            "l_distance": float(dist.min()) if n else np.inf, "l_ratio": 0.0, "flipped": flipped,
            "lin_ratio": 0.0, "o_step_ratio": 0.0, "l_step_distance": np.inf}
    return O, sorted(events), diag


def efta_rows(Q: np.ndarray, row_idx: np.ndarray, K: np.ndarray, V: np.ndarray,
              prm: Params, faults: Sequence[Fault] = (),
              max_shift: Optional[Dict[Tuple[int, int], float]] = None
              ) -> Tuple[np.ndarray, List[Event], Dict[str, float]]:
    """Algorithm 1 for query rows ``row_idx`` of one head: ``efta_rows_unified`` (the paper's method),
    or, when ``prm`` asks for one of the verification variants, ``efta_rows_with_modes``."""
    if prm.rowsum_fold or prm.per_step or prm.softmax_dmr or prm.rescale_margin > 0:
        return efta_rows_with_modes(Q, row_idx, K, V, prm, faults, max_shift)
    return efta_rows_unified(Q, row_idx, K, V, prm, faults, max_shift)


def efta_rows_with_modes(Q: np.ndarray, row_idx: np.ndarray, K: np.ndarray, V: np.ndarray,
              prm: Params, faults: Sequence[Fault] = (),
              max_shift: Optional[Dict[Tuple[int, int], float]] = None
              ) -> Tuple[np.ndarray, List[Event], Dict[str, float]]:
    """Algorithm 1 with the verification variants of ``Params`` (``rowsum_fold``, ``per_step``,
    ``softmax_dmr``) for query rows ``row_idx`` of one head.  With every variant off it takes
    exactly the steps of ``efta_rows_unified`` (a test holds the two against each other).

    Q: [n, d] float64 (rows row_idx of the head's query matrix), K, V: [N, d].
    Returns (O [n, d], sorted events, diagnostics).  Diagnostics hold the largest
    check statistic over all evaluated checks relative to its threshold
    (``lambda_ratio``, ``o_ratio``) and the smallest relative distance of a final
    row-sum to its range boundaries (``l_distance``); the fault generator uses
    them to keep clear of decisions that hinge on rounding.  ``flipped`` lists
    (stage, value before the flip) for every fault that was applied.

    ``max_shift`` maps (kv_tile, row) to an error added to the running maximum the
    moment it is formed (Section 3.4, case 1: such an error needs no protection
    because it cancels between numerator and denominator); tests use it to show
    exactly that.
    """
    s, Bc, sc = prm.stride, prm.block_n, prm.scale
    n, d = Q.shape
    N = K.shape[0]
    assert Bc % s == 0 and d % s == 0
    nK, nV = Bc // s, d // s
    row_idx = np.asarray(row_idx, dtype=np.int64)
    pos = {int(r): i for i, r in enumerate(row_idx)}
    by_tile: Dict[Tuple[int, int], List[Tuple[int, int, int]]] = {}
    for (st, kt, row, col, bit) in faults:
        if int(row) in pos:
            by_tile.setdefault((int(st), int(kt)), []).append((pos[int(row)], int(col), int(bit)))

    m = np.full(n, -np.inf)
    ell = np.zeros(n)
    lower = np.zeros(n)
    Ot = np.zeros((n, d))
    Oc1 = np.zeros((n, s))
    Oc2 = np.zeros((n, s))
    events: List[Event] = []
    flipped: List[Tuple[int, float]] = []     # (stage, value before the flip) of every applied fault
    lam_ratio = 0.0
    lin_ratio = 0.0            # per_step: largest linear residual over its threshold
    o_step_ratio = 0.0         # per_step: largest per-iteration output residual over its threshold
    l_step_distance = np.inf   # per_step: smallest relative distance of a row-sum to its range, any iteration
    assert not (prm.per_step and prm.rowsum_fold)
    assert prm.per_step or not prm.softmax_dmr
    lazy = prm.rescale_margin > 0
    assert not (lazy and (prm.per_step or prm.rowsum_fold))
    m_true = np.full(n, -np.inf)   # running maximum (with rescale_margin, m holds the reference maximum)
    n_rescales = 0                 # (row, iteration) pairs with a rescale factor other than one
    n_tiles = (N + Bc - 1) // Bc

    for j in range(n_tiles):
        k0 = j * Bc
        act = np.flatnonzero(row_idx >= k0) if prm.causal else np.arange(n)
        if act.size == 0:
            break
        keys = k0 + np.arange(Bc)
        Kj = np.zeros((Bc, d)); Vj = np.zeros((Bc, d))
        kv = min(N, k0 + Bc) - k0
        Kj[:kv] = K[k0:k0 + kv]; Vj[:kv] = V[k0:k0 + kv]
        valid = np.broadcast_to(keys[None, :] < N, (act.size, Bc)).copy()
        if prm.causal:
            valid &= keys[None, :] <= row_idx[act, None]

        # encode (Algorithm 1, "Encode tensor checksum")
        Kc1, Kc2 = encode_k(Kj, s)
        Vc1, Vc2 = encode_v(Vj, s)
        if prm.rowsum_fold:
            Vc1[:kv, 0] += 1.0
            Vc2[:kv, 0] += nV + 1.0
        # GEMM I
        Qa = Q[act]
        S = Qa @ Kj.T
        Sc1 = Qa @ Kc1.T
        Sc2 = Qa @ Kc2.T
        loc = {int(a): i for i, a in enumerate(act)}
        for (ri, col, bit) in by_tile.get((ST_S, j), []):
            if ri in loc:
                flipped.append((ST_S, float(S[loc[ri], col - k0])))
                S[loc[ri], col - k0] = bitflip32(S[loc[ri], col - k0], bit)

        def softmax_part(Srows, vrows, m_old, mt_old=None):
            with np.errstate(all="ignore"):
                mh = np.where(vrows, sc * Srows, -np.inf).max(axis=1)
                if lazy:
                    mt = np.maximum(mt_old, mh)
                    mn = np.where(mt > m_old + prm.rescale_margin, mt, m_old)     # renewed only beyond the margin
                else:
                    mn = np.maximum(m_old, mh)
                x = sc * Srows - mn[:, None]
                P = np.where(vrows, np.exp(x), 0.0)
            return mh, mn, x, P

        # reduce max, element-wise exp
        m_hat, m_new, x, P = softmax_part(S, valid, m[act], m_true[act])
        for (jt, row), dm in (max_shift or {}).items():
            if jt == j and int(row) in pos and pos[int(row)] in loc:
                i = loc[pos[int(row)]]
                m_new[i] += dm
                x[i] = sc * S[i] - m_new[i]
                P[i] = np.where(valid[i], np.exp(x[i]), 0.0)
        touched = np.zeros_like(valid)
        for (ri, col, bit) in by_tile.get((ST_EXP, j), []):
            if ri in loc and valid[loc[ri], col - k0]:
                flipped.append((ST_EXP, float(P[loc[ri], col - k0])))
                P[loc[ri], col - k0] = bitflip32(P[loc[ri], col - k0], bit)
                touched[loc[ri], col - k0] = True

        # unified verification of GEMM I, subtraction and exp
        with np.errstate(all="ignore"):
            sum1, _ = fold(S, s)
            R1 = Sc1 - sum1
            e = np.where(touched & valid, np.log(P) - x, 0.0)
            E, _ = fold(e, s)
            lam = E - sc * R1
        has_valid = valid.reshape(act.size, nK, s).any(axis=1)
        with np.errstate(invalid="ignore"):
            ok = np.abs(lam) <= prm.eps1
        det = has_valid & ~ok
        if prm.softmax_dmr:
            # duplication: any stored exponential that differs from its re-evaluation
            with np.errstate(all="ignore"):
                differs = touched & valid & (P != np.exp(x))
            det = differs.reshape(act.size, nK, s).any(axis=1)
        if prm.per_step:
            with np.errstate(invalid="ignore"):
                lin_all = ~(sc * np.abs(R1) <= prm.eps1 / 2)
            det |= has_valid & lin_all
            finl = has_valid & np.isfinite(R1)
            if finl.any():
                lin_ratio = max(lin_ratio, float((sc * np.abs(R1[finl])).max()) / (prm.eps1 / 2))
            if (has_valid & ~np.isfinite(R1)).any():
                lin_ratio = np.inf
        fin = has_valid & np.isfinite(lam)
        if not prm.softmax_dmr:
            if fin.any():
                lam_ratio = max(lam_ratio, float(np.abs(lam[fin]).max()) / prm.eps1)
            if (has_valid & ~np.isfinite(lam)).any():
                lam_ratio = np.inf
        redo = []
        for (i, c) in zip(*np.nonzero(det)):
            cols = c + s * np.arange(nK)
            with np.errstate(invalid="ignore"):
                linear = not (sc * abs(R1[i, c]) <= prm.eps1 / 2)
            if linear:
                lstar, val = locate_and_restore(S[i, cols], Sc1[i, c], Sc2[i, c])
                col = k0 + int(cols[lstar]) if lstar >= 0 else -1
                events.append((CHECK_S, j, int(row_idx[act[i]]), col))
                if prm.correct and lstar >= 0:
                    S[i, cols[lstar]] = val
                    redo.append(i)
            else:
                with np.errstate(all="ignore"):
                    good = np.exp(x[i, cols])
                for l in range(nK):
                    if valid[i, cols[l]] and touched[i, cols[l]] and P[i, cols[l]] != good[l]:
                        events.append((CHECK_EXP, j, int(row_idx[act[i]]), k0 + int(cols[l])))
                        if prm.correct:
                            P[i, cols[l]] = good[l]
        for i in sorted(set(redo)):
            mh, mn, xx, PP = softmax_part(S[i:i + 1], valid[i:i + 1], m[act[i]:act[i] + 1], m_true[act[i]:act[i] + 1])
            m_hat[i], m_new[i], x[i], P[i] = mh[0], mn[0], xx[0], PP[0]
        m_true[act] = np.maximum(m_true[act], m_hat)

        # reduce sum, GEMM II with rescale
        with np.errstate(all="ignore"):
            alpha = np.exp(m[act] - m_new)
            n_rescales += int(np.count_nonzero(np.isfinite(m[act]) & (alpha != 1.0)))
            ell[act] = alpha * ell[act] + P.sum(axis=1)
            lower[act] = alpha * lower[act] + np.where(np.isfinite(m_hat), np.exp(m_hat - m_new), 0.0)
            ell_dup = ell.copy()               # the second evaluation of the reduce-sum (softmax_dmr)
            for (ri, col, bit) in by_tile.get((ST_ROWSUM, j), []):
                flipped.append((ST_ROWSUM, float(ell[ri])))
                ell[ri] = bitflip32(ell[ri], bit)
            Ot[act] = alpha[:, None] * Ot[act] + P @ Vj
            Oc1[act] = alpha[:, None] * Oc1[act] + P @ Vc1
            Oc2[act] = alpha[:, None] * Oc2[act] + P @ Vc2
            for (ri, col, bit) in by_tile.get((ST_OACC, j), []):
                flipped.append((ST_OACC, float(Ot[ri, col])))
                Ot[ri, col] = bitflip32(Ot[ri, col], bit)
        m[act] = m_new
        if prm.per_step:
            # (b) range of the row-sum so far
            seen = np.minimum(row_idx[act] + 1, min(N, k0 + Bc)) if prm.causal else np.full(act.size, float(min(N, k0 + Bc)))
            seen = seen.astype(np.float64)
            la, lo_ = ell[act], lower[act]
            if prm.softmax_dmr:
                same = (la == ell_dup[act]) | (np.isnan(la) & np.isnan(ell_dup[act]))
                for i in np.flatnonzero(~same):
                    events.append((CHECK_L, j, int(row_idx[act[i]]), 0))
                    if prm.correct:
                        ell[act[i]] = ell_dup[act[i]]
            else:
                with np.errstate(all="ignore"):
                    in_rng = (lo_ * (1 - prm.delta_l) <= la) & (la <= seen * (1 + prm.delta_l))
                    dst = np.minimum(np.abs(la / (lo_ * (1 - prm.delta_l)) - 1), np.abs(la / (seen * (1 + prm.delta_l)) - 1))
                dst = np.where(np.isfinite(dst), dst, np.inf)
                if dst.size:
                    l_step_distance = min(l_step_distance, float(dst.min()))
                for i in np.flatnonzero(~in_rng):
                    events.append((CHECK_L, j, int(row_idx[act[i]]), 0))
                    if prm.correct:
                        ell[act[i]] = lower[act[i]]
            # (c) GEMM II and the rescale, on the unnormalised accumulator
            with np.errstate(all="ignore"):
                f1, _ = fold(Ot[act], s)
                Rs = Oc1[act] - f1
                thr = prm.tau_o * ell[act][:, None]
                okS = np.abs(Rs) <= thr
                stat = np.abs(Rs) / thr
            finS = np.isfinite(stat)
            if finS.any():
                o_step_ratio = max(o_step_ratio, float(stat[finS].max()))
            if (~finS).any():
                o_step_ratio = np.inf
            for (i, c) in zip(*np.nonzero(~okS)):
                cols = c + s * np.arange(nV)
                r = act[i]
                lstar, val = locate_and_restore(Ot[r, cols], Oc1[r, c], Oc2[r, c])
                events.append((CHECK_O, j, int(row_idx[r]), int(cols[lstar]) if lstar >= 0 else -1))
                if prm.correct and lstar >= 0:
                    Ot[r, cols[lstar]] = val

    U = np.minimum(row_idx + 1, N).astype(np.float64) if prm.causal else np.full(n, float(N))
    if lazy:
        with np.errstate(all="ignore"):
            U = U * np.exp(m_true - m)         # exponentials reach exp(running maximum - reference maximum)
    l_ratio = 0.0
    if prm.rowsum_fold:
        # exact check of the row-sum against the one the class-0 checksum implies
        dist = np.full(n, np.inf)
        cols0 = s * np.arange(nV)
        for i in range(n):
            x = Ot[i, cols0]
            with np.errstate(all="ignore"):
                l_c = Oc1[i, 0] - x.sum()
                r = (l_c - ell[i]) / l_c
                ok = np.isfinite(r) and abs(r) <= prm.tau_o
            l_ratio = max(l_ratio, abs(r) / prm.tau_o if np.isfinite(r) else np.inf)
            if ok:
                continue
            lstar, val = locate_and_restore(np.append(x, ell[i]), Oc1[i, 0], Oc2[i, 0])
            if lstar == nV:
                events.append((CHECK_L, -1, int(row_idx[i]), 0))
                if prm.correct:
                    ell[i] = val
    elif prm.softmax_dmr:
        dist = np.full(n, np.inf)
    else:
        # range restriction of the row-sum
        with np.errstate(all="ignore"):
            in_range = (lower * (1 - prm.delta_l) <= ell) & (ell <= U * (1 + prm.delta_l))
            dist = np.minimum(np.abs(ell / (lower * (1 - prm.delta_l)) - 1), np.abs(ell / (U * (1 + prm.delta_l)) - 1))
        dist = np.where(np.isfinite(dist), dist, np.inf)
        for i in np.flatnonzero(~in_range):
            events.append((CHECK_L, -1, int(row_idx[i]), 0))
            if prm.correct:
                ell[i] = lower[i]
    # normalisation
    with np.errstate(all="ignore"):
        O = Ot / ell[:, None]
        C1 = Oc1 / ell[:, None]
        C2 = Oc2 / ell[:, None]
        extra = ell / ell                      # the normalised extra fold of class 0 (rowsum_fold)
        # unified verification of GEMM II, rescale and normalisation
        sum1, _ = fold(O, s)
        if prm.rowsum_fold:
            sum1[:, 0] += extra
        R = C1 - sum1
        okO = np.abs(R) <= prm.tau_o
    finR = np.isfinite(R)
    o_ratio = float(np.abs(R[finR]).max()) / prm.tau_o if finR.any() else 0.0
    if (~finR).any():
        o_ratio = np.inf
    for (i, c) in zip(*np.nonzero(~okO)):
        cols = c + s * np.arange(nV)
        if prm.rowsum_fold and c == 0:
            lstar, val = locate_and_restore(np.append(O[i, cols], extra[i]), C1[i, c], C2[i, c])
            if lstar == nV:
                continue                       # the row-sum itself: reported by the check above
        else:
            lstar, val = locate_and_restore(O[i, cols], C1[i, c], C2[i, c])
        events.append((CHECK_O, -1, int(row_idx[i]), int(cols[lstar]) if lstar >= 0 else -1))
        if prm.correct and lstar >= 0:
            O[i, cols[lstar]] = val
    diag = {"lambda_ratio": float(lam_ratio), "o_ratio": float(o_ratio),
            "l_distance": float(dist.min()) if n else np.inf, "l_ratio": float(l_ratio), "flipped": flipped,
            "lin_ratio": float(lin_ratio), "o_step_ratio": float(o_step_ratio), "l_step_distance": float(l_step_distance),
            "rescales": n_rescales}
    return O, sorted(events), diag


def fault_is_robust(diag: Dict[str, float], band: float = 4.0, l_band: float = 2.0 ** -11) -> bool:
    """True when no check decision of the run sits near its threshold.

    Used by the fault generator: a candidate fault is kept only if every check
    statistic is either below threshold/band or above threshold*band, and the
    final row-sum is further than ``l_band`` (relative) from both range bounds.
    """
    for key in ("lambda_ratio", "o_ratio", "l_ratio", "lin_ratio", "o_step_ratio"):
        r = diag.get(key, 0.0)
        if 1.0 / band <= r <= band:
            return False
    return diag["l_distance"] > l_band and diag.get("l_step_distance", np.inf) > l_band


def fp32_is_fragile(x: float, stage: int, bit: Optional[int] = None) -> bool:
    """True when what a flipped bit does to the fp32 value x depends on rounding, i.e. when an
    fp32 evaluation of the same quantity in another summation order (or from operands rounded to
    16 bits first) could see another outcome of the same flip:

    * x sits so close to a power of two (or to zero, or to the bottom of the normal range) that
      the other evaluation could land in the neighbouring binade;
    * (row-sum, with ``bit`` given) the flipped mantissa bit could have the other present value.
      A flip of mantissa bit b adds 2^(b-23) 2^e when the bit is clear and subtracts it when set;
      a row-sum formed from exponentials rounded to 16 bits differs from the exact one by up to
      about 2^-9 of its size, so the bit is uncertain when x lies that close to a multiple of
      2^(b-23) 2^e.  Bits below 10 move the row-sum by less than 2^-13 of its size in either
      direction and are harmless whatever their value."""
    if not np.isfinite(x) or x == 0.0:
        return True
    ax = abs(float(x))
    if ax < 2.0 ** -100:
        return True
    mant, ex = np.frexp(ax)                    # ax = mant * 2**ex, mant in [0.5, 1)
    gap = min(mant - 0.5, 1.0 - mant) * 2.0 ** ex   # absolute distance to a binade edge
    if stage == ST_S:
        return gap < 2.0 ** -11                # raw scores: absolute accumulation noise
    rel = 2.0 ** -14 if stage == ST_EXP else 2.0 ** -9
    if gap < rel * ax:
        return True
    if stage == ST_ROWSUM and bit is not None and 10 <= bit <= 22:
        step = 2.0 ** (bit - 23) * 2.0 ** (ex - 1)      # weight of mantissa bit `bit` in x
        off = ax % step
        return min(off, step - off) < rel * ax
    return False
