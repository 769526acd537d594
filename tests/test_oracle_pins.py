"""Pins for the CPU oracle: closed forms, invariants, library routines and brute force.

Each test checks the oracle against something other than itself, chosen so that a
dropped term, a wrong sign or index, or a transposed operand in the oracle fails
at least one of them.  No GPU is needed.
"""
import math
import os

import numpy as np
import pytest

from oracle import efta_oracle as orc
from oracle.efta_oracle import (CHECK_EXP, CHECK_L, CHECK_O, CHECK_S, ST_EXP, ST_OACC,
                                ST_ROWSUM, ST_S, Params, attention_clean, bitflip32,
                                efta_rows, encode_k, encode_v, fold, locate_and_restore)

HERE = os.path.dirname(os.path.abspath(__file__))


def _rand(N, d, seed, scale=1.0):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, d)) * scale, rng.standard_normal((N, d)) * scale,
            rng.standard_normal((N, d)) * scale)


# ---------------------------------------------------------------- definition

def _parse_rows(txt):
    def val(t):
        t = t.strip()
        return math.log(float(t[2:])) if t.startswith("ln") else float(t)
    return np.array([[val(t) for t in row.split(",")] for row in txt.split("/")], dtype=np.float64)


def test_clean_against_printed_closed_forms():
    """eq. (8): exact rational softmax weights, expected O written by hand."""
    n = 0
    for line in open(os.path.join(HERE, "golden", "softmax_closed_form.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, causal, scale, q, k, v, o = [f.strip() for f in line.split(";")]
        Q, K, V, O = map(_parse_rows, (q, k, v, o))
        got = attention_clean(Q, K, V, float(scale), bool(int(causal)))
        assert np.allclose(got, O, rtol=0, atol=1e-13), name
        prm = Params(scale=float(scale), causal=bool(int(causal)), block_n=8)
        Kp = np.vstack([K, np.zeros((0, K.shape[1]))])
        # the tiled algorithm needs d % 8 == 0: pad the feature axis with zeros
        pad = lambda X: np.hstack([X, np.zeros((X.shape[0], 8 - X.shape[1]))])
        got2, ev, _ = efta_rows(pad(Q), np.arange(Q.shape[0]), pad(Kp), pad(V), prm)
        assert ev == [] and np.allclose(got2[:, :O.shape[1]], O, rtol=0, atol=1e-13), name
        n += 1
    assert n == 5


@pytest.mark.parametrize("causal", [False, True])
def test_clean_against_library_sdpa(causal):
    torch = pytest.importorskip("torch")
    Q, K, V = _rand(96, 32, 1)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q)[None, None], torch.from_numpy(K)[None, None], torch.from_numpy(V)[None, None],
        is_causal=causal, scale=0.3)[0, 0].numpy()
    got = attention_clean(Q, K, V, 0.3, causal)
    assert np.abs(got - ref).max() < 1e-13


def test_clean_invariants():
    """Softmax rows sum to one; colsum(P V) = colsum(P) V; colsum(Q K^T) = colsum(Q) K^T."""
    Q, K, V = _rand(40, 16, 2)
    ones = attention_clean(Q, K, np.ones((40, 16)), 0.25, True)
    assert np.abs(ones - 1).max() < 1e-14
    P = attention_clean(Q, K, np.eye(40), 0.25, False)          # V = I returns P itself
    assert np.abs(P.sum(axis=1) - 1).max() < 1e-14
    O = attention_clean(Q, K, V, 0.25, False)
    assert np.abs(O.sum(axis=0) - P.sum(axis=0) @ V).max() < 1e-13
    # a permutation of the keys (with their values) must not change O: catches index slips
    perm = np.random.default_rng(3).permutation(40)
    assert np.abs(attention_clean(Q, K[perm], V[perm], 0.25, False) - O).max() < 1e-13
    # transposition slip: scores must be Q K^T, not K Q^T -> one-hot query picks a K column
    Q1 = np.zeros((1, 16)); Q1[0, 3] = 1.0
    w = attention_clean(Q1, K, np.eye(40), 1.0, False)[0]
    e = np.exp(K[:, 3] - K[:, 3].max())
    assert np.abs(w - e / e.sum()).max() < 1e-14
    S = Q @ K.T
    assert np.abs(S.sum(axis=0) - Q.sum(axis=0) @ K.T).max() < 1e-12


# ---------------------------------------------------------------- tiled recurrence

@pytest.mark.parametrize("N,d,Bc,causal", [(128, 64, 64, False), (128, 64, 32, True), (200, 16, 64, True),
                                           (77, 8, 16, False), (64, 128, 128, True), (1, 8, 8, True)])
def test_tiled_equals_definition(N, d, Bc, causal):
    """eq. (2)-(8): the online recurrence with checksums attached reaches the definition,
    raises no flag, and keeps every check statistic at rounding level."""
    Q, K, V = _rand(N, d, 10 + N)
    prm = Params(scale=d ** -0.5, causal=causal, block_n=Bc)
    O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm)
    assert ev == []
    assert np.abs(O - attention_clean(Q, K, V, prm.scale, causal)).max() < 1e-12
    assert dg["lambda_ratio"] < 1e-9 and dg["o_ratio"] < 1e-9
    # a subset of rows gives the same rows
    rows = np.arange(N)[::3]
    O2, _, _ = efta_rows(Q[rows], rows, K, V, prm)
    assert np.abs(O2 - O[rows]).max() < 1e-13


# ---------------------------------------------------------------- checksums

def test_encode_closed_forms():
    """eq. (13)-(16): products with the encoded tiles equal strided sums of the plain product."""
    rng = np.random.default_rng(5)
    Qi = rng.standard_normal((7, 24)); Kj = rng.standard_normal((32, 24)); Vj = rng.standard_normal((32, 24))
    Kc1, Kc2 = encode_k(Kj, 8)
    S = Qi @ Kj.T
    for c in range(8):
        assert np.allclose(Qi @ Kc1[c], sum(S[:, c + 8 * l] for l in range(4)), atol=1e-12)
        assert np.allclose(Qi @ Kc2[c], sum((l + 1) * S[:, c + 8 * l] for l in range(4)), atol=1e-12)
    f1, f2 = fold(S, 8)
    assert np.allclose(f1, Qi @ Kc1.T, atol=1e-12) and np.allclose(f2, Qi @ Kc2.T, atol=1e-12)
    P = rng.random((7, 32))
    Vc1, Vc2 = encode_v(Vj, 8)
    Ot = P @ Vj
    for c in range(8):
        assert np.allclose(P @ Vc1[:, c], sum(Ot[:, c + 8 * l] for l in range(3)), atol=1e-12)
        assert np.allclose(P @ Vc2[:, c], sum((l + 1) * Ot[:, c + 8 * l] for l in range(3)), atol=1e-12)


def test_classical_abft_locate_correct():
    """eq. (9), (10): one checksum class per column (stride 1 fold over all rows)."""
    rng = np.random.default_rng(6)
    A = rng.standard_normal((6, 5)); B = rng.standard_normal((5, 4))
    C = A @ B
    c1 = np.ones(6) @ A @ B
    c2 = np.arange(1, 7) @ A @ B
    for i in range(6):
        for j in range(4):
            for delta in (0.5, -3.0, 1e6):
                Cb = C.copy(); Cb[i, j] += delta
                # the paper's index formula: (c2' - c2) / (c1' - c1) names row i (1-based weight)
                ratio = (np.arange(1, 7) @ Cb[:, j] - c2[j]) / (Cb[:, j].sum() - c1[j])
                assert round(ratio) - 1 == i
                l, val = locate_and_restore(Cb[:, j], c1[j], c2[j])
                assert l == i and abs(val - C[i, j]) < 1e-9 * max(1, abs(delta))


def test_strided_locate_bruteforce():
    """Text after eq. (16): every position of a tile, several error sizes incl. Inf/NaN."""
    rng = np.random.default_rng(7)
    Qi = rng.standard_normal((4, 16)); Kj = rng.standard_normal((32, 16))
    S = Qi @ Kj.T
    Kc1, Kc2 = encode_k(Kj, 8)
    Sc1, Sc2 = Qi @ Kc1.T, Qi @ Kc2.T
    for i in range(4):
        for col in range(32):
            for delta in (1.0, -0.01, 1e30, np.inf, -np.inf, np.nan):
                Sb = S.copy(); Sb[i, col] = Sb[i, col] + delta
                c = col % 8
                cols = c + 8 * np.arange(4)
                l, val = locate_and_restore(Sb[i, cols], Sc1[i, c], Sc2[i, c])
                assert cols[l] == col
                assert abs(val - S[i, col]) < 1e-12


def test_strided_multi_error_rows():
    """Errors in distinct stride-8 classes of one row are all repaired; two in one class are
    detected but cannot be located (the limitation the paper states)."""
    Q, K, V = _rand(64, 16, 8)
    prm = Params(scale=0.25, causal=False, block_n=32)
    clean = attention_clean(Q, K, V, 0.25, False)
    faults = [(ST_S, 1, 5, 32 + c + 8 * (c % 4), 28) for c in range(8)]    # 8 classes, row 5, tile 1
    O, ev, _ = efta_rows(Q, np.arange(64), K, V, prm, faults)
    assert ev == sorted((CHECK_S, 1, 5, f[3]) for f in faults)
    assert np.abs(O - clean).max() < 1e-11
    same = [(ST_S, 0, 9, 3, 29), (ST_S, 0, 9, 19, 29)]                     # both class 3
    O, ev, _ = efta_rows(Q, np.arange(64), K, V, prm, same)
    assert len(ev) >= 1 and ev[0][0] == CHECK_S                            # noticed ...
    assert np.abs(O[9] - clean[9]).max() > 1e-6                            # ... but not repaired



def test_element_wide_checksum_versus_stride_8():
    """The traditional checksum (one class over the whole tile row: stride 1) against the stride-8
    tensor checksum (Section 3.3, and the coverage comparison of Section 4.2): without faults both
    are silent and exact, one error per (row, key tile) is repaired by both, and of several errors
    in one (row, key tile) the stride-8 fold repairs every one that has its class to itself while
    the single class notices them and repairs none."""
    Q, K, V = _rand(64, 16, 8)
    clean = attention_clean(Q, K, V, 0.25, False)
    wide = Params(scale=0.25, causal=False, block_n=32, stride=1)
    tensor = Params(scale=0.25, causal=False, block_n=32, stride=8)
    rows = np.arange(64)
    for prm in (wide, tensor):
        O, ev, _ = efta_rows(Q, rows, K, V, prm, [])
        assert ev == [] and np.abs(O - clean).max() < 1e-12
        one = [(ST_S, 1, 5, 41, 28)]
        O, ev, _ = efta_rows(Q, rows, K, V, prm, one)
        assert ev == [(CHECK_S, 1, 5, 41)] and np.abs(O - clean).max() < 1e-11
        one = [(ST_OACC, 1, 7, 11, 27)]
        O, ev, _ = efta_rows(Q, rows, K, V, prm, one)
        assert [e[0] for e in ev] == [CHECK_O] and ev[0][3] == 11 and np.abs(O - clean).max() < 1e-11
    rng = np.random.default_rng(77)
    repaired = {1: 0, 8: 0}
    noticed = {1: 0, 8: 0}
    trials = 40
    for t in range(trials):
        row, tile = int(rng.integers(0, 64)), int(rng.integers(0, 2))
        c0, c1 = rng.choice(8, size=2, replace=False)                      # two different classes
        cols = [32 * tile + int(c0) + 8 * int(rng.integers(0, 4)), 32 * tile + int(c1) + 8 * int(rng.integers(0, 4))]
        faults = [(ST_S, tile, row, cols[0], 28), (ST_S, tile, row, cols[1], 29)]
        for prm in (wide, tensor):
            O, ev, _ = efta_rows(Q, rows, K, V, prm, faults)
            noticed[prm.stride] += len(ev) >= 1
            repaired[prm.stride] += np.abs(O - clean).max() < 2e-3     # the parity tolerance: harmless residue counts as repaired
    assert noticed[8] == trials and noticed[1] >= trials - 2      # (two errors may offset each other in one sum)
    assert repaired[8] == trials and repaired[1] <= trials // 4, (noticed, repaired)


# ---------------------------------------------------------------- softmax protection

def test_case1_max_error_cancels():
    """Section 3.4, case 1: an error in the row maximum cancels between numerator and
    denominator.  (A maximum that ends the loop too LOW inflates the row-sum by the same factor,
    which the upper range bound may then notice; the shifts below stay inside the range.)"""
    Q, K, V = _rand(96, 16, 9)
    prm = Params(scale=0.25, causal=False, block_n=32)
    base, _, _ = efta_rows(Q, np.arange(96), K, V, prm)
    for dm in (0.7, -1.0, 11.0):
        O, ev, dg = efta_rows(Q, np.arange(96), K, V, prm, max_shift={(1, 50): dm, (0, 7): abs(dm), (2, 90): dm})
        assert ev == [] and np.abs(O - base).max() < 1e-12
        assert dg["lambda_ratio"] < 1e-9


def _row_state(q, K, scale, Bc, j, row, causal):
    """Independent evaluation of m (running max through tile j) and the tile's scores."""
    hi = min(K.shape[0], (j + 1) * Bc)
    keys = np.arange(hi)
    ok = keys <= row if causal else np.ones(hi, bool)
    s_all = scale * (K[:hi] @ q)
    m = s_all[ok].max()
    return m, s_all[j * Bc:hi], ok[j * Bc:hi]


def test_case2_product_identity_and_signatures():
    """prod_l exp(S_l - m) = exp(check1 - n*m) on clean data (masked classes included), and the
    oracle's log-ratio statistic equals ln(P'/P) for an exp fault and scale*delta for a score fault."""
    N, d, Bc = 96, 16, 32
    Q, K, V = _rand(N, d, 11)
    scale = 0.25
    for causal in (False, True):
        prm = Params(scale=scale, causal=causal, block_n=Bc)
        for (row, j) in ((40, 1), (95, 2), (33, 1)):
            m, sj, ok = _row_state(Q[row], K, scale, Bc, j, row, causal)
            Kc1, _ = encode_k(K[j * Bc:(j + 1) * Bc], 8)
            for c in range(8):
                cols = c + 8 * np.arange(Bc // 8)
                okc = ok[cols]
                if not okc.any():
                    continue
                prod = np.prod(np.exp(sj[cols][okc] - m))
                chk_eff = scale * (Q[row] @ Kc1[c]) - sj[cols][~okc].sum()
                assert abs(prod / np.exp(chk_eff - okc.sum() * m) - 1) < 1e-12
            col = j * Bc + (3 if not causal else 1)
            p = math.exp(sj[col - j * Bc] - m)
            for bit in (20, 22, 24, 30):
                pf = bitflip32(p, bit)
                _, ev, dg = efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [(ST_EXP, j, row, col, bit)])
                want = abs(math.log(pf / p)) if 0 < pf < np.inf else np.inf   # incl. the fp32 rounding of P
                if np.isfinite(want):
                    assert abs(dg["lambda_ratio"] * prm.eps1 - want) < 1e-9 * max(1, want)
                assert ((CHECK_EXP, j, row, col) in ev) == (want > prm.eps1)
            s_raw = float(Q[row] @ K[col])
            for bit in (21, 25, 29):
                delta = bitflip32(s_raw, bit) - float(np.float32(s_raw))
                _, ev, dg = efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [(ST_S, j, row, col, bit)])
                # the fp32 rounding of the score is itself part of the injected error
                delta_total = bitflip32(s_raw, bit) - s_raw
                assert abs(dg["lambda_ratio"] * prm.eps1 - scale * abs(delta_total)) < 1e-6 * max(1.0, scale * abs(delta))
                assert ((CHECK_S, j, row, col) in ev) == (scale * abs(delta_total) > prm.eps1)


def test_case2_minimum_signature():
    """Any flip of bits 20..30 of a normal fp32 in (0, 1] moves its log by more than 2*eps1."""
    worst = np.inf
    for mant in np.linspace(1.0, 2.0, 4097)[:-1]:
        for ex in (-1, -20, -60):
            p = float(np.float32(mant * 2.0 ** ex))
            for bit in range(20, 31):
                pf = bitflip32(p, bit)
                if 0 < pf < np.inf:
                    worst = min(worst, abs(math.log(pf / p)))
    assert worst >= math.log(1 + 2.0 ** -4) - 1e-12
    assert worst > 2 * Params(scale=1, causal=False, block_n=8).eps1


def test_case3_rowsum_bounds_and_counterexample():
    """lower <= l <= upper on assorted inputs, equality for a single key, and the running-max
    reading of the lower bound is not a bound."""
    for seed, scale, causal in ((1, 0.1, False), (2, 3.0, True), (3, 1.0, True)):
        Q, K, V = _rand(80, 8, 20 + seed)
        K[::7] *= 8
        prm = Params(scale=scale, causal=causal, block_n=16, delta_l=0.0)
        _, ev, _ = efta_rows(Q, np.arange(80), K, V, prm)
        assert ev == []                      # with zero slack: lower <= l <= upper exactly
    # single unmasked key: lower = l = upper = 1 (row 0 of a causal head), slack zero, no flag
    prm = Params(scale=1.0, causal=True, block_n=8, delta_l=0.0)
    Q, K, V = _rand(8, 8, 30)
    O, ev, _ = efta_rows(Q[:1], np.array([0]), K, V, prm)
    assert ev == [] and np.allclose(O[0], V[0], atol=1e-14)
    # counter-example: one dominant score in the first of four tiles.
    scores = np.full(32, -30.0); scores[0] = 0.0
    l_true = np.exp(scores).sum()
    run_max = np.maximum.accumulate(scores.reshape(4, 8).max(axis=1))
    loc_max = scores.reshape(4, 8).max(axis=1)
    assert np.exp(run_max - run_max[-1]).sum() > l_true          # "bound" of 4 above l ~ 1
    assert np.exp(loc_max - run_max[-1]).sum() <= l_true         # local maxima: a true bound


def test_case3_substitution_closed_form():
    """When the row-sum leaves its range it is replaced by the lower bound, so the row of O is
    the clean row times l_true / lower."""
    N, d, Bc = 64, 8, 16
    Q, K, V = _rand(N, d, 40)
    prm = Params(scale=0.5, causal=False, block_n=Bc)
    clean = attention_clean(Q, K, V, 0.5, False)
    row = 17
    s = 0.5 * (K @ Q[row]); m = s.max()
    l_true = np.exp(s - m).sum()
    lower = np.exp(s.reshape(N // Bc, Bc).max(axis=1) - m).sum()
    O, ev, _ = efta_rows(Q, np.arange(N), K, V, prm, [(ST_ROWSUM, 3, row, 0, 30)])
    assert ev == [(CHECK_L, -1, row, 0)]
    assert np.abs(O[row] - clean[row] * l_true / lower).max() < 1e-12
    others = np.delete(np.arange(N), row)
    assert np.abs(O[others] - clean[others]).max() < 1e-12


def test_oacc_fault_located_and_restored():
    N, d, Bc = 64, 32, 16
    Q, K, V = _rand(N, d, 41)
    prm = Params(scale=0.3, causal=True, block_n=Bc)
    clean = attention_clean(Q, K, V, 0.3, True)
    for (row, col, kt, bit) in ((63, 0, 0, 28), (40, 31, 2, 22), (20, 13, 1, 30), (33, 8, 0, 25)):
        O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm, [(ST_OACC, kt, row, col, bit)])
        if dg["o_ratio"] > 1:
            assert ev == [(CHECK_O, -1, row, col)]
            assert np.abs(O - clean).max() < 1e-10
        else:
            assert ev == []


# ---------------------------------------------------------------- whole pipeline, brute force

def _exhaustive(stage, rows, N=32, d=16, Bc=16, causal=True):
    Q, K, V = _rand(N, d, 50)
    scale = 0.4
    prm = Params(scale=scale, causal=causal, block_n=Bc)
    clean = attention_clean(Q, K, V, scale, causal)
    vmax = np.abs(V).max()
    n_det = n_tot = 0
    for row in rows:
        q = Q[row:row + 1]; ridx = np.array([row])
        s = scale * (K @ Q[row]); ok = np.arange(N) <= row if causal else np.ones(N, bool)
        m = s[ok].max(); l_true = np.exp(s[ok] - m).sum()
        nt = (row if causal else N - 1) // Bc + 1
        if stage in (ST_S, ST_EXP):
            targets = [(c // Bc, c) for c in range(row + 1 if causal else N)]
        elif stage == ST_ROWSUM:
            targets = [(t, 0) for t in range(nt)]
        else:
            targets = [(t, c) for t in range(nt) for c in range(0, d, 3)]
        for (kt, col) in targets:
            for bit in range(31):
                O, ev, dg = efta_rows(q, ridx, K, V, prm, [(stage, kt, row, col, bit)])
                n_tot += 1
                dev = np.abs(O[0] - clean[row]).max()
                if stage == ST_ROWSUM:
                    if ev:
                        assert ev == [(CHECK_L, -1, row, 0)]
                        lower = sum(np.exp(s[t * Bc:(t + 1) * Bc][ok[t * Bc:(t + 1) * Bc]].max() - m) for t in range(nt))
                        assert np.abs(O[0] - clean[row] * l_true / lower).max() < 1e-10
                        n_det += 1
                    else:     # undetected: row is the clean row times l_true / l', l' inside the range
                        k = np.abs(clean[row]).argmax()
                        f = O[0, k] / clean[row, k]
                        assert np.abs(O[0] - f * clean[row]).max() < 1e-10
                        assert l_true / ((row + 1 if causal else N) * (1 + prm.delta_l)) - 1e-12 <= f
                    continue
                if ev:
                    n_det += 1
                    want = {ST_S: CHECK_S, ST_EXP: CHECK_EXP, ST_OACC: CHECK_O}[stage]
                    assert ev == [(want, kt if stage != ST_OACC else -1, row, col)], (ev, row, col, bit)
                    assert dev < 1e-9, (stage, row, col, bit, dev)
                else:
                    assert max(dg["lambda_ratio"], dg["o_ratio"]) <= 1.0
                    if stage == ST_OACC:
                        assert dev <= prm.tau_o * (1 + 1e-9)
                    else:     # one softmax weight moved by a factor within exp(+-eps1)
                        assert dev <= 2 * vmax * (math.exp(prm.eps1) - 1) * 1.0001
    return n_det, n_tot


def test_exhaustive_bitflips_scores():
    det, tot = _exhaustive(ST_S, rows=(0, 9, 17, 31))
    assert tot == (1 + 10 + 18 + 32) * 31 and det > tot // 4


def test_exhaustive_bitflips_exp():
    det, tot = _exhaustive(ST_EXP, rows=(3, 16, 30))
    assert det > tot // 4


def test_exhaustive_bitflips_rowsum():
    det, tot = _exhaustive(ST_ROWSUM, rows=range(0, 32, 3))
    assert det > 0


def test_exhaustive_bitflips_oacc():
    det, tot = _exhaustive(ST_OACC, rows=(1, 15, 16, 31), causal=False)
    assert det > tot // 4


# ---------------------------------------------------------------- helper predicates

def test_bitflip_and_fragility_helpers():
    assert bitflip32(1.0, 22) == 1.5 and bitflip32(1.0, 23) == 0.5 and bitflip32(0.75, 30) > 1e38
    assert orc.fp32_is_fragile(1.0, ST_EXP) and orc.fp32_is_fragile(0.0, ST_S)
    assert not orc.fp32_is_fragile(0.75, ST_EXP) and not orc.fp32_is_fragile(3.1, ST_S)
    assert orc.fp32_is_fragile(4.0001, ST_S) and orc.fp32_is_fragile(1e-40, ST_EXP)
    # row-sum, mantissa bit 20 of a value in [4, 8) weighs 0.5: 5.25 is a quarter away from the
    # next multiple (bit certain), 5.5 + 2^-10 is not (a sum rounded elsewhere may see the bit clear);
    # bits below 10 never matter, exponent bits are not subject to this rule
    assert not orc.fp32_is_fragile(5.25, ST_ROWSUM, 20)
    assert orc.fp32_is_fragile(5.5 + 2.0 ** -10, ST_ROWSUM, 20) and orc.fp32_is_fragile(5.5 - 2.0 ** -10, ST_ROWSUM, 20)
    assert orc.fp32_is_fragile(5.25, ST_ROWSUM, 12)           # weight 2^-9: always within the rounding distance
    assert not orc.fp32_is_fragile(5.5 + 2.0 ** -10, ST_ROWSUM, 5) and not orc.fp32_is_fragile(5.5 + 2.0 ** -10, ST_ROWSUM, 27)
    for b in range(10, 23):                                  # the rule is about the bit it names
        w = 2.0 ** (b - 23) * 4.0
        assert bitflip32(5.25, b) in (5.25 + w, 5.25 - w)
    assert orc.fault_is_robust({"lambda_ratio": 10.0, "o_ratio": 1e-9, "l_distance": 0.5})
    assert not orc.fault_is_robust({"lambda_ratio": 1.5, "o_ratio": 1e-9, "l_distance": 0.5})
    assert not orc.fault_is_robust({"lambda_ratio": 0.0, "o_ratio": 0.0, "l_distance": 1e-5})


# ---------------------------------------------------------------- row-sum as an extra checksum fold

@pytest.mark.parametrize("N,d,Bc,causal", [(128, 64, 64, False), (200, 16, 64, True), (77, 8, 16, False), (1, 8, 8, True)])
def test_rowsum_fold_is_silent_and_exact_without_faults(N, d, Bc, causal):
    """A column of ones appended to V accumulates exactly the row-sum (eq. (2)-(8) applied to
    that column), so the class-0 checksum minus the class-0 output folds equals the row-sum."""
    Q, K, V = _rand(N, d, 70 + N)
    prm = Params(scale=d ** -0.5, causal=causal, block_n=Bc, rowsum_fold=True)
    O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm)
    assert ev == []
    assert np.abs(O - attention_clean(Q, K, V, prm.scale, causal)).max() < 1e-12
    assert dg["l_ratio"] < 1e-9 and dg["o_ratio"] < 1e-9 and dg["lambda_ratio"] < 1e-9


def test_rowsum_fold_repairs_every_harmful_rowsum_flip():
    """Every bit of the row-sum, at several rows and iterations: with the extra fold a flip that
    changes the output beyond the threshold is named as the row-sum and put right exactly, where
    the range restriction leaves most of them in place."""
    N, d, Bc = 96, 16, 32
    Q, K, V = _rand(N, d, 71)
    clean = attention_clean(Q, K, V, 0.4, True)
    exact = Params(scale=0.4, causal=True, block_n=Bc, rowsum_fold=True)
    ranged = Params(scale=0.4, causal=True, block_n=Bc)
    left_wrong = 0
    for row, kt in ((95, 0), (95, 2), (40, 1), (5, 0), (64, 2)):
        for bit in range(32):
            f = [(ST_ROWSUM, kt, row, 0, bit)]
            O, ev, dg = efta_rows(Q[row:row + 1], np.array([row]), K, V, exact, f)
            if dg["l_ratio"] > 1:
                assert ev == [(CHECK_L, -1, row, 0)], (row, kt, bit, ev)
                assert np.abs(O[0] - clean[row]).max() < 1e-10
            else:
                assert ev == [] and np.abs(O[0] - clean[row]).max() < 4 * exact.tau_o * np.abs(clean[row]).max() + 1e-12
            O2, _, _ = efta_rows(Q[row:row + 1], np.array([row]), K, V, ranged, f)
            left_wrong += bool(np.abs(O2[0] - clean[row]).max() > 1e-3)
    assert left_wrong > 20          # what the extension is for


def test_rowsum_fold_keeps_class0_output_faults_apart():
    N, d, Bc = 64, 32, 16
    Q, K, V = _rand(N, d, 72)
    prm = Params(scale=0.3, causal=True, block_n=Bc, rowsum_fold=True)
    clean = attention_clean(Q, K, V, 0.3, True)
    for (row, col, kt, bit) in ((63, 0, 0, 28), (40, 24, 2, 22), (20, 8, 1, 30), (33, 16, 0, 25), (50, 5, 1, 27)):
        O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm, [(ST_OACC, kt, row, col, bit)])
        assert ev == [(CHECK_O, -1, row, col)], (row, col, ev)
        assert np.abs(O - clean).max() < 1e-10


def test_rowsum_fold_detect_only_reports_once():
    N, d, Bc = 64, 16, 16
    Q, K, V = _rand(N, d, 73)
    prm = Params(scale=0.3, causal=False, block_n=Bc, rowsum_fold=True, correct=False)
    clean = attention_clean(Q, K, V, 0.3, False)
    O, ev, _ = efta_rows(Q, np.arange(N), K, V, prm, [(ST_ROWSUM, 1, 10, 0, 24)])
    assert ev == [(CHECK_L, -1, 10, 0)]
    assert np.abs(O[10] - clean[10]).max() > 1e-2
    O[10] = clean[10]
    assert np.abs(O - clean).max() < 1e-12


def test_rowsum_fold_non_finite_rowsum():
    N, d, Bc = 32, 8, 16
    Q, K, V = _rand(N, d, 74)
    prm = Params(scale=0.3, causal=False, block_n=Bc, rowsum_fold=True)
    clean = attention_clean(Q, K, V, 0.3, False)
    for bit in (30, 31):
        O, ev, _ = efta_rows(Q, np.arange(N), K, V, prm, [(ST_ROWSUM, 1, 7, 0, bit)])
        assert ev == [(CHECK_L, -1, 7, 0)]
        assert np.abs(O - clean).max() < 1e-10


# ---------------------------------------------------------------- per-step verification (EFTA before unification)

@pytest.mark.parametrize("N,d,Bc,causal", [(128, 64, 64, False), (200, 16, 64, True), (77, 8, 16, False), (1, 8, 8, True)])
def test_per_step_is_silent_and_exact_without_faults(N, d, Bc, causal):
    """Each step's own identity holds without faults (eq. (15) for GEMM I, the same identity applied
    to the running accumulator for GEMM II and the rescale, the range of Section 3.4 case 3 at every
    iteration), so verifying after every step changes nothing and reports nothing."""
    Q, K, V = _rand(N, d, 170 + N)
    prm = Params(scale=d ** -0.5, causal=causal, block_n=Bc, per_step=True)
    O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm)
    assert ev == []
    assert np.abs(O - attention_clean(Q, K, V, prm.scale, causal)).max() < 1e-12
    assert dg["lin_ratio"] < 1e-9 and dg["o_step_ratio"] < 1e-9 and dg["l_step_distance"] > 0


def test_per_step_output_identity_is_exact_on_integers():
    """K = 0 makes every P equal to one, so with integer V the running accumulator and its checksum
    are exact sums of integers: the per-iteration residual is exactly zero (a threshold at
    rounding level passes) and any flipped accumulator bit is found in its own iteration and
    restored exactly."""
    N, d, Bc = 48, 16, 16
    rng = np.random.default_rng(171)
    Q = rng.standard_normal((N, d)); K = np.zeros((N, d)); V = rng.integers(-4, 5, size=(N, d)).astype(np.float64)
    prm = Params(scale=1.0, causal=False, block_n=Bc, per_step=True, tau_o=1e-12)
    O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm)
    assert ev == [] and dg["o_step_ratio"] == 0.0
    clean = attention_clean(Q, K, V, 1.0, False)
    for (row, col, kt, bit) in ((0, 0, 0, 23), (17, 15, 1, 30), (47, 9, 2, 3), (5, 8, 1, 31)):
        _, _, dgu = efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [(ST_OACC, kt, row, col, bit)])
        before = dgu["flipped"][0][1]
        O, ev, _ = efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [(ST_OACC, kt, row, col, bit)])
        if bitflip32(before, bit) == before:
            continue
        assert ev == [(CHECK_O, kt, row, col)], (row, col, kt, bit, ev)
        assert np.abs(O[0] - clean[row]).max() < 1e-12


def test_per_step_names_the_iteration_unified_does_not():
    N, d, Bc = 64, 32, 16
    Q, K, V = _rand(N, d, 172)
    clean = attention_clean(Q, K, V, 0.3, True)
    step = Params(scale=0.3, causal=True, block_n=Bc, per_step=True)
    uni = Params(scale=0.3, causal=True, block_n=Bc)
    for (row, col, kt, bit) in ((63, 0, 0, 28), (40, 31, 1, 29), (20, 13, 0, 30), (33, 8, 1, 27)):
        f = [(ST_OACC, kt, row, col, bit)]
        O, ev, dg = efta_rows(Q, np.arange(N), K, V, step, f)
        assert dg["o_step_ratio"] > 1
        assert ev == [(CHECK_O, kt, row, col)]
        assert np.abs(O - clean).max() < 1e-10
        O2, ev2, _ = efta_rows(Q, np.arange(N), K, V, uni, f)
        assert ev2 == [(CHECK_O, -1, row, col)] and np.abs(O2 - clean).max() < 1e-10
    # a row-sum pushed out of its range is seen in the iteration it happens in
    f = [(ST_ROWSUM, 1, 50, 0, 30)]
    O, ev, _ = efta_rows(Q, np.arange(N), K, V, step, f)
    assert ev == [(CHECK_L, 1, 50, 0)]
    _, ev2, _ = efta_rows(Q, np.arange(N), K, V, uni, f)
    assert ev2 == [(CHECK_L, -1, 50, 0)]
    # the substituted lower bound at iteration 1 is then carried on like the row-sum itself
    assert np.all(np.isfinite(O)) and np.abs(O[np.arange(N) != 50] - clean[np.arange(N) != 50]).max() < 1e-12


def test_per_step_catches_a_linear_fault_the_unified_statistic_lets_pass():
    """A score error e with eps1/2 < scale*e <= eps1 changes the product-form statistic by less than
    eps1 (the exponential follows the damaged score, so only the checksum side moves) but exceeds
    the GEMM I threshold on its own."""
    N, d, Bc = 32, 16, 16
    Q, K, V = _rand(N, d, 173)
    sc = 0.25
    row, col, kt, bit = 20, 19, 1, 14
    S = Q[row] @ K[col]
    e = abs(bitflip32(S, bit) - np.float32(S))
    eps1 = float(sc * e * 1.5)
    clean = attention_clean(Q, K, V, sc, False)
    f = [(ST_S, kt, row, col, bit)]
    uni = Params(scale=sc, causal=False, block_n=Bc, eps1=eps1)
    _, ev, dg = efta_rows(Q[row:row + 1], np.array([row]), K, V, uni, f)
    assert ev == [] and 0.5 < dg["lambda_ratio"] < 1.0
    step = Params(scale=sc, causal=False, block_n=Bc, eps1=eps1, per_step=True)
    O, ev, dg = efta_rows(Q[row:row + 1], np.array([row]), K, V, step, f)
    assert ev == [(CHECK_S, kt, row, col)] and 1.0 < dg["lin_ratio"] < 2.0
    assert np.abs(O[0] - clean[row]).max() < 1e-6


def test_per_step_rejects_the_rowsum_fold():
    Q, K, V = _rand(16, 8, 174)
    with pytest.raises(AssertionError):
        efta_rows(Q, np.arange(16), K, V, Params(scale=1.0, causal=False, block_n=8, per_step=True, rowsum_fold=True))


# ---------------------------------------------------------------- softmax protected by duplication (eq. (11), (12))

def test_dmr_is_silent_and_exact_without_faults():
    for (N, d, Bc, causal) in ((128, 64, 64, False), (200, 16, 64, True), (1, 8, 8, True)):
        Q, K, V = _rand(N, d, 270 + N)
        prm = Params(scale=d ** -0.5, causal=causal, block_n=Bc, per_step=True, softmax_dmr=True)
        O, ev, _ = efta_rows(Q, np.arange(N), K, V, prm)
        assert ev == []
        assert np.abs(O - attention_clean(Q, K, V, prm.scale, causal)).max() < 1e-12


def test_dmr_finds_every_changed_exponential_and_rowsum_bit():
    """Duplication compares exactly: every bit of an exponential or of the row-sum, however small
    its effect, is reported and the output is the fault-free one; the product-form check and the
    range restriction (thresholds) let the small ones pass."""
    N, d, Bc = 48, 16, 16
    Q, K, V = _rand(N, d, 271)
    clean = attention_clean(Q, K, V, 0.4, True)
    dmr = Params(scale=0.4, causal=True, block_n=Bc, per_step=True, softmax_dmr=True)
    snvr = Params(scale=0.4, causal=True, block_n=Bc, per_step=True)
    silent_snvr = 0
    for (row, col, kt) in ((47, 3, 0), (47, 40, 2), (20, 17, 1), (5, 5, 0)):
        for bit in range(32):
            f = [(ST_EXP, kt, row, col, bit)]
            O, ev, _ = efta_rows(Q[row:row + 1], np.array([row]), K, V, dmr, f)
            assert ev == [(CHECK_EXP, kt, row, col)], (row, col, kt, bit, ev)
            assert np.abs(O[0] - clean[row]).max() < 1e-12
            _, ev2, _ = efta_rows(Q[row:row + 1], np.array([row]), K, V, snvr, f)
            silent_snvr += ev2 == []
    assert silent_snvr > 20
    for (row, kt) in ((47, 0), (47, 2), (30, 1)):
        for bit in range(32):
            f = [(ST_ROWSUM, kt, row, 0, bit)]
            O, ev, _ = efta_rows(Q[row:row + 1], np.array([row]), K, V, dmr, f)
            assert ev == [(CHECK_L, kt, row, 0)]
            assert np.abs(O[0] - clean[row]).max() < 1e-12


def test_dmr_leaves_the_matrix_products_to_their_checksums():
    N, d, Bc = 64, 32, 16
    Q, K, V = _rand(N, d, 272)
    clean = attention_clean(Q, K, V, 0.3, True)
    dmr = Params(scale=0.3, causal=True, block_n=Bc, per_step=True, softmax_dmr=True)
    O, ev, _ = efta_rows(Q, np.arange(N), K, V, dmr, [(ST_S, 1, 40, 20, 27), (ST_OACC, 0, 63, 9, 28)])
    assert ev == [(CHECK_S, 1, 40, 20), (CHECK_O, 0, 63, 9)]
    assert np.abs(O - clean).max() < 1e-9
    with pytest.raises(AssertionError):
        efta_rows(Q, np.arange(N), K, V, Params(scale=0.3, causal=True, block_n=Bc, softmax_dmr=True))


def test_unified_path_and_the_variant_function_take_the_same_steps():
    """``efta_rows_unified`` is Algorithm 1 written out without any variant; ``efta_rows_with_modes``
    with every variant off must agree with it bit for bit (outputs, events, diagnostics), with and
    without faults, for both strides, masks and ragged lengths."""
    rng = np.random.default_rng(77)
    for (N, d, Bc, causal, stride) in ((96, 16, 32, True, 8), (70, 16, 16, False, 8), (64, 8, 64, True, 1), (50, 24, 16, True, 8)):
        Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
        prm = orc.Params(scale=0.4, causal=causal, block_n=Bc, stride=stride)
        rows = np.arange(N)
        fl = []
        for st in (ST_S, ST_EXP, ST_ROWSUM, ST_OACC):
            for _ in range(6):
                row = int(rng.integers(0, N))
                kt = int(rng.integers(0, (row if causal else N - 1) // Bc + 1))
                hi = min(N - 1, kt * Bc + Bc - 1, row if causal else N - 1)
                col = int(rng.integers(kt * Bc, hi + 1)) if st in (ST_S, ST_EXP) else int(rng.integers(0, d))
                fl.append((st, kt, row, col, int(rng.integers(0, 32))))
        for faults in ([], fl):
            for correct in (True, False):
                prm.correct = correct
                a = orc.efta_rows_unified(Q, rows, K, V, prm, faults)
                b = orc.efta_rows_with_modes(Q, rows, K, V, prm, faults)
                assert a[1] == b[1]
                assert np.array_equal(a[0], b[0], equal_nan=True)
                for key in ("lambda_ratio", "o_ratio", "l_distance", "flipped"):
                    assert a[2][key] == b[2][key] or (a[2][key] != a[2][key] and b[2][key] != b[2][key]), key


# ---------------------------------------------------------------- lazily renewed reference maximum (rescale_margin)

def test_rescale_margin_leaves_the_result_alone_and_saves_rescales():
    """The subtracted value cancels between numerator and denominator (Section 3.4, case 1), so a
    reference maximum that lags behind the running one by at most the margin gives the definition's
    result, silently, with far fewer iterations whose rescale factor differs from one."""
    rng = np.random.default_rng(91)
    for (N, d, Bc, causal) in ((300, 16, 32, True), (257, 8, 64, False), (96, 24, 16, True)):
        Q, K, V = (rng.standard_normal((N, d)) * 1.5 for _ in range(3))
        ref = attention_clean(Q, K, V, 0.5, causal)
        counts = []
        for margin in (1e-9, 0.7, 3.0, 5.5):
            prm = orc.Params(scale=0.5, causal=causal, block_n=Bc, rescale_margin=margin)
            O, ev, dg = efta_rows(Q, np.arange(N), K, V, prm)
            assert ev == [] and np.abs(O - ref).max() < 1e-12
            counts.append(dg["rescales"])
        assert counts[0] > 2 * max(1, counts[2]) and counts[0] > 4 * max(1, counts[3]) and counts == sorted(counts, reverse=True)


def test_rescale_margin_row_sum_range_uses_the_lagging_reference():
    """With a lagging reference the exponentials reach exp(running maximum - reference), and so does
    the row-sum per key: the upper bound carries that factor (a row built to exceed the plain key
    count stays silent), the lower bound is unchanged, and a flipped row-sum is still replaced by the
    lower bound with the closed form O_ft = O_clean * l_true / L."""
    d, Bc = 8, 16
    N = 4 * Bc
    K = np.zeros((N, d)); K[:, 0] = 1.0
    K[Bc:, 0] = 1.9                       # every later key scores 0.9 above the first tile's, within the margin
    Q = np.zeros((1, d)); Q[0, 0] = 1.0
    V = np.random.default_rng(5).standard_normal((N, d))
    prm = orc.Params(scale=1.0, causal=False, block_n=Bc, rescale_margin=1.0)
    O, ev, dg = efta_rows(Q, np.array([0]), K, V, prm)
    ell = Bc + 3 * Bc * np.exp(0.9)        # relative to the reference (the first tile's maximum)
    assert ell > N and ev == [] and dg["rescales"] == 0
    assert np.abs(O - attention_clean(Q, K, V, 1.0, False)).max() < 1e-13
    # the same row under Algorithm 1 proper: the maximum moves once, the row-sum is below the key count
    _, ev0, _ = efta_rows(Q, np.array([0]), K, V, orc.Params(scale=1.0, causal=False, block_n=Bc))
    assert ev0 == []
    # a row-sum flipped far out of range is replaced by the lower bound L = sum of exp(tile maximum - reference)
    O2, ev2, _ = efta_rows(Q, np.array([0]), K, V, prm, [(ST_ROWSUM, 3, 0, 0, 30)])
    assert ev2 == [(CHECK_L, -1, 0, 0)]
    L = 1.0 + 3 * np.exp(0.9)
    assert np.abs(O2 - attention_clean(Q, K, V, 1.0, False) * ell / L).max() < 1e-12


def test_rescale_margin_faults_are_found_where_algorithm_1_finds_them():
    rng = np.random.default_rng(92)
    N, d, Bc = 128, 16, 32
    Q, K, V = (rng.standard_normal((N, d)) for _ in range(3))
    base = orc.Params(scale=0.4, causal=True, block_n=Bc)
    lazy = orc.Params(scale=0.4, causal=True, block_n=Bc, rescale_margin=4.0)
    ref = attention_clean(Q, K, V, 0.4, True)
    faults, rows = [], set()
    while len(faults) < 24:
        st = (ST_S, ST_EXP, ST_OACC)[len(faults) % 3]
        row = int(rng.integers(8, N))
        if row in rows:
            continue
        rows.add(row)
        kt = int(rng.integers(0, row // Bc + 1))
        col = int(rng.integers(kt * Bc, min(row, kt * Bc + Bc - 1) + 1)) if st != ST_OACC else int(rng.integers(0, d))
        faults.append((st, kt, row, col, int(rng.integers(26, 31))))
    O0, ev0, _ = efta_rows(Q, np.arange(N), K, V, base, faults)
    O1, ev1, _ = efta_rows(Q, np.arange(N), K, V, lazy, faults)
    assert ev0 == ev1 and len(ev0) >= 20
    assert np.abs(O1 - ref).max() < 1e-9 and np.abs(O0 - ref).max() < 1e-9
