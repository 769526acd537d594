"""Pins of the decoupled-scheme oracle (Section 3.1: ABFT-GEMM I, DMR row-softmax of eq. (11), (12),
ABFT-GEMM II) against the definition, closed forms and its stated control flow.  CPU only."""
import numpy as np
import pytest

from oracle import decoupled_oracle as dorc
from oracle import efta_oracle as eorc
from oracle.decoupled_oracle import ST_EXP, ST_GEMM1, ST_GEMM2, ST_PNORM


def _qkv(seed, n=48, d=16):
    rng = np.random.default_rng(seed)
    return [rng.standard_normal((n, d)) for _ in range(3)]


@pytest.mark.parametrize("causal", [False, True])
def test_fault_free_result_is_the_definition(causal):
    Q, K, V = _qkv(1)
    O, ev, _ = dorc.decoupled_attention(Q, K, V, dorc.Params(scale=0.3, causal=causal))
    assert ev == []
    assert np.abs(O - eorc.attention_clean(Q, K, V, 0.3, causal)).max() < 1e-13
    # the rational closed-form cases of the attention oracle hold for this path too: logits that are
    # logs of small integers give weights k / sum(k)
    Qh = np.array([[1.0, 0.0]]); Kh = np.array([[0.0, 0.0], [np.log(2.0), 0.0], [np.log(5.0), 0.0]])
    Vh = np.array([[8.0, 0.0], [8.0, 16.0], [12.8, 12.8]])
    Oh, _, _ = dorc.decoupled_attention(Qh, Kh, Vh, dorc.Params(scale=1.0, causal=False))
    assert np.allclose(Oh, [[(1 * 8 + 2 * 8 + 5 * 12.8) / 8, (2 * 16 + 5 * 12.8) / 8]], atol=1e-13)


def test_dmr_row_control_flow():
    """eq. (11): a difference of the two evaluations at or above eps is flagged, the row is evaluated
    again and comes out clean; below eps the mean of the two evaluations is kept (closed form).
    eq. (12): a normalised weight moved by eps or more is flagged through the row sum."""
    rng = np.random.default_rng(2)
    s = rng.standard_normal(32) * 2
    x = 0.5 * s
    e = np.exp(x - x.max()); clean = e / e.sum()
    eps = 2.0 ** -12
    P, ev, attempts, st = dorc.dmr_softmax_row(s, 0.5, eps)
    assert ev == [] and attempts == 1 and np.allclose(P, clean, atol=1e-15) and abs(P.sum() - 1) < 1e-14
    # exponent-bit flip of one exponential: far above eps
    P, ev, attempts, st = dorc.dmr_softmax_row(s, 0.5, eps, exp_faults=[(7, 27)])
    assert ev == [(ST_EXP, 7)] and attempts == 2 and np.allclose(P, clean, atol=1e-15)
    # low mantissa bit: below eps, silent; DMR(e) = (e_a + e_b) / 2 enters the row
    col, bit = 7, 3
    ea = dorc.gorc.bitflip32(e[col], bit); delta = ea - e[col]
    assert 0 < abs(delta) < eps / 4
    P, ev, attempts, st = dorc.dmr_softmax_row(s, 0.5, eps, exp_faults=[(col, bit)])
    em = e.copy(); em[col] += delta / 2
    assert ev == [] and attempts == 1 and np.allclose(P, em / em.sum(), atol=1e-15)
    assert st["exp_delta"] == [pytest.approx(abs(delta))]
    # the two evaluations must agree element by element: the largest element (value 1) flipped in its sign bit
    top = int(np.argmax(s))
    P, ev, attempts, _ = dorc.dmr_softmax_row(s, 0.5, eps, exp_faults=[(top, 31)])
    assert ev == [(ST_EXP, top)] and attempts == 2
    # eq. (12): a weight of about 0.1 with a flipped high mantissa bit moves the row sum by more than eps
    big = int(np.argmax(clean))
    P, ev, attempts, st = dorc.dmr_softmax_row(s, 0.5, eps, p_faults=[(big, 22)])
    assert ev == [(ST_PNORM, -1)] and attempts == 2 and np.allclose(P, clean, atol=1e-15) and st["p_delta"][0] > eps
    # ... and a low bit does not, and stays in the stored row
    P, ev, attempts, st = dorc.dmr_softmax_row(s, 0.5, eps, p_faults=[(big, 2)])
    assert ev == [] and P[big] != clean[big] and abs(P[big] - clean[big]) < eps


def test_faults_of_every_stage_are_reported_and_repaired():
    Q, K, V = _qkv(3, n=64, d=16)
    prm = dorc.Params(scale=0.25, causal=True)
    ref = eorc.attention_clean(Q, K, V, 0.25, True)
    faults = [(ST_GEMM1, 5, 3, 27), (ST_EXP, 17, 2, 25), (ST_PNORM, 29, 4, 29), (ST_GEMM2, 41, 5, 26)]
    O, ev, dg = dorc.decoupled_attention(Q, K, V, prm, faults)
    assert ev == [(ST_GEMM1, 5, 3), (ST_EXP, 17, 2), (ST_PNORM, 29, -1), (ST_GEMM2, 41, 5)]
    assert np.abs(O - ref).max() < 1e-12 and dorc.fault_is_robust(dg, prm)
    # a score error above the diagonal of a causal row is repaired too (S is computed in full)
    O, ev, _ = dorc.decoupled_attention(Q, K, V, prm, [(ST_GEMM1, 5, 40, 28)])
    assert ev == [(ST_GEMM1, 5, 40)] and np.abs(O - ref).max() < 1e-12
    # masked keys take no part: their scores may hold anything
    O2, ev2, _ = dorc.decoupled_attention(Q, K * np.where(np.arange(64)[:, None] > 50, 1e3, 1.0), V, prm)
    assert np.abs(O2[:51] - ref[:51]).max() < 1e-12 and ev2 == []


def test_row_subsets_equal_the_whole_head():
    """Every check is local to a query row: rows taken alone give the same outputs and events."""
    Q, K, V = _qkv(4, n=40, d=8)
    prm = dorc.Params(scale=0.35, causal=True)
    faults = [(ST_GEMM1, 9, 30, 26), (ST_EXP, 20, 11, 28), (ST_GEMM2, 33, 2, 27)]
    O, ev, _ = dorc.decoupled_attention(Q, K, V, prm, faults)
    rows = np.array([9, 20, 21, 33])
    Os, evs, _ = dorc.decoupled_attention(Q[rows], K, V, prm, faults, row_idx=rows)
    assert evs == ev and np.abs(Os - O[rows]).max() < 1e-13


def test_guard_band_predicate():
    prm = dorc.Params(scale=1.0, causal=False)
    base = {"gemm1": {"ratio_near": np.inf}, "gemm2": {"ratio_near": np.inf}, "exp_delta": [], "p_delta": []}
    assert dorc.fault_is_robust(base, prm)
    assert not dorc.fault_is_robust(dict(base, exp_delta=[prm.eps_dmr * 2]), prm)
    assert dorc.fault_is_robust(dict(base, exp_delta=[prm.eps_dmr * 8]), prm)
    assert not dorc.fault_is_robust(dict(base, p_delta=[prm.eps_dmr / 3]), prm)
    assert not dorc.fault_is_robust(dict(base, gemm1={"ratio_near": 2.0}), prm)
