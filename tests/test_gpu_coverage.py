"""GPU: the coverage sweep (detection and false-alarm rates against thresholds) behaves like the
method says it must, and the library's decisions at non-default thresholds match the oracle's."""
import numpy as np
import pytest

from oracle import efta_oracle as orc
from paper_2504_02211_amd import coverage, ftattn, synth
import ft_harness as H

pytestmark = pytest.mark.gpu


def test_sweep_shape_and_oracle_agreement():
    shape = (1, 2, 640, 64)
    dtype, causal = synth.F16, True
    q, k, v = synth.gen_qkv(shape, dtype, 0xC0FE)
    faults = coverage.draw_faults(*shape, causal, 64, 24, 0xC0FF)
    assert len(faults) == 48 and len({(f[0], f[1], f[4]) for f in map(tuple, faults)}) == 48
    grids = {"product": (1e-3, 3e-2, 1.0), "sum": (1e-5, 0.75 * 2.0 ** -9, 2e-2), "range": (1e-6, 2.0 ** -10, 1e-1)}
    res = coverage.sweep(q, k, v, dtype, causal, faults, grids)
    print(coverage.to_markdown(res), flush=True)
    for fam in coverage.FAMILIES:
        curve = res["curves"][fam]
        det = [c["harmful_detected"] + c["benign_detected"] for c in curve]
        fa = [c["false_alarms"] for c in curve]
        # a looser threshold never detects more and never raises more false alarms
        assert det == sorted(det, reverse=True), (fam, det)
        assert fa == sorted(fa, reverse=True), (fam, fa)
        # the library's default thresholds are silent on clean data
        assert curve[1]["false_alarms"] == 0, (fam, curve[1])
    # at the default thresholds every harmful flip of S, exp and the output accumulator is detected,
    # and the checksum-based corrections bring the output back to within the tolerance
    for fam in ("product", "sum"):
        c, a = res["curves"][fam][1], res["after_correction"][fam]
        assert c["harmful"] > 0 and c["harmful_detected"] == c["harmful"], (fam, c)
        assert a["within_tol"] == a["harmful"], (fam, a)

    # ---- per-fault decisions at a non-default threshold against the oracle (faults whose statistic
    # lies within 4x of the threshold are left out: the decision would hinge on rounding)
    r = coverage.Runner(q, k, v, dtype, causal)
    for fam, kw in (("product", {"eps1": 0.3}), ("sum", {"tau_o": 2e-2}), ("range", {"delta_l": 1e-1})):
        _, rep, cfg = r.run(faults, ftattn.FT_DETECT, **kw)
        prm = H.oracle_params(shape[2], shape[3], causal, block_n=cfg.block_n, scale=cfg.softmax_scale,
                              eps1=cfg.eps1, tau_o=cfg.tau_o, delta_l=cfg.delta_l, correct=False)
        got = rep.event_set()
        compared = 0
        for f in faults:
            b, h, row = int(f[0]), int(f[1]), int(f[4])
            Q, K, V = H.head_f64(q, dtype, b, h), H.head_f64(k, dtype, b, h), H.head_f64(v, dtype, b, h)
            _, ev, dg = orc.efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [tuple(int(x) for x in f[2:])])
            if not orc.fault_is_robust(dg) or len(dg["flipped"]) != 1 or orc.fp32_is_fragile(dg["flipped"][0][1], int(f[2])):
                continue
            compared += 1
            mine = {e for e in got if e[0] == b and e[1] == h and e[4] == row}
            assert mine == {(b, h) + e for e in ev}, (fam, tuple(f), sorted(mine), ev)
        assert compared >= 24, compared


@pytest.mark.parametrize("stride", [8, 1])
def test_bit_error_rate_sweep(stride):
    """(stride 1: the traditional single-class checksum.)  Unconstrained flips at two rates: no event on a row that no flip hit; at the low rate (flips on
    separate rows) every row that is still wrong after correction carries a row-sum flip (the range
    restriction is the weak check), and the events of every hit row equal the oracle's."""
    shape = (1, 2, 640, 64)
    dtype, causal = synth.F16, True
    q, k, v = synth.gen_qkv(shape, dtype, 0xC0FE)
    rows = coverage.ber_sweep(q, k, v, dtype, causal, (2e-5, 1e-3), 0xBE7, stride=stride)
    print(coverage.ber_markdown(rows), flush=True)
    lo, hi = rows
    assert lo["faults"] >= 8 and hi["faults"] > 20 * lo["faults"]
    for r in rows:
        assert r["flagged_not_hit"] == 0 and r["events_dropped"] == 0
        assert r["harmed_flagged"] >= 0.6 * r["rows_harmed"] > 0
    st = lo["rows_bad_after_by_stage"]
    assert lo["rows_bad_after"] == st["ROWSUM"]

    faults = coverage.draw_ber_faults(*shape, causal, 64, 2e-5, 0xBE7)
    r = coverage.Runner(q, k, v, dtype, causal, stride=stride)
    _, rep, cfg = r.run(faults, ftattn.FT_CORRECT)
    assert cfg.stride == stride
    prm = H.oracle_params(shape[2], shape[3], causal, block_n=cfg.block_n, scale=cfg.softmax_scale,
                          eps1=cfg.eps1, tau_o=cfg.tau_o, delta_l=cfg.delta_l, stride=stride)
    got = rep.event_set()
    compared = 0
    for (b, h, row) in sorted({(int(f[0]), int(f[1]), int(f[4])) for f in faults}):
        fl = [tuple(int(x) for x in f[2:]) for f in faults if (int(f[0]), int(f[1]), int(f[4])) == (b, h, row)]
        Q, K, V = H.head_f64(q, dtype, b, h), H.head_f64(k, dtype, b, h), H.head_f64(v, dtype, b, h)
        _, ev, dg = orc.efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, fl)
        if not orc.fault_is_robust(dg) or any(orc.fp32_is_fragile(x, st_) for st_, x in dg["flipped"]):
            continue
        compared += 1
        mine = {e for e in got if e[0] == b and e[1] == h and e[4] == row}
        assert mine == {(b, h) + e for e in ev}, (fl, sorted(mine), ev)
    assert compared >= 5, compared


def test_linear_layer_threshold_sweep():
    """Shape of the coverage curve of the linear layer's check: at the default threshold every
    harmful flip is flagged and repaired and a fault-free run raises nothing; detection can only
    fall as the threshold grows; a threshold below the rounding noise of the two-word checksums
    fires on clean data."""
    res = coverage.linear_sweep(512, 768, 256, synth.BF16, 96, 0xC0FE, grid=(2.0 ** -24, 2.0 ** -15, 2.0 ** -11, 2.0 ** -7))
    c = {r["tau_rel"]: r for r in res["curve"]}
    d = c[2.0 ** -15]
    assert d["harmful"] > 20 and d["harmful_detected"] == d["harmful"] == d["harmful_repaired"] and d["false_alarms"] == 0
    det = [r["harmful_detected"] for r in res["curve"]]
    assert all(a >= b for a, b in zip(det, det[1:])) and det[-1] < det[0]
    assert c[2.0 ** -24]["false_alarms"] > 0
    print(coverage.linear_markdown(res))
    tok = coverage.linear_sweep(512, 768, 256, synth.F16, 96, 0xC0FE, fold_tokens=True, grid=(2.0 ** -15,))["curve"][0]
    assert tok["harmful_detected"] == tok["harmful"] == tok["harmful_repaired"] and tok["false_alarms"] == 0
