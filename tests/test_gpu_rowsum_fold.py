"""GPU parity of the exact row-sum check (rowsum_fold = 1: the row-sum rides through GEMM II as an
extra fold of checksum class 0 of the value tiles) against the oracle run in the same mode.
Same bars as the main parity tests: fault-free O within max-abs 2e-3 / relative Frobenius 1e-3 of
the definition, event sets identical, repaired rows within the same tolerance."""
import numpy as np
import pytest

from paper_2504_02211_amd import synth
import ft_harness as H

pytestmark = pytest.mark.gpu

MAX_ABS, REL_FRO = 2e-3, 1e-3


@pytest.mark.parametrize("shape,dtype,causal,scale", [((1, 2, 640, 64), synth.F16, True, 1.0),
                                                      ((2, 3, 1000, 128), synth.BF16, True, 1.0),
                                                      ((1, 2, 333, 128), synth.F16, False, 1.0),
                                                      ((2, 2, 512, 64), synth.BF16, False, 0.125)])
def test_rowsum_fold_parity(shape, dtype, causal, scale):
    B, Hh, N, d = shape
    print(f"[rowsum fold] shape {shape} dtype {dtype} causal {causal}", flush=True)
    q, k, v = synth.gen_qkv(shape, dtype, 0xF01D + N, value_scale=scale)
    out, rep, c = H.run_gpu(q, k, v, dtype, causal, rowsum_fold=True)
    assert c.rowsum_fold == 1
    prm = H.oracle_params(N, d, causal, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o,
                          delta_l=c.delta_l, rowsum_fold=True)
    assert rep.n_events == 0, rep.events[:8]
    # the largest fault-free row-sum residual sits far below the threshold
    assert 0.0 <= rep.residual_max[..., 2].max() < 0.1 * c.tau_o
    rows = np.unique(np.concatenate([np.arange(0, N, 7), [N - 1]]))
    got, ref = [], []
    for b in range(B):
        for h in range(Hh):
            clean, _, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, rows, np.zeros((0, 7), np.int32))
            assert ev == set()
            got.append(out[b, h][rows]); ref.append(clean)
    ma, rf = H.tolerance_ok(np.concatenate(got), np.concatenate(ref))
    assert ma <= MAX_ABS and rf <= REL_FRO

    # ---- seeded flips of all four stages, four per head, bits 10..30
    slots = [(b, h, s, (stage,)) for b in range(B) for h in range(Hh)
             for s, stage in enumerate((synth.ST_ROWSUM, synth.ST_ROWSUM, synth.ST_OACC, synth.ST_S, synth.ST_EXP, synth.ST_ROWSUM))]
    faults, redraws = H.select_faults(slots, 0xF01E + N, q, k, v, dtype, prm, 10, 30)
    H.assert_skip_share(redraws, len(faults))
    all_faults = faults
    for mode, correct in ((1, True), (2, False)):
        prm.correct = correct
        faults = all_faults
        if not correct:
            # left in place, a fault can turn every later statistic of its row into garbage (a
            # non-finite row-sum, say); keep the row-sum flips whose only consequence is their own event
            keep = []
            for f in all_faults:
                if f[2] != synth.ST_ROWSUM:
                    continue
                _, _, ev1 = H.oracle_rows(q, k, v, dtype, prm, int(f[0]), int(f[1]), np.array([int(f[4])]), f[None, :])
                if {e[2] for e in ev1} == {2}:
                    keep.append(f)
            faults = np.array(keep, np.int32)
            assert len(faults) >= 3
        out2, rep2, _ = H.run_gpu(q, k, v, dtype, causal, faults, ft_mode=mode, rowsum_fold=True)
        expected = set()
        got, ref, cleanref = [], [], []
        for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
            frows = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
            clean, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, frows, faults)
            expected |= ev
            got.append(out2[b, h][frows]); ref.append(oft); cleanref.append(clean)
        assert rep2.event_set() == expected, (sorted(rep2.event_set() - expected)[:5], sorted(expected - rep2.event_set())[:5])
        n_l = sum(1 for e in expected if e[2] == 2)
        print(f"[rowsum fold] mode {mode}: {len(expected)} events identical ({n_l} row-sum), {redraws} candidates skipped", flush=True)
        assert n_l > 0
        g, r_ = np.concatenate(got), np.concatenate(ref)
        fin = np.isfinite(r_)
        assert np.array_equal(np.isfinite(g), fin)
        if correct:
            ma, rf = H.tolerance_ok(g, r_)
            assert ma <= MAX_ABS and rf <= REL_FRO
            # with the extra fold a detected row-sum flip is repaired exactly, not approximated
            ma, _ = H.tolerance_ok(g, np.concatenate(cleanref))
            assert ma <= 2 * MAX_ABS
