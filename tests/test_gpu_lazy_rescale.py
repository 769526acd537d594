"""GPU parity of the lazily renewed reference maximum (rescale_margin > 0, an extension) against the
oracle run with the same margin.  Same bars as the main parity tests: fault-free O within max-abs
2e-3 / relative Frobenius 1e-3 of the definition and no event, also with the checks compiled out;
with injected faults the event sets are identical and the repaired rows stay within tolerance."""
import numpy as np
import pytest

from paper_2504_02211_amd import ftattn, synth
import ft_harness as H

pytestmark = pytest.mark.gpu

MAX_ABS, REL_FRO = 2e-3, 1e-3


@pytest.mark.parametrize("margin", [0.5, 5.5])
@pytest.mark.parametrize("shape,dtype,causal,scale", [((1, 2, 640, 64), synth.F16, True, 1.0),
                                                      ((2, 2, 1000, 128), synth.BF16, True, 2.0),
                                                      ((1, 2, 333, 128), synth.F16, False, 1.0)])
def test_lazy_rescale_parity(shape, dtype, causal, scale, margin):
    B, Hh, N, d = shape
    print(f"[lazy rescale] margin {margin} shape {shape} dtype {dtype} causal {causal}", flush=True)
    q, k, v = synth.gen_qkv(shape, dtype, 0x1A27 + N, value_scale=scale)
    out, rep, c = H.run_gpu(q, k, v, dtype, causal, rescale_margin=margin)
    assert abs(c.rescale_margin - margin) < 1e-6
    prm = H.oracle_params(N, d, causal, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o,
                          delta_l=c.delta_l, rescale_margin=float(c.rescale_margin))
    assert rep.n_events == 0, rep.events[:8]
    out0, rep0, _ = H.run_gpu(q, k, v, dtype, causal, ft_mode=ftattn.FT_OFF, rescale_margin=margin)
    rows = np.unique(np.concatenate([np.arange(0, N, 7), [N - 1]]))
    got, got0, ref = [], [], []
    for b in range(B):
        for h in range(Hh):
            clean, _, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, rows, np.zeros((0, 7), np.int32))
            assert ev == set()
            got.append(out[b, h][rows]); got0.append(out0[b, h][rows]); ref.append(clean)
    for g in (got, got0):
        ma, rf = H.tolerance_ok(np.concatenate(g), np.concatenate(ref))
        assert ma <= MAX_ABS and rf <= REL_FRO

    # ---- seeded flips of all four stages, five per head
    slots = [(b, h, s, (stage,)) for b in range(B) for h in range(Hh)
             for s, stage in enumerate((synth.ST_OACC, synth.ST_ROWSUM, synth.ST_S, synth.ST_EXP, synth.ST_S))]
    faults, redraws = H.select_faults(slots, 0x1A28 + N, q, k, v, dtype, prm, 16, 30)
    H.assert_skip_share(redraws, len(faults))
    out2, rep2, _ = H.run_gpu(q, k, v, dtype, causal, faults, rescale_margin=margin)
    expected, got, ref = set(), [], []
    for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
        fr = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
        _, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, fr, faults)
        expected |= ev
        got.append(out2[b, h][fr]); ref.append(oft)
    assert rep2.event_set() == expected, (sorted(rep2.event_set() - expected)[:5], sorted(expected - rep2.event_set())[:5])
    assert len(expected) >= len(faults) // 2
    ma, rf = H.tolerance_ok(np.concatenate(got), np.concatenate(ref))
    print(f"[lazy rescale] {len(expected)} events identical; faulted rows max-abs {ma:.3e} rel-Frobenius {rf:.3e}", flush=True)
    assert ma <= MAX_ABS and rf <= REL_FRO
