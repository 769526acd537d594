"""GPU parity of the per-step verification modes (per_step = 1: every step verified where it
happens, the paper's EFTA before the unified verification of Section 3.4; per_step = 2: the same
with the softmax protected by duplication, eq. (11), (12)) against the oracle run in the same mode.  Same bars as the main parity tests: fault-free O within max-abs 2e-3 / relative
Frobenius 1e-3 of the definition and no event; with injected faults the event sets (check, key
tile, row, column) are identical and the repaired rows stay within the same tolerance."""
import numpy as np
import pytest

from paper_2504_02211_amd import synth
import ft_harness as H

pytestmark = pytest.mark.gpu

MAX_ABS, REL_FRO = 2e-3, 1e-3


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("shape,dtype,causal,scale", [((1, 2, 640, 64), synth.F16, True, 1.0),
                                                      ((2, 3, 1000, 128), synth.BF16, True, 1.0),
                                                      ((1, 2, 333, 128), synth.F16, False, 1.0),
                                                      ((2, 2, 512, 64), synth.BF16, False, 0.125)])
def test_per_step_parity(shape, dtype, causal, scale, mode):
    B, Hh, N, d = shape
    print(f"[per step] mode {mode} shape {shape} dtype {dtype} causal {causal}", flush=True)
    q, k, v = synth.gen_qkv(shape, dtype, 0x57E9 + N, value_scale=scale)
    out, rep, c = H.run_gpu(q, k, v, dtype, causal, per_step=mode)
    assert c.per_step == mode
    prm = H.oracle_params(N, d, causal, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o,
                          delta_l=c.delta_l, per_step=True, softmax_dmr=mode == 2)
    assert rep.n_events == 0, rep.events[:8]
    rows = np.unique(np.concatenate([np.arange(0, N, 7), [N - 1]]))
    got, ref = [], []
    for b in range(B):
        for h in range(Hh):
            clean, _, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, rows, np.zeros((0, 7), np.int32))
            assert ev == set()
            got.append(out[b, h][rows]); ref.append(clean)
    ma, rf = H.tolerance_ok(np.concatenate(got), np.concatenate(ref))
    assert ma <= MAX_ABS and rf <= REL_FRO

    # ---- seeded flips of all four stages, six per head, bits 10..30
    slots = [(b, h, s, (stage,)) for b in range(B) for h in range(Hh)
             for s, stage in enumerate((synth.ST_OACC, synth.ST_OACC, synth.ST_ROWSUM, synth.ST_S, synth.ST_EXP, synth.ST_S))]
    # (duplication compares exactly: with it every bit of an exponential or of the row-sum is in range)
    faults, redraws = H.select_faults(slots, 0x57EA + N, q, k, v, dtype, prm, 10 if mode == 1 else 0, 30 if mode == 1 else 31)
    H.assert_skip_share(redraws, len(faults))
    out2, rep2, _ = H.run_gpu(q, k, v, dtype, causal, faults, per_step=mode)
    expected = set()
    got, ref = [], []
    for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
        frows = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
        _, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, frows, faults)
        expected |= ev
        got.append(out2[b, h][frows]); ref.append(oft)
    assert rep2.event_set() == expected, (sorted(rep2.event_set() - expected)[:5], sorted(expected - rep2.event_set())[:5])
    in_loop = sum(1 for e in expected if e[2] in (2, 3) and e[3] >= 0)
    print(f"[per step] {len(expected)} events identical ({in_loop} row-sum / output events inside the loop), "
          f"{redraws} candidates skipped", flush=True)
    assert in_loop > 0 or (scale < 1.0 and mode == 1)      # (small values: few flips reach the output threshold)
    g, r_ = np.concatenate(got), np.concatenate(ref)
    fin = np.isfinite(r_)
    assert np.array_equal(np.isfinite(g), fin)
    ma, rf = H.tolerance_ok(g, r_)
    assert ma <= MAX_ABS and rf <= REL_FRO
    # rows without a fault are untouched by the extra checks
    clean_rows = np.setdiff1d(rows, faults[:, 4])
    ma, _ = H.tolerance_ok(out2[0, 0][clean_rows], H.oracle_rows(q, k, v, dtype, prm, 0, 0, clean_rows, np.zeros((0, 7), np.int32))[0])
    assert ma <= MAX_ABS


def test_per_step_needs_the_correcting_mode():
    from paper_2504_02211_amd import ftattn
    for kw in (dict(ft_mode=ftattn.FT_DETECT), dict(ft_mode=ftattn.FT_OFF), dict(rowsum_fold=True)):
        with pytest.raises(ftattn.FtAttnError) as ei:
            ftattn.FtAttn(1, 1, 128, 64, synth.F16, True, per_step=1, **kw)
        assert ei.value.code == ftattn.EINVAL
