"""GPU parity of the traditional-checksum mode (stride = 1: one class over the whole tile row and
one over all features, the scheme the paper compares its strided tensor checksum with in
Sections 3.3 and 4.2) against the oracle run with the same stride.  Same bars as the main parity
tests: fault-free O within max-abs 2e-3 / relative Frobenius 1e-3 of the definition and no event;
with injected faults the event sets (check, key tile, row, column) are identical and the repaired
rows stay within the same tolerance.  A last test shows the difference in coverage on the GPU:
two errors in one (row, key tile) in different stride-8 classes."""
import numpy as np
import pytest

from paper_2504_02211_amd import ftattn, synth
import ft_harness as H

pytestmark = pytest.mark.gpu

MAX_ABS, REL_FRO = 2e-3, 1e-3


@pytest.mark.parametrize("shape,dtype,causal,scale", [((1, 2, 640, 64), synth.F16, True, 1.0),
                                                      ((2, 3, 1000, 128), synth.BF16, True, 1.0),
                                                      ((1, 2, 333, 128), synth.F16, False, 1.0),
                                                      ((2, 2, 512, 64), synth.BF16, False, 0.125)])
def test_element_wide_parity(shape, dtype, causal, scale):
    B, Hh, N, d = shape
    print(f"[element-wide] shape {shape} dtype {dtype} causal {causal}", flush=True)
    q, k, v = synth.gen_qkv(shape, dtype, 0xE1E0 + N, value_scale=scale)
    out, rep, c = H.run_gpu(q, k, v, dtype, causal, stride=1)
    assert c.stride == 1
    prm = H.oracle_params(N, d, causal, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o,
                          delta_l=c.delta_l, stride=1)
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

    # ---- seeded flips of all four stages, six per head, bits 20..30
    slots = [(b, h, s, (stage,)) for b in range(B) for h in range(Hh)
             for s, stage in enumerate((synth.ST_OACC, synth.ST_OACC, synth.ST_ROWSUM, synth.ST_S, synth.ST_EXP, synth.ST_S))]
    faults, redraws = H.select_faults(slots, 0xE1E1 + N, q, k, v, dtype, prm, 20, 30)
    H.assert_skip_share(redraws, len(faults))
    out2, rep2, _ = H.run_gpu(q, k, v, dtype, causal, faults, stride=1)
    expected = set()
    got, ref = [], []
    for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
        frows = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
        _, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, frows, faults)
        expected |= ev
        got.append(out2[b, h][frows]); ref.append(oft)
    assert rep2.event_set() == expected, (sorted(rep2.event_set() - expected)[:5], sorted(expected - rep2.event_set())[:5])
    print(f"[element-wide] {len(expected)} events identical, {redraws} candidates skipped", flush=True)
    assert len(expected) >= len(faults) // 3     # (the lower of these bits stay below the thresholds)
    g, r_ = np.concatenate(got), np.concatenate(ref)
    fin = np.isfinite(r_)
    assert np.array_equal(np.isfinite(g), fin)
    assert np.abs(g[fin] - r_[fin]).max() <= MAX_ABS


def test_two_errors_in_one_tile_row():
    """Two score errors in one (row, key tile), in different stride-8 classes: the strided fold
    repairs both, the single class reports the row and leaves it wrong."""
    B, Hh, N, d = 1, 2, 512, 128
    dtype = synth.BF16
    q, k, v = synth.gen_qkv((B, Hh, N, d), dtype, 0xE1E7)
    clean, _, _ = H.run_gpu(q, k, v, dtype, False)          # the protected kernel without faults
    # (b, h, stage, key tile, row, column, bit): exponent bit 30 of two scores of one tile row
    rows = [37, 200, 411]
    faults = []
    for h in range(Hh):
        for r in rows:
            tile = (r * 7 + h) % (N // 64)
            faults.append((0, h, synth.ST_S, tile, r, 64 * tile + 3, 30))         # class 3
            faults.append((0, h, synth.ST_S, tile, r, 64 * tile + 8 * 5 + 6, 30))  # class 6
    fa = np.array(faults, np.int32)
    out8, rep8, _ = H.run_gpu(q, k, v, dtype, False, fa, stride=8)
    out1, rep1, _ = H.run_gpu(q, k, v, dtype, False, fa, stride=1)
    assert {(e[1], e[3], e[4], e[5]) for e in rep8.event_set()} == {(int(f[1]), int(f[3]), int(f[4]), int(f[5])) for f in fa}
    assert np.abs(out8 - clean).max() <= 2e-5                  # both scores rebuilt from their checksums
    hit1 = {(e[1], e[4]) for e in rep1.event_set()}
    assert hit1 == {(h, r) for h in range(Hh) for r in rows}
    for h in range(Hh):
        for r in rows:
            d1 = out1[0, h, r] - clean[0, h, r]
            assert not (np.isfinite(d1).all() and np.abs(d1).max() <= 1e-4), (h, r, np.abs(d1).max())
    mask = np.ones(N, bool); mask[rows] = False
    assert np.abs(out1[:, :, mask] - clean[:, :, mask]).max() <= 2e-5
