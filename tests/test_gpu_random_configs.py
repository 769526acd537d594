"""Randomised parity sweep: seeded random shapes, dtypes, masks, value scales and verification modes
of the attention path (and random shapes of the linear layer), each run through the C ABI and
compared with the oracle as in the fixed-shape parity tests: fault-free output within max-abs 2e-3 /
relative Frobenius 1e-3 on sampled rows and no event; then a few seeded robust faults whose event
sets must be identical and whose rows must come out as the oracle's."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import ftgemm_oracle as gorc
from paper_2504_02211_amd import ftgemm, synth
import ft_harness as H

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("seed", [101, 202, 303, 404, 505, 606])
def test_random_attention_configurations(seed):
    rng = np.random.default_rng(seed)
    skipped = accepted = unselectable = 0
    for it in range(30):
        B, Hh, N = int(rng.integers(1, 3)), int(rng.integers(1, 4)), int(rng.integers(1, 900))
        d, dtype, causal = int(rng.choice([64, 128])), int(rng.integers(0, 2)), bool(rng.integers(0, 2))
        mode = int(rng.integers(0, 3))                       # 0 unified, 1 after every step, 2 + duplicated softmax
        fold = bool(rng.integers(0, 2)) and mode == 0
        stride = 1 if mode == 0 and not fold and bool(rng.integers(0, 2)) else 8      # 1: the traditional checksum
        scale = float(rng.choice([1.0, 0.25, 2.0]))
        # (drawn from a generator of its own so that the configurations of earlier versions of this test stay as they were)
        margin = float(np.random.default_rng(31 * seed + it).choice([0.0, 0.0, 0.7, 4.0])) if mode == 0 and not fold and stride == 8 else 0.0
        tag = f"B{B} H{Hh} N{N} d{d} dtype{dtype} causal{causal} rowsum_fold{fold} per_step{mode} stride{stride} scale{scale} margin{margin}"
        print(f"[random attention] {tag}", flush=True)
        q, k, v = synth.gen_qkv((B, Hh, N, d), dtype, 1000 * seed + it, value_scale=scale)
        out, rep, c = H.run_gpu(q, k, v, dtype, causal, rowsum_fold=fold, per_step=mode, stride=stride, rescale_margin=margin)
        prm = H.oracle_params(N, d, causal, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o,
                              delta_l=c.delta_l, rowsum_fold=fold, per_step=mode > 0, softmax_dmr=mode == 2, stride=stride,
                              rescale_margin=float(c.rescale_margin))
        assert rep.n_events == 0, (tag, rep.events[:4])
        rows = np.unique(rng.integers(0, N, size=min(N, 24)))
        for b in range(B):
            for h in range(Hh):
                clean, _, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, rows, np.zeros((0, 7), np.int32))
                ma, rf = H.tolerance_ok(out[b, h][rows], clean)
                assert ev == set() and ma <= 2e-3 and rf <= 1e-3, (tag, b, h, ma, rf)
        if N < 8:
            continue
        slots = [(b, h, s, (int(rng.integers(0, 4)),)) for b in range(B) for h in range(Hh) for s in range(min(3, max(1, N // 4)))]
        try:
            faults, redraws = H.select_faults(slots, 5000 * seed + it, q, k, v, dtype, prm, int(rng.integers(0, 22)), 31)
        except RuntimeError as e:
            unselectable += 1                                # no candidate of a slot is clear of every threshold
            print(f"[random attention] {tag}: {e}", flush=True)
            continue
        skipped += redraws
        accepted += len(faults)
        out2, rep2, _ = H.run_gpu(q, k, v, dtype, causal, faults, rowsum_fold=fold, per_step=mode, stride=stride, rescale_margin=margin)
        expected, got, ref = set(), [], []
        for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
            fr = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
            _, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, fr, faults)
            expected |= ev
            got.append(out2[b, h][fr]); ref.append(oft)
        assert rep2.event_set() == expected, (tag, sorted(rep2.event_set() - expected)[:4], sorted(expected - rep2.event_set())[:4])
        g, r = np.concatenate(got), np.concatenate(ref)
        fin = np.isfinite(r)
        assert np.array_equal(np.isfinite(g), fin), tag
        assert not fin.any() or np.abs(g[fin] - r[fin]).max() <= 2e-3, tag
    # the selector may pass over ill-posed candidates, not over most of the stream, and a
    # configuration without any selectable fault must stay an exception
    print(f"[random attention] seed {seed}: {accepted} faults, {skipped} candidates skipped, {unselectable} configurations without faults", flush=True)
    assert unselectable <= 2
    H.assert_skip_share(skipped, accepted, 0.5)


def test_random_linear_configurations():
    rng = np.random.default_rng(303)
    TT = {0: torch.float16, 1: torch.bfloat16, 2: torch.float32}
    for it in range(12):
        m, n, k = int(rng.integers(1, 700)), int(rng.integers(1, 900)), 8 * int(rng.integers(1, 65))
        dt = int(rng.integers(0, 2))
        od = int(rng.choice([2, dt]))
        print(f"[random linear] m{m} n{n} k{k} dtype{dt} out{od}", flush=True)
        xb, wb = synth.gen_linear(m, n, k, 7000 + it, dtype=dt)
        X, W = synth.bits_to_f64(xb, dt), synth.bits_to_f64(wb, dt)
        prm = gorc.Params()
        faults, used = [], set()
        for s in range(6):
            stream = synth.linear_fault_stream(8000 + it, s, m, n, 0, 31)
            for _ in range(60):
                r, c, b = next(stream)
                if r in used:
                    continue
                _, _, dg = gorc.ftgemm(X[r:r + 1], W, prm, [(0, c, b)])
                if gorc.fault_is_robust(dg) and not gorc.fp32_is_fragile(dg["flipped"][0]):
                    faults.append((r, c, b)); used.add(r)
                    break
        fa = np.array(faults, np.int32).reshape(-1, 3)
        ctx = ftgemm.FtGemm(m, n, k, out_dtype=od, in_dtype=dt)
        x = torch.from_numpy(xb.view(np.int16)).cuda().view(TT[dt])
        w = torch.from_numpy(wb.view(np.int16)).cuda().view(TT[dt])
        y = torch.full((m, n), float("nan"), dtype=TT[od], device="cuda")
        ctx.encode_weights(w)
        ctx.forward(x, w, y, fa if len(fa) else None)
        rep = ctx.report()
        ctx.close()
        want, ev, _ = gorc.ftgemm(X, W, prm, [tuple(f) for f in faults])
        assert rep.event_list() == ev
        got = y.double().cpu().numpy()
        tol = {2: (1e-4 if dt == 0 else 4e-3), 0: 2.0 ** -10, 1: 2.0 ** -7}[od]
        assert np.all(np.abs(got - want) <= tol * np.maximum(1.0, np.abs(want)))
