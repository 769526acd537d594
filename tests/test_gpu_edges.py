"""GPU edge cases through the C ABI: ragged and tiny sequences, both head sizes and dtypes,
output types, the unprotected and detect-only variants, several faults in one row, error paths."""
import numpy as np
import pytest

from paper_2504_02211_amd import synth
import ft_harness as H

pytestmark = pytest.mark.gpu


def _clean_all(q, k, v, dtype, prm):
    B, Hh, N, d = q.shape
    out = np.empty((B, Hh, N, d))
    for b in range(B):
        for h in range(Hh):
            out[b, h] = H.oracle_rows(q, k, v, dtype, prm, b, h, np.arange(N), np.zeros((0, 7), np.int32))[0]
    return out


@pytest.mark.parametrize("N", [1, 7, 63, 64, 65, 200, 333])
@pytest.mark.parametrize("d,dtype,causal", [(64, synth.F16, True), (128, synth.BF16, False), (128, synth.F16, True),
                                            (64, synth.BF16, False)])
def test_ragged_shapes(N, d, dtype, causal):
    q, k, v = synth.gen_qkv((2, 3, N, d), dtype, 1234 + N + d)
    out, rep, c = H.run_gpu(q, k, v, dtype, causal)
    prm = H.oracle_params(N, d, causal, scale=c.softmax_scale)
    assert rep.n_events == 0
    ma, rf = H.tolerance_ok(out, _clean_all(q, k, v, dtype, prm))
    assert ma <= 2e-3 and rf <= 1e-3, (ma, rf)


@pytest.mark.parametrize("d,block_m", [(128, 0), (128, 256), (64, 0), (64, 128)])
def test_row_tile_sizes_and_output_types(d, block_m):
    N = 640
    q, k, v = synth.gen_qkv((1, 2, N, d), synth.BF16, 77)
    prm = H.oracle_params(N, d, True)
    ref = _clean_all(q, k, v, synth.BF16, prm)
    out, rep, c = H.run_gpu(q, k, v, synth.BF16, True, block_m=block_m)
    assert c.block_m == (256 if d == 128 else 128) and rep.n_events == 0      # the row tile goes with the head size
    ma, rf = H.tolerance_ok(out, ref)
    assert ma <= 2e-3 and rf <= 1e-3
    out16, _, _ = H.run_gpu(q, k, v, synth.BF16, True, block_m=block_m, out_dtype=synth.BF16)
    assert np.abs(out16 - ref).max() <= 2e-3 + np.abs(ref).max() * 2.0 ** -8     # bf16 output rounding
    # the unprotected variant computes the same numbers
    out0, rep0, _ = H.run_gpu(q, k, v, synth.BF16, True, block_m=block_m, ft_mode=0)
    assert np.abs(out0 - out).max() <= 1e-6 and rep0.n_events == 0


def test_modes_with_a_fault():
    """Correct / detect-only / unprotected variants on a fault whose damage is visible."""
    import dataclasses
    from oracle import efta_oracle as orc
    N, d = 256, 64
    q, k, v = synth.gen_qkv((1, 1, N, d), synth.F16, 5)
    prm = H.oracle_params(N, d, False)
    ref = _clean_all(q, k, v, synth.F16, prm)
    Q, K, V = (H.head_f64(x, synth.F16, 0, 0) for x in (q, k, v))
    row = 100
    col = int(np.argmax(K @ Q[row]))                    # the row's largest score
    prm_det = dataclasses.replace(prm, correct=False)
    for bit in range(20, 31):                           # pick a flip that visibly damages the row
        f = (synth.ST_S, col // 64, row, col, bit)
        damaged, ev, dg = orc.efta_rows(Q[row:row + 1], np.array([row]), K, V, prm_det, [f])
        if np.abs(damaged[0] - ref[0, 0, row]).max() > 0.05 and orc.fault_is_robust(dg):
            break
    else:
        raise AssertionError("no damaging flip found")
    fault = np.array([[0, 0, *f]], np.int32)
    want = {(0, 0, 0, col // 64, row, col)}
    out1, rep1, _ = H.run_gpu(q, k, v, synth.F16, False, fault, ft_mode=1)
    assert rep1.event_set() == want and rep1.events["action"][0] == 1
    assert np.abs(out1 - ref).max() <= 2e-3
    out2, rep2, _ = H.run_gpu(q, k, v, synth.F16, False, fault, ft_mode=2)       # detect only
    assert rep2.event_set() == want and rep2.events["action"][0] == 0
    assert np.abs(out2[0, 0, row] - damaged[0]).max() <= 2e-3                       # damage left in place
    out0, rep0, _ = H.run_gpu(q, k, v, synth.F16, False, fault, ft_mode=0)       # unprotected
    assert rep0.n_events == 0 and np.abs(out0[0, 0, row] - damaged[0]).max() <= 2e-3
    others = np.delete(np.arange(N), row)
    assert np.abs(out0[0, 0, others] - ref[0, 0, others]).max() <= 2e-3
    assert np.abs(out2[0, 0, others] - ref[0, 0, others]).max() <= 2e-3


def test_many_faults_in_one_row_and_all_stages():
    """Errors in distinct stride-8 classes of one row are all repaired (Section 3.3); the four
    stages can be hit in one call; detection of non-finite results."""
    N, d = 192, 128
    q, k, v = synth.gen_qkv((1, 2, N, d), synth.BF16, 9)
    out_a, _, c = H.run_gpu(q, k, v, synth.BF16, True)
    prm = H.oracle_params(N, d, True, scale=c.softmax_scale)
    faults = [(0, 0, synth.ST_S, 1, 150, 64 + cc + 8 * (cc % 5), 27) for cc in range(8)]
    faults += [(0, 1, synth.ST_EXP, 0, 40, 13, 24), (0, 1, synth.ST_ROWSUM, 2, 180, 0, 29), (0, 1, synth.ST_OACC, 0, 100, 77, 30),
               (0, 1, synth.ST_S, 2, 191, 130, 30)]
    faults = np.array(faults, np.int32)
    out, rep, _ = H.run_gpu(q, k, v, synth.BF16, True, faults)
    expected = set()
    for h in (0, 1):
        rows = np.array(sorted({int(f[4]) for f in faults if f[1] == h}))
        _, oft, ev = H.oracle_rows(q, k, v, synth.BF16, prm, 0, h, rows, faults)
        expected |= ev
        assert np.abs(out[0, h][rows] - oft).max() <= 2e-3
    assert rep.event_set() == expected and len(expected) >= 11
    assert np.isfinite(out).all()


def test_context_reuse_and_event_overflow():
    import torch
    from paper_2504_02211_amd import ftattn
    N, d = 128, 64
    q, k, v = synth.gen_qkv((1, 1, N, d), synth.F16, 11)
    tq, tk, tv = (H.to_torch(x, synth.F16) for x in (q, k, v))
    o = torch.empty((1, 1, N, d), dtype=torch.float32, device="cuda")
    ctx = ftattn.FtAttn(1, 1, N, d, synth.F16, False, max_events=2)
    faults = np.array([[0, 0, synth.ST_OACC, 1, r, 3, 30] for r in range(5)], np.int32)
    ctx.forward(tq, tk, tv, o, faults)
    rep = ctx.report()
    assert rep.n_events == 2 and rep.n_events_dropped == 3 and (rep.rowtile_flags & 16).all()
    ctx.forward(tq, tk, tv, o, None)                 # a second call starts from clean counters
    rep = ctx.report()
    assert rep.n_events == 0 and rep.n_events_dropped == 0 and not rep.rowtile_flags.any()
    ctx.close()


def test_error_paths():
    import torch
    from paper_2504_02211_amd import ftattn
    with pytest.raises(ftattn.FtAttnError) as e:
        ftattn.FtAttn(1, 1, 128, 96, synth.F16, False)
    assert e.value.code == ftattn.EUNSUPPORTED
    ctx = ftattn.FtAttn(1, 1, 128, 64, synth.F16, True)
    t = torch.zeros((1, 1, 128, 64), dtype=torch.float16, device="cuda")
    o = torch.zeros((1, 1, 128, 64), dtype=torch.float32, device="cuda")
    for bad in ([0, 0, synth.ST_S, 0, 10, 20, 3],      # masked position (key > query)
                [0, 0, synth.ST_S, 1, 100, 20, 3],     # kv_tile does not hold the key
                [0, 0, synth.ST_OACC, 0, 10, 64, 3],   # feature out of range
                [0, 0, synth.ST_ROWSUM, 1, 10, 0, 3],  # iteration the row never runs
                [0, 1, synth.ST_S, 0, 10, 2, 3],       # head out of range
                [0, 0, 7, 0, 10, 2, 3]):               # unknown stage
        with pytest.raises(ftattn.FtAttnError) as e:
            ctx.forward(t, t, t, o, np.array([bad], np.int32))
        assert e.value.code == ftattn.EINVAL
    with pytest.raises(ftattn.FtAttnError):
        ctx.forward(t.data_ptr() + 2, t, t, o)         # misaligned pointer
    ctx.close()


def test_forward_in_a_captured_graph():
    """A fault-free forward call launches kernels only (no allocation, no memset, no copy), so a
    caller may capture it in a HIP graph: several replays, with eager work and new inputs between
    them, each equal bit for bit to the eager call on the same inputs."""
    import torch
    from paper_2504_02211_amd import ftattn
    B, Hh, N, d = 2, 3, 700, 128
    dtype = synth.BF16
    ctx = ftattn.FtAttn(B, Hh, N, d, dtype, True)
    inputs = [tuple(H.to_torch(x, dtype) for x in synth.gen_qkv((B, Hh, N, d), dtype, 0x6A0 + i)) for i in range(3)]
    q, k, v = (t.clone() for t in inputs[0])
    o = torch.empty((B, Hh, N, d), dtype=torch.float32, device="cuda")
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        ctx.forward(q, k, v, o, None, side.cuda_stream)          # warm-up on the capturing stream
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        ctx.forward(q, k, v, o, None, torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        src = inputs[rep % 3]
        for dst, s_ in zip((q, k, v), src):
            dst.copy_(s_)
        o.fill_(float("nan"))
        junk = (q.float() * 2).sum()                               # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = o.clone()
        assert ctx.report().n_events == 0
        ref = torch.empty_like(o)
        ctx.forward(q, k, v, ref, None, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.isfinite(junk) and torch.equal(got, ref), rep
    ctx.close()


def test_long_ragged_sequence_on_sampled_rows():
    """A sequence longer than any workload of the paper's evaluation, not a multiple of either tile
    size (626 key tiles, the last with one key): sampled rows against the oracle, and one fault
    late in the sequence located where the oracle says."""
    B, Hh, N, d = 1, 2, 40001, 128
    dtype = synth.BF16
    q, k, v = synth.gen_qkv((B, Hh, N, d), dtype, 0x10A6)
    out, rep, c = H.run_gpu(q, k, v, dtype, True)
    assert rep.n_events == 0
    prm = H.oracle_params(N, d, True, block_n=c.block_n, scale=c.softmax_scale, eps1=c.eps1, tau_o=c.tau_o, delta_l=c.delta_l)
    rows = np.array([0, 63, 64, 255, 256, 12345, 39935, 39936, 39999, 40000])
    for h in range(Hh):
        clean, _, ev = H.oracle_rows(q, k, v, dtype, prm, 0, h, rows, np.zeros((0, 7), np.int32))
        ma, rf = H.tolerance_ok(out[0, h][rows], clean)
        assert ev == set() and ma <= 2e-3 and rf <= 1e-3, (h, ma, rf)
    slots = [(0, h, 0, (synth.ST_S,)) for h in range(Hh)] + [(0, h, 1, (synth.ST_OACC,)) for h in range(Hh)]
    faults, redraws = H.select_faults(slots, 0x10A7, q, k, v, dtype, prm, 24, 30)
    H.assert_skip_share(redraws, len(faults))
    out2, rep2, _ = H.run_gpu(q, k, v, dtype, True, faults)
    expected = set()
    for (b, h) in sorted({(int(f[0]), int(f[1])) for f in faults}):
        fr = np.array(sorted({int(f[4]) for f in faults if f[0] == b and f[1] == h}))
        _, oft, ev = H.oracle_rows(q, k, v, dtype, prm, b, h, fr, faults)
        expected |= ev
        assert np.abs(out2[b, h][fr] - oft).max() <= 2e-3
    assert rep2.event_set() == expected and len(expected) >= 2


def test_two_contexts_on_two_streams():
    """Contexts own their scratch: two of them (different shapes) run on two streams at the same
    time and give what they give one after the other."""
    import torch
    from paper_2504_02211_amd import ftattn
    specs = [((1, 4, 1500, 128), synth.BF16, True), ((2, 3, 900, 64), synth.F16, False)]
    ctxs, tens, refs = [], [], []
    for i, (shape, dtype, causal) in enumerate(specs):
        q, k, v = (H.to_torch(x, dtype) for x in synth.gen_qkv(shape, dtype, 0x2C0 + i))
        ctx = ftattn.FtAttn(*shape, dtype, causal)
        o = torch.empty(shape, dtype=torch.float32, device="cuda")
        ctx.forward(q, k, v, o, None, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ctxs.append(ctx); tens.append((q, k, v)); refs.append(o.clone())
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.empty_like(r) for r in refs]
    torch.cuda.synchronize()
    for rep in range(5):
        for o in outs:
            o.fill_(float("nan"))
        torch.cuda.synchronize()
        for ctx, (q, k, v), o, st in zip(ctxs, tens, outs, streams):
            ctx.forward(q, k, v, o, None, st.cuda_stream)
        torch.cuda.synchronize()
        for ctx, o, r in zip(ctxs, outs, refs):
            assert torch.equal(o, r) and ctx.report().n_events == 0, rep
    for ctx in ctxs:
        ctx.close()


def test_range_flags_report_operands_that_do_not_survive_the_conversion_to_fp16():
    import torch
    from paper_2504_02211_amd import ftattn
    """bf16 inputs are converted to fp16 on entry: exact for 2^-14 <= |x| <= 65504, to 2^-25 below.  The report says
    when an operand (Q, K or V) or a tensor checksum leaves that range; ordinary data raises nothing."""
    shape = (1, 2, 200, 128)
    q, k, v = synth.gen_qkv(shape, synth.BF16, 0xF1A6)
    bf = lambda x: int(np.array([x], np.float32).view(np.uint32)[0] >> 16)
    def flags(qq, kk, vv, dtype=synth.BF16):
        _, rep, _ = H.run_gpu(qq, kk, vv, dtype, True)
        return rep.range_flags
    assert flags(q, k, v) == 0
    k2 = k.copy(); k2[0, 1, 77, 5] = bf(1.0e5)              # becomes Inf in fp16
    assert flags(q, k2, v) & ftattn.RANGE_OPERAND_OVERFLOW
    v2 = v.copy(); v2[0, 0, 3, 100] = bf(1.0e-9)            # below 2^-24: nothing left of it in fp16
    assert flags(q, k, v2) == ftattn.RANGE_OPERAND_UNDERFLOW
    q2 = q.copy(); q2[0, 1, 199, 0] = bf(-7.0e4)
    assert flags(q2, k, v) == ftattn.RANGE_OPERAND_OVERFLOW
    k3 = k.copy(); k3[0, 0, 64:128, 9] = bf(3000.0)         # every key finite in fp16, the weighted checksum (36 x 3000) is not
    assert flags(q, k3, v) == ftattn.RANGE_CHECKSUM_OVERFLOW
    # a context reports each call on its own: a clean call after a flagged one reads 0
    ctx = ftattn.FtAttn(*shape, synth.BF16, True)
    o = torch.empty(shape, dtype=torch.float32, device="cuda")
    for kk, want in ((k2, True), (k, False), (k, False), (k2, True)):
        ctx.forward(H.to_torch(q, synth.BF16), H.to_torch(kk, synth.BF16), H.to_torch(v, synth.BF16), o)
        assert bool(ctx.report().range_flags & ftattn.RANGE_OPERAND_OVERFLOW) == want
    ctx.close()
    # fp16 inputs need no conversion; their checksums can still overflow
    qh, kh, vh = synth.gen_qkv(shape, synth.F16, 0xF1A7)
    assert flags(qh, kh, vh, synth.F16) == 0
    kh[0, 0, 0:64, 3] = int(np.array([3000.0], np.float16).view(np.uint16)[0])
    assert flags(qh, kh, vh, synth.F16) == ftattn.RANGE_CHECKSUM_OVERFLOW
