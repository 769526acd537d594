"""CPU-only checks of the host side: the library loads, exports what the header declares, and
rejects bad configurations before touching a device.  Also covers the synthetic-input module."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2504_02211_amd import ftattn, ftdecoupled, ftgemm, synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions(header, prefix):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ftattn.load_library()
    for header, prefix, exports in (("ftattn.h", "ftattn", ftattn.EXPORTS), ("ftgemm.h", "ftgemm", ftgemm.EXPORTS),
                                    ("ftdecoupled.h", "ftdec", ftdecoupled.EXPORTS)):
        names = _declared_functions(header, prefix)
        assert set(names) == set(exports)
        for n in names:
            assert hasattr(lib, n), n
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["ftattn.h", "ftdecoupled.h", "ftgemm.h"]


def test_struct_layouts_match_header():
    assert C.sizeof(ftattn.Config) == 21 * 4
    assert C.sizeof(ftattn.Fault) == 7 * 4
    assert C.sizeof(ftattn.Event) == 8 * 4 == ftattn.EVENT_DTYPE.itemsize


def test_create_rejects_bad_configs_without_a_device():
    lib = ftattn.load_library()
    def create(**kw):
        base = dict(struct_size=C.sizeof(ftattn.Config), batch=1, heads=1, seq=128, head_dim=64, in_dtype=0, out_dtype=2,
                    causal=0, softmax_scale=0.0, ft_mode=1, stride=8, block_m=0, block_n=0, eps1=0.0, tau_o=0.0,
                    delta_l=0.0, rowsum_fold=0, per_step=0, rescale_margin=0.0, max_events=0, device=0)
        base.update(kw)
        cfg = ftattn.Config(**base)
        h = C.c_void_p()
        rc = lib.ftattn_create(C.byref(cfg), C.byref(h))
        return rc, lib.ftattn_last_error(None).decode()
    assert create(struct_size=12)[0] == ftattn.EINVAL
    assert create(head_dim=80)[0] == ftattn.EUNSUPPORTED
    assert create(seq=0)[0] == ftattn.EINVAL
    assert create(in_dtype=2)[0] == ftattn.EINVAL
    assert create(out_dtype=1)[0] == ftattn.EINVAL          # bf16 out for fp16 in
    assert create(stride=4)[0] == ftattn.EUNSUPPORTED
    assert create(block_n=128)[0] == ftattn.EUNSUPPORTED
    assert create(ft_mode=5)[0] == ftattn.EINVAL
    assert create(rowsum_fold=2)[0] == ftattn.EINVAL
    assert create(per_step=3)[0] == ftattn.EINVAL
    assert create(per_step=2, ft_mode=2)[0] == ftattn.EINVAL
    assert create(per_step=1, ft_mode=2)[0] == ftattn.EINVAL       # per-step verification repairs as it goes
    assert create(per_step=1, rowsum_fold=1)[0] == ftattn.EINVAL
    assert create(stride=4)[0] == ftattn.EUNSUPPORTED
    assert create(stride=1, ft_mode=0)[0] == ftattn.EINVAL           # the traditional checksum is a mode of the protected kernel
    assert create(stride=1, rowsum_fold=1)[0] == ftattn.EINVAL
    assert create(stride=1, per_step=1)[0] == ftattn.EINVAL
    assert create(rescale_margin=2.0, per_step=1)[0] == ftattn.EINVAL      # the lazily renewed maximum is a mode of the unified scheme
    assert create(rescale_margin=2.0, rowsum_fold=1)[0] == ftattn.EINVAL
    assert create(rescale_margin=2.0, stride=1)[0] == ftattn.EINVAL
    assert create(rescale_margin=9.0)[0] == ftattn.EINVAL                  # exponentials beyond the fp16 range
    rc, msg = create(block_m=96)
    assert rc == ftattn.EUNSUPPORTED and "block_m" in msg
    assert create(block_m=256)[0] == ftattn.EUNSUPPORTED       # head_dim 64 runs 128-query row tiles
    assert lib.ftattn_forward(None, None, None, None, None, None, 0, None) == ftattn.EINVAL
    assert lib.ftattn_report(None, None) == ftattn.EINVAL
    assert lib.ftattn_destroy(None) == ftattn.EINVAL


def test_gemm_create_rejects_bad_configs_without_a_device():
    lib = ftgemm.load_library()
    assert C.sizeof(ftgemm.Config) == 14 * 4 and C.sizeof(ftgemm.Fault) == 12
    assert C.sizeof(ftgemm.Event) == 16 == ftgemm.EVENT_DTYPE.itemsize
    def create(**kw):
        base = dict(struct_size=C.sizeof(ftgemm.Config), m=256, n=256, k=128, in_dtype=0, out_dtype=2, ft_mode=1,
                    stride=8, block_n=0, tau_rel=0.0, tau_abs=-1.0, fold_tokens=0, max_events=0, device=0)
        base.update(kw)
        cfg = ftgemm.Config(**base)
        h = C.c_void_p()
        rc = lib.ftgemm_create(C.byref(cfg), C.byref(h))
        return rc, lib.ftgemm_last_error(None).decode()
    assert create(struct_size=8)[0] == ftgemm.EINVAL
    assert create(m=0)[0] == ftgemm.EINVAL
    assert create(k=100)[0] == ftgemm.EUNSUPPORTED
    assert create(k=0)[0] == ftgemm.EUNSUPPORTED
    assert create(in_dtype=2)[0] == ftgemm.EINVAL
    assert create(out_dtype=1)[0] == ftgemm.EINVAL          # bf16 out for fp16 in
    assert create(in_dtype=1, out_dtype=0)[0] == ftgemm.EINVAL
    assert create(stride=4)[0] == ftgemm.EUNSUPPORTED
    assert create(ft_mode=3)[0] == ftgemm.EINVAL
    assert create(fold_tokens=2)[0] == ftgemm.EINVAL
    rc, msg = create(block_n=128)
    assert rc == ftgemm.EUNSUPPORTED and "block_n" in msg
    assert lib.ftgemm_forward(None, None, None, None, None, 0, None) == ftgemm.EINVAL
    assert lib.ftgemm_encode_weights(None, None, None) == ftgemm.EINVAL
    assert lib.ftgemm_report(None, None) == ftgemm.EINVAL
    assert lib.ftgemm_destroy(None) == ftgemm.EINVAL


def test_linear_inputs_are_deterministic():
    x1, w1 = synth.gen_linear(300, 520, 128, 7)
    x2, w2 = synth.gen_linear(300, 520, 128, 7)
    assert np.array_equal(x1, x2) and np.array_equal(w1, w2)
    xf, wf = synth.bits_to_f64(x1, synth.F16), synth.bits_to_f64(w1, synth.F16)
    assert abs(xf.std() - 1) < 0.05 and abs(wf.std() * np.sqrt(128) - 1) < 0.05
    s = synth.linear_fault_stream(3, 0, 300, 520, 20, 30)
    a = [next(s) for _ in range(50)]
    s = synth.linear_fault_stream(3, 0, 300, 520, 20, 30)
    assert a == [next(s) for _ in range(50)]
    assert all(0 <= r < 300 and 0 <= c < 520 and 20 <= b <= 30 for r, c, b in a)


def test_synth_is_deterministic_and_exact():
    q1, k1, v1 = synth.gen_workload(1)
    q2, k2, v2 = synth.gen_workload(1)
    assert np.array_equal(q1, q2) and np.array_equal(k1, k2) and np.array_equal(v1, v2)
    x = synth.bits_to_f64(q1, synth.F16)
    assert abs(x.mean()) < 0.05 and abs(x.std() - 1) < 0.05
    # bf16 round trip and round-to-nearest-even
    vals = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -3.1415926, 65280.0], np.float32)
    bits = synth.f32_to_bf16_bits(vals)
    back = synth.bf16_bits_to_f64(bits)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.0 + 2.0 ** -6 and back[4] == 65280.0
    assert abs(back[3] + 3.1415926) < 2.0 ** -7
    # a subset of heads reproduces the same bits; outlier rows are scaled
    qa, ka, va = synth.gen_workload(4, heads_subset=[(1, 3)])
    qb, kb, vb = synth.gen_workload(4, heads_subset=[(0, 0), (1, 3)])
    assert np.array_equal(ka[1, 3], kb[1, 3]) and not ka[0, 0].any()
    kk = synth.bits_to_f64(ka[1, 3], synth.BF16)
    assert (np.abs(kk).max(axis=1) > 12).sum() >= 30


def test_candidate_streams_respect_the_mask_and_the_seu_rule():
    w = synth.WORKLOADS[3]
    s = synth.candidate_stream(1, 0, 0, 0, w.seq, w.head_dim, 64, True, (synth.ST_S, synth.ST_EXP, synth.ST_ROWSUM, synth.ST_OACC), 20, 30)
    seen = [next(s) for _ in range(500)]
    for (b, h, st, kt, row, col, bit) in seen:
        assert 20 <= bit <= 30 and 0 <= row < w.seq and kt < synth.n_kv_tiles(row, w.seq, 64, True)
        if st in (synth.ST_S, synth.ST_EXP):
            assert col <= row and kt == col // 64
        if st == synth.ST_OACC:
            assert 0 <= col < w.head_dim
    s2 = synth.candidate_stream(1, 0, 0, 0, w.seq, w.head_dim, 64, True, (synth.ST_S, synth.ST_EXP, synth.ST_ROWSUM, synth.ST_OACC), 20, 30)
    assert [next(s2) for _ in range(500)] == seen
    assert synth.conflicts((0, 0, synth.ST_EXP, 1, 5, 70, 3), [(0, 0, synth.ST_S, 1, 5, 90, 4)])
    assert not synth.conflicts((0, 0, synth.ST_EXP, 2, 5, 130, 3), [(0, 0, synth.ST_S, 1, 5, 90, 4)])
    assert synth.conflicts((0, 0, synth.ST_OACC, 2, 5, 11, 3), [(0, 0, synth.ST_OACC, 0, 5, 3, 4)])
    assert len(list(synth.workload_fault_slots(4))) == 4 * 32 * 4


def test_binding_checks_tensors_before_passing_raw_pointers():
    """The C ABI sees addresses only; the binding refuses a tensor whose type, size, layout or
    device does not fit the configured shape (it would be an out-of-bounds access on the GPU)."""
    class FakeDevice:
        index = 0
    class FakeTensor:
        def __init__(self, n, dtype="torch.float16", contiguous=True, cuda=True):
            self._n, self.dtype, self._c, self.is_cuda, self.device = n, dtype, contiguous, cuda, FakeDevice()
        def data_ptr(self): return 4096
        def numel(self): return self._n
        def is_contiguous(self): return self._c
    ok = ftattn.device_pointer(FakeTensor(64), "q", 64, ftattn.F16, 0)
    assert ok.value == 4096 and ftattn.device_pointer(12345, "q", 64, ftattn.F16, 0).value == 12345
    for bad in (FakeTensor(63), FakeTensor(64, "torch.bfloat16"), FakeTensor(64, contiguous=False), FakeTensor(64, cuda=False)):
        with pytest.raises(ValueError):
            ftattn.device_pointer(bad, "q", 64, ftattn.F16, 0)
    with pytest.raises(ValueError):
        ftattn.device_pointer(FakeTensor(64), "q", 64, ftattn.F16, 1)
    with pytest.raises(TypeError):
        ftattn.device_pointer(object(), "q", 64, ftattn.F16, 0)


def test_decoupled_create_rejects_bad_configs_without_a_device():
    lib = ftdecoupled.load_library()
    assert C.sizeof(ftdecoupled.Config) == 13 * 4 and C.sizeof(ftdecoupled.Fault) == 24 == C.sizeof(ftdecoupled.Event)
    def create(**kw):
        base = dict(struct_size=C.sizeof(ftdecoupled.Config), batch=1, heads=1, seq=64, head_dim=64, in_dtype=0, causal=0,
                    softmax_scale=0.0, ft_mode=1, tau_rel=0.0, eps_dmr=0.0, max_events=0, device=0)
        base.update(kw)
        h = C.c_void_p()
        return lib.ftdec_create(C.byref(ftdecoupled.Config(**base)), C.byref(h))
    assert create(struct_size=8) == ftdecoupled.EINVAL
    assert create(seq=0) == ftdecoupled.EINVAL
    assert create(head_dim=60) == ftdecoupled.EUNSUPPORTED and create(head_dim=512) == ftdecoupled.EUNSUPPORTED
    assert create(in_dtype=2) == ftdecoupled.EINVAL and create(causal=2) == ftdecoupled.EINVAL
    assert create(ft_mode=2) == ftdecoupled.EINVAL
    assert b"ft_mode" in lib.ftdec_last_error(None)
    assert lib.ftdec_forward(None, None, None, None, None, None, 0, None) == ftdecoupled.EINVAL
    assert lib.ftdec_report(None, None) == ftdecoupled.EINVAL and lib.ftdec_destroy(None) == ftdecoupled.EINVAL
