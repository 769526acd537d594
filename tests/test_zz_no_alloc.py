"""The entry point that allocates nothing (ftattn_forward_static) against ftattn_forward: same
kernels on the library's static scratch array instead of a context's buffers, so the outputs must
be identical bit for bit.  Two calls in a row on one stream, the second with a smaller input (the
array keeps the first call's contents), then a shape that does not fit the array."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2504_02211_amd import ftattn, synth
import ft_harness as H

pytestmark = pytest.mark.gpu


def _both(shape, dtype, causal, ft_mode, seed):
    B, Hh, N, d = shape
    q, k, v = synth.gen_qkv(shape, dtype, seed)
    tq, tk, tv = (H.to_torch(x, dtype) for x in (q, k, v))
    st = torch.cuda.current_stream().cuda_stream
    want = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    ctx = ftattn.FtAttn(B, Hh, N, d, dtype, causal, ft_mode=ft_mode)
    ctx.forward(tq, tk, tv, want, None, st)
    rep = ctx.report()
    ctx.close()
    got = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    nev = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    ftattn.forward_static(tq, tk, tv, got, B, Hh, N, d, dtype, causal, ft_mode=ft_mode, n_events=nev, stream=st)
    torch.cuda.synchronize()
    return got, want, int(nev.item()), rep.n_events


def test_static_entry_point_matches_the_context_path_on_two_calls_in_a_row():
    print("[no alloc] first call: 2 x 3 x 1000 x 128 bf16 causal", flush=True)
    got, want, nev, nref = _both((2, 3, 1000, 128), synth.BF16, True, ftattn.FT_CORRECT, 0x5A71)
    assert torch.isfinite(got).all() and torch.equal(got, want) and nev == nref == 0
    print("[no alloc] second call, smaller: 1 x 2 x 333 x 64 fp16", flush=True)
    got, want, nev, nref = _both((1, 2, 333, 64), synth.F16, False, ftattn.FT_CORRECT, 0x5A72)
    assert torch.isfinite(got).all() and torch.equal(got, want) and nev == nref == 0
    print("[no alloc] third call: checks compiled out, 1 x 1 x 77 x 128", flush=True)
    got, want, nev, nref = _both((1, 1, 77, 128), synth.F16, True, ftattn.FT_OFF, 0x5A73)
    assert torch.isfinite(got).all() and torch.equal(got, want) and nev == 0


def test_static_entry_point_rejects_what_does_not_fit():
    x = torch.zeros(16, dtype=torch.float16, device="cuda")
    a = x.data_ptr()                                     # raw addresses: the C entry point must refuse before any launch
    with pytest.raises(ftattn.FtAttnError) as ei:        # 8 x 16 x 2048 x 64: 100 MB of encoded tiles
        ftattn.forward_static(a, a, a, a, 8, 16, 2048, 64, synth.BF16, True)
    assert ei.value.code == ftattn.EUNSUPPORTED and "scratch" in str(ei.value)
    with pytest.raises(ftattn.FtAttnError) as ei:
        ftattn.forward_static(a, a, a, None, 1, 1, 64, 64, synth.F16, False)
    assert ei.value.code == ftattn.EINVAL
    with pytest.raises(ValueError):                      # the binding refuses a tensor of the wrong size
        ftattn.forward_static(x, x, x, x, 1, 1, 64, 64, synth.F16, False)
