"""Shared helpers of the parity tests: fault selection through the oracle, and running the
GPU library on synthetic workloads.  (Test infrastructure; imports both sides.)"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from oracle import efta_oracle as orc
from paper_2504_02211_amd import synth


def head_f64(bits: np.ndarray, dtype: int, b: int, h: int) -> np.ndarray:
    return synth.bits_to_f64(bits[b, h], dtype)


def oracle_params(seq: int, head_dim: int, causal: bool, block_n: int = 64, scale: Optional[float] = None,
                  **kw) -> orc.Params:
    return orc.Params(scale=scale if scale is not None else float(np.float32(1.0) / np.sqrt(np.float32(head_dim))),
                      causal=causal, block_n=block_n, **kw)


def select_faults(slots, seed: int, q, k, v, dtype: int, prm: orc.Params, bit_lo: int, bit_hi: int,
                  max_attempts: int = 200) -> Tuple[np.ndarray, int]:
    """Draws one fault per slot from the seeded candidate streams, skipping candidates whose
    detection would hinge on rounding (oracle statistics within 4x of a threshold), whose flipped
    value sits on a binade edge or (row-sum) has an uncertain value of the flipped mantissa bit, whose
    substituted row-sum blows the output row up (more than twofold, beyond +-2), that break the one-fault-per-cycle rule, or
    that share a row with an accepted fault.  Returns (int32
    [n,7] fault array, number of skipped candidates); callers bound the skipped share with
    ``assert_skip_share``."""
    B, H, N, d = q.shape
    accepted: List[Tuple[int, ...]] = []
    redraws = 0
    cache: Dict[Tuple[int, int], Tuple[np.ndarray, np.ndarray, np.ndarray]] = {}
    for (b, h, slot, stages) in slots:
        if (b, h) not in cache:
            cache.clear()
            cache[(b, h)] = (head_f64(q, dtype, b, h), head_f64(k, dtype, b, h), head_f64(v, dtype, b, h))
        Q, K, V = cache[(b, h)]
        stream = synth.candidate_stream(seed, b, h, slot, N, d, prm.block_n, prm.causal, stages, bit_lo, bit_hi)
        for _ in range(max_attempts):
            f = next(stream)
            row = f[4]
            if synth.conflicts(f, accepted) or any(g[0] == b and g[1] == h and g[4] == row for g in accepted):
                redraws += 1
                continue
            o_ft, ev, dg = orc.efta_rows(Q[row:row + 1], np.array([row]), K, V, prm, [f[2:]])
            ok = orc.fault_is_robust(dg) and len(dg["flipped"]) == 1 and not orc.fp32_is_fragile(dg["flipped"][0][1], f[2], f[6])
            # A row-sum replaced by its lower bound (the paper's approximate repair) multiplies the whole output row
            # by l_true / L, and with it the kernel's rounding error (fp16 weights: up to 1e-3 of the output): blown
            # up by more than 2x to beyond +-2, that error alone can pass the absolute bar of 2e-3, so such a
            # candidate decides nothing.
            if ok and any(e[0] == orc.CHECK_L for e in ev) and np.isfinite(o_ft).all() and np.abs(o_ft).max() > 2.0:
                clean = orc.attention_clean(Q[row:row + 1], K, V, prm.scale, prm.causal, np.array([row]))
                if np.abs(o_ft).max() > 2.0 * np.abs(clean).max():
                    ok = False
            if ok:
                accepted.append(f)
                break
            redraws += 1
        else:
            raise RuntimeError(f"no robust fault found for slot {(b, h, slot)}")
    return synth.faults_to_array(accepted), redraws


MAX_SKIP_SHARE = 0.6


def assert_skip_share(skipped: int, accepted: int, bound: float = MAX_SKIP_SHARE) -> None:
    """The fault selector may pass over ill-posed candidates, but not over most of them: a filter
    that rejects the bulk of the stream would hide a real disagreement behind "ill-posed"."""
    share = skipped / max(1, skipped + accepted)
    assert share <= bound, f"{skipped} of {skipped + accepted} fault candidates skipped ({share:.0%} > {bound:.0%})"


def oracle_rows(q, k, v, dtype: int, prm: orc.Params, b: int, h: int, rows: np.ndarray, faults: np.ndarray):
    """Oracle results for some rows of one head: (O_clean, O_ft, events as (b,h,check,kv_tile,row,col) set)."""
    Q, K, V = head_f64(q, dtype, b, h), head_f64(k, dtype, b, h), head_f64(v, dtype, b, h)
    rows = np.asarray(rows)
    fl = [tuple(int(x) for x in f[2:]) for f in faults if f[0] == b and f[1] == h]
    clean = orc.attention_clean(Q[rows], K, V, prm.scale, prm.causal, rows)
    O, ev, _ = orc.efta_rows(Q[rows], rows, K, V, prm, fl)
    return clean, O, {(b, h) + e for e in ev}


def to_torch(bits: np.ndarray, dtype: int, device: str = "cuda"):
    import torch
    t = torch.from_numpy(bits.view(np.int16)).to(device)
    return t.view(torch.float16 if dtype == synth.F16 else torch.bfloat16)


def run_gpu(q, k, v, dtype: int, causal: bool, faults: Optional[np.ndarray] = None, ft_mode: int = 1,
            out_dtype: int = 2, **kw):
    """One forward call through the C ABI; returns (O as float64 numpy, Report, effective Config)."""
    import torch
    from paper_2504_02211_amd import ftattn
    B, H, N, d = q.shape
    ctx = ftattn.FtAttn(B, H, N, d, dtype, causal, out_dtype=out_dtype, ft_mode=ft_mode, **kw)
    tq, tk, tv = (to_torch(x, dtype) for x in (q, k, v))
    odt = {0: torch.float16, 1: torch.bfloat16, 2: torch.float32}[out_dtype]
    o = torch.full((B, H, N, d), float("nan"), dtype=odt, device="cuda")
    ctx.forward(tq, tk, tv, o, faults, torch.cuda.current_stream().cuda_stream)
    rep = ctx.report()
    torch.cuda.synchronize()
    out = o.double().cpu().numpy()
    cfg = ctx.config
    ctx.close()
    return out, rep, cfg


def tolerance_ok(got: np.ndarray, ref: np.ndarray) -> Tuple[float, float]:
    """(max-abs error, relative Frobenius error)."""
    diff = got - ref
    return float(np.abs(diff).max()), float(np.linalg.norm(diff) / max(np.linalg.norm(ref), 1e-300))
