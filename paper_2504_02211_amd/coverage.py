#!/usr/bin/env python3
"""Error coverage of the three checks of Algorithm 1 against their thresholds.

The paper's evaluation (Section 4.2, "Error Coverage of Strided ABFT" and "Error Coverage of
Selective Neuron Value Restriction") reports, for a range of thresholds, how many injected
computational errors a check detects and how often it fires on error-free data.  This module
measures the same three curves on the GPU library with its seeded injector:

  product  the per-iteration product-form check (threshold eps1) against flips of S and exp(S - m);
  sum      the final sum-form check of the output (threshold tau_o) against flips of the output accumulator;
  range    the range restriction of the row-sum (relative slack delta_l) against flips of the row-sum;

and the error that is left in the output after correction (the approximation of the row-sum by
its lower bound included).  Every flip hits its own query row, so a detection is attributed to a
fault by (batch, head, row).  A fault counts as harmful when, left alone, it moves some output of
its row by more than the parity tolerance of the library (2e-3).

A second mode (``--ber``) injects flips at a given rate per computed fp32 intermediate with no
constraint on where they fall, and counts the rows that are wrong without protection, flagged
under protection, and right again after correction.

A third mode (``--linear``) does the threshold sweep for the strided ABFT of the linear layer
(relative threshold tau_rel): one flip per output row, both checksum orientations.

Everything here goes through the C ABI; the inputs are synthetic and seeded.

    python -m paper_2504_02211_amd.coverage --seq 2048 --heads 8 --faults-per-head 48
    python -m paper_2504_02211_amd.coverage --seq 2048 --heads 8 --ber 1e-7 1e-6 1e-5 1e-4
    python -m paper_2504_02211_amd.coverage --linear [--fold-tokens]
"""
from __future__ import annotations

import argparse
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import ftattn, ftgemm, synth

HARM_TOL = 2e-3
FAMILIES = ("product", "sum", "range")
STAGES_OF = {"product": (synth.ST_S, synth.ST_EXP), "sum": (synth.ST_OACC,), "range": (synth.ST_ROWSUM,)}
CHECKS_OF = {"product": (ftattn.CHECK_S, ftattn.CHECK_EXP), "sum": (ftattn.CHECK_O,), "range": (ftattn.CHECK_L,)}
DEFAULT_GRIDS = {
    "product": (1e-4, 1e-3, 3e-3, 1e-2, 3e-2, 1e-1, 3e-1, 1.0, 3.0),
    "sum": (1e-6, 1e-5, 1e-4, 4e-4, 0.75 * 2.0 ** -9, 5e-3, 2e-2, 1e-1),
    "range": (1e-7, 1e-6, 1e-5, 1e-4, 2.0 ** -10, 1e-2, 1e-1, 1.0),
}


def draw_faults(batch: int, heads: int, seq: int, head_dim: int, causal: bool, block_n: int, per_head: int,
                seed: int, bit_lo: int = 0, bit_hi: int = 30) -> np.ndarray:
    """Seeded single-bit flips, `per_head` per (batch, head), each on a query row of its own."""
    out: List[Tuple[int, ...]] = []
    stages = (synth.ST_S, synth.ST_EXP, synth.ST_ROWSUM, synth.ST_OACC)
    for b in range(batch):
        for h in range(heads):
            rows = set()
            for slot in range(per_head):
                stream = synth.candidate_stream(seed, b, h, slot, seq, head_dim, block_n, causal,
                                                (stages[slot % 4],), bit_lo, bit_hi)
                for _ in range(1000):
                    f = next(stream)
                    if f[4] not in rows:
                        rows.add(f[4])
                        out.append(f)
                        break
    return synth.faults_to_array(out)


def _to_torch(bits: np.ndarray, dtype: int):
    import torch
    t = torch.from_numpy(bits.view(np.int16)).to("cuda")
    return t.view(torch.float16 if dtype == synth.F16 else torch.bfloat16)


class Runner:
    """Keeps the operands on the device and runs one forward call per threshold setting."""

    def __init__(self, q: np.ndarray, k: np.ndarray, v: np.ndarray, dtype: int, causal: bool, rowsum_fold: bool = False,
                 per_step: int = 0, stride: int = 8):
        import torch
        self.torch = torch
        self.rowsum_fold = rowsum_fold
        self.per_step = per_step
        self.stride = stride
        self.shape = q.shape
        self.dtype, self.causal = dtype, causal
        self.tq, self.tk, self.tv = (_to_torch(x, dtype) for x in (q, k, v))

    def run(self, faults: Optional[np.ndarray], ft_mode: int, **thresholds):
        torch = self.torch
        B, H, N, d = self.shape
        ctx = ftattn.FtAttn(B, H, N, d, self.dtype, self.causal, ft_mode=ft_mode, max_events=1 << 20,
                            rowsum_fold=self.rowsum_fold,
                            per_step=self.per_step if ft_mode == ftattn.FT_CORRECT else 0,
                            stride=self.stride if ft_mode != ftattn.FT_OFF else 8, **thresholds)
        o = torch.empty((B, H, N, d), dtype=torch.float32, device="cuda")
        ctx.forward(self.tq, self.tk, self.tv, o, faults, torch.cuda.current_stream().cuda_stream)
        rep = ctx.report()
        out = o.cpu().numpy()
        cfg = ctx.config
        ctx.close()
        return out, rep, cfg


def _rows_with_events(rep, checks: Sequence[int]) -> set:
    e = rep.events
    m = np.isin(e["check"], checks)
    return set(zip(e["b"][m].tolist(), e["h"][m].tolist(), e["row"][m].tolist()))


def sweep(q: np.ndarray, k: np.ndarray, v: np.ndarray, dtype: int, causal: bool, faults: np.ndarray,
          grids: Optional[Dict[str, Sequence[float]]] = None) -> Dict[str, object]:
    """Runs the sweep; returns per-family curves and the post-correction error statistics."""
    grids = dict(DEFAULT_GRIDS if grids is None else grids)
    r = Runner(q, k, v, dtype, causal)
    B, H, N, d = q.shape
    clean, _, cfg = r.run(None, ftattn.FT_OFF)
    damaged, _, _ = r.run(faults, ftattn.FT_OFF)
    with np.errstate(all="ignore"):
        dmg = np.array([np.nanmax(np.abs(damaged[f[0], f[1], f[4]] - clean[f[0], f[1], f[4]]))
                        if np.isfinite(damaged[f[0], f[1], f[4]]).all() else np.inf for f in faults])
    harmful = dmg > HARM_TOL
    rows_per_check = {"product": None, "sum": B * H * N * 8, "range": B * H * N}
    bn = cfg.block_n
    n_tiles = sum((row // bn + 1) if causal else -(-N // bn) for row in range(N))
    rows_per_check["product"] = B * H * n_tiles * 8
    key = {"product": "eps1", "sum": "tau_o", "range": "delta_l"}
    result: Dict[str, object] = {"n_faults": int(len(faults)), "harm_tol": HARM_TOL, "curves": {}}
    for fam in FAMILIES:
        sel = np.isin(faults[:, 2], STAGES_OF[fam])
        curve = []
        for thr in grids[fam]:
            _, rep_f, _ = r.run(faults, ftattn.FT_DETECT, **{key[fam]: float(thr)})
            _, rep_c, _ = r.run(None, ftattn.FT_DETECT, **{key[fam]: float(thr)})
            hit_rows = _rows_with_events(rep_f, CHECKS_OF[fam])
            det = np.array([(int(f[0]), int(f[1]), int(f[4])) in hit_rows for f in faults])
            fa_rows = _rows_with_events(rep_c, CHECKS_OF[fam])
            n_h, n_b = int((sel & harmful).sum()), int((sel & ~harmful).sum())
            curve.append({
                "threshold": float(thr),
                "harmful": n_h, "harmful_detected": int((sel & harmful & det).sum()),
                "benign": n_b, "benign_detected": int((sel & ~harmful & det).sum()),
                # (the other checks run at their defaults and stay silent on clean data; events beyond
                # the capacity of the log are counted by the library)
                "false_alarms": int(np.isin(rep_c.events["check"], CHECKS_OF[fam]).sum()) + int(rep_c.n_events_dropped),
                "false_alarm_rows": len(fa_rows), "checks": rows_per_check[fam],
            })
        result["curves"][fam] = curve
    # what is left after correction at the default thresholds
    fixed, rep_fix, _ = r.run(faults, ftattn.FT_CORRECT)
    with np.errstate(all="ignore"):
        left = np.array([np.nanmax(np.abs(fixed[f[0], f[1], f[4]] - clean[f[0], f[1], f[4]]))
                         if np.isfinite(fixed[f[0], f[1], f[4]]).all() else np.inf for f in faults])
    result["after_correction"] = {}
    for fam in FAMILIES:
        sel = np.isin(faults[:, 2], STAGES_OF[fam]) & harmful
        x = left[sel]
        result["after_correction"][fam] = {
            "harmful": int(sel.sum()),
            "within_tol": int((x <= HARM_TOL).sum()),
            "median": float(np.median(x)) if len(x) else 0.0,
            "p90": float(np.quantile(x, 0.9)) if len(x) else 0.0,
            "max": float(x.max()) if len(x) else 0.0,
        }
    result["unprotected_damage"] = {"harmful": int(harmful.sum()), "median": float(np.median(dmg[harmful])) if harmful.any() else 0.0}
    result["per_fault"] = {"damage": dmg, "left": left, "harmful": harmful}
    return result


def population(batch: int, heads: int, seq: int, head_dim: int, causal: bool, block_n: int) -> int:
    """Number of fp32 intermediates the injector can hit: raw scores and exponentials of every
    unmasked position, one row-sum and head_dim output accumulators per (row, key-tile iteration)."""
    scores = seq * (seq + 1) // 2 if causal else seq * seq
    iters = sum(synth.n_kv_tiles(r, seq, block_n, causal) for r in range(seq))
    return batch * heads * (2 * scores + iters * (1 + head_dim))


def draw_ber_faults(batch: int, heads: int, seq: int, head_dim: int, causal: bool, block_n: int, ber: float,
                    seed: int, limit: int = 60000) -> np.ndarray:
    """round(ber * population) single-bit flips (at least one, at most `limit`) at seeded positions
    spread evenly over the heads, with no constraint on how they fall: several may share a row, a
    key tile or a checksum class (the bit-error-rate experiments of Section 4.2)."""
    n = int(min(limit, max(1, round(ber * population(batch, heads, seq, head_dim, causal, block_n)))))
    stages = (synth.ST_S, synth.ST_EXP, synth.ST_ROWSUM, synth.ST_OACC)
    streams = {}
    out: List[Tuple[int, ...]] = []
    for i in range(n):
        bh = i % (batch * heads)
        b, h = divmod(bh, heads)
        if bh not in streams:
            streams[bh] = synth.candidate_stream(seed, b, h, 0, seq, head_dim, block_n, causal, stages, 0, 30)
        out.append(next(streams[bh]))
    return synth.faults_to_array(out)


def ber_sweep(q: np.ndarray, k: np.ndarray, v: np.ndarray, dtype: int, causal: bool, bers: Sequence[float],
              seed: int, rowsum_fold: bool = False, per_step: int = 0, stride: int = 8) -> List[Dict[str, object]]:
    """For every bit error rate: how many rows the flips damage when nothing protects them, how
    many of those rows raise an event under protection, and how many are back within the
    tolerance after correction (default thresholds)."""
    r = Runner(q, k, v, dtype, causal, rowsum_fold, per_step, stride)
    B, H, N, d = q.shape
    clean, _, cfg = r.run(None, ftattn.FT_OFF)
    rows_out = []
    for ber in bers:
        faults = draw_ber_faults(B, H, N, d, causal, cfg.block_n, ber, seed)
        damaged, _, _ = r.run(faults, ftattn.FT_OFF)
        fixed, rep, _ = r.run(faults, ftattn.FT_CORRECT)
        with np.errstate(all="ignore"):
            dmg = np.abs(damaged - clean).max(axis=-1)
            left = np.abs(fixed - clean).max(axis=-1)
        dmg = np.where(np.isfinite(dmg), dmg, np.inf)
        left = np.where(np.isfinite(left), left, np.inf)
        harmful = dmg > HARM_TOL                                   # [B, H, N] rows
        flagged = np.zeros_like(harmful)
        e = rep.events
        flagged[e["b"], e["h"], e["row"]] = True
        hit = np.zeros_like(harmful)
        hit[faults[:, 0], faults[:, 1], faults[:, 4]] = True
        rows_out.append({
            "ber": float(ber), "faults": int(len(faults)), "rows_hit": int(hit.sum()),
            "rows_harmed": int(harmful.sum()), "harmed_flagged": int((harmful & flagged).sum()),
            "harmed_repaired": int((harmful & (left <= HARM_TOL)).sum()),
            "rows_bad_after": int((left > HARM_TOL).sum()),
            "flagged_unharmed_hit": int((flagged & ~harmful & hit).sum()),
            "flagged_not_hit": int((flagged & ~hit).sum()),
            "events": int(rep.n_events), "events_dropped": int(rep.n_events_dropped),
            "rows_bad_after_by_stage": {synth.STAGE_NAMES[st]: int(((left > HARM_TOL) & _rows_of(faults, st, harmful.shape)).sum())
                                         for st in range(4)},
        })
    return rows_out


def _rows_of(faults: np.ndarray, stage: int, shape) -> np.ndarray:
    m = np.zeros(shape, bool)
    f = faults[faults[:, 2] == stage]
    m[f[:, 0], f[:, 1], f[:, 4]] = True
    return m


def ber_markdown(rows: List[Dict[str, object]]) -> str:
    out = ["| bit error rate | flips | rows harmed (unprotected) | of those flagged | of those repaired | rows still wrong "
           "(by stage of a flip in the row: S / EXP / ROWSUM / OACC) | events on rows no flip hit |", "|---|---|---|---|---|---|---|"]
    for r in rows:
        st = r["rows_bad_after_by_stage"]
        pct = lambda a, b: f"{a} ({100.0 * a / b:.1f} %)" if b else f"{a}"
        out.append(f"| {r['ber']:.0e} | {r['faults']} | {r['rows_harmed']} | {pct(r['harmed_flagged'], r['rows_harmed'])} | "
                   f"{pct(r['harmed_repaired'], r['rows_harmed'])} | {r['rows_bad_after']} ({st['S']} / {st['EXP']} / "
                   f"{st['ROWSUM']} / {st['OACC']}) | {r['flagged_not_hit']} |")
    return "\n".join(out)


def to_markdown(res: Dict[str, object]) -> str:
    names = {"product": "product-form check, threshold eps1 (flips of S and exp)",
             "sum": "sum-form check of O, threshold tau_o (flips of the output accumulator)",
             "range": "row-sum range restriction, slack delta_l (flips of the row-sum)"}
    out = [f"{res['n_faults']} single-bit flips (bits 0-30), harmful = output of the row moves by more than {res['harm_tol']:g}", ""]
    for fam in FAMILIES:
        out += [f"**{names[fam]}**", "", "| threshold | harmful detected | benign detected | false alarms on clean data (of checks) |",
                "|---|---|---|---|"]
        for c in res["curves"][fam]:
            hd = f"{c['harmful_detected']}/{c['harmful']}" + (f" ({100.0 * c['harmful_detected'] / c['harmful']:.1f} %)" if c["harmful"] else "")
            out.append(f"| {c['threshold']:.3g} | {hd} | {c['benign_detected']}/{c['benign']} | {c['false_alarms']} of {c['checks']} |")
        out.append("")
    out += ["**left after correction (default thresholds), harmful faults only**", "",
            "| check | harmful | back within tolerance | median error | 90 % | max |", "|---|---|---|---|---|---|"]
    for fam in FAMILIES:
        a = res["after_correction"][fam]
        out.append(f"| {fam} | {a['harmful']} | {a['within_tol']} | {a['median']:.2e} | {a['p90']:.2e} | {a['max']:.2e} |")
    return "\n".join(out)



LINEAR_GRID = tuple(2.0 ** e for e in (-21, -19, -17, -16, -15, -14, -13, -11, -9, -7))
LINEAR_HARM = 1e-3          # a flip is harmful when it moves its output by more than this (outputs are of order one)


def linear_sweep(m: int, n: int, k: int, dtype: int, n_faults: int, seed: int, fold_tokens: bool = False,
                 grid: Sequence[float] = LINEAR_GRID) -> Dict[str, object]:
    """Threshold sweep of the linear layer's check: for every tau_rel, how many of the harmful and of the
    harmless flips (one per output row and column, bits 0..31) are flagged, how many of the harmful ones
    are back within tolerance, and how many events a fault-free run raises."""
    import torch
    xb, wb = synth.gen_linear(m, n, k, seed, dtype=dtype)
    tt = torch.float16 if dtype == synth.F16 else torch.bfloat16
    x = torch.from_numpy(xb.view(np.int16)).cuda().view(tt)
    w = torch.from_numpy(wb.view(np.int16)).cuda().view(tt)
    rows, cols, faults = set(), set(), []
    for slot in range(n_faults):
        stream = synth.linear_fault_stream(seed + 1, slot, m, n, 0, 31)
        for _ in range(1000):
            r, c, b = next(stream)
            if r not in rows and c not in cols:
                rows.add(r); cols.add(c); faults.append((r, c, b))
                break
    fa = np.asarray(faults, np.int32)

    def run(ft_mode, flt, tau_rel=0.0):
        ctx = ftgemm.FtGemm(m, n, k, out_dtype=ftgemm.F32, ft_mode=ft_mode, tau_rel=tau_rel, in_dtype=dtype,
                            fold_tokens=fold_tokens, max_events=1 << 20)
        y = torch.empty((m, n), dtype=torch.float32, device="cuda")
        if ft_mode != ftgemm.FT_OFF:
            ctx.encode_weights(w)
        ctx.forward(x, w, y, flt)
        rep = ctx.report()
        out = y.cpu().numpy()
        ctx.close()
        return out, rep

    clean, _ = run(ftgemm.FT_OFF, None)
    damaged, _ = run(ftgemm.FT_OFF, fa)
    with np.errstate(all="ignore"):
        dmg = np.abs(damaged[fa[:, 0], fa[:, 1]] - clean[fa[:, 0], fa[:, 1]])
    harmful = ~(dmg <= LINEAR_HARM)                       # non-finite counts as harmful
    curve = []
    for tau in grid:
        _, rep0 = run(ftgemm.FT_CORRECT, None, tau)
        fixed, rep = run(ftgemm.FT_CORRECT, fa, tau)
        ev = {(int(e["row"]), int(e["col"])) for e in rep.events}
        hit = np.array([(int(f[0]), int(f[1])) in ev for f in fa])
        with np.errstate(all="ignore"):
            left = np.abs(fixed[fa[:, 0], fa[:, 1]] - clean[fa[:, 0], fa[:, 1]])
        curve.append({"tau_rel": float(tau), "harmful": int(harmful.sum()), "harmful_detected": int((harmful & hit).sum()),
                      "harmful_repaired": int((harmful & (left <= LINEAR_HARM)).sum()),
                      "benign": int((~harmful).sum()), "benign_detected": int((~harmful & hit).sum()),
                      "false_alarms": int(rep0.n_events), "residual_max": float(rep0.residual_max),
                      "checks": int(m) * 8 * ((n + 255) // 256) if not fold_tokens else int(n) * 8 * ((m + 255) // 256)})
    return {"m": m, "n": n, "k": k, "faults": int(len(fa)), "curve": curve}


def linear_markdown(res: Dict[str, object]) -> str:
    out = ["| tau_rel | harmful flips flagged | ... repaired | harmless flips flagged | events on a fault-free run (of checks) | largest fault-free residual / threshold |",
           "|---|---|---|---|---|---|"]
    for c in res["curve"]:
        out.append(f"| 2^{int(np.log2(c['tau_rel']))} | {c['harmful_detected']}/{c['harmful']} | {c['harmful_repaired']}/{c['harmful']} | "
                   f"{c['benign_detected']}/{c['benign']} | {c['false_alarms']} of {c['checks']} | {c['residual_max']:.3g} |")
    return "\n".join(out)

def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--batch", type=int, default=2)
    ap.add_argument("--heads", type=int, default=8)
    ap.add_argument("--seq", type=int, default=2048)
    ap.add_argument("--head-dim", type=int, default=128)
    ap.add_argument("--dtype", choices=("fp16", "bf16"), default="bf16")
    ap.add_argument("--non-causal", action="store_true")
    ap.add_argument("--faults-per-head", type=int, default=48)
    ap.add_argument("--seed", type=lambda s: int(s, 0), default=0xC0FE)
    ap.add_argument("--rowsum-fold", action="store_true",
                    help="protect the row-sum as an extra fold of checksum class 0 (exact check) instead of the range restriction")
    ap.add_argument("--per-step", type=int, choices=(0, 1, 2), default=0,
                    help="bit-error-rate sweep: 1 = verification after every step, 2 = the same with the softmax "
                         "protected by duplication (0 = unified verification)")
    ap.add_argument("--stride", type=int, choices=(8, 1), default=8,
                    help="bit-error-rate sweep: 1 = the traditional checksum (one class per tile row) instead of the "
                         "stride-8 tensor checksum")
    ap.add_argument("--linear", action="store_true", help="threshold sweep of the linear layer's check instead of attention")
    ap.add_argument("--fold-tokens", action="store_true", help="--linear: checksums over the token rows")
    ap.add_argument("--ber", type=float, nargs="*", default=None,
                    help="run the bit-error-rate sweep at these rates instead of the threshold sweep")
    args = ap.parse_args()
    dtype = synth.F16 if args.dtype == "fp16" else synth.BF16
    if args.linear:
        res = linear_sweep(2048, 2048, 1024, dtype, 512, args.seed, args.fold_tokens)
        print(f"workload: linear layer 2048 tokens, 1024 -> 2048 features, {args.dtype}, X ~ N(0,1), W ~ N(0,1/k), seed {args.seed:#x}; "
              f"{res['faults']} flips of bits 0..31, one per output row and column; checksums over the "
              f"{'token' if args.fold_tokens else 'weight'} rows; harmful = moves its output by more than {LINEAR_HARM}")
        print(linear_markdown(res))
        return
    shape = (args.batch, args.heads, args.seq, args.head_dim)
    q, k, v = synth.gen_qkv(shape, dtype, args.seed)
    if args.ber is not None:
        bers = args.ber or [1e-7, 1e-6, 1e-5, 1e-4]
        print(f"workload: batch {args.batch}, heads {args.heads}, seq {args.seq}, head_dim {args.head_dim}, {args.dtype}, "
              f"{'non-causal' if args.non_causal else 'causal'}, N(0,1) inputs, seed {args.seed:#x}; "
              f"{population(*shape, not args.non_causal, 64)} fp32 intermediates per pass; row-sum protection: "
              f"{'extra checksum fold' if args.rowsum_fold else 'range restriction'}; verification: "
              f"{('unified', 'after every step', 'after every step, duplicated softmax')[args.per_step]}; checksum: "
              f"{'stride 8 (tensor checksum)' if args.stride == 8 else 'stride 1 (traditional, one class per tile row)'}")
        print(ber_markdown(ber_sweep(q, k, v, dtype, not args.non_causal, bers, args.seed + 2, args.rowsum_fold, args.per_step,
                                     args.stride)))
        return
    faults = draw_faults(*shape, not args.non_causal, 64, args.faults_per_head, args.seed + 1)
    res = sweep(q, k, v, dtype, not args.non_causal, faults)
    print(f"workload: batch {args.batch}, heads {args.heads}, seq {args.seq}, head_dim {args.head_dim}, {args.dtype}, "
          f"{'non-causal' if args.non_causal else 'causal'}, N(0,1) inputs, seed {args.seed:#x}")
    print(to_markdown(res))


if __name__ == "__main__":
    main()
