"""Comparison of csv_decode_step outputs with the CPU oracle, with tie-band accounting.

The oracle decides in float64, the kernels in float32.  A comparison whose two sides are closer than
TAU * max(1,|x|,|y|) may legitimately flip; the oracle reports the margin of every comparison it made.
  - out of band: flags, rounds, rows, opened cluster SET, and ordered top-k ids must be identical;
  - in band: either outcome is accepted, but what the GPU returns must still be valid for the set of
    clusters it opened (top-k of that set, its log-sum-exp, certificates sound against brute force).
"""
from __future__ import annotations

import numpy as np

from oracle import csv_oracle as O

TAU = 1e-5          # relative tie band for decisions
LOGIT_RTOL = 1e-3   # bar for logits (float32 accumulation), relative to max(1,|l|)
LOGIT_TIGHT = 2e-5  # what the kernels are actually expected to achieve; reported, asserted


def tau(scale: float) -> float:
    return TAU * scale


class Tally:
    def __init__(self):
        self.exact = self.inband = self.id_ties = 0
        self.mismatch: list[str] = []
        self.max_logit_err = 0.0
        self.max_lse_err = 0.0
        self.fallbacks = 0
        self.rows = 0
        self.n = 0
        self.relaxed = 0          # sequences accepted at the relaxed tolerance
        self.late_rounds = 0      # sequences that went through more than two scoring rounds

    def summary(self) -> str:
        return (f"exact={self.exact} in-band={self.inband} id-ties={self.id_ties} mismatch={len(self.mismatch)} "
                f"fallback={self.fallbacks}/{self.n} relaxed={self.relaxed} late={self.late_rounds} mean_rows={self.rows / max(self.n, 1):.1f} "
                f"max_logit_err={self.max_logit_err:.2e} max_lse_err={self.max_lse_err:.2e}")


def _check_ids(tag, t: Tally, L_row, S_rows, k, g_ids, g_vals):
    """Rank-wise: the GPU's r-th id is the oracle's r-th id over the same row set, or its exact logit is within
    the tie band of the oracle's r-th logit.  Returns True when ids are identical."""
    exp_ids, exp_vals = O.topk_bruteforce(L_row[S_rows], k, S_rows) if S_rows is not None else O.topk_bruteforce(L_row, k)
    if len(set(g_ids.tolist())) != k:
        t.mismatch.append(f"{tag}: duplicate or missing ids {g_ids.tolist()}")
        return False
    same = np.array_equal(g_ids, exp_ids)
    if S_rows is not None:
        inS = np.isin(g_ids, S_rows)
        if not inS.all():
            t.mismatch.append(f"{tag}: ids outside the opened rows")
            return False
    for r in range(k):
        lv = L_row[g_ids[r]]
        err = abs(float(g_vals[r]) - lv) / max(1.0, abs(lv))
        t.max_logit_err = max(t.max_logit_err, err)
        if err > LOGIT_TIGHT:
            t.mismatch.append(f"{tag}: logit[{r}] off by {err:.2e} (rel)")
            return False
        if g_ids[r] != exp_ids[r] and abs(lv - exp_vals[r]) > tau(max(1.0, abs(lv), abs(exp_vals[r]))):
            t.mismatch.append(f"{tag}: rank {r} id {g_ids[r]} (l={lv:.6f}) vs oracle {exp_ids[r]} (l={exp_vals[r]:.6f})")
            return False
    return same


def compare_step(tag: str, t: Tally, orc: list, gpu: dict, L: np.ndarray, index: O.OracleIndex, k: int, eps: float,
                 K_max: int, combine: int) -> None:
    """orc: oracle decode_step output (list per sequence); gpu: numpy arrays of the step outputs; L: oracle logits [B,V]."""
    B = len(orc)
    for b in range(B):
        t.n += 1
        r = orc[b]
        tg = f"{tag} b={b}"
        gf = int(gpu["flags"][b])
        if r["flags"] == O.FLAG_INVALID:
            if gf != O.FLAG_INVALID:
                t.mismatch.append(f"{tg}: expected INVALID, got flags={gf}")
            else:
                t.exact += 1
            continue
        band = [name for name, (gap, scale) in r["margins"].items() if name != "id_gap" and gap < tau(scale)]
        g_fb = bool(gf & O.FLAG_FALLBACK)
        t.fallbacks += g_fb
        g_rows, g_ncl, g_rounds = int(gpu["n_rows"][b]), int(gpu["n_clusters"][b]), int(gpu["rounds"][b])
        t.rows += g_rows
        t.relaxed += bool(gf & O.FLAG_SOFTMAX_RELAXED)
        t.late_rounds += g_rounds > 2
        same_dec = (gf == r["flags"] and g_rows == r["n_rows"] and g_ncl == r["n_clusters"] and g_rounds == r["rounds"])
        if g_fb:
            S_rows = None
            sel = None
        else:
            sel = gpu["sel"][b][:g_ncl]
            same_dec = same_dec and set(sel.tolist()) == set(r["clusters"].tolist())
            S_rows = np.concatenate([index.rows(c) for c in sel]) if g_ncl else np.empty(0, dtype=np.int64)
        if not same_dec and not band:
            t.mismatch.append(f"{tg}: decisions differ out of band: gpu(flags={gf}, rows={g_rows}, cl={g_ncl}, rounds={g_rounds}) "
                              f"oracle(flags={r['flags']}, rows={r['n_rows']}, cl={r['n_clusters']}, rounds={r['rounds']}) "
                              f"margins={r['margins']}")
            continue
        # validity of what the GPU returned, for the set it opened
        U = r["U"]
        if not g_fb:
            if S_rows.size != g_rows:
                t.mismatch.append(f"{tg}: n_rows {g_rows} != rows of opened clusters {S_rows.size}")
                continue
            if g_rows > K_max:
                t.mismatch.append(f"{tg}: {g_rows} rows scored above the budget {K_max}")
                continue
            mask = np.ones(index.C, bool); mask[sel] = False
            rest = U[mask & (index.n > 0)]
            if rest.size and sel.size and rest.max() > U[sel].min() + tau(max(1.0, abs(rest.max()))):
                t.mismatch.append(f"{tg}: opened set is not a prefix of the bound order")
                continue
        Lrow = L[b]
        lse_ref = O.logsumexp(Lrow if g_fb else Lrow[S_rows])
        lerr = abs(float(gpu["lse"][b]) - lse_ref) / max(1.0, abs(lse_ref))
        t.max_lse_err = max(t.max_lse_err, lerr)
        if lerr > LOGIT_TIGHT:
            t.mismatch.append(f"{tg}: lse off by {lerr:.2e}")
            continue
        ids_same = True
        if k >= 1:
            nbad = len(t.mismatch)
            ids_same = _check_ids(tg, t, Lrow, S_rows, k, gpu["ids"][b].astype(np.int64), gpu["logits"][b])
            if len(t.mismatch) > nbad:
                continue
            # Theorem 1: a top-k certificate must agree with brute force over the whole vocabulary
            if gf & O.FLAG_TOPK_CERT:
                nb = len(t.mismatch)
                _check_ids(tg + " (vs full vocabulary)", t, Lrow, None, k, gpu["ids"][b].astype(np.int64), gpu["logits"][b])
                if len(t.mismatch) > nb:
                    continue
        if (gf & O.FLAG_SOFTMAX_CERT) and not g_fb and eps < 1:
            inS = np.zeros(index.V, bool); inS[S_rows] = True
            p_out = float(np.exp(Lrow[~inS] - O.logsumexp(Lrow)).sum())
            if p_out > eps * (1 + 1e-6):
                t.mismatch.append(f"{tg}: softmax certificate set but outside mass {p_out:.3e} > eps")
                continue
        if (gf & O.FLAG_SOFTMAX_RELAXED) and eps < 0.5:
            inS = np.zeros(index.V, bool); inS[S_rows] = True
            p_out = float(np.exp(Lrow[~inS] - O.logsumexp(Lrow)).sum())
            if g_fb or (gf & O.FLAG_SOFTMAX_CERT) or p_out > 2 * eps * (1 + 1e-6):
                t.mismatch.append(f"{tg}: relaxed flag set but flags={gf}, outside mass {p_out:.3e} vs 2 eps")
                continue
        if same_dec:
            if ids_same:
                t.exact += 1
            else:
                t.id_ties += 1
        else:
            t.inband += 1


def gpu_step_to_numpy(buf) -> dict:
    return {"ids": buf.ids.cpu().numpy(), "logits": buf.logits.cpu().numpy(), "lse": buf.lse.cpu().numpy(),
            "flags": buf.flags.cpu().numpy(), "n_rows": buf.n_rows.cpu().numpy(),
            "n_clusters": buf.n_clusters.cpu().numpy(), "rounds": buf.rounds.cpu().numpy(),
            "sel": buf.sel_clusters.cpu().numpy() if buf.sel_clusters is not None else None}
