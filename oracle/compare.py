"""Comparison rules between a candidate result and the CPU oracle -- TEST INFRASTRUCTURE.

Holds only the acceptance rules (no part of the method): which index sets count as
equal to the oracle's under rounding of the scores, and the output tolerances.

Index-set rule.  Let s be the oracle's float64 scores of one (batch, kv head),
s_(k) and s_(k+1) its k-th and (k+1)-th largest (ties toward the lower index), and
gap_rel = (s_(k) - s_(k+1)) / max(|s_(k)|, |s_(k+1)|, 1e-30).
  * gap_rel > 1e-3: the candidate set must equal the oracle set exactly.
  * otherwise, with tau = 1e-3 * max(|s_(k)|, |s_(k+1)|): every j with
    s_j > s_(k) + tau must be in the candidate set, every member of the candidate
    set must have s_j >= s_(k) - tau, and the set must have k_b distinct in-range
    members; the number of tokens with |s_j - s_(k)| <= tau (the boundary tie
    count) is reported.
Output tolerance: max-abs 2e-3 for fp16 caches, 1e-5 for fp32 caches.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np

GAP_REL = 1e-3
OUT_TOL = {np.dtype(np.float16): 2e-3, np.dtype(np.float32): 1e-5}


@dataclass
class SetReport:
    problems: int = 0
    exact_rule: int = 0          # problems judged by exact equality
    band_rule: int = 0           # problems judged by the tie band
    equal_sets: int = 0          # candidate set == oracle set
    boundary_ties: List[int] = field(default_factory=list)   # |band| per band-rule problem
    failures: List[str] = field(default_factory=list)

    @property
    def ok(self) -> bool:
        return not self.failures

    def summary(self) -> dict:
        bt = self.boundary_ties
        return dict(problems=self.problems, exact_rule=self.exact_rule, band_rule=self.band_rule,
                    equal_sets=self.equal_sets,
                    boundary_ties_total=int(np.sum(bt)) if bt else 0,
                    boundary_ties_median=float(np.median(bt)) if bt else 0.0,
                    boundary_ties_max=int(np.max(bt)) if bt else 0,
                    failures=len(self.failures))


def check_index_sets(scores64: np.ndarray, k: int, vis_len, idx: np.ndarray, count: np.ndarray) -> SetReport:
    """Applies the index-set rule to every (b, g); also checks order, padding and count."""
    B, Hkv, Nv = scores64.shape
    rep = SetReport()
    for b in range(B):
        n = int(vis_len[b]) if vis_len is not None else Nv
        kb = min(k, n)
        for g in range(Hkv):
            rep.problems += 1
            tag = f"(b={b},g={g})"
            c = int(count[b, g])
            row = idx[b, g]
            if c != kb:
                rep.failures.append(f"{tag} count {c} != {kb}")
                continue
            sel = row[:c]
            if np.any(row[c:] != -1):
                rep.failures.append(f"{tag} slots past count are not -1")
            if c and (sel.min() < 0 or sel.max() >= n):
                rep.failures.append(f"{tag} index out of range")
                continue
            if np.any(np.diff(sel) <= 0):
                rep.failures.append(f"{tag} indices not strictly ascending")
                continue
            s = scores64[b, g, :n]
            order = np.lexsort((np.arange(n), -s))
            want = np.sort(order[:kb])
            same = np.array_equal(sel, want)
            rep.equal_sets += int(same)
            if kb == 0 or kb == n:
                rep.exact_rule += 1
                if not same:
                    rep.failures.append(f"{tag} trivial set differs")
                continue
            sk, sk1 = s[order[kb - 1]], s[order[kb]]
            ref = max(abs(sk), abs(sk1), 1e-30)
            if (sk - sk1) / ref > GAP_REL:
                rep.exact_rule += 1
                if not same:
                    rep.failures.append(f"{tag} gap_rel {(sk - sk1) / ref:.2e} > 1e-3 but sets differ")
                continue
            rep.band_rule += 1
            tau = GAP_REL * max(abs(sk), abs(sk1))
            rep.boundary_ties.append(int(np.count_nonzero(np.abs(s - sk) <= tau)))
            must = np.nonzero(s > sk + tau)[0]
            if not np.all(np.isin(must, sel)):
                rep.failures.append(f"{tag} a token above the tie band is missing")
            if np.any(s[sel] < sk - tau):
                rep.failures.append(f"{tag} a token below the tie band was kept")
    return rep


def out_tolerance(dtype) -> float:
    return OUT_TOL[np.dtype(dtype)]
