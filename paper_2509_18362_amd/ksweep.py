"""Draft-length sweep (Sec. 3.5, Fig. 3): a MODEL of end-to-end speed-up against the number of draft steps K, built
from a measured time per draft step and an ASSUMED time of the target model's verification forward.

Nothing here runs the 7B model or the paper's benchmarks.  Inputs:
  * accept[j-1] = probability that draft position j is accepted given that all earlier ones were (conditional
    rates).  The default comes from the cumulative acceptance the paper reports for its head, 0.81 / 0.56 / 0.36 at
    positions 1-3 (Sec. 3.4; they sum with the bonus token to the reported tau = 2.73); positions beyond the third
    repeat the third conditional rate - an assumption, marked as such in the output.
  * t_mtp: seconds per K-step draft chain, measured by bench.py for every K = 1..7 (or one time per draft step, taken
    K times), t_accept: seconds for the acceptance kernel,
  * t_target: seconds of one target forward over K+1 positions (assumed constant in K: the verification of a few
    tokens is bandwidth-bound like a single-token step).
One cycle drafts K tokens, verifies them in one target forward and emits tau(K) = 1 + sum_j prod_{i<=j} accept[i]
tokens on average; plain decoding emits one token per target forward.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

PAPER_CUMULATIVE = (0.81, 0.56, 0.36)  # Sec. 3.4, acceptance at draft positions 1..3


def conditional_rates(k_max: int, cumulative: Sequence[float] = PAPER_CUMULATIVE) -> List[float]:
    cond, prev = [], 1.0
    for c in cumulative:
        cond.append(c / prev)
        prev = c
    while len(cond) < k_max:
        cond.append(cond[-1])  # assumption: later positions keep the last conditional rate
    return cond[:k_max]


def expected_tokens(k: int, cond: Sequence[float]) -> float:
    """tau(K): mean tokens emitted per cycle = accepted drafts + the target's own token."""
    tau, run = 1.0, 1.0
    for j in range(k):
        run *= cond[j]
        tau += run
    return tau


def sweep(t_mtp, t_accept: float, t_target: float, k_max: int = 7,
          cumulative: Sequence[float] = PAPER_CUMULATIVE) -> List[Dict[str, float]]:
    """t_mtp: seconds per draft step, or a sequence of MEASURED seconds per K-step chain for K = 1 .. k_max."""
    cond = conditional_rates(k_max, cumulative)
    rows = []
    for k in range(1, k_max + 1):
        tau = expected_tokens(k, cond)
        chain = t_mtp[k - 1] if hasattr(t_mtp, "__len__") else k * t_mtp
        cycle = t_target + chain + t_accept
        rows.append({"K": k, "tau": tau, "cycle_s": cycle, "speedup_vs_plain_decoding": tau * t_target / cycle,
                     "extrapolated_acceptance": k > len(cumulative)})
    return rows
