"""CPU oracle for the paper's latency model and the sender queue's ordering.

TEST INFRASTRUCTURE ONLY (see oracle/oracle.py).  Plain restatements of:
  * the latency of cloud autoregressive decoding, edge-cloud speculative decoding and
    speculative decoding with early exits (Experiments, table "Latency calculation", with the
    notation table's symbols);
  * the projected speed-up of early exits over plain speculative decoding when communication
    and thread synchronisation cost nothing (Appendix "Speedup Projection Analysis", Eq. 9);
  * the order in which the server's SENDER releases exit results: by confidence score,
    s = the largest confidence among the tokens of the exit's result (Appendix "System
    Design", Algorithm 2; confidence = Eq. 4).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple


def latency_ar(n: int, T_q: float, T_c: float) -> float:
    """Cloud autoregressive decoding of n tokens: the request and the answer cross the
    network once, every token costs one pass of the target model."""
    return 2.0 * T_c + n * T_q


def latency_sd(n: int, tau: float, gamma: int, T_p: float, T_q: float, T_c: float) -> float:
    """Edge-cloud speculative decoding: n / tau rounds, each drafting gamma tokens, crossing
    the network twice and verifying once."""
    return (n / tau) * (2.0 * T_c + gamma * T_p + T_q)


def latency_fsd(n: int, tau: float, gamma: int, T_p: float, T_q: float, T_c: float, r: float, T_r: float) -> float:
    """With early exits: a round drafts only on a cache miss (rate r); on a hit it pays the
    thread synchronisation T_r instead."""
    return (n / tau) * (2.0 * T_c + r * gamma * T_p + (1.0 - r) * T_r + T_q)


def projected_speedup(gamma: int, c: float, r: float) -> float:
    """Eq. 9: SD -> FSD speed-up per round for T_c = T_r = 0, c = T_p / T_q."""
    return (gamma * c + 1.0) / (r * gamma * c + 1.0)


def exit_score(conf_rows: Sequence[float], accept_len: int) -> float:
    """Score of one exit's result: its tokens are rows 0..accept_len of the exit head."""
    return max(float(x) for x in conf_rows[: accept_len + 1])


def sender_order(exit_conf: Sequence[Sequence[float]], exit_accept_len: Sequence[int]) -> Tuple[List[int], List[float]]:
    """All exits of a pass in the order a full queue releases them: highest score first,
    equal scores in exit order."""
    scores = [exit_score(exit_conf[e], int(exit_accept_len[e])) for e in range(len(exit_accept_len))]
    order = sorted(range(len(scores)), key=lambda e: (-scores[e], e))
    return order, [scores[e] for e in order]
