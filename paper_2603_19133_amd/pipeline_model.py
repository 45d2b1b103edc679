"""The paper's analytic model of the edge-cloud pipeline (Sections 3.2 and 3.4, Eq. 1-3 and 5-10), as host code.

It turns what this library measures -- verified draft positions per second of the sampling path -- and an
acceptance rate into the quantities the paper reasons with: expected tokens per cycle, cycle time of the
synchronous and of the asynchronous schedule, throughput and speedup.  Nothing here runs on the GPU and
nothing here is on the timed path; times are in seconds, rates in tokens per second.

    gamma     draft length per cycle            alpha     per-token acceptance probability
    t_draft   time to draft gamma tokens        t_rtt     network round trip
    t_verify  time of the cloud's verification  t_pre     lead of a pre-verify (Fast Verification)
"""
from __future__ import annotations

import numpy as np


def expected_length(alpha: float, gamma: int) -> float:
    """Eq. 5: tokens per cycle, L truncated geometric on 1..gamma: (1 - alpha^gamma) / (1 - alpha)."""
    if not (0.0 <= alpha <= 1.0) or gamma < 1:
        raise ValueError("alpha in [0,1], gamma >= 1")
    return float(gamma) if alpha == 1.0 else (1.0 - alpha ** gamma) / (1.0 - alpha)


def length_distribution(alpha: float, gamma: int) -> np.ndarray:
    """P(L = k), k = 1..gamma: k-1 acceptances and a rejection, or everything up to the last position."""
    k = np.arange(1, gamma + 1)
    p = alpha ** (k - 1) * (1.0 - alpha)
    p[-1] = alpha ** (gamma - 1)
    return p


def latency_sync(t_draft: float, t_rtt: float, t_verify: float) -> float:
    """Eq. 1 / Eq. 6: stop-and-wait cycle."""
    return t_draft + t_rtt + t_verify


def latency_async_full_hit(t_draft: float, t_rtt: float, t_verify: float) -> float:
    """Eq. 2: drafting of cycle i+1 overlaps the verification of cycle i."""
    return max(t_draft, t_rtt + t_verify)


def bubble(t_draft: float, t_rtt: float, t_verify: float, t_pre: float = 0.0) -> float:
    """Eq. 3: idle time left in the pipeline with a pre-verify lead of t_pre."""
    return max(0.0, t_rtt + t_verify - t_draft - t_pre)


def throughput_sync(alpha: float, gamma: int, t_draft: float, t_rtt: float, t_verify: float) -> float:
    """Eq. 7."""
    return expected_length(alpha, gamma) / latency_sync(t_draft, t_rtt, t_verify)


def expected_time_async(alpha: float, gamma: int, t_draft: float, t_rtt: float, t_verify: float) -> float:
    """Eq. 8-9: a full hit (probability alpha^gamma) costs the overlapped time, a miss the serial one."""
    hit = alpha ** gamma
    return hit * latency_async_full_hit(t_draft, t_rtt, t_verify) + (1.0 - hit) * latency_sync(t_draft, t_rtt, t_verify)


def throughput_async(alpha: float, gamma: int, t_draft: float, t_rtt: float, t_verify: float) -> float:
    return expected_length(alpha, gamma) / expected_time_async(alpha, gamma, t_draft, t_rtt, t_verify)


def speedup(alpha: float, gamma: int, t_draft: float, t_rtt: float, t_verify: float) -> float:
    """S = R_async / R_sync; Eq. 10 is its limit for alpha -> 1 with t_draft >= t_rtt + t_verify."""
    return throughput_async(alpha, gamma, t_draft, t_rtt, t_verify) / throughput_sync(alpha, gamma, t_draft, t_rtt, t_verify)


def speedup_limit(t_draft: float, t_rtt: float, t_verify: float) -> float:
    """Eq. 10."""
    return 1.0 + (t_rtt + t_verify) / t_draft


def sampling_time(n_positions: int, positions_per_s: float) -> float:
    """Share of t_verify that the sampling path (compress + verify + residual) takes for n_positions draft
    positions at the measured rate (the target model's forward pass is the rest of t_verify)."""
    return n_positions / positions_per_s


def simulate(alpha: float, gamma: int, t_draft: float, t_rtt: float, t_verify: float, cycles: int,
             rng: np.random.Generator) -> tuple[float, float]:
    """Monte-Carlo of the two-case process behind Eq. 8: every position is accepted independently with
    probability alpha; a cycle whose draft is accepted whole costs the overlapped time, any other the serial
    one.  Returns (tokens per cycle, tokens per second)."""
    acc = rng.random((cycles, gamma)) < alpha
    all_hit = acc.all(axis=1)
    first_rej = np.where(all_hit, gamma, acc.argmin(axis=1))
    tokens = np.where(all_hit, gamma, first_rej + 1)          # accepted ones and the corrected token, capped at gamma
    time = np.where(all_hit, latency_async_full_hit(t_draft, t_rtt, t_verify), latency_sync(t_draft, t_rtt, t_verify))
    return float(tokens.mean()), float(tokens.sum() / time.sum())


def truncated_gammas(gamma_max: int, t_token: float, jitter: float, budget: float, n: int,
                     rng: np.random.Generator) -> np.ndarray:
    """Latency-aware truncation (Section 3.3, last paragraph): a segment is cut and sent as soon as its drafting
    time exceeds `budget`.  Token times are t_token * (1 + jitter * Exp(1)); returns the n segment lengths
    (1..gamma_max), the source of ragged draft lengths."""
    t = t_token * (1.0 + jitter * rng.exponential(size=(n, gamma_max)))
    done = np.cumsum(t, axis=1)
    return np.clip((done <= budget).sum(axis=1), 1, gamma_max).astype(np.int32)
