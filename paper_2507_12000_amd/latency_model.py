"""Closed-form communication and inference latency of DSD and DSSD (Sec. 2.2, 2.3 and 3.1 of
arXiv 2507.12000), fed either by an acceptance rate alpha or by the per-session `rejected`
flags a verification step produced (the paper's indicator a: a = 1 iff a draft was rejected,
which is when DSSD has to send one vocabulary distribution down).

Times in seconds, rates in bit/s, b_prob in bits per probability value.
"""
from dataclasses import dataclass


@dataclass(frozen=True)
class Link:
    t_ntt: float            # non-transmission time per round (processing, propagation, queuing)
    rate_up: float          # R_up
    rate_down: float        # R_down


def distribution_bits(vocab_size: int, b_prob: int) -> float:
    """Payload of one vocabulary distribution: |V| * b_prob."""
    return float(vocab_size) * float(b_prob)


def dsd_comm_time(gamma: int, vocab_size: int, b_prob: int, link: Link) -> float:
    """Sec. 2.2: the uplink carries gamma distributions; T_comm = gamma |V| b_prob / R_up + T_NTT."""
    return gamma * distribution_bits(vocab_size, b_prob) / link.rate_up + link.t_ntt


def dssd_comm_time_given_a(a: float, vocab_size: int, b_prob: int, link: Link) -> float:
    """Sec. 3.1: T_down = a |V| b_prob / R_down with a = 1 iff there was a rejection (or the mean
    of that indicator over many rounds); T_comm = T_down + T_NTT."""
    return a * distribution_bits(vocab_size, b_prob) / link.rate_down + link.t_ntt


def reject_probability(alpha: float, gamma: int) -> float:
    """Probability that a round of gamma drafts contains a rejection: 1 - alpha^gamma."""
    return 1.0 - alpha ** gamma


def dssd_expected_comm_time(alpha: float, gamma: int, vocab_size: int, b_prob: int, link: Link) -> float:
    """Sec. 3.1: E[T_comm] = (1 - alpha^gamma) |V| b_prob / R_down + T_NTT."""
    return dssd_comm_time_given_a(reject_probability(alpha, gamma), vocab_size, b_prob, link)


def dssd_comm_bounds(vocab_size: int, b_prob: int, link: Link):
    """Corollary of Sec. 3.1: T_NTT <= T_comm <= T_down + T_NTT."""
    return link.t_ntt, distribution_bits(vocab_size, b_prob) / link.rate_down + link.t_ntt


def inference_time(gamma: int, t_slm: float, t_llm: float, t_comm: float) -> float:
    """Sec. 2.3: one draft-verify round costs gamma T_SLM + T_LLM + T_comm."""
    return gamma * t_slm + t_llm + t_comm


def dssd_comm_time_from_flags(rejected, vocab_size: int, b_prob: int, link: Link) -> float:
    """Mean DSSD communication time over the rounds whose `rejected` flags are given (any
    iterable of 0/1, e.g. the accepted-or-not record of a verification step)."""
    flags = [int(x) for x in rejected]
    return dssd_comm_time_given_a(sum(flags) / max(len(flags), 1), vocab_size, b_prob, link)
