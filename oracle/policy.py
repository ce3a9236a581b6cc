"""Oracle for the state-update and stride-selection arithmetic around the verification step.

TEST INFRASTRUCTURE ONLY (see oracle.py).  Plain Python, fp64, written from the definitions:

  - step latency  T_step(K, R) = T_fixed(R) + K * T_marginal(R)                      (Sec. IV-B, refined latency model)
        T_fixed    = T_prop + T_base + T_down + O_header / R + beta
        T_marginal = alpha_edge + b / R + delta_cloud
  - stride        K* = argmax_{K in 1..K_max}  E[tokens | K] / T_step(K, R)           (Sec. IV-B objective; Alg. 2 step 1)
        E[tokens | K] = 1 + gamma_hat * K            (the numerator Alg. 2 prints: accepted drafts plus the correction token)
                      or 1 + sum_{i=1..K} gamma_hat^i (the geometric decay model Sec. IV-B names as the alternative)
        ties go to the smallest K
  - EMA           gamma_hat <- (1 - mu) * gamma_hat + mu * tau / K                    (Alg. 2 step 3), started at 0.8
  - pages         a session holding n positions owns ceil(n / page_size) pages; growing takes free pages, trimming after
                  a rollback returns the tail pages (Sec. IV-C: invalid KV pairs are discarded)
"""
from __future__ import annotations

from dataclasses import dataclass

LINEAR, GEOMETRIC = 0, 1
GAMMA_INIT = 0.8


@dataclass
class LatencyModel:
    alpha_edge: float      # s per drafted token on the edge
    beta: float            # s fixed edge cost
    bits_per_token: float  # b
    header_bits: float     # O_header
    t_prop: float          # s
    t_base: float          # s, cloud base cost
    delta_cloud: float     # s per verified token
    t_down: float          # s


def t_fixed(m: LatencyModel, rate: float) -> float:
    return m.t_prop + m.t_base + m.t_down + m.header_bits / rate + m.beta


def t_marginal(m: LatencyModel, rate: float) -> float:
    return m.alpha_edge + m.bits_per_token / rate + m.delta_cloud


def t_step(m: LatencyModel, rate: float, k: int) -> float:
    return t_fixed(m, rate) + k * t_marginal(m, rate)


def expected_tokens(gamma_hat: float, k: int, model: int) -> float:
    if model == LINEAR:
        return 1.0 + gamma_hat * k
    total = 1.0
    p = 1.0
    for _ in range(k):
        p *= gamma_hat
        total += p
    return total


def stride(m: LatencyModel, rate: float, gamma_hat: float, k_max: int, model: int):
    """(K*, objective at K*): tokens per second the model expects."""
    best_k, best = 1, -1.0
    for k in range(1, k_max + 1):
        f = expected_tokens(gamma_hat, k, model) / t_step(m, rate, k)
        if f > best:
            best_k, best = k, f
    return best_k, best


def ema(gamma_hat: float, tau: int, k: int, mu: float) -> float:
    return (1.0 - mu) * gamma_hat + mu * (tau / k)


class Pager:
    """Reference page bookkeeping: sets and lists, nothing clever."""

    def __init__(self, num_pages: int, page_size: int = 16):
        self.page_size = page_size
        self.free = list(range(num_pages - 1, -1, -1))   # popped from the end: lowest id first
        self.owned: dict[int, list[int]] = {}

    def reserve(self, session: int, n_positions: int) -> bool:
        have = self.owned.setdefault(session, [])
        need = -(-n_positions // self.page_size)
        if need - len(have) > len(self.free):
            return False
        while len(have) < need:
            have.append(self.free.pop())
        return True

    def trim(self, session: int, n_positions: int) -> int:
        have = self.owned.setdefault(session, [])
        keep = -(-n_positions // self.page_size)
        released = 0
        while len(have) > keep:
            self.free.append(have.pop())
            released += 1
        return released

    def release(self, session: int) -> int:
        return self.trim(session, 0)
