"""Service-rate and queueing relations of the paper (host-side calculator).

These closed forms tie a measured prefill throughput and an exact-prefix hit
rate to a sustainable request rate (Sec. 2.4 and Appendix "queueing").  They
are plain arithmetic on host numbers; nothing here touches the GPU path.

Notation: L mean prompt length (tokens), h full-prompt token-level exact-prefix
hit rate, M mean wave size, R effective prefill throughput (tokens/s/request
slot), mu request-level service rate (requests/s), c2 squared coefficient of
variation of the per-request service time.
"""
from __future__ import annotations


def wave_service_time(L: float, h: float, R: float) -> float:
    """E[S_wave] = L (1 - h) / R  (Eq. 5, left)."""
    return L * (1.0 - h) / R


def service_rate(M: float, L: float, h: float, R: float) -> float:
    """mu = M R / (L (1 - h)) requests/s: a wave releases M completions (Eq. 5, right)."""
    return M / wave_service_time(L, h, R)


def calibrate_prefill_throughput(mu: float, M: float, L: float, h: float) -> float:
    """R that reproduces a sustained mu (Eq. 5 solved for R)."""
    return mu * L * (1.0 - h) / M


def service_ratio(M1, R1, L1, h1, M0, R0, L0, h0) -> float:
    """mu_1 / mu_0 as the product of batching, throughput, length and reuse factors (Eq. 6)."""
    return (M1 / M0) * (R1 / R0) * (L0 / L1) * ((1.0 - h0) / (1.0 - h1))


def service_gap(mu_lru: float, h_prism: float, h_lru: float) -> float:
    """mu_PRISM - mu_LRU = mu_LRU * dh / (1 - h_PRISM) with L, M, R held fixed (Eq. 7)."""
    return mu_lru * (h_prism - h_lru) / (1.0 - h_prism)


def stability_expansion(M: float, R: float, L: float, h_lru: float, dh: float) -> float:
    """Delta lambda* = (M R / L) * dh / ((1 - h_lru - dh)(1 - h_lru))  (Eq. 8)."""
    return (M * R / L) * dh / ((1.0 - h_lru - dh) * (1.0 - h_lru))


def full_prompt_gap(dh_reuse: float, L_reuse: float, L: float) -> float:
    """A hit-rate gap over the reusable tokens only, as a full-prompt token gap (Thm. 1, last line)."""
    return dh_reuse * L_reuse / L


def admission_wait(lam: float, mu: float, c2: float, dt_win: float = 0.0) -> float:
    """E[W_admit] = dt_win/2 + rho/(1-rho) * (1+c2)/2 * 1/mu  (Eq. 14); inf at rho >= 1."""
    rho = lam / mu
    if rho >= 1.0:
        return float("inf")
    return 0.5 * dt_win + rho / (1.0 - rho) * (1.0 + c2) / 2.0 / mu


def crossover_rate(mu: float, M: float, c2: float = 1.0) -> float:
    """lambda* = mu * 2M / (1 + c2 + 2M): where the queueing wait equals the wave duration (Eq. 15)."""
    return mu * 2.0 * M / (1.0 + c2 + 2.0 * M)


def effective_prefill_throughput(R: float, X: float, L_out: float, R_dec: float) -> float:
    """R_eff = R (1 - X L_out / R_dec): decode contention as an attenuation (Eq. 16)."""
    return R * (1.0 - X * L_out / R_dec)
