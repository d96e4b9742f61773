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


def attention_only_knee(layer_call_s: float, n_layers: int, M: float, L: float, h: float, c2: float = 1.0) -> dict:
    """The service knee that the measured attention path alone would allow.

    layer_call_s is the measured time of one layer call (paged KV append +
    prefill attention) for a wave of M requests with mean prompt length L and
    exact-prefix hit rate h.  A model of n_layers layers spends n_layers such
    calls per wave on attention, so with every other cost of the model left
    out (projections, MLP, sampling, decode) a wave takes n_layers *
    layer_call_s.  From there Eq. 5 gives the per-request prefill throughput
    R = L (1 - h) / E[S_wave] and the service rate mu = M / E[S_wave], and
    Eq. 15 the crossover lambda*.  These are ceilings of the attention path,
    not predictions for a serving system."""
    wave_s = n_layers * layer_call_s
    R = L * (1.0 - h) / wave_s
    mu = service_rate(M, L, h, R)
    return {"scope": "attention-only (KV append + prefill attention of every layer; nothing else of the model)",
            "wave_s": wave_s, "R_attn_tokens_per_s_per_request": R, "mu_requests_per_s": mu,
            "lambda_star_requests_per_s": crossover_rate(mu, M, c2), "M": M, "L": L, "h": h, "c2": c2,
            "n_layers": n_layers}
