"""Queueing model of a streaming inference server (paper, Section "Streaming inference").

The server is modelled as an M/D/1 queue: one server with constant compute latency D per
request (serving rate mu = 1/D), requests arriving as a Poisson process of rate lam.  The mean
total latency of a request is its compute latency plus its mean wait in the queue,

    omega = 1/mu + lam / (2 mu (mu - lam)),        lam < mu.

A request here is one batched chunk (all channels of the batch advance by one chunk); with
chunks of `chunk_seconds` of audio, `groups` such batches served in real time arrive at rate
lam = groups / chunk_seconds.
"""
from __future__ import annotations

import math


def total_latency(compute_latency: float, arrival_rate: float) -> float:
    """Mean total latency (same unit as compute_latency) at the given arrival rate (requests per
    unit of time).  Infinite when the server is saturated (arrival_rate >= 1 / compute_latency)."""
    if compute_latency <= 0.0:
        raise ValueError("compute latency must be positive")
    if arrival_rate < 0.0:
        raise ValueError("arrival rate must be non-negative")
    mu = 1.0 / compute_latency
    if arrival_rate >= mu:
        return math.inf
    return 1.0 / mu + arrival_rate / (2.0 * mu * (mu - arrival_rate))


def load_table(compute_latency_s: float, chunk_seconds: float, channels_per_request: int,
               loads=(0.1, 0.25, 0.5, 0.75, 0.9)):
    """For each utilisation rho = lam / mu: the real-time streams it corresponds to and the
    model's queue and total latency in milliseconds."""
    rows = []
    for rho in loads:
        lam = rho / compute_latency_s
        total = total_latency(compute_latency_s, lam)
        rows.append({"load": rho,
                     "streams_at_realtime": int(lam * chunk_seconds * channels_per_request),
                     "queue_ms": (total - compute_latency_s) * 1e3,
                     "total_ms": total * 1e3})
    return rows
