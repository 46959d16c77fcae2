"""Latency model of the split deployment (float64): test infrastructure, see the package header.

Section 6.3 splits the wall time of one decode step into the network round trip and everything
that does not depend on the network (cloud compute, local compute, serialization), and projects
throughput at other round-trip times from the tokens a step commits on average, which does not
depend on the network either.  Section 4.2 gives the corresponding relation for Jacobi decoding.
All times in milliseconds, throughput in tokens per second.
"""


def per_step_ms(rtt_ms: float, fixed_ms: float) -> float:
    """Wall time of one step: round trip plus fixed overhead (Section 6.3, latency decomposition)."""
    return float(rtt_ms) + float(fixed_ms)


def fixed_overhead_ms(per_step_wall_ms: float, rtt_ms: float) -> float:
    """The part of a measured step that the network does not account for (Section 6.3)."""
    return float(per_step_wall_ms) - float(rtt_ms)


def projected_tok_s(tokens_per_step: float, target_rtt_ms: float, fixed_ms: float) -> float:
    """Throughput projected at another round-trip time (Section 6.3, projection model):
    tokens committed per step over the step's wall time in seconds."""
    return float(tokens_per_step) / (per_step_ms(target_rtt_ms, fixed_ms) / 1000.0)


def jacobi_tok_s(k: int, iterations: float, rtt_ms: float) -> float:
    """Section 4.2: a block of k tokens that converges after `iterations` round trips."""
    return float(k) / (float(iterations) * float(rtt_ms) / 1000.0)
