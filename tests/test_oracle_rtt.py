"""Pins of the latency model (oracle/rtt.py) and of the library's host-side calculator against
the numbers the paper prints (tests/golden/rtt_projection_seq.txt)."""
import os

import pytest

from oracle import rtt

HERE = os.path.dirname(os.path.abspath(__file__))


def _rows():
    out = []
    for ln in open(os.path.join(HERE, "golden", "rtt_projection_seq.txt")):
        ln = ln.strip()
        if ln and not ln.startswith("#"):
            out.append(ln.split())
    return out


def test_sequential_projection_columns_are_reproduced_to_the_printed_digit():
    rows = [r for r in _rows() if r[0] in ("7B", "12B")]
    assert len(rows) == 15
    for _, fixed, r, want in rows:
        got = rtt.projected_tok_s(1.0, float(r), float(fixed))
        assert round(got, 1) == float(want), (fixed, r, got, want)


def test_decomposition_tables_are_consistent_with_the_model():
    for row in (r for r in _rows() if r[0] == "decomp"):
        net, local, cloud, ser, wall, fixed = map(float, row[2:8])
        shares = list(map(float, row[8:11]))
        # the printed entries are rounded to 0.1 ms: the identities hold to a few roundings
        assert abs(rtt.fixed_overhead_ms(wall, net) - fixed) <= 0.15
        assert abs((local + cloud + ser) - fixed) <= 0.25
        assert abs(rtt.per_step_ms(net, fixed) - wall) <= 0.15
        for part, pct in zip((net, local, cloud), shares):
            assert round(100.0 * part / wall) == pct


def test_lookahead_entry_and_sequential_85ms():
    for row in _rows():
        if row[0] == "la":
            assert round(rtt.projected_tok_s(float(row[2]), float(row[4]), float(row[3])), 1) == float(row[5])
        if row[0] == "seq85":
            assert round(rtt.projected_tok_s(1.0, float(row[3]), float(row[2])), 1) == float(row[4])


def test_model_identities():
    # a dropped term, a swapped operand or a unit slip fails one of these
    assert rtt.projected_tok_s(1.0, 0.0, 1000.0) == 1.0
    assert rtt.projected_tok_s(2.0, 250.0, 250.0) == 4.0
    assert rtt.projected_tok_s(1.0, 100.0, 0.0) != rtt.projected_tok_s(1.0, 0.0, 50.0)
    assert rtt.fixed_overhead_ms(rtt.per_step_ms(33.0, 9.5), 33.0) == 9.5
    # Section 4.2: k tokens per converged block; one iteration per token is sequential decoding at zero overhead
    assert rtt.jacobi_tok_s(4, 4, 100.0) == rtt.projected_tok_s(1.0, 100.0, 0.0)
    assert rtt.jacobi_tok_s(8, 2, 100.0) == 40.0


def test_library_calculator_matches_the_oracle():
    from paper_2602_16760_amd import binding as B
    for acc, r, fixed in ((1.0, 20.0, 42.9), (1.17, 80.0, 42.9), (2.5, 0.0, 3.7), (1.0, 150.0, 46.3)):
        assert B.la_rtt_project(acc, r, fixed) == pytest.approx(rtt.projected_tok_s(acc, r, fixed), rel=1e-15)
    assert B.la_rtt_fixed_overhead(120.2, 77.4) == pytest.approx(rtt.fixed_overhead_ms(120.2, 77.4), rel=1e-15)
    assert B.la_jacobi_project(8, 2.0, 100.0) == pytest.approx(rtt.jacobi_tok_s(8, 2.0, 100.0), rel=1e-15)
    for bad in ((1.0, -1.0, 3.0), (0.0, 1.0, 1.0), (1.0, 0.0, 0.0)):
        with pytest.raises(B.LaError):
            B.la_rtt_project(*bad)
