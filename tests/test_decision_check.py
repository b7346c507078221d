"""CPU tests of the decision comparison that the GPU parity tests use (tests/helpers.py).

The comparison may relax bit-exactness only where the oracle's statistic lies within the statistics tolerance
of a threshold (b_k for pass/fail, an integer for the ceiling, Alg. 1's If-branch), and even there only to the
answers the oracle itself gives inside that band.  Each case plants a wrong answer on the "GPU" side and checks
that the comparison rejects it; the oracle's own answers on either side of a threshold must be accepted.
"""
import pytest

import helpers as H
from paper_2412_21124_amd import synth

J, ETA = 4, 0.1


def make_ref(T, h):
    # T = (C / (J - 1)) / (eta^2 B / J^2) with B = 1  ->  C = T (J - 1) eta^2 / J^2
    B = 1.0
    C = T * (J - h.ddof) * h.eta * h.eta / (J * J)
    A = C + B / J
    ref = H.OracleOut(A, B, C, H.oracle_decide(A, B, C, J, h), J)
    assert ref.dec.T == pytest.approx(T, rel=1e-12)
    return ref


def res_of(passed, next_b, status=0):
    return {"pass": int(passed), "next_b": next_b, "status": status}


def rejected(res, ref, h):
    with pytest.raises(AssertionError):
        H.assert_decision_matches(res, ref, h)
    return True


def test_far_from_any_threshold_is_exact():
    h = synth.Hyper(eta=ETA, b_k=256, round_to=128, b_max=8192, ddof=1)
    ref = make_ref(1000.5, h)
    assert (ref.dec.passed, ref.dec.next_b) == (False, 1024)
    H.assert_decision_matches(res_of(0, 1024), ref, h)
    assert rejected(res_of(1, 256), ref, h)
    assert rejected(res_of(1, 1024), ref, h)
    assert rejected(res_of(0, 1152), ref, h)
    assert rejected(res_of(0, 896), ref, h)
    assert rejected(res_of(0, 1024, status=4), ref, h)


def test_near_an_integer_far_from_b_k_checks_pass_and_both_ceilings_only():
    # the case the earlier comparison let through: T next to an integer, nowhere near b_k
    h = synth.Hyper(eta=ETA, b_k=256, round_to=1, b_max=0, ddof=1)
    ref = make_ref(1000.0 + 1e-4, h)            # within 2e-5 relative of 1000
    assert (ref.dec.passed, ref.dec.next_b) == (False, 1001)
    H.assert_decision_matches(res_of(0, 1001), ref, h)
    H.assert_decision_matches(res_of(0, 1000), ref, h)   # the kernel's T may fall just below 1000
    assert rejected(res_of(1, 256), ref, h)              # pass may not flip: b_k is far away
    assert rejected(res_of(1, 1000), ref, h)
    assert rejected(res_of(0, 1002), ref, h)
    assert rejected(res_of(0, 999), ref, h)
    assert rejected(res_of(0, 256), ref, h)
    assert rejected(res_of(0, 100000), ref, h)           # "anything >= b_k" is not enough


def test_near_b_k_accepts_exactly_the_two_sides():
    h = synth.Hyper(eta=ETA, b_k=256, round_to=128, b_max=8192, ddof=1)
    for T in (256.0 - 1e-3, 256.0, 256.0 + 1e-3):
        ref = make_ref(T, h)
        H.assert_decision_matches(res_of(1, 256), ref, h)
        H.assert_decision_matches(res_of(0, 384), ref, h)
        assert rejected(res_of(0, 256), ref, h)          # failing without growing is neither side's answer
        assert rejected(res_of(1, 384), ref, h)
        assert rejected(res_of(0, 512), ref, h)


def test_equality_passes_and_just_outside_the_band_is_exact():
    h = synth.Hyper(eta=ETA, b_k=256, round_to=128, b_max=8192, ddof=1)
    ref = make_ref(256.0 * (1 + 1e-4), h)        # 5 band-widths above b_k
    assert not ref.dec.passed
    assert rejected(res_of(1, 256), ref, h)
    ref = make_ref(256.0 * (1 - 1e-4), h)
    assert ref.dec.passed
    assert rejected(res_of(0, 384), ref, h)


def test_large_statistic_band_spans_integers_but_not_everything():
    # from T = 25000 on the band 2e-5 T exceeds half a unit: every case used to count as "near"
    h = synth.Hyper(eta=ETA, b_k=256, round_to=1, b_max=0, ddof=1)
    ref = make_ref(40000.3, h)
    assert ref.dec.next_b == 40001
    for nb in (40000, 40001, 40002):
        H.assert_decision_matches(res_of(0, nb), ref, h)
    assert rejected(res_of(1, 256), ref, h)
    assert rejected(res_of(0, 39998), ref, h)
    assert rejected(res_of(0, 40004), ref, h)
    # with the rounding chain the same band collapses to one value
    h2 = synth.Hyper(eta=ETA, b_k=256, round_to=128, b_max=0, ddof=1)
    ref2 = make_ref(40000.3, h2)
    H.assert_decision_matches(res_of(0, 40064), ref2, h2)
    assert rejected(res_of(0, 40192), ref2, h2)
    assert rejected(res_of(0, 39936), ref2, h2)


def test_band_too_wide_to_enumerate_still_bounds_the_answer():
    h = synth.Hyper(eta=ETA, b_k=256, round_to=1, b_max=0, ddof=1)
    ref = make_ref(3.0e8 + 0.5, h)
    assert H.admissible_decisions(ref, h) is None
    H.assert_decision_matches(res_of(0, ref.dec.next_b + 5000), ref, h)
    assert rejected(res_of(0, ref.dec.next_b + 50000), ref, h)
    assert rejected(res_of(1, 256), ref, h)
    assert rejected(res_of(0, 256), ref, h)


def test_cap_and_status_bits_are_part_of_the_answer():
    h = synth.Hyper(eta=ETA, b_k=256, round_to=128, b_max=512, ddof=1)
    ref = make_ref(1000.5, h)
    assert (ref.dec.next_b, ref.dec.status) == (512, 4)
    H.assert_decision_matches(res_of(0, 512, status=4), ref, h)
    assert rejected(res_of(0, 512, status=0), ref, h)
    assert rejected(res_of(0, 1024, status=0), ref, h)
    # zero gradient norm with variance: infinite statistic, exact answer required
    B, C = 0.0, 1.0
    ref0 = H.OracleOut(C, B, C, H.oracle_decide(C, B, C, J, h), J)
    assert ref0.dec.T == float("inf")
    H.assert_decision_matches(res_of(0, 512, status=2), ref0, h)
    assert rejected(res_of(1, 256, status=2), ref0, h)
    assert rejected(res_of(0, 512, status=0), ref0, h)
