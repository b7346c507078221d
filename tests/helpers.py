"""Shared test plumbing: run the oracle over a workload (chunked, optionally threaded) and compare the
GPU library's outputs with it to the stated tolerances."""
from __future__ import annotations

import math
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np
import torch

import oracle
from paper_2412_21124_amd import synth

STATS_RTOL = 1e-5   # A, B, C, ||gbar||^2, ||Var||_1, T
ADAMW_RTOL = 1e-6   # w', m', v' relative to max(|x_ref|, rms(x_ref)); also max-norm relative
ORACLE_CHUNK = 1 << 22


def n_threads() -> int:
    return max(1, min(16, os.cpu_count() or 1))


@dataclass
class OracleOut:
    A: float
    B: float
    C: float
    dec: oracle.Decision
    J: int = 0


def oracle_stats(grads: torch.Tensor, d: int, chunk: int = ORACLE_CHUNK, threads: int | None = None):
    """(A, B, C) over the first d columns of a (J, ld) tensor on any device, streamed in chunks."""
    threads = n_threads() if threads is None else threads
    ranges = [(lo, min(d, lo + chunk)) for lo in range(0, d, chunk)]

    def work(r):
        G = synth.grads_as_numpy(grads, r[0], r[1])
        return oracle.stats(G)

    if len(ranges) <= 1 or threads == 1:
        parts = [work(r) for r in ranges]
    else:
        with ThreadPoolExecutor(threads) as ex:
            parts = list(ex.map(work, ranges))
    return oracle.combine_chunks(parts) if parts else (0.0, 0.0, 0.0)


def oracle_decide(A, B, C, J, h: synth.Hyper) -> oracle.Decision:
    return oracle.decide(A, B, C, J, h.eta, h.b_k, h.b_max, h.round_to, h.ddof)


def oracle_full(grads, d, J, h: synth.Hyper) -> OracleOut:
    A, B, C = oracle_stats(grads, d)
    return OracleOut(A, B, C, oracle_decide(A, B, C, J, h), J)


def assert_stats_close(res: dict, ref: OracleOut, rtol: float = STATS_RTOL, partial: bool = False):
    for key, want in (("A", ref.A), ("B", ref.B), ("C", ref.C)):
        got = res[key]
        assert abs(got - want) <= rtol * abs(want), "%s: gpu %r oracle %r rel %.3g" % (
            key, got, want, abs(got - want) / max(abs(want), 1e-300))
    if partial:
        return
    for key, want in (("gbar_sq", ref.dec.gbar_sq), ("var_l1", ref.dec.var_l1), ("T", ref.dec.T)):
        got = res[key]
        if math.isnan(want) or math.isinf(want):
            assert (math.isnan(got) and math.isnan(want)) or got == want, key
        else:
            assert abs(got - want) <= rtol * abs(want), "%s: gpu %r oracle %r" % (key, got, want)


def near_threshold(T: float, b_k: int, rtol: float = STATS_RTOL) -> bool:
    """The statistic lies within tolerance of b_k or of an integer: the decision may legitimately differ."""
    if not math.isfinite(T):
        return False
    return abs(T - b_k) <= 2 * rtol * max(abs(T), 1.0) or abs(T - round(T)) <= 2 * rtol * max(abs(T), 1.0)


def near_b_k(T: float, b_k: int, rtol: float = STATS_RTOL) -> bool:
    """The statistic lies within tolerance of b_k itself: only then may `pass` differ."""
    return math.isfinite(T) and abs(T - b_k) <= 2 * rtol * max(abs(T), 1.0)


def admissible_decisions(ref: OracleOut, h: synth.Hyper, rtol: float = STATS_RTOL, max_points: int = 4097):
    """Every (pass, next_b, status) the oracle itself gives when the centred sum moves within the band that the
    statistics tolerance allows (B and C may each be off by rtol, so T by 2 rtol): the oracle's decision on
    C (1 - 2 rtol) ... C (1 + 2 rtol), sampled densely enough that T moves by at most half a unit between
    samples, so that every value of the ceiling inside the band is met.  Returns None if the band would
    need more than max_points samples (a statistic so large that the band spans thousands of integers)."""
    J = ref.J
    assert J >= 2, "OracleOut.J must be set for the decision check"
    T = ref.dec.T
    if not math.isfinite(T):
        d = ref.dec
        return {(d.passed, d.next_b, d.status)}
    width = 4 * rtol * abs(T)                       # T(1 + 2 rtol) - T(1 - 2 rtol)
    n = max(1, int(math.ceil(2.0 * width)))         # half-unit spacing
    if 2 * n + 1 > max_points:
        return None
    out = set()
    for k in range(-n, n + 1):
        d = oracle_decide(ref.A, ref.B, ref.C * (1.0 + 2 * rtol * k / n), J, h)
        out.add((d.passed, d.next_b, d.status))
    return out


def assert_decision_matches(res: dict, ref: OracleOut, h: synth.Hyper, rtol: float = STATS_RTOL):
    """Alg. 1's decision must be the oracle's.  Where the oracle's statistic lies within the statistics
    tolerance of b_k or of an integer, the kernel's fp32-accumulated sums may put T on the other side:
    then the answer must still be one the oracle gives somewhere inside that band (so `pass` can only
    differ next to b_k, and next_b only between the two neighbouring values of the rounding chain)."""
    got = (bool(res["pass"]), int(res["next_b"]), int(res["status"]))
    want = (ref.dec.passed, ref.dec.next_b, ref.dec.status)
    if got == want:
        return
    allowed = admissible_decisions(ref, h, rtol)
    if allowed is None:
        # band too wide to enumerate: the ends bound the answer (pass and next_b are monotone in T)
        lo = oracle_decide(ref.A, ref.B, ref.C * (1.0 - 2 * rtol), ref.J, h)
        hi = oracle_decide(ref.A, ref.B, ref.C * (1.0 + 2 * rtol), ref.J, h)
        assert got[0] in (lo.passed, hi.passed), "pass %r, oracle %r..%r" % (got[0], lo.passed, hi.passed)
        assert lo.next_b <= got[1] <= hi.next_b, "next_b %d outside [%d, %d]" % (got[1], lo.next_b, hi.next_b)
        assert got[1] == h.b_k if got[0] else (got[1] % h.round_to == 0 or got[1] in (h.b_max, h.b_k))
        assert got[2] in (lo.status, hi.status)
        return
    assert got in allowed, "decision (pass, next_b, status) = %r; oracle %r (T = %r, b_k = %d); admissible within the band: %r" % (
        got, want, ref.dec.T, h.b_k, sorted(allowed))


def assert_state_close(name: str, got: np.ndarray, want: np.ndarray, rtol: float = ADAMW_RTOL):
    """|got - want| <= rtol * max(|want|, rms(want)) elementwise, and max-norm relative error <= rtol."""
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if want.size == 0:
        return
    rms = math.sqrt(float(np.mean(want * want)))
    err = np.abs(got - want)
    bound = rtol * np.maximum(np.abs(want), rms)
    bad = err > bound
    if bad.any():
        i = int(np.argmax(err / np.maximum(bound, 1e-300)))
        raise AssertionError("%s[%d]: gpu %r oracle %r err %.3g bound %.3g (%d of %d out of tolerance)" % (
            name, i, got[i], want[i], err[i], bound[i], int(bad.sum()), want.size))
    assert err.max() <= rtol * np.abs(want).max(), name


def oracle_adamw_check(grads, d, w0, m0, v0, w1, m1, v1, h: synth.Hyper, ranges=None,
                       chunk: int = ORACLE_CHUNK, threads: int | None = None, gbar=None, grad_scale: float = 1.0):
    """Compare the GPU's updated state (w1, m1, v1) with the oracle's AdamW on the pre-step state
    (w0, m0, v0), over all of [0, d) or over the given coordinate ranges.  rms is taken per range."""
    threads = n_threads() if threads is None else threads
    if ranges is None:
        ranges = [(lo, min(d, lo + chunk)) for lo in range(0, d, chunk)]

    def work(r):
        lo, hi = r
        G = synth.grads_as_numpy(grads, lo, hi)
        a = [t[lo:hi].cpu().numpy() for t in (w0, m0, v0)]
        out = oracle.adamw(G, a[0], a[1], a[2], h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step,
                           want_gbar=gbar is not None, grad_scale=grad_scale)
        for name, got, want in zip("wmv", (w1, m1, v1), out[:3]):
            assert_state_close("%s[%d:%d]" % (name, lo, hi), got[lo:hi].cpu().numpy(), want)
        if gbar is not None:
            assert_state_close("gbar[%d:%d]" % (lo, hi), gbar[lo:hi].cpu().numpy(), out[3], rtol=1e-6)
        return hi - lo

    if len(ranges) <= 1 or threads == 1:
        return sum(work(r) for r in ranges)
    with ThreadPoolExecutor(threads) as ex:
        return sum(ex.map(work, ranges))


def oracle_coord_counts(grads, d, h: synth.Hyper, band: float = STATS_RTOL, chunk: int = ORACLE_CHUNK,
                        threads: int | None = None):
    """(fail, near, pass, max_ratio) of the coordinate-wise test over the first d columns, streamed in chunks:
    the three counts and the largest ratio Var_i / (eta^2 b_k gbar_i^2)."""
    threads = n_threads() if threads is None else threads
    ranges = [(lo, min(d, lo + chunk)) for lo in range(0, d, chunk)]

    def work(r):
        G = synth.grads_as_numpy(grads, r[0], r[1])
        return oracle.coord_test(G, h.eta, h.b_k, h.ddof, band) + (oracle.coord_max_ratio(G, h.eta, h.b_k, h.ddof),)

    if len(ranges) <= 1 or threads == 1:
        parts = [work(r) for r in ranges]
    else:
        with ThreadPoolExecutor(threads) as ex:
            parts = list(ex.map(work, ranges))
    return tuple(sum(p[k] for p in parts) for k in range(3)) + (max([p[3] for p in parts], default=0.0),)


def assert_coord_count(got: int, counts):
    """The kernel decides each coordinate in fp32: coordinates within the band of equality may fall either way."""
    fail, near = counts[0], counts[1]
    assert fail <= got <= fail + near, "coord_fail %d not in [%d, %d]" % (got, fail, fail + near)


def assert_coord_ratio(got: float, want: float, rtol: float = STATS_RTOL):
    """Largest coordinate-wise ratio: the kernel forms each ratio in fp32 (about 1e-6 relative), so the largest
    agrees to the statistics tolerance; an infinite one (spread around an exactly zero mean) must be infinite."""
    if math.isinf(want):
        assert got == want, "coord_max_ratio %r, oracle inf" % got
    else:
        assert abs(got - want) <= rtol * abs(want), "coord_max_ratio %r, oracle %r" % (got, want)


def assert_coord_matches(res: dict, counts):
    """Count and largest ratio of a result against oracle_coord_counts' 4-tuple."""
    assert_coord_count(res["coord_fail"], counts)
    assert_coord_ratio(res["coord_max_ratio"], counts[3])
