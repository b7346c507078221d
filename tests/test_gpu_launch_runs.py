"""A long vector is walked by several kernel launches, each over a run of consecutive tiles (2^27 coordinates for the
fused step up to 16 rows, 2^25 for AdamW only and for AdamW from a stored mean, 2^23 beyond 16 rows).  These cases
sit just past one or two such runs, with a ragged end and, in one variant each, with every buffer misaligned so that
all tiles of all launches take the guarded path; each is compared with the oracle element by element, and the
misaligned call with the aligned one bit for bit."""
import math

import pytest
import torch

import oracle
from paper_2412_21124_amd import binding as B
from paper_2412_21124_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FULL = B.NT_DO_STATS | B.NT_DO_ADAMW


def hyper_of(h: synth.Hyper, flags=FULL) -> B.nt_hyper:
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                        step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)


def step(wl, flags=FULL, d=None):
    res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, flags), d=d)
    torch.cuda.synchronize()
    return B.read_result(res).as_dict()


def shifted_copy(wl: synth.Workload):
    """The same rows and state one element further on in fresh buffers: nothing is 16-byte aligned any more."""
    J, d = wl.J, wl.d
    g = torch.empty((J, d + 9), dtype=wl.grads.dtype, device=DEV)[:, 1:d + 1]
    g.copy_(wl.grads[:, :d])
    state = []
    for t in (wl.w, wl.m, wl.v):
        s = torch.empty(d + 9, dtype=torch.float32, device=DEV)[1:d + 1]
        s.copy_(t)
        state.append(s)
    return g, state


@pytest.mark.parametrize("J,gdtype", [(24, torch.bfloat16), (17, torch.float32)])
def test_many_rows_in_one_pass_over_several_launches(J, gdtype):
    """More than 16 rows, state updated in the same pass: launches of 2^23 coordinates; two whole runs, a third of
    three tiles and a ragged tile."""
    d = 2 * (1 << 23) + 3 * 2048 + 77
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=31, device=DEV, hyper=synth.Hyper(b_k=64, round_to=J, step=3))
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    res = step(wl, FULL | B.NT_ONE_PASS)
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    assert H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper) == d


def test_adamw_only_over_several_launches_equals_the_fused_step():
    """AdamW only (the test skipped): launches of 2^25 coordinates.  Same bits in w, m, v as the fused step, whose
    launches are four times as long, and within the bound of the oracle's AdamW."""
    d = 2 * (1 << 25) + 5 * 4096 + 13
    wl = synth.make("t", 8, d, gdtype=torch.bfloat16, sigma=1e-2, seed=32, device=DEV)
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    res = step(wl, B.NT_DO_ADAMW)
    assert res["status"] == B.NT_STATUS_NO_STATS
    only = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), (w0, m0, v0)):
        t.copy_(s)
    step(wl, FULL)
    for a, b in zip((wl.w, wl.m, wl.v), only):
        assert torch.equal(a, b)
    assert H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper) == d


def test_fused_step_over_two_launches_aligned_and_misaligned():
    """The fused step just past one run of 2^27 coordinates: statistics, decision and every updated element against
    the oracle; then the same data in misaligned buffers (every tile of both launches on the guarded path, the
    ragged tile first) must give the same bits."""
    d = (1 << 27) + 2 * 4096 + 5
    wl = synth.flat_1p5b(d=d, seed=33, device=DEV)     # the headline's rows and state, 8 bf16 rows
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    g2, (w2, m2, v2) = shifted_copy(wl)
    res = step(wl, FULL | B.NT_COORD_TEST)
    ref = H.oracle_full(wl.grads, d, wl.J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    H.assert_coord_matches(res, H.oracle_coord_counts(wl.grads, d, wl.hyper))
    assert H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper) == d
    res2 = B.normtest_step(g2, w2, m2, v2, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST), d=d)
    torch.cuda.synchronize()
    res2 = B.read_result(res2).as_dict()
    for k in ("A", "B", "C", "T", "next_b", "pass", "status", "coord_fail", "coord_max_ratio"):
        assert res2[k] == res[k], k
    for a, b in zip((w2, m2, v2), (wl.w, wl.m, wl.v)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("misaligned", [False, True])
def test_clipped_step_over_several_launches(misaligned):
    """Two-phase clipped step past one run of each phase's kernel: statistics + stored mean in launches of 2^27
    coordinates (one here), AdamW from the stored mean in launches of 2^25 (three here, the last one ragged)."""
    J, d = 4, 2 * (1 << 25) + 3 * 4096 + 9
    wl = synth.make("t", J, d, gdtype=torch.float32, sigma=1e-2, seed=34, device=DEV, hyper=synth.Hyper(b_k=64, round_to=J, step=4))
    grads, w, m, v = wl.grads, wl.w, wl.m, wl.v
    if misaligned:
        grads, (w, m, v) = shifted_copy(wl)
    ref = H.oracle_full(grads, d, J, wl.hyper)
    max_norm = 0.5 * math.sqrt(ref.dec.gbar_sq)
    w0, m0, v0 = w.clone(), m.clone(), v.clone()
    gbar = torch.full((d + 4,), 7.0, dtype=torch.float32, device=DEV)[1 if misaligned else 0:][:d]
    res = B.normtest_step_clipped(grads, w, m, v, gbar, max_norm, hyper_of(wl.hyper), d=d)
    torch.cuda.synchronize()
    res = B.read_result(res).as_dict()
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    coef = oracle.clip_coef(ref.dec.gbar_sq, max_norm)
    assert coef < 1.0 and res["clip_coef"] == pytest.approx(coef, rel=1e-6)
    assert H.oracle_adamw_check(grads, d, w0, m0, v0, w, m, v, wl.hyper, gbar=gbar, grad_scale=coef) == d
