"""Are the GPU parity comparisons sharp?  The library's outputs on a handful of small cases are computed once;
then every planted mistake of test_oracle_mutants.py is compiled into a copy of the ORACLE (never into the
GPU code) and the same comparisons that the parity tests make must notice the disagreement.  With the
unmodified oracle they must all pass."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2412_21124_amd import binding as B
from paper_2412_21124_amd import synth

import helpers as H
import test_library_host as HOST
import test_oracle_mutants as M

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FULL = B.NT_DO_STATS | B.NT_DO_ADAMW

# not observable at the parity tolerances: dropping the compensation changes an fp64 sum of 3e4 terms by ~1e-13
NOT_OBSERVABLE = {"compensation_dropped"}


def hyper_of(h, flags):
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                        step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)


class Case:
    """One GPU call with everything the comparison needs kept on the host."""

    def __init__(self, name, grads, w, m, v, h, max_norm=None, coord=True, exact=False):
        self.name, self.h, self.max_norm, self.coord, self.exact = name, h, max_norm, coord, exact
        self.J, self.d = grads.shape
        self.G = synth.grads_as_numpy(grads)
        self.before = [t.cpu().numpy().copy() for t in (w, m, v)]
        flags = FULL | (B.NT_COORD_TEST if coord else 0)
        if max_norm is None:
            res = B.normtest_step(grads, w, m, v, hyper_of(h, flags))
        else:
            gbar = torch.empty(self.d, dtype=torch.float32, device=DEV)
            res = B.normtest_step_clipped(grads, w, m, v, gbar, max_norm, hyper_of(h, flags))
        torch.cuda.synchronize()
        self.res = B.read_result(res).as_dict()
        self.after = [t.cpu().numpy().copy() for t in (w, m, v)]

    def compare(self):
        h = self.h
        A, Bs, C = oracle.stats(self.G)
        ref = H.OracleOut(A, Bs, C, oracle.decide(A, Bs, C, self.J, h.eta, h.b_k, h.b_max, h.round_to, h.ddof), self.J)
        H.assert_stats_close(self.res, ref)
        H.assert_decision_matches(self.res, ref, h)
        if self.exact:      # every step is exact in binary arithmetic: no threshold tolerance applies
            assert (self.res["T"], self.res["pass"], self.res["next_b"]) == (ref.dec.T, int(ref.dec.passed), ref.dec.next_b)
        coef = 1.0
        if self.max_norm is not None:
            coef = oracle.clip_coef(ref.dec.gbar_sq, self.max_norm)
            assert self.res["clip_coef"] == pytest.approx(coef, rel=1e-6)
        out = oracle.adamw(self.G, self.before[0], self.before[1], self.before[2], h.lr, h.beta1, h.beta2, h.eps,
                           h.weight_decay, h.step, grad_scale=coef)
        if not (math.isnan(self.res["T"]) or math.isinf(self.res["T"])):
            for name, got, want in zip("wmv", self.after, out):
                H.assert_state_close(name, got, want)
        if self.coord:
            band = 0.0 if self.exact else H.STATS_RTOL
            H.assert_coord_count(self.res["coord_fail"], oracle.coord_test(self.G, h.eta, h.b_k, h.ddof, band))
            H.assert_coord_ratio(self.res["coord_max_ratio"], oracle.coord_max_ratio(self.G, h.eta, h.b_k, h.ddof))


@pytest.fixture(scope="module")
def cases():
    out = []

    def add(name, wl, h=None, max_norm=None, grads=None, coord=True):
        g = wl.grads if grads is None else grads
        out.append(Case(name, g, wl.w, wl.m, wl.v, h or wl.hyper, max_norm, coord))

    # fails the test, rounding to a multiple of 16, cut by the cap
    add("fp32_fail_capped", synth.make("s", 4, 20001, sigma=1e-2, seed=1, device=DEV,
                                       hyper=synth.Hyper(b_k=32, b_max=64, round_to=16, step=10)))
    # fails, plain ceiling, no cap; and rounding to 16 without a cap
    add("fp32_fail_ceiling", synth.make("s", 4, 20001, sigma=1e-2, seed=1, device=DEV,
                                        hyper=synth.Hyper(b_k=32, b_max=0, round_to=1, step=10)))
    add("fp32_fail_round16", synth.make("s", 4, 20001, sigma=1e-2, seed=1, device=DEV,
                                        hyper=synth.Hyper(b_k=32, b_max=0, round_to=16, step=10)))
    # current batch already above the cap: must not shrink
    add("above_cap", synth.make("s", 4, 20001, sigma=3e-2, seed=2, device=DEV,
                                hyper=synth.Hyper(b_k=256, b_max=64, round_to=4, step=3)))
    # bf16, Alg. 1's normaliser, passes, second step
    add("bf16_pass_ddof0", synth.make("s", 8, 30000, gdtype=torch.bfloat16, sigma=1e-3, seed=3, device=DEV,
                                      hyper=synth.Hyper(b_k=32, ddof=0, step=2, eps=1e-8)))
    # the row-walking path
    add("bf16_rows33", synth.make("s", 33, 9000, gdtype=torch.bfloat16, sigma=1e-2, seed=4, device=DEV,
                                  hyper=synth.Hyper(b_k=64, round_to=1, step=5)))
    # clipping active, and a bound that does not bind
    add("clip_active", synth.make("s", 8, 30000, gdtype=torch.bfloat16, sigma=1e-2, seed=5, device=DEV,
                                  hyper=synth.Hyper(b_k=256, round_to=128, step=4)), max_norm=0.05)
    add("clip_idle", synth.make("s", 8, 30000, gdtype=torch.bfloat16, sigma=1e-2, seed=5, device=DEV,
                                hyper=synth.Hyper(b_k=256, round_to=128, step=4)), max_norm=1e6)
    # rows that cancel exactly: zero mean with spread
    wl = synth.make("s", 2, 5000, sigma=1e-2, seed=6, device=DEV, hyper=synth.Hyper(b_k=32, b_max=512, round_to=4))
    g = wl.grads.clone()
    g[1] = -g[0]
    add("zero_mean", wl, grads=g, coord=False)
    # coordinates that carry nothing (all rows zero) next to live ones: their ratio is 0, not 0/0
    wl = synth.make("s", 8, 12000, gdtype=torch.bfloat16, sigma=1e-2, seed=7, device=DEV, hyper=synth.Hyper(b_k=64, round_to=1))
    g = wl.grads.clone()
    g[:, :50] = 0
    add("dead_coordinates", wl, grads=g)
    # ... and coordinates whose rows cancel exactly: spread around a zero mean, the largest ratio is infinite
    g = g.clone()
    g[:, 50:60] = 0
    g[0, 50:60] = 1.0
    g[1, 50:60] = -1.0
    add("cancelling_coordinates", wl, grads=g)
    # exact equalities (hand example g_1 = (1,2), g_2 = (3,6), eta = 1/2, ddof 0: T = 1; per coordinate ratio 4 at eta 1/4)
    two = torch.tensor([[1.0, 2.0], [3.0, 6.0]], device=DEV)
    z = lambda: torch.zeros(2, device=DEV)
    out.append(Case("T_equals_b_k", two, z(), z(), z(), synth.Hyper(eta=0.5, b_k=1, ddof=0, round_to=2, step=1), coord=False, exact=True))
    out.append(Case("coordinate_equality", two, z(), z(), z(), synth.Hyper(eta=0.25, b_k=4, ddof=0, round_to=1, step=1), exact=True))
    return out


def compare_all(cases):
    for c in cases:
        try:
            c.compare()
        except AssertionError as e:
            raise AssertionError("%s: %s" % (c.name, e))
    # host-side entry points of the library against the same oracle
    HOST.test_resplit_matches_oracle()
    HOST.test_schedule_flags_match_oracle()
    HOST.test_clip_coef_matches_oracle()
    HOST.test_combine_decision_agrees_with_oracle_on_random_sums()
    HOST.test_combine_special_cases_agree_with_oracle()


def test_unmodified_oracle_agrees_with_the_gpu(cases, tmp_path, monkeypatch):
    monkeypatch.setattr(oracle, "_lib", oracle._bind(M.compile_variant(open(M.SRC).read(), str(tmp_path / "clean.so"))))
    compare_all(cases)
    assert cases[0].res["status"] & B.NT_STATUS_CLAMPED and cases[3].res["next_b"] == 256
    assert cases[-2].res["pass"] == 1 and cases[-1].res["coord_fail"] == 0


@pytest.mark.parametrize("mutant", [m for m in M.MUTANTS if m[0] not in NOT_OBSERVABLE], ids=lambda m: m[0])
def test_gpu_comparison_notices_each_planted_oracle_mistake(mutant, cases, tmp_path, monkeypatch):
    name, find, repl = mutant[:3]
    text = M.plant(open(M.SRC).read(), find, repl, mutant[3] if len(mutant) > 3 else None)
    monkeypatch.setattr(oracle, "_lib", oracle._bind(M.compile_variant(text, str(tmp_path / (name + ".so")))))
    with pytest.raises(AssertionError):
        compare_all(cases)
