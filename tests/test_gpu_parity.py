"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle on the same seeded
inputs, element by element; plus bit-exactness properties (determinism, path and shard invariance)."""
import math

import numpy as np
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
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay,
                        eta=h.eta, step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to,
                        ddof=h.ddof, flags=flags)


def gpu_step(grads, w, m, v, h: synth.Hyper, d=None, flags=FULL, **kw) -> dict:
    res = B.normtest_step(grads, w, m, v, hyper_of(h, flags), d=d, **kw)
    torch.cuda.synchronize()
    return B.read_result(res).as_dict()


def full_parity(wl: synth.Workload, d=None, flags=FULL, check_gbar=False):
    """One full step on the GPU, everything compared with the oracle."""
    d = wl.d if d is None else d
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    gbar = torch.full((max(d, 1),), 7.0, dtype=torch.float32, device=wl.grads.device) if check_gbar else None
    fl = flags | (B.NT_WRITE_GBAR if check_gbar else 0)
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, d=d, flags=fl, gbar_out=gbar)
    ref = H.oracle_full(wl.grads, d, wl.J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper, gbar=gbar)
    # coordinates past d are never written
    for a, b in ((wl.w, w0), (wl.m, m0), (wl.v, v0)):
        assert torch.equal(a[d:], b[d:])
    return res, ref


# ------------------------------------------------------------------ the paper-shaped workloads, small

@pytest.mark.parametrize("sigma,expect_pass", [(1e-3, True), (1e-2, False)])
def test_tiny_config(sigma, expect_pass):
    wl = synth.tiny(sigma, device=DEV)
    res, ref = full_parity(wl, check_gbar=True)
    assert bool(res["pass"]) == expect_pass == ref.dec.passed
    assert res["next_b"] == ref.dec.next_b


@pytest.mark.parametrize("ratio", [0.1, 0.3, 1.0, 1.9, 2.0, 3.0, 10.0])
def test_gpt2_small_scaled_ratio_sweep(ratio):
    sizes = synth.scaled_blocks(synth.gpt2_small_blocks(), 1 << 21, multiple=8)
    wl = synth.gpt2_small(ratio, block_sizes=sizes, seed=2, device=DEV)
    res, ref = full_parity(wl)
    assert res["C"] < res["A"]


def test_per_sample_scaled():
    wl = synth.per_sample(b=512, d=1 << 16, n_blocks=64, seed=3, device=DEV)
    full_parity(wl)


def test_fsdp_shard_scaled_and_combine():
    """Eight shards with fresh seeds, each a PARTIAL call; the host combine equals the oracle on the concatenation."""
    d_shard, J = 100_003, 16
    parts, accs = [], []
    hyper = None
    for sid in range(8):
        wl = synth.fsdp_shard(sid, d_shard=d_shard, J=J, seed=5, device=DEV)
        hyper = wl.hyper
        w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
        shard = B.nt_shard_info(sid, 8, sid * d_shard, 8 * d_shard)
        res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(hyper, FULL | B.NT_PARTIAL), shard=shard)
        torch.cuda.synchronize()
        r = B.read_result(res)
        assert r.status == B.NT_STATUS_PARTIAL_ONLY and math.isnan(r.T) and r.next_b == hyper.b_k
        ref = H.oracle_full(wl.grads, d_shard, J, hyper)
        H.assert_stats_close(r.as_dict(), ref, partial=True)
        H.oracle_adamw_check(wl.grads, d_shard, w0, m0, v0, wl.w, wl.m, wl.v, hyper)
        parts.append(r)
        accs.append((ref.A, ref.B, ref.C))
    comb = B.normtest_combine(parts, J, hyper_of(hyper)).as_dict()
    A, Bs, C = oracle.combine_chunks(accs)
    ref = H.OracleOut(A, Bs, C, H.oracle_decide(A, Bs, C, J, hyper), J)
    H.assert_stats_close(comb, ref)
    H.assert_decision_matches(comb, ref, hyper)


# ------------------------------------------------------------------ shapes: every J path, ragged tails

@pytest.mark.parametrize("J", [2, 3, 4, 5, 6, 7, 8, 9, 11, 13, 15, 16])
@pytest.mark.parametrize("gdtype", [torch.float32, torch.bfloat16])
def test_small_J_ragged(J, gdtype):
    d = 3 * 16384 + 4321          # three full tiles, a ragged tile whose end is not a multiple of the vector width
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=2e-2, seed=J, device=DEV,
                    hyper=synth.Hyper(b_k=16, round_to=J, step=3))
    full_parity(wl, check_gbar=(J % 4 == 0))


@pytest.mark.parametrize("J", [17, 20, 21, 31, 32, 48, 100])
@pytest.mark.parametrize("gdtype", [torch.float32, torch.bfloat16])
def test_large_J_ragged(J, gdtype):
    d = 5 * 4096 + 777
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=J, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=1, step=7))
    full_parity(wl, check_gbar=True)


@pytest.mark.parametrize("d", [0, 1, 7, 8, 2047, 2048, 16383, 16384, 16385])
def test_small_d(d):
    wl = synth.make("t", 8, max(d, 1), gdtype=torch.bfloat16, sigma=1e-2, seed=d, device=DEV)
    full_parity(wl, d=d)


def test_d_zero_result():
    wl = synth.make("t", 4, 8, device=DEV)
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, d=0)
    assert (res["A"], res["B"], res["C"]) == (0.0, 0.0, 0.0)
    assert res["pass"] == 1 and res["next_b"] == wl.hyper.b_k and res["status"] == B.NT_STATUS_ZERO_GRAD_NORM


# ------------------------------------------------------------------ bit-exactness properties

def test_two_runs_bit_identical():
    wl = synth.gpt2_small(1.0, block_sizes=synth.scaled_blocks(synth.gpt2_small_blocks(), 1 << 20, 8), device=DEV)
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    r1 = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    out1 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    wl.w.copy_(w0), wl.m.copy_(m0), wl.v.copy_(v0)
    r2 = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    assert r1 == r2
    for a, b in zip(out1, (wl.w, wl.m, wl.v)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("J,gdtype", [(8, torch.bfloat16), (4, torch.float32), (40, torch.bfloat16)])
def test_misaligned_and_padded_rows_same_bits(J, gdtype):
    """Rows that start 1 element off a 16-byte boundary, or with a padded stride, take the guarded
    kernel; the sums and the updated state must have the same bits as on the aligned fast path."""
    d = 2 * B.normtest_tile_coords(J) + 1000
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=1, device=DEV)
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    ref = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    ref_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for pad, off in ((3, 1), (8, 0), (0, 1)):
        big = torch.zeros((J, d + pad + off), dtype=gdtype, device=DEV)
        big[:] = 9.0                                 # poison the padding
        view = big[:, off:off + d]
        view.copy_(wl.grads)
        st = [torch.full((d + 1,), 5.0, device=DEV)[off:off + d] for _ in range(3)]
        for t, s in zip(st, state0):
            t.copy_(s)
        res = gpu_step(view, st[0], st[1], st[2], wl.hyper, d=d)
        assert res == ref
        for a, b in zip(st, ref_state):
            assert torch.equal(a, b)


@pytest.mark.parametrize("J,gdtype", [(8, torch.bfloat16), (16, torch.bfloat16), (4, torch.float32), (64, torch.bfloat16)])
def test_tile_aligned_shards_add_up_bit_exactly(J, gdtype):
    tc = B.normtest_tile_coords(J)
    d = 11 * tc + 517
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=4, device=DEV)
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    whole = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    whole_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    cuts = [0, 2 * tc, 3 * tc, 8 * tc, d]
    parts = []
    for sid, (lo, hi) in enumerate(zip(cuts[:-1], cuts[1:])):
        res = B.normtest_step(wl.grads[:, lo:hi], wl.w[lo:hi], wl.m[lo:hi], wl.v[lo:hi],
                              hyper_of(wl.hyper, FULL | B.NT_PARTIAL),
                              shard=B.nt_shard_info(sid, len(cuts) - 1, lo, d))
        torch.cuda.synchronize()
        parts.append(B.read_result(res))
    comb = B.normtest_combine(parts, J, hyper_of(wl.hyper)).as_dict()
    for k in ("A", "B", "C", "gbar_sq", "var_l1", "T", "next_b", "pass", "status"):
        assert comb[k] == whole[k], k
    for a, b in zip((wl.w, wl.m, wl.v), whole_state):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ flags

def test_stats_only_leaves_state_untouched():
    wl = synth.tiny(1e-2, d=50_000, device=DEV)
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_STATS)
    ref = H.oracle_full(wl.grads, wl.d, wl.J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    assert torch.equal(wl.w, w0) and torch.equal(wl.m, m0) and torch.equal(wl.v, v0)
    # state pointers may be absent altogether
    res2 = gpu_step(wl.grads, None, None, None, wl.hyper, flags=B.NT_DO_STATS)
    assert res2 == res
    # the fused step adds the same per-lane fp32 terms, in fp64 but over differently sized tiles
    res3 = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=FULL)
    assert (res3["A"], res3["B"], res3["C"]) == pytest.approx((res["A"], res["B"], res["C"]), rel=1e-13)


def test_adamw_only_reports_no_stats():
    wl = synth.make("t", 8, 70_001, gdtype=torch.bfloat16, seed=8, device=DEV)
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_ADAMW)
    assert res["status"] == B.NT_STATUS_NO_STATS and res["pass"] == 1 and res["next_b"] == wl.hyper.b_k
    assert math.isnan(res["A"]) and math.isnan(res["T"])
    H.oracle_adamw_check(wl.grads, wl.d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper)


def test_first_step_from_zero_moments():
    """k = 1 with m = v = 0 (Alg. 1's initial state): the update is a sign step of size lr."""
    wl = synth.make("t", 8, 40_000, gdtype=torch.bfloat16, seed=9, device=DEV,
                    hyper=synth.Hyper(step=1, lr=4e-4, b_k=256, round_to=128))
    wl.m.zero_(), wl.v.zero_()
    w0 = wl.w.clone()
    full_parity(wl)
    moved = (wl.w - (1 - 4e-4 * 0.1) * w0).abs()
    assert float(moved.max()) <= 4e-4 * (1 + 1e-5)


def test_ddof_zero_is_alg1_estimator():
    wl = synth.tiny(1e-2, d=100_000, device=DEV)
    wl.hyper.ddof = 0
    res, ref = full_parity(wl)
    assert res["var_l1"] == pytest.approx(res["C"] / wl.J, rel=1e-15)


# ------------------------------------------------------------------ degenerate inputs

@pytest.mark.parametrize("J", [4, 8, 32])
def test_identical_rows_have_exactly_zero_variance(J):
    wl = synth.make("t", J, 40_000, gdtype=torch.bfloat16, seed=10, device=DEV)
    wl.grads[:] = wl.grads[0].clone()
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    assert res["C"] == 0.0 and res["T"] == 0.0 and res["pass"] == 1 and res["next_b"] == wl.hyper.b_k
    n2 = float((wl.grads[0].double() ** 2).sum())
    assert res["gbar_sq"] == pytest.approx(n2, rel=1e-6)


def test_zero_gradients_and_zero_mean():
    wl = synth.make("t", 4, 20_000, seed=11, device=DEV)
    wl.grads.zero_()
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    assert res["status"] == B.NT_STATUS_ZERO_GRAD_NORM and res["pass"] == 1 and res["next_b"] == wl.hyper.b_k
    # rows that cancel exactly: zero mean, positive spread -> cannot pass, go to the cap
    wl.grads[0] = 1.0
    wl.grads[1] = -1.0
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    assert res["status"] == B.NT_STATUS_ZERO_GRAD_NORM and res["pass"] == 0 and res["next_b"] == wl.hyper.b_max
    assert math.isinf(res["T"]) and res["C"] == 2.0 * 20_000


@pytest.mark.parametrize("bad", [float("nan"), float("inf")])
def test_nonfinite_gradient_is_flagged_and_batch_kept(bad):
    wl = synth.make("t", 8, 50_000, gdtype=torch.bfloat16, seed=12, device=DEV)
    wl.grads[3, 31_337] = bad
    res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    assert res["status"] & B.NT_STATUS_NONFINITE and res["pass"] == 1 and res["next_b"] == wl.hyper.b_k
    ref = H.oracle_full(wl.grads, wl.d, wl.J, wl.hyper)
    assert ref.dec.status & oracle.NONFINITE and ref.dec.next_b == res["next_b"]


def test_threshold_and_cap():
    """A statistic far above b_max is cut to it; b_k above the statistic passes."""
    wl = synth.tiny(1e-2, d=100_000, device=DEV)
    wl.hyper.b_max = 64
    res, ref = full_parity(wl)
    assert res["next_b"] == 64 and res["status"] == B.NT_STATUS_CLAMPED == ref.dec.status
    wl2 = synth.tiny(1e-2, d=100_000, device=DEV)
    wl2.hyper.b_k = 4096
    res, ref = full_parity(wl2)
    assert res["pass"] == 1 and res["next_b"] == 4096


# ------------------------------------------------------------------ gradient-clipped two-phase variant

def clipped_step(wl, max_norm, d=None):
    d = wl.d if d is None else d
    gbar = torch.full((max(d, 1),), 7.0, dtype=torch.float32, device=wl.grads.device)
    res = B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, max_norm, hyper_of(wl.hyper), d=d)
    torch.cuda.synchronize()
    return B.read_result(res).as_dict(), gbar


@pytest.mark.parametrize("J,gdtype,d", [(8, torch.bfloat16, 5 * 4096 + 123), (4, torch.float32, 1 << 20),
                                        (40, torch.bfloat16, 3 * 4096 + 5), (16, torch.bfloat16, 4096)])
def test_clipped_step_matches_oracle(J, gdtype, d):
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=21, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=J, step=4))
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    norm = math.sqrt(ref.dec.gbar_sq)
    for max_norm, clipped in ((0.5 * norm, True), (2.0 * norm, False)):
        w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
        res, gbar = clipped_step(wl, max_norm)
        H.assert_stats_close(res, ref)                      # the test uses the unclipped mean
        H.assert_decision_matches(res, ref, wl.hyper)
        coef = oracle.clip_coef(ref.dec.gbar_sq, max_norm)
        assert (coef < 1.0) == clipped
        assert res["clip_coef"] == pytest.approx(coef, rel=1e-6)
        H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper, gbar=gbar, grad_scale=coef)


def test_clipped_step_without_bound_equals_fused_step_bit_for_bit():
    wl = synth.make("t", 8, 9 * 4096 + 77, gdtype=torch.bfloat16, seed=22, device=DEV)
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    fused = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    fused_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for max_norm in (0.0, 1e30):
        for t, s in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s)
        res, _ = clipped_step(wl, max_norm)
        assert res["clip_coef"] == 1.0
        for k in ("A", "B", "C", "T"):
            assert res[k] == pytest.approx(fused[k], rel=1e-13), k
        for k in ("next_b", "pass", "status"):
            assert res[k] == fused[k], k
        for a, b in zip((wl.w, wl.m, wl.v), fused_state):
            assert torch.equal(a, b)


def test_clipped_shards_via_host_combine_equal_one_call():
    """FSDP flow: per-shard statistics with the mean written out, host combine, then AdamW on each shard
    with the host-computed factor; same bits as one clipped call over the whole vector."""
    J = 16
    tc = B.normtest_tile_coords(J)
    d = 6 * tc + 1001
    wl = synth.make("t", J, d, gdtype=torch.bfloat16, sigma=1e-2, seed=23, device=DEV)
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    max_norm = 0.3 * math.sqrt(ref.dec.gbar_sq)
    whole, gbar_whole = clipped_step(wl, max_norm)
    whole_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    cuts = [0, 2 * tc, 5 * tc, d]
    gbar = torch.zeros(d, dtype=torch.float32, device=DEV)
    parts = []
    flags = B.NT_DO_STATS | B.NT_PARTIAL | B.NT_WRITE_GBAR
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        r = B.normtest_step(wl.grads[:, lo:hi], None, None, None, hyper_of(wl.hyper, flags), gbar_out=gbar[lo:hi])
        torch.cuda.synchronize()
        parts.append(B.read_result(r))
    comb = B.normtest_combine(parts, J, hyper_of(wl.hyper))
    coef = B.normtest_clip_coef(comb.gbar_sq, max_norm)
    assert coef == whole["clip_coef"] and coef < 1.0
    assert torch.equal(gbar, gbar_whole)
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        B.normtest_adamw_gbar(gbar[lo:hi], wl.w[lo:hi], wl.m[lo:hi], wl.v[lo:hi], hyper_of(wl.hyper), coef)
    torch.cuda.synchronize()
    for a, b in zip((wl.w, wl.m, wl.v), whole_state):
        assert torch.equal(a, b)
    assert (comb.T, comb.next_b, comb.pass_) == (whole["T"], whole["next_b"], whole["pass"])


def test_adamw_gbar_misaligned_matches_aligned():
    d = 4096 + 333
    wl = synth.make("t", 4, d, seed=24, device=DEV)
    gbar = torch.randn(d + 1, device=DEV) * 1e-2
    ref = [t.clone() for t in (wl.w, wl.m, wl.v)]
    B.normtest_adamw_gbar(gbar[:d].clone(), ref[0], ref[1], ref[2], hyper_of(wl.hyper), 0.75)
    off = [torch.zeros(d + 1, device=DEV)[1:] for _ in range(3)]
    for t, s in zip(off, (wl.w, wl.m, wl.v)):
        t.copy_(s)
    g1 = gbar.clone()
    g1[1:] = gbar[:d]
    B.normtest_adamw_gbar(g1[1:], off[0], off[1], off[2], hyper_of(wl.hyper), 0.75, d=d)
    torch.cuda.synchronize()
    for a, b in zip(off, ref):
        assert torch.equal(a, b)


# ------------------------------------------------------------------ a short run: schedule, growth, bias corrections

def test_short_run_with_test_interval_and_maximum():
    """Ten consecutive steps as a training loop would issue them: flags from normtest_schedule_flags (interval 2,
    maximum 512), step counter k = 1.., b_k fed back from next_b, fresh gradients each step.  Every step is compared with the oracle from the same pre-step state; the sequence of
    batch sizes must be the oracle's."""
    J, d, M = 4, 3 * 4096 + 100, 4
    b_k, b_max, interval = 32, 512, 2
    dev_state = None
    sizes, tested = [], []
    for k in range(1, 11):
        # T = r^2 / (eta^2 (1 + r^2/J)) for noise-to-signal ratio r: about 100, 300, 700 on the steps that test
        sigma = 1e-2 * {1: 0.52, 3: 0.96, 5: 1.76}.get(k, 1.0)
        h = synth.Hyper(lr=3e-3, step=k, b_k=b_k, b_max=b_max, round_to=J * M, ddof=1, eta=0.05)
        wl = synth.make("run", J, d, gdtype=torch.bfloat16, sigma=sigma, seed=100 + k, device=DEV, hyper=h)
        if dev_state is None:
            dev_state = (wl.w, wl.m, wl.v)
        w, m, v = dev_state
        w0, m0, v0 = w.clone(), m.clone(), v.clone()
        flags = B.normtest_schedule_flags(k, interval, b_k, b_max, FULL)
        due = oracle.test_due(k, interval, b_k, b_max)
        assert bool(flags & B.NT_DO_STATS) == due
        res = gpu_step(wl.grads, w, m, v, h, flags=flags)
        H.oracle_adamw_check(wl.grads, d, w0, m0, v0, w, m, v, h)      # AdamW runs on every step, bias terms at k
        if due:
            ref = H.oracle_full(wl.grads, d, J, h)
            H.assert_stats_close(res, ref)
            assert not H.near_threshold(ref.dec.T, b_k), "choose another seed: T too close to b_k"
            H.assert_decision_matches(res, ref, h)
            assert res["next_b"] == ref.dec.next_b
        else:
            assert res["status"] == B.NT_STATUS_NO_STATS and res["next_b"] == b_k and res["pass"] == 1
        tested.append(due)
        sizes.append(res["next_b"])
        b_k = res["next_b"]
    assert tested[:2] == [True, False] and sizes[-1] == b_max            # grew to the maximum ...
    first_max = sizes.index(b_max)
    assert not any(tested[first_max + 1:])                                # ... after which no step tests
    assert all(b >= a for a, b in zip(sizes, sizes[1:])) and all(s % (J * M) == 0 for s in sizes if s != 32)


# ------------------------------------------------------------------ coordinate-wise form of the test

@pytest.mark.parametrize("J,gdtype,d,sigma,b_k", [
    (8, torch.bfloat16, 5 * 16384 + 321, 1e-2, 256), (8, torch.bfloat16, 40_000, 1e-3, 32),
    (4, torch.float32, 1 << 20, 1e-2, 32), (4, torch.float32, 1 << 20, 1e-3, 8192),
    (16, torch.bfloat16, 70_001, 3e-3, 64), (40, torch.bfloat16, 30_003, 1e-2, 512), (3, torch.float32, 9_999, 1e-2, 1)])
def test_coordinatewise_count_matches_oracle(J, gdtype, d, sigma, b_k):
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=sigma, seed=60 + J, device=DEV,
                    hyper=synth.Hyper(b_k=b_k, round_to=1, b_max=0))
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    plain = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper)
    plain_state = [t.clone() for t in (wl.w, wl.m, wl.v)]
    assert plain["coord_fail"] == -1 and plain["coord_max_ratio"] == -1.0
    counts = H.oracle_coord_counts(wl.grads, d, wl.hyper)
    assert sum(counts[:3]) == d and counts[1] < max(10, d // 1000)      # the band must stay a thin sliver
    assert counts[3] > 0.0
    for mode_flags in (FULL, B.NT_DO_STATS):
        for t, s0 in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s0)
        res = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=mode_flags | B.NT_COORD_TEST)
        H.assert_coord_matches(res, counts)
        if mode_flags == FULL:                                          # asking for the count changes nothing else
            for k in ("A", "B", "C", "T", "next_b", "pass", "status"):
                assert res[k] == plain[k], k
            for a, b in zip((wl.w, wl.m, wl.v), plain_state):
                assert torch.equal(a, b)


def test_coordinatewise_count_degenerate_and_sharded():
    J, d = 8, 3 * 16384 + 500
    wl = synth.make("t", J, d, gdtype=torch.bfloat16, sigma=1e-2, seed=61, device=DEV, hyper=synth.Hyper(b_k=64))
    # identical rows: no spread, nothing fails; all-zero coordinates: 0 > 0 is false
    same = wl.grads[0:1].repeat(J, 1).contiguous()
    same[:, :100] = 0
    res = gpu_step(same, wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_STATS | B.NT_COORD_TEST)
    assert res["coord_fail"] == 0 and res["coord_max_ratio"] == 0.0
    # zero mean with spread fails whatever the batch size
    same[0, :100] = 1.0
    same[1, :100] = -1.0
    res = gpu_step(same, wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_STATS | B.NT_COORD_TEST)
    assert res["coord_fail"] == 100 and res["coord_max_ratio"] == math.inf
    # shards: counts add up in normtest_combine, and the guarded (misaligned) path counts the same
    whole = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_STATS | B.NT_COORD_TEST)
    cuts = [0, 16384, 2 * 16384, d]
    parts = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        r = B.normtest_step(wl.grads[:, lo:hi], None, None, None,
                            hyper_of(wl.hyper, B.NT_DO_STATS | B.NT_PARTIAL | B.NT_COORD_TEST))
        torch.cuda.synchronize()
        parts.append(B.read_result(r))
    comb = B.normtest_combine(parts, J, hyper_of(wl.hyper))
    assert comb.coord_fail == whole["coord_fail"]
    # the largest ratio over the shards is the largest of the shards' values, bit for bit
    assert comb.coord_max_ratio == whole["coord_max_ratio"] == max(p.coord_max_ratio for p in parts)
    big = torch.zeros((J, d + 1), dtype=torch.bfloat16, device=DEV)
    big[:, 1:] = wl.grads
    off = gpu_step(big[:, 1:], wl.w, wl.m, wl.v, wl.hyper, flags=B.NT_DO_STATS | B.NT_COORD_TEST)
    assert off["coord_fail"] == whole["coord_fail"] and off["coord_max_ratio"] == whole["coord_max_ratio"]
    # the clipped two-phase step counts too (its statistics phase uses another tile shape)
    gbar = torch.empty(d, dtype=torch.float32, device=DEV)
    r = B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, 1.0, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST))
    torch.cuda.synchronize()
    assert B.read_result(r).coord_fail == whole["coord_fail"]
    assert B.read_result(r).coord_max_ratio == whole["coord_max_ratio"]
    r = B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, 1.0, hyper_of(wl.hyper, FULL))
    torch.cuda.synchronize()
    assert B.read_result(r).coord_fail == -1 and B.read_result(r).coord_max_ratio == -1.0


# ------------------------------------------------------------------ rows given as separate allocations

@pytest.mark.parametrize("J,gdtype,flags", [(8, torch.bfloat16, FULL), (4, torch.float32, FULL),
                                            (37, torch.bfloat16, FULL), (18, torch.float32, FULL),
                                            (8, torch.bfloat16, B.NT_DO_STATS)])
def test_row_table_gives_the_same_bits_as_the_strided_matrix(J, gdtype, flags):
    d = 3 * 16384 + 2222
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=50 + J, device=DEV)
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    ref = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=flags)
    ref_state = [t.clone() for t in (wl.w, wl.m, wl.v)]
    oracle_ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(ref, oracle_ref)
    for misalign in (False, True):
        # separate allocations of different lengths, in shuffled address order; optionally one row off by one element
        rows = []
        for j in range(J):
            buf = torch.full((d + 64 + 8 * j,), 5.0, dtype=gdtype, device=DEV)
            off = 1 if (misalign and j == J // 2) else 0
            r = buf[off:off + d]
            r.copy_(wl.grads[j, :d])
            rows.append(r)
        for t, s0 in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s0)
        res = B.normtest_step_rows(rows, wl.w, wl.m, wl.v, hyper_of(wl.hyper, flags))
        torch.cuda.synchronize()
        got = B.read_result(res).as_dict()
        assert got == ref
        for a, b in zip((wl.w, wl.m, wl.v), ref_state):
            assert torch.equal(a, b)


# ------------------------------------------------------------------ seeded random sweep over the argument space

def test_random_configurations_against_oracle():
    """60 seeded draws of (J, d, dtype, alignment offset, row padding, flags, ddof, step, eta, b_k, rounding)."""
    rng = np.random.default_rng(2024)
    for case in range(60):
        J = int(rng.choice([2, 3, 4, 6, 8, 12, 16, 17, 24, 33, 70]))
        d = int(rng.choice([1, 5, 100, 1023, 1024, 2049, 4096, 4097, 9000, 20000, 40001]))
        gdtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
        off = int(rng.choice([0, 0, 1, 2, 4]))
        pad = int(rng.choice([0, 0, 3, 8, 64]))
        mode = str(rng.choice(["full", "full", "stats", "adamw"]))
        flags = {"full": FULL, "stats": B.NT_DO_STATS, "adamw": B.NT_DO_ADAMW}[mode]
        want_gbar = bool(rng.random() < 0.3)
        h = synth.Hyper(lr=float(rng.choice([1e-3, 4e-4, 0.0])), beta1=float(rng.choice([0.9, 0.0, 0.5])),
                        beta2=float(rng.choice([0.95, 0.999])), eps=1e-8, weight_decay=float(rng.choice([0.1, 0.0])),
                        eta=float(rng.choice([0.05, 0.1, 0.275])), step=int(rng.choice([1, 2, 10, 1000])),
                        b_k=int(rng.choice([1, 32, 256])), b_max=int(rng.choice([0, 512, 8192])),
                        round_to=int(rng.choice([1, 4, 128])), ddof=int(rng.integers(0, 2)))
        sigma = float(rng.choice([1e-3, 1e-2, 1e-1]))
        src = synth.make("r", J, d, gdtype=gdtype, sigma=sigma, seed=1000 + case, device=DEV, hyper=h)
        big = torch.full((J, off + d + pad), 3.0, dtype=gdtype, device=DEV)
        grads = big[:, off:off + d]
        grads.copy_(src.grads)
        st = [torch.full((off + d + 1,), 9.0, device=DEV)[off:off + d] for _ in range(3)]
        for t, s0 in zip(st, (src.w, src.m, src.v)):
            t.copy_(s0)
        before = [t.clone() for t in st]
        gbar = torch.full((off + d,), 7.0, device=DEV)[off:] if want_gbar else None
        fl = flags | (B.NT_WRITE_GBAR if want_gbar else 0)
        ctx = "case %d: J=%d d=%d %s off=%d pad=%d mode=%s gbar=%s" % (case, J, d, gdtype, off, pad, mode, want_gbar)
        res = gpu_step(grads, st[0], st[1], st[2], h, d=d, flags=fl, gbar_out=gbar)
        ref = H.oracle_full(grads, d, J, h)
        try:
            if mode != "adamw":
                H.assert_stats_close(res, ref)
                H.assert_decision_matches(res, ref, h)
            else:
                assert res["status"] == B.NT_STATUS_NO_STATS and res["next_b"] == h.b_k
            if mode != "stats":
                H.oracle_adamw_check(grads, d, before[0], before[1], before[2], st[0], st[1], st[2], h, gbar=gbar)
            else:
                for a, b in zip(st, before):
                    assert torch.equal(a, b)
                if want_gbar:
                    g64 = grads.double().mean(dim=0)
                    H.assert_state_close("gbar", gbar.cpu().numpy(), g64.cpu().numpy())
        except AssertionError as e:
            raise AssertionError(ctx + ": " + str(e))
        assert bool((big[:, :off] == 3.0).all()) and bool((big[:, off + d:] == 3.0).all()), ctx


def test_noisy_gradients_and_tiny_second_moments_stay_within_the_adamw_bound():
    """Noise far above the state's scale with a small epsilon makes w sensitive to the relative error of gbar
    wherever gbar and v are both small.  300 seeded draws over every row-count path; the row sums must be
    exact enough (fp64 sums of the unshifted values, also for more than 16 rows) for all of them."""
    rng = np.random.default_rng(7)
    for case in range(300):
        J = int(rng.choice([2, 3, 4, 7, 8, 16, 17, 20, 24, 31, 32, 33, 40, 64, 70, 95, 96, 128, 200]))
        d = int(rng.choice([20000, 40001, 100000]))
        gdtype = torch.bfloat16 if rng.random() < 0.6 else torch.float32
        h = synth.Hyper(lr=float(rng.choice([1e-3, 4e-4, 1e-2])), beta1=float(rng.choice([0.9, 0.0, 0.5])),
                        beta2=float(rng.choice([0.95, 0.999])), eps=float(rng.choice([1e-8, 1e-12])),
                        weight_decay=float(rng.choice([0.1, 0.0])), eta=0.1, step=int(rng.choice([1, 2, 10, 1000])),
                        b_k=32, b_max=0, round_to=1, ddof=1)
        sigma = float(rng.choice([1e-3, 1e-2, 1e-1, 1.0]))
        mu = str(rng.choice(["normal", "sign"]))
        if sigma < 0.1 and case % 4:          # keep the run short: the quiet draws are covered elsewhere
            continue
        wl = synth.make("r", J, d, gdtype=gdtype, sigma=sigma, mu=mu, seed=5000 + case, device=DEV, hyper=h)
        w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
        res = gpu_step(wl.grads, wl.w, wl.m, wl.v, h)
        try:
            H.assert_stats_close(res, H.oracle_full(wl.grads, d, J, h))
            H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, h)
        except AssertionError as e:
            raise AssertionError("case %d: J=%d %s sigma=%g mu=%s lr=%g step=%d eps=%g: %s" % (
                case, J, gdtype, sigma, mu, h.lr, h.step, h.eps, e))


@pytest.mark.parametrize("J", [8, 33])
def test_subnormal_second_moment_keeps_the_sign_step(J):
    """Gradients around 1e-19 put (1 - beta2) gbar^2 into fp32's subnormal range.  From zero moments at k = 1 the
    update is lr * gbar / (|gbar| + eps), a sign step for eps far below |gbar| (closed form).  The stored v has
    few significant bits there, so only 1e-3 of the step is asked for; a square root that flushes subnormals
    would instead divide by eps alone and throw w off by many orders of magnitude."""
    d = 20000
    h = synth.Hyper(lr=1e-2, beta1=0.9, beta2=0.95, eps=1e-30, weight_decay=0.0, step=1, b_k=32)
    wl = synth.make("t", J, d, gdtype=torch.float32, sigma=1e-3, mu="sign", seed=77, device=DEV, hyper=h)
    g = wl.grads * 3e-17                                  # |gbar| about 3e-19: gbar^2 * 0.05 about 5e-39
    wl.m.zero_()
    wl.v.zero_()
    w0 = wl.w.clone()
    res = gpu_step(g, wl.w, wl.m, wl.v, h)
    assert res["status"] == 0
    gbar = g.double().mean(dim=0)
    v_expect = 0.05 * gbar * gbar
    assert float(v_expect.max()) < 1.2e-38 and float(v_expect.min()) > 1e-42      # all subnormal, none flushed
    expect = w0.double() - h.lr * torch.sign(gbar)
    assert bool(torch.isfinite(wl.w).all())
    assert float((wl.w.double() - expect).abs().max()) <= 1e-3 * h.lr
    assert float((wl.v.double() - v_expect).abs().max()) <= 1.5e-45              # within one subnormal step


def test_structural_sweep_over_entry_points_flags_and_alignment():
    """250 seeded draws of row count (2 .. 3000, every path and both routes), length, dtype, misalignment of rows
    and of state, row padding, entry point (strided, pointer table, clipped), mode, and the optional flags; all
    outputs against the oracle, and guard words around every buffer the library may write."""
    structural_sweep(21, 250, [2, 3, 5, 8, 13, 16, 17, 31, 47, 48, 64, 95, 96, 97, 300, 1000, 3000], 20000)


def test_structural_sweep_as_parts_of_a_long_vector():
    """The same sweep with a shard record that names a vector of 2^26 coordinates, which selects the launch classes
    for long vectors: up to 16 rows from 28 bytes of gradient per coordinate on (all the fp32 draws from 7 rows, bf16
    from 14 rows; AdamW only: from 20 bytes), and beyond 16 rows always (without the record these short vectors
    run in one launch of short tiles)."""
    structural_sweep(23, 260, [5, 6, 7, 8, 9, 10, 12, 14, 15, 16, 17, 20, 24, 47, 64, 300], 30000, whole=1 << 26)


def structural_sweep(seed, cases, J_choices, seed0, whole=None):
    rng = np.random.default_rng(seed)
    guard = 16
    for case in range(cases):
        J = int(rng.choice(J_choices))
        d = int(rng.choice([1, 3, 4, 100, 2047, 2048, 2049, 4095, 4097, 8192, 16383, 16385, 30000]))
        if J * d > 20_000_000:
            d = 2049
        gdtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        off = int(rng.choice([0, 0, 1, 2, 3, 4, 8]))
        pad = int(rng.choice([0, 0, 1, 3, 8, 64]))
        soff = int(rng.choice([0, 0, 1, 2, 4]))
        entry = str(rng.choice(["step", "rows", "clipped"]))
        mode = str(rng.choice(["full", "full", "stats", "adamw"])) if entry != "clipped" else "full"
        flags = {"full": FULL, "stats": B.NT_DO_STATS, "adamw": B.NT_DO_ADAMW}[mode]
        coord = mode != "adamw" and rng.random() < 0.5
        want_gbar = entry != "clipped" and rng.random() < 0.3
        partial = mode != "adamw" and entry != "clipped" and rng.random() < 0.2
        one_pass = rng.random() < 0.2
        h = synth.Hyper(eta=float(rng.choice([0.05, 0.2])), step=int(rng.choice([1, 7])), b_k=int(rng.choice([1, 32, 256])),
                        b_max=int(rng.choice([0, 512])), round_to=int(rng.choice([1, 16])), ddof=int(rng.integers(0, 2)))
        sigma = float(rng.choice([1e-3, 1e-2, 1e-1]))
        max_norm = float(rng.choice([0.0, 0.01, 100.0]))
        src = synth.make("r", J, d, gdtype=gdtype, sigma=sigma, seed=seed0 + case, device=DEV, hyper=h)
        if d == 1:
            continue                      # a one-element vector has no rms to measure AdamW errors against
        big = torch.full((J, off + d + pad), 3.0, dtype=gdtype, device=DEV)
        grads = big[:, off:off + d]
        grads.copy_(src.grads)
        st = []
        for s0 in (src.w, src.m, src.v):
            t = torch.full((guard + soff + d + guard,), 9.0, device=DEV)
            t[guard + soff:guard + soff + d] = s0
            st.append(t)
        view = lambda t: t[guard + soff:guard + soff + d]
        before = [view(t).clone() for t in st]
        gb = torch.full((guard + soff + d + guard,), 7.0, device=DEV)
        fl = (flags | (B.NT_COORD_TEST if coord else 0) | (B.NT_WRITE_GBAR if want_gbar else 0)
              | (B.NT_PARTIAL if partial else 0) | (B.NT_ONE_PASS if one_pass else 0))
        need = B.normtest_workspace_bytes(J, d)
        wsraw = torch.full((64 + need + 64,), 0x5A, dtype=torch.uint8, device=DEV)
        ws = wsraw[64:64 + need]
        ctx = "case %d J=%d d=%d %s off=%d pad=%d soff=%d entry=%s mode=%s coord=%s gbar=%s partial=%s one_pass=%s" % (
            case, J, d, gdtype, off, pad, soff, entry, mode, coord, want_gbar, partial, one_pass)
        shard = B.nt_shard_info(0, 1, 0, whole) if whole else None
        try:
            a = [view(t) if mode != "stats" else None for t in st]
            if entry == "step":
                res = B.normtest_step(grads, a[0], a[1], a[2], hyper_of(h, fl), d=d, shard=shard,
                                      gbar_out=view(gb) if want_gbar else None, workspace=ws)
            elif entry == "rows":
                res = B.normtest_step_rows([big[j, off:off + d] for j in range(J)], a[0], a[1], a[2], hyper_of(h, fl),
                                           d=d, shard=shard, gbar_out=view(gb) if want_gbar else None, workspace=ws)
            else:
                res = B.normtest_step_clipped(grads, a[0], a[1], a[2], view(gb), max_norm, hyper_of(h, fl), d=d,
                                              shard=shard, workspace=ws)
            torch.cuda.synchronize()
            r = B.read_result(res).as_dict()
            ref = H.oracle_full(grads, d, J, h)
            if mode != "adamw":
                H.assert_stats_close(r, ref, partial=partial)
                if not partial:
                    H.assert_decision_matches(r, ref, h)
                if coord:
                    H.assert_coord_matches(r, H.oracle_coord_counts(grads, d, h))
                else:
                    assert r["coord_fail"] == -1
            else:
                assert r["status"] == B.NT_STATUS_NO_STATS
            if mode != "stats":
                coef = oracle.clip_coef(ref.dec.gbar_sq, max_norm) if entry == "clipped" else 1.0
                H.oracle_adamw_check(grads, d, before[0], before[1], before[2], view(st[0]), view(st[1]), view(st[2]), h,
                                     gbar=view(gb) if want_gbar else None, grad_scale=coef)
            else:
                for t, b0 in zip(st, before):
                    assert torch.equal(view(t), b0)
            for t in st:
                assert bool((t[:guard + soff] == 9.0).all()) and bool((t[guard + soff + d:] == 9.0).all()), "state guard"
            assert bool((gb[:guard + soff] == 7.0).all()) and bool((gb[guard + soff + d:] == 7.0).all()), "gbar guard"
            if not (want_gbar or entry == "clipped"):
                assert bool((gb == 7.0).all()), "gbar touched"
            assert bool((big[:, :off] == 3.0).all()) and bool((big[:, off + d:] == 3.0).all()), "gradients written"
            assert bool((wsraw[:64] == 0x5A).all()) and bool((wsraw[64 + need:] == 0x5A).all()), "workspace guard"
        except AssertionError as e:
            raise AssertionError(ctx + ": " + str(e))


def test_maximum_row_count():
    """J = 2^20 rows (the largest the entry points accept) of a 9-coordinate vector: 65536 chunks per coordinate."""
    J, d = 1 << 20, 9
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    mu = torch.randn(d, device=DEV, generator=gen) * 1e-2
    grads = (mu + 1e-2 * torch.randn(J, d, device=DEV, generator=gen)).to(torch.bfloat16)
    h = synth.Hyper(b_k=64, round_to=1, step=2)
    w = torch.randn(d, device=DEV, generator=gen) * 0.02
    m = torch.randn(d, device=DEV, generator=gen) * 0.02
    v = (torch.randn(d, device=DEV, generator=gen) * 0.02) ** 2
    w0, m0, v0 = w.clone(), m.clone(), v.clone()
    res = gpu_step(grads, w, m, v, h, flags=FULL | B.NT_COORD_TEST)
    ref = H.oracle_full(grads, d, J, h)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, h)
    H.oracle_adamw_check(grads, d, w0, m0, v0, w, m, v, h)
    H.assert_coord_matches(res, H.oracle_coord_counts(grads, d, h))


# ------------------------------------------------------------------ memory safety and graph capture

@pytest.mark.parametrize("J,gdtype,flags", [(8, torch.bfloat16, FULL), (4, torch.float32, FULL),
                                            (33, torch.bfloat16, FULL), (8, torch.bfloat16, B.NT_DO_STATS),
                                            (16, torch.bfloat16, B.NT_DO_ADAMW), (19, torch.bfloat16, B.NT_DO_ADAMW),
                                            (20, torch.float32, FULL)])
def test_canaries_around_every_buffer_survive(J, gdtype, flags):
    """Every buffer the library may write sits between guard words; after a step (ragged d, with and
    without alignment) the guards and everything past d are untouched."""
    d = 2 * 16384 + 3001
    guard = 64
    for off in (0, 1):                                     # off = 1 breaks 16-byte alignment: guarded kernel path
        wl = synth.make("t", J, d, gdtype=gdtype, seed=31, device=DEV)
        bufs = {}
        for name, src in (("w", wl.w), ("m", wl.m), ("v", wl.v), ("gbar", torch.zeros(d, device=DEV))):
            big = torch.full((guard + off + d + guard,), 123.25, dtype=torch.float32, device=DEV)
            big[guard + off:guard + off + d] = src
            bufs[name] = big
        need = B.normtest_workspace_bytes(J, d)
        ws = torch.full((guard * 8 + need + guard * 8,), 0x5A, dtype=torch.uint8, device=DEV)
        resbuf = torch.full((guard * 8 + B.RESULT_BYTES + guard * 8,), 0x5A, dtype=torch.uint8, device=DEV)
        view = lambda n: bufs[n][guard + off:guard + off + d]
        res = B.normtest_step(wl.grads, view("w"), view("m"), view("v"), hyper_of(wl.hyper, flags | B.NT_WRITE_GBAR),
                              gbar_out=view("gbar"), workspace=ws[guard * 8:guard * 8 + need],
                              result=resbuf[guard * 8:guard * 8 + B.RESULT_BYTES])
        torch.cuda.synchronize()
        for name, big in bufs.items():
            assert bool((big[:guard + off] == 123.25).all()) and bool((big[guard + off + d:] == 123.25).all()), name
        assert bool((ws[:guard * 8] == 0x5A).all()) and bool((ws[guard * 8 + need:] == 0x5A).all())
        assert bool((resbuf[:guard * 8] == 0x5A).all()) and bool((resbuf[guard * 8 + B.RESULT_BYTES:] == 0x5A).all())
        r = B.read_result(res)
        assert r.status in (0, B.NT_STATUS_NO_STATS)


@pytest.mark.parametrize("J,gdtype,flags", [(64, torch.bfloat16, FULL), (64, torch.float32, FULL | B.NT_ONE_PASS),
                                            (96, torch.bfloat16, FULL | B.NT_ONE_PASS), (96, torch.bfloat16, FULL),
                                            (64, torch.float32, FULL), (512, torch.bfloat16, B.NT_DO_STATS)])
def test_workspace_of_exactly_the_size_for_this_call_is_enough(J, gdtype, flags):
    """normtest_workspace_bytes_for(gdtype, J, d, flags) is what the call needs and all it touches: guard bytes
    right behind a workspace of exactly that size survive, the result matches the oracle, and no call is asked for
    anything d-sized (the step is one pass at every row count; NT_ONE_PASS changes nothing)."""
    d = 5 * 2048 + 333
    guard = 512
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=77 + J, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=1, step=5))
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    need = B.normtest_workspace_bytes_for(B._gdtype(wl.grads), J, d, flags)
    upper = B.normtest_workspace_bytes(J, d)
    assert need == upper and need < 4096
    raw = torch.full((guard + need + guard,), 0x5A, dtype=torch.uint8, device=DEV)
    res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, flags), workspace=raw[guard:guard + need])
    torch.cuda.synchronize()
    assert bool((raw[:guard] == 0x5A).all()) and bool((raw[guard + need:] == 0x5A).all())
    got = B.read_result(res).as_dict()
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(got, ref)
    H.assert_decision_matches(got, ref, wl.hyper)
    if flags & B.NT_DO_ADAMW:
        H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper)
    with pytest.raises(B.NormtestError):
        B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, flags), workspace=raw[guard:guard + need - 8])


@pytest.mark.parametrize("J,gdtype", [(96, torch.bfloat16), (48, torch.float32), (100, torch.float32),
                                      (257, torch.bfloat16)])
def test_many_rows_in_one_pass_equal_the_explicit_two_phases(J, gdtype):
    """With many rows the step stays one pass (the state update of a tile deferred to the end of the block's walk):
    results match the oracle, NT_ONE_PASS changes nothing, the explicit two-phase entry point without a bound
    leaves the same bits, and nothing outside the declared workspace size is touched, whatever its alignment."""
    d = 3 * 8192 + 777
    guard = 64
    for shift in (0, 8):                                   # workspace base 16-byte aligned, or only 8-byte aligned
        wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=40 + J, device=DEV,
                        hyper=synth.Hyper(b_k=64, round_to=1, step=5))
        w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
        need = B.normtest_workspace_bytes(J, d)
        assert need < 4096                                  # a record and a few partials: no room for gbar, none needed
        raw = torch.full((guard * 8 + shift + need + guard * 8,), 0x5A, dtype=torch.uint8, device=DEV)
        lo = guard * 8 + shift
        assert (raw.data_ptr() + lo) % 16 == shift
        res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST),
                              workspace=raw[lo:lo + need])
        torch.cuda.synchronize()
        assert bool((raw[:lo] == 0x5A).all()) and bool((raw[lo + need:] == 0x5A).all())
        got = B.read_result(res).as_dict()
        ref = H.oracle_full(wl.grads, d, J, wl.hyper)
        H.assert_stats_close(got, ref)
        H.assert_decision_matches(got, ref, wl.hyper)
        H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, wl.hyper)
        H.assert_coord_matches(got, H.oracle_coord_counts(wl.grads, d, wl.hyper))
        # the flag that once forced the single pass is accepted and leaves the same bits
        w1, m1, v1 = w0.clone(), m0.clone(), v0.clone()
        res1 = B.normtest_step(wl.grads, w1, m1, v1, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST | B.NT_ONE_PASS))
        torch.cuda.synchronize()
        assert B.read_result(res1).as_dict() == got
        for a, b in zip((wl.w, wl.m, wl.v), (w1, m1, v1)):
            assert torch.equal(a, b)
        # the explicit two-phase entry point without a bound leaves the same bits
        w2, m2, v2 = w0.clone(), m0.clone(), v0.clone()
        gbar = torch.empty(d, dtype=torch.float32, device=DEV)
        res2 = B.normtest_step_clipped(wl.grads, w2, m2, v2, gbar, 0.0, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST))
        torch.cuda.synchronize()
        assert B.read_result(res2).as_dict() == got
        for a, b in zip((wl.w, wl.m, wl.v), (w2, m2, v2)):
            assert torch.equal(a, b)
        # and the per-layer table finds its partials in the workspace
        off = torch.tensor([0, 1000, d], dtype=torch.int64, device=DEV)
        lay = B.normtest_layer_stats(wl.grads, off, raw[lo:lo + need])
        torch.cuda.synchronize()
        layers = B.read_layers(lay)
        assert layers[0].status == 0 and layers[0].A + layers[1].A == pytest.approx(got["A"], rel=1e-7)


def test_result_in_pinned_host_memory_and_two_streams():
    """The result struct may live in pinned host memory, and calls on different streams with their own
    buffers do not interfere (the library keeps no state)."""
    wls = [synth.make("t", 8, 6 * 16384 + 11 * k, gdtype=torch.bfloat16, seed=40 + k, device=DEV) for k in range(2)]
    refs = []
    for wl in wls:
        st = [t.clone() for t in (wl.w, wl.m, wl.v)]
        refs.append((gpu_step(wl.grads, st[0], st[1], st[2], wl.hyper), st))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    pinned = [torch.zeros(B.RESULT_BYTES, dtype=torch.uint8).pin_memory() for _ in wls]
    ws = [torch.empty(B.normtest_workspace_bytes(wl.J, wl.d), dtype=torch.uint8, device=DEV) for wl in wls]
    torch.cuda.synchronize()
    for wl, s, pin, wsp in zip(wls, streams, pinned, ws):
        s.wait_stream(torch.cuda.current_stream())
        lib_rc = B.lib().normtest_step(wl.grads.data_ptr(), B.NT_BF16, wl.J, wl.d, wl.ld, wl.w.data_ptr(),
                                       wl.m.data_ptr(), wl.v.data_ptr(), None, hyper_of(wl.hyper), None,
                                       wsp.data_ptr(), wsp.numel(), pin.data_ptr(), s.cuda_stream)
        assert lib_rc == B.NT_OK
    for s in streams:
        s.synchronize()
    for wl, pin, (ref, st) in zip(wls, pinned, refs):
        got = B.nt_result.from_buffer_copy(pin.numpy().tobytes()).as_dict()
        assert got == ref
        for a, b in zip((wl.w, wl.m, wl.v), st):
            assert torch.equal(a, b)


@pytest.mark.parametrize("J,d", [(8, 5 * 16384 + 99), (24, 2 * 8388608 + 3 * 8192 + 99)])
def test_step_can_be_captured_in_a_hip_graph(J, d):
    """The step allocates nothing and records only kernel launches, so it can be captured; every replay,
    with eager work and synchronisation in between, must reproduce the eager result bit for bit.  The second case
    has more than 16 rows and is long enough for several launches of the step kernel (one generation of blocks
    each) inside the captured graph."""
    wl = synth.make("t", J, d, gdtype=torch.bfloat16, seed=32, device=DEV)
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    hy = hyper_of(wl.hyper)
    ws = torch.empty(B.normtest_workspace_bytes(wl.J, wl.d), dtype=torch.uint8, device=DEV)
    result = torch.zeros(B.RESULT_BYTES, dtype=torch.uint8, device=DEV)
    # eager reference: two consecutive steps
    eager = []
    for _ in range(2):
        B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, workspace=ws, result=result)
        torch.cuda.synchronize()
        eager.append((B.read_result(result).as_dict(), [t.clone() for t in (wl.w, wl.m, wl.v)]))
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, workspace=ws, result=result, stream=side)   # warm-up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, workspace=ws, result=result,
                        stream=torch.cuda.current_stream())
    for rounds in range(2):
        for t, s in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s)
        for k in range(2):
            result.zero_()
            graph.replay()
            torch.cuda.synchronize()
            got = B.read_result(result).as_dict()
            assert got == eager[k][0]
            for a, b in zip((wl.w, wl.m, wl.v), eager[k][1]):
                assert torch.equal(a, b)
            _ = (torch.randn(1 << 16, device=DEV) * 2).sum().item()        # unrelated eager work between replays


def test_clipped_step_and_layer_table_can_be_captured_together():
    """Both phases of the clipped step and the per-layer table in one graph (five kernel launches, no memsets,
    no allocation); replays must reproduce the eager results bit for bit."""
    wl = synth.make("t", 8, 6 * 4096 + 55, gdtype=torch.bfloat16, seed=33, device=DEV, sigma=3e-2)
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    hy = hyper_of(wl.hyper, FULL | B.NT_COORD_TEST)
    ws = torch.empty(B.normtest_workspace_bytes(wl.J, wl.d), dtype=torch.uint8, device=DEV)
    result = torch.zeros(B.RESULT_BYTES, dtype=torch.uint8, device=DEV)
    gbar = torch.empty(wl.d, dtype=torch.float32, device=DEV)
    off = torch.tensor([0, 5000, 5001, 20000, wl.d], dtype=torch.int64, device=DEV)
    layers = torch.zeros(4 * B.LAYER_BYTES, dtype=torch.uint8, device=DEV)

    def enqueue(stream):
        B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, 0.05, hy, workspace=ws, result=result, stream=stream)
        B.normtest_layer_stats(wl.grads, off, ws, layers=layers, stream=stream)

    eager = []
    for _ in range(2):
        enqueue(torch.cuda.current_stream())
        torch.cuda.synchronize()
        eager.append((B.read_result(result).as_dict(), layers.clone(), [t.clone() for t in (wl.w, wl.m, wl.v)]))
    assert eager[0][0]["clip_coef"] < 1.0 and eager[0][0]["coord_fail"] > 0
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(torch.cuda.current_stream())
    for rounds in range(2):
        for t, s in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s)
        for k in range(2):
            result.zero_()
            layers.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert B.read_result(result).as_dict() == eager[k][0]
            assert torch.equal(layers, eager[k][1])
            for a, b in zip((wl.w, wl.m, wl.v), eager[k][2]):
                assert torch.equal(a, b)
            _ = (torch.randn(1 << 16, device=DEV) * 2).sum().item()


def test_calib_copy():
    src = torch.randn(1 << 20, device=DEV)
    dst = torch.zeros_like(src)
    B.normtest_calib_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_calib_streams_touches_only_its_streams():
    """The stream-mix yardstick: written streams change, read streams and the bytes behind the declared size do
    not; in-place streams keep the exclusive-or structure (a second call restores nothing but stays in bounds);
    unsupported mixes and short buffers are refused before any launch."""
    coords = 3 * 4096 + 8
    for row_reads, reads, writes, rmw, lc in ((8, 0, 3, True, 0), (0, 11, 3, False, 0), (16, 0, 0, False, 0), (0, 0, 1, False, 0),
                                              (8, 3, 3, False, 0), (8, 0, 3, True, 4096), (8, 0, 3, True, 8192 + 4),
                                              (0, 2, 2, False, 4)):
        need = B.calib_streams_bytes(coords, row_reads, reads, writes)
        guard = 4096
        buf = torch.randint(0, 255, (need + guard,), dtype=torch.uint8, device=DEV)
        before = buf.clone()
        B.normtest_calib_streams(buf[:need], coords, row_reads, reads, writes, rmw, launch_coords=lc)
        torch.cuda.synchronize()
        if lc:
            # split into several launches the walk leaves the same bytes as in one
            once = before.clone()
            B.normtest_calib_streams(once[:need], coords, row_reads, reads, writes, rmw)
            torch.cuda.synchronize()
            assert torch.equal(buf, once), (row_reads, reads, writes, rmw, lc)
        r2 = (coords * 2 + 255) // 256 * 256
        r4 = (coords * 4 + 255) // 256 * 256
        read_end = row_reads * r2 + reads * r4
        assert torch.equal(buf[:read_end], before[:read_end])                       # read streams untouched
        assert torch.equal(buf[need - 16:], before[need - 16:])                      # spare word and guard untouched
        for k in range(writes):
            lo = read_end + k * r4
            assert not torch.equal(buf[lo:lo + 4 * coords], before[lo:lo + 4 * coords])   # written
            assert torch.equal(buf[lo + 4 * coords:lo + r4], before[lo + 4 * coords:lo + r4])  # padding of the stream
    small = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    for args, code in (((coords, 8, 0, 3, True), B.NT_ERR_WORKSPACE_TOO_SMALL), ((4, 7, 0, 3, True), B.NT_ERR_UNSUPPORTED),
                       ((4, 0, 0, 0, False), B.NT_ERR_UNSUPPORTED), ((5, 0, 1, 0, False), B.NT_ERR_BAD_ARG),
                       ((4, 17, 0, 0, False), B.NT_ERR_UNSUPPORTED)):
        with pytest.raises(B.NormtestError) as e:
            B.normtest_calib_streams(small, *args)
        assert e.value.code == code, args


def test_long_row_table_with_one_misaligned_row_at_the_end():
    """300 separately allocated rows: the alignment of all of them is checked once per call by a small kernel
    (more rows than that kernel has threads); a single row off by one element, the last one, must send the whole
    call down the guarded path, with the same bits as the aligned call and as the strided matrix."""
    J, d = 300, 2 * 2048 + 100
    wl = synth.make("t", J, d, gdtype=torch.bfloat16, sigma=1e-2, seed=91, device=DEV, hyper=synth.Hyper(b_k=512, round_to=1))
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    ref = gpu_step(wl.grads, wl.w, wl.m, wl.v, wl.hyper, flags=FULL | B.NT_COORD_TEST)
    ref_state = [t.clone() for t in (wl.w, wl.m, wl.v)]
    oracle_ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(ref, oracle_ref)
    H.assert_decision_matches(ref, oracle_ref, wl.hyper)
    for misaligned_row in (None, J - 1):
        rows = []
        for j in range(J):
            buf = torch.zeros(d + 16, dtype=torch.bfloat16, device=DEV)
            off = 1 if j == misaligned_row else 0
            rows.append(buf[off:off + d])
            rows[-1].copy_(wl.grads[j, :d])
        assert all(r.data_ptr() % 16 == 0 for r in rows[:J - 1]) and (rows[-1].data_ptr() % 16 == 0) == (misaligned_row is None)
        for t, s0 in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s0)
        res = B.normtest_step_rows(rows, wl.w, wl.m, wl.v, hyper_of(wl.hyper, FULL | B.NT_COORD_TEST))
        torch.cuda.synchronize()
        assert B.read_result(res).as_dict() == ref
        for a, b in zip((wl.w, wl.m, wl.v), ref_state):
            assert torch.equal(a, b)
