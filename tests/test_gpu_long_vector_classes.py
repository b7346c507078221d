"""Up to 16 rows with at least 28 bytes of gradient per coordinate (14 bf16 or 7 fp32 rows; AdamW only: 20 bytes),
in a vector of at least 2^26 coordinates: steps that write per coordinate run in a second launch class (rows in
registers, the state update deferred to the end of an 8192-coordinate tile, one generation of blocks per launch).
More than 16 rows run that way from 2^24 coordinates on (more than 32 rows: 3 * 2^21) and in one launch of
2048-coordinate tiles below.  The class is chosen by the length of the whole vector, which a call that covers a
part of it states in its shard record; the small cases here use that to reach the classes for long vectors with
vectors the oracle finishes in a moment, the last ones run them at their real size."""
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
WHOLE = 1 << 26                      # shortest vector that takes the class
TILE = 8192                          # its tile


def hyper_of(h: synth.Hyper, flags=FULL) -> B.nt_hyper:
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                        step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)


def part_of_long_vector(d):
    """Shard record of a call whose d coordinates are the head of a vector of 2^26."""
    return B.nt_shard_info(0, 1, 0, max(d, WHOLE))


def run(wl, flags=FULL, shard=None, grads=None, state=None, d=None, gbar_out=None):
    w, m, v = state if state is not None else (wl.w, wl.m, wl.v)
    res = B.normtest_step(wl.grads if grads is None else grads, w, m, v, hyper_of(wl.hyper, flags), d=d, shard=shard,
                          gbar_out=gbar_out)
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


CASES = [(14, torch.bfloat16), (15, torch.bfloat16), (16, torch.bfloat16),
         (7, torch.float32), (8, torch.float32), (11, torch.float32), (16, torch.float32),
         # more than 16 rows: short vectors run in one launch of 2048-coordinate tiles, long ones like the above
         (17, torch.bfloat16), (20, torch.float32), (21, torch.bfloat16), (33, torch.bfloat16), (100, torch.bfloat16)]


@pytest.mark.parametrize("J,gdtype", CASES)
def test_fused_step_in_the_deferred_class(J, gdtype):
    """Statistics, decision, coordinate-wise count and every updated element against the oracle; the same bits in
    w, m, v as the interleaved class leaves (the arithmetic per coordinate is the same), the sums to rounding of a
    differently ordered fp64 addition; and the same bits again from misaligned buffers (guarded tiles)."""
    d = 5 * TILE + 3 * 512 + 77
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=41 + J, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=J, step=3))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    flags = FULL | B.NT_COORD_TEST
    plain = run(wl, flags)
    plain_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    g2, st2 = shifted_copy(wl)
    res = run(wl, flags, shard=part_of_long_vector(d))
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    H.assert_coord_matches(res, H.oracle_coord_counts(wl.grads, d, wl.hyper))
    assert H.oracle_adamw_check(wl.grads, d, *state0, wl.w, wl.m, wl.v, wl.hyper) == d
    for a, b in zip((wl.w, wl.m, wl.v), plain_state):
        assert torch.equal(a, b)
    for k in ("A", "B", "C", "T"):
        assert res[k] == pytest.approx(plain[k], rel=1e-13), k
    for k in ("next_b", "pass", "status", "coord_fail", "coord_max_ratio"):
        assert res[k] == plain[k], k
    res2 = run(wl, flags, shard=part_of_long_vector(d), grads=g2, state=st2, d=d)
    assert res2 == res
    for a, b in zip(st2, (wl.w, wl.m, wl.v)):
        assert torch.equal(a, b)


@pytest.mark.parametrize("J,gdtype", [(14, torch.bfloat16), (9, torch.float32)])
def test_adamw_only_and_stored_mean_in_the_deferred_class(J, gdtype):
    """AdamW only: same bits as the fused step's update.  Statistics with the mean stored (first phase of the clipped
    step): the stored mean is the oracle's and the state stays untouched."""
    d = 3 * TILE + 1029
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=47, device=DEV, hyper=synth.Hyper(b_k=32, round_to=J, step=5))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    shard = part_of_long_vector(d)
    run(wl, FULL, shard=shard)
    fused = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    res = run(wl, B.NT_DO_ADAMW, shard=shard)
    assert res["status"] == B.NT_STATUS_NO_STATS
    for a, b in zip((wl.w, wl.m, wl.v), fused):
        assert torch.equal(a, b)
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    gbar = torch.full((d,), 7.0, dtype=torch.float32, device=DEV)
    res = run(wl, B.NT_DO_STATS | B.NT_WRITE_GBAR, shard=shard, gbar_out=gbar)
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    h = wl.hyper
    out = oracle.adamw(synth.grads_as_numpy(wl.grads, 0, d), *(t.cpu().numpy() for t in state0), h.lr, h.beta1, h.beta2,
                       h.eps, h.weight_decay, h.step, want_gbar=True)
    H.assert_state_close("gbar", gbar.cpu().numpy(), out[3], rtol=1e-6)
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        assert torch.equal(t, s)


@pytest.mark.parametrize("J,gdtype", [(10, torch.bfloat16), (13, torch.bfloat16), (5, torch.float32), (6, torch.float32)])
def test_adamw_only_takes_the_deferred_class_from_fewer_rows(J, gdtype):
    """AdamW only (no sums, so nothing depends on the tiles): the class from 20 bytes of gradient per coordinate on.
    Same bits as the call that stands alone, aligned and misaligned, and within the bound of the oracle's AdamW."""
    d = 4 * TILE + 2 * 512 + 5
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=60 + J, device=DEV, hyper=synth.Hyper(b_k=32, round_to=J, step=4))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    run(wl, B.NT_DO_ADAMW)
    alone = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    g2, st2 = shifted_copy(wl)
    res = run(wl, B.NT_DO_ADAMW, shard=part_of_long_vector(d))
    assert res["status"] == B.NT_STATUS_NO_STATS
    run(wl, B.NT_DO_ADAMW, shard=part_of_long_vector(d), grads=g2, state=st2, d=d)
    for a, b, c in zip((wl.w, wl.m, wl.v), alone, st2):
        assert torch.equal(a, b) and torch.equal(a, c)
    assert H.oracle_adamw_check(wl.grads, d, *state0, wl.w, wl.m, wl.v, wl.hyper) == d


@pytest.mark.parametrize("J,gdtype", [(2, torch.bfloat16), (8, torch.bfloat16), (16, torch.bfloat16), (4, torch.float32)])
def test_read_only_statistics_in_both_tile_sizes(J, gdtype):
    """Statistics only, up to 16 rows: vectors shorter than 2^21 coordinates are cut into 4096-coordinate tiles,
    longer ones into 16384.  Both against the oracle (the second reached through the shard record), aligned and
    misaligned with the same bits, and nothing but the result written."""
    d = 3 * 16384 + 4096 + 3 * 512 + 7
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=70 + J, device=DEV, hyper=synth.Hyper(b_k=64, round_to=J, step=3))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    g2, _ = shifted_copy(wl)
    flags = B.NT_DO_STATS | B.NT_COORD_TEST
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    counts = H.oracle_coord_counts(wl.grads, d, wl.hyper)
    got = []
    for shard in (None, part_of_long_vector(d)):
        res = run(wl, flags, shard=shard)
        H.assert_stats_close(res, ref)
        H.assert_decision_matches(res, ref, wl.hyper)
        H.assert_coord_matches(res, counts)
        res2 = B.normtest_step(g2, None, None, None, hyper_of(wl.hyper, flags), d=d, shard=shard)
        torch.cuda.synchronize()
        assert B.read_result(res2).as_dict() == res
        got.append(res)
    for k in ("A", "B", "C", "T"):
        assert got[0][k] == pytest.approx(got[1][k], rel=1e-13), k
    for k in ("next_b", "pass", "status", "coord_fail", "coord_max_ratio"):
        assert got[0][k] == got[1][k], k
    for t, s0 in zip((wl.w, wl.m, wl.v), state0):
        assert torch.equal(t, s0)


def test_row_table_and_clipped_step_in_the_deferred_class():
    """Row pointers instead of a matrix, and the two-phase clipped step, both as parts of a long vector."""
    J, d = 8, 4 * TILE + 333
    wl = synth.make("t", J, d, gdtype=torch.float32, sigma=1e-2, seed=48, device=DEV, hyper=synth.Hyper(b_k=32, round_to=J, step=2))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    shard = part_of_long_vector(d)
    res = run(wl, FULL, shard=shard)
    fused = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    rows = [wl.grads[j, :d].clone() for j in range(J)]
    r2 = B.normtest_step_rows(rows, wl.w, wl.m, wl.v, hyper_of(wl.hyper), shard=shard)
    torch.cuda.synchronize()
    assert B.read_result(r2).as_dict() == res
    for a, b in zip((wl.w, wl.m, wl.v), fused):
        assert torch.equal(a, b)
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    ref = H.oracle_full(wl.grads, d, J, wl.hyper)
    max_norm = 0.5 * math.sqrt(ref.dec.gbar_sq)
    gbar = torch.zeros(d, dtype=torch.float32, device=DEV)
    r3 = B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, max_norm, hyper_of(wl.hyper), shard=shard)
    torch.cuda.synchronize()
    r3 = B.read_result(r3).as_dict()
    H.assert_stats_close(r3, ref)
    coef = oracle.clip_coef(ref.dec.gbar_sq, max_norm)
    assert r3["clip_coef"] == pytest.approx(coef, rel=1e-6) and coef < 1.0
    assert H.oracle_adamw_check(wl.grads, d, *state0, wl.w, wl.m, wl.v, wl.hyper, gbar=gbar, grad_scale=coef) == d


@pytest.mark.parametrize("J,whole", [(16, WHOLE), (24, 1 << 24)])
def test_parts_of_a_long_vector_add_up_bit_exactly(J, whole):
    """A vector long enough for the class, cut at multiples of normtest_tile_coords into parts that are far too short
    for it on their own: with the whole length in their shard records they are cut into the same tiles, so the
    combined sums and the state equal the one call's bit for bit."""
    tc = B.normtest_tile_coords(J)
    d = whole + 3 * tc + 517
    wl = synth.make("t", J, d, gdtype=torch.bfloat16, sigma=1e-2, seed=49, device=DEV, hyper=synth.Hyper(b_k=64, round_to=J, step=2))
    state0 = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    full = run(wl, FULL)
    whole_state = (wl.w.clone(), wl.m.clone(), wl.v.clone())
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    cuts = [0, 2 * tc, 100 * tc, whole // 2 + tc, d]
    parts = []
    for sid, (lo, hi) in enumerate(zip(cuts[:-1], cuts[1:])):
        res = B.normtest_step(wl.grads[:, lo:hi], wl.w[lo:hi], wl.m[lo:hi], wl.v[lo:hi],
                              hyper_of(wl.hyper, FULL | B.NT_PARTIAL), shard=B.nt_shard_info(sid, len(cuts) - 1, lo, d))
        torch.cuda.synchronize()
        parts.append(B.read_result(res))
    comb = B.normtest_combine(parts, J, hyper_of(wl.hyper)).as_dict()
    for k in ("A", "B", "C", "gbar_sq", "var_l1", "T", "next_b", "pass", "status"):
        assert comb[k] == full[k], k
    for a, b in zip((wl.w, wl.m, wl.v), whole_state):
        assert torch.equal(a, b)


@pytest.mark.parametrize("J,gdtype,misaligned", [(14, torch.bfloat16, False), (7, torch.float32, True)])
def test_deferred_class_at_its_real_size(J, gdtype, misaligned):
    """Just past 2^26 coordinates without any shard record: eight full generations of blocks, a launch with a few
    tiles and a ragged tile; everything against the oracle."""
    d = WHOLE + 5 * TILE + 13
    wl = synth.make("t", J, d, gdtype=gdtype, sigma=1e-2, seed=50, device=DEV, hyper=synth.Hyper(b_k=64, round_to=J, step=3))
    grads, state = (wl.grads, (wl.w, wl.m, wl.v))
    if misaligned:
        grads, state = shifted_copy(wl)
    state0 = tuple(t.clone() for t in state)
    res = run(wl, FULL, grads=grads, state=state, d=d)
    ref = H.oracle_full(grads, d, J, wl.hyper)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, wl.hyper)
    assert H.oracle_adamw_check(grads, d, *state0, *state, wl.hyper) == d
