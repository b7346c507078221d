"""GPU parity of the per-layer table: normtest_layer_stats, called through the C ABI after each kind of
step, against the oracle evaluated on every layer's columns."""
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
RTOL = H.STATS_RTOL


def hyper_of(h: synth.Hyper, flags=FULL) -> B.nt_hyper:
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay,
                        eta=h.eta, step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to,
                        ddof=h.ddof, flags=flags)


def offsets_for(d, tile, rng, n_cuts=12):
    """Ascending offsets that exercise every case: aligned and unaligned cuts, several cuts inside one tile,
    empty layers, a layer inside one tile, layers that do not start at 0 / end at d."""
    cuts = set(int(x) for x in rng.integers(0, d + 1, size=n_cuts))
    if d > 3 * tile:
        cuts |= {tile, 2 * tile, 2 * tile + 1, 2 * tile + 5, 2 * tile + 5, 3 * tile - 1}
    off = sorted(cuts)
    off = off[:3] + [off[2]] + off[3:]          # an empty layer
    return off


def run_layers(wl, flags, offsets, *, rows=False, clipped=False, coord=False, whole=None):
    h = wl.hyper
    d, J = wl.d, wl.J
    shard = B.nt_shard_info(0, 1, 0, whole) if whole else None     # the step as a part of a vector of `whole`
    if coord:
        flags |= B.NT_COORD_TEST
    ws = torch.empty(B.normtest_workspace_bytes(J, d), dtype=torch.uint8, device=DEV)
    off = torch.tensor(offsets, dtype=torch.int64, device=DEV)
    hy = hyper_of(h, flags)
    if rows:
        rws = [wl.grads[j, :d].clone() for j in range(J)]
        res = B.normtest_step_rows(rws, wl.w, wl.m, wl.v, hy, d=d, shard=shard, workspace=ws)
        lay = B.normtest_layer_stats(rws, off, ws, d=d)
    elif clipped:
        gbar = torch.empty(d, dtype=torch.float32, device=DEV)
        res = B.normtest_step_clipped(wl.grads, wl.w, wl.m, wl.v, gbar, 1.0, hy, d=d, shard=shard, workspace=ws)
        lay = B.normtest_layer_stats(wl.grads, off, ws, d=d)
    else:
        res = B.normtest_step(wl.grads, wl.w if flags & B.NT_DO_ADAMW else None, wl.m if flags & B.NT_DO_ADAMW else None,
                              wl.v if flags & B.NT_DO_ADAMW else None, hy, d=d, shard=shard, workspace=ws)
        lay = B.normtest_layer_stats(wl.grads, off, ws, d=d)
    torch.cuda.synchronize()
    return B.read_result(res).as_dict(), [x.as_dict() for x in B.read_layers(lay)]


def check_layers(wl, res, layers, offsets, coord=False):
    h = wl.hyper
    G = synth.grads_as_numpy(wl.grads, 0, wl.d)
    ref = oracle.layer_stats(G, offsets, h.eta, h.b_k, h.ddof, band=RTOL if coord else None)
    assert len(layers) == len(ref) == len(offsets) - 1
    for l, (got, want) in enumerate(zip(layers, ref)):
        tag = "layer %d [%d, %d)" % (l, offsets[l], offsets[l + 1])
        assert got["n"] == want["n"], tag
        assert not got["status"] & (B.NT_STATUS_BAD_RANGE | B.NT_STATUS_NO_STATS), tag
        for k in "ABC":
            assert got[k] == pytest.approx(want[k], rel=RTOL, abs=0.0), (tag, k)
        dec = want["dec"]
        if want["n"] == 0:
            assert got["A"] == got["B"] == got["C"] == 0.0 and math.isnan(got["T"]) and got["pass"] == 1, tag
            assert got["status"] & B.NT_STATUS_ZERO_GRAD_NORM
            continue
        assert got["gbar_sq"] == pytest.approx(dec.gbar_sq, rel=RTOL), tag
        assert got["var_l1"] == pytest.approx(dec.var_l1, rel=RTOL), tag
        assert got["T"] == pytest.approx(dec.T, rel=2 * RTOL), tag
        if not H.near_b_k(dec.T, h.b_k):   # no rounding chain per layer: only b_k itself is a threshold
            assert bool(got["pass"]) == dec.passed, tag
        if coord:
            fail, near, _ = want["coord"]
            assert fail <= got["coord_fail"] <= fail + near, (tag, got["coord_fail"], fail, near)
            H.assert_coord_ratio(got["coord_max_ratio"], want["coord_max_ratio"])
        else:
            assert got["coord_fail"] == -1 and got["coord_max_ratio"] == -1.0
    # the layers of a partition add up to the step's own sums (pieces of tiles are re-added coordinate by
    # coordinate, the step adds four fp32 terms at a time: agreement to fp32 rounding, averaged over the piece)
    if offsets[0] == 0 and offsets[-1] == wl.d:
        for k in "ABC":
            assert math.fsum(x[k] for x in layers) == pytest.approx(res[k], rel=1e-7), k
        if coord:
            assert sum(x["coord_fail"] for x in layers) == res["coord_fail"]
            assert max(x["coord_max_ratio"] for x in layers) == res["coord_max_ratio"]


CASES = [
    # J, dtype, d, mode
    (8, torch.bfloat16, 5 * 16384 + 1237, "full"),
    (8, torch.bfloat16, 5 * 16384 + 1237, "stats"),
    (8, torch.bfloat16, 5 * 16384 + 1237, "clipped"),
    (8, torch.bfloat16, 5 * 16384 + 1237, "rows"),
    (4, torch.float32, 3 * 16384 + 5, "full"),
    (2, torch.float32, 70001, "stats"),
    (16, torch.bfloat16, 4 * 16384, "full"),
    (3, torch.bfloat16, 40000, "full"),
    (33, torch.bfloat16, 9 * 2048 + 77, "full"),
    (40, torch.float32, 9 * 2048 + 77, "stats"),
]


@pytest.mark.parametrize("J,gdtype,d,mode", CASES)
def test_layers_match_oracle(J, gdtype, d, mode):
    rng = np.random.default_rng(J * 1000 + d % 997)
    wl = synth.make("layers", J, d, gdtype=gdtype, sigma=2e-2, seed=J + d % 13, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=J, step=4))
    flags = B.NT_DO_STATS if mode == "stats" else FULL
    tile = {"full": 4096, "stats": 16384, "clipped": 4096, "rows": 4096}[mode] if J <= 16 else 2048
    offsets = [0] + offsets_for(d, tile, rng) + [d]
    res, layers = run_layers(wl, flags, offsets, rows=mode == "rows", clipped=mode == "clipped", coord=True)
    check_layers(wl, res, layers, offsets, coord=True)


LONG_CASES = [
    # J, dtype, d, mode: with a shard record that names a vector of 2^26 coordinates these steps leave 8192-coordinate
    # tiles (statistics only, up to 16 rows: 16384 instead of the 4096 of a short vector)
    (16, torch.bfloat16, 5 * 8192 + 1237, "full"),
    (14, torch.bfloat16, 5 * 8192 + 1237, "clipped"),
    (8, torch.float32, 5 * 8192 + 1237, "rows"),
    (8, torch.bfloat16, 5 * 16384 + 1237, "stats"),
    (33, torch.bfloat16, 6 * 8192 + 77, "full"),
    (20, torch.float32, 6 * 8192 + 77, "clipped"),
]


@pytest.mark.parametrize("J,gdtype,d,mode", LONG_CASES)
def test_layers_after_a_step_in_the_long_vector_classes(J, gdtype, d, mode):
    rng = np.random.default_rng(J * 1000 + d % 991)
    wl = synth.make("layers", J, d, gdtype=gdtype, sigma=2e-2, seed=J + d % 11, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=J, step=4))
    flags = B.NT_DO_STATS if mode == "stats" else FULL
    tile = 16384 if mode == "stats" else 8192
    offsets = [0] + offsets_for(d, tile, rng) + [d]
    res, layers = run_layers(wl, flags, offsets, rows=mode == "rows", clipped=mode == "clipped", coord=True, whole=1 << 26)
    check_layers(wl, res, layers, offsets, coord=True)


def test_layers_without_coordinate_count_and_partial_cover():
    """No NT_COORD_TEST: counts are -1; layers that cover only the middle of the vector."""
    d = 3 * 4096 + 100
    wl = synth.make("layers", 8, d, gdtype=torch.bfloat16, sigma=1e-2, seed=3, device=DEV)
    offsets = [17, 4095, 4096, 4097, 9000, d - 3]
    res, layers = run_layers(wl, FULL, offsets)
    check_layers(wl, res, layers, offsets)


def test_single_layer_equals_the_step():
    d = 7 * 4096 + 11
    wl = synth.make("layers", 8, d, gdtype=torch.bfloat16, sigma=1e-2, seed=4, device=DEV)
    res, layers = run_layers(wl, FULL, [0, d], coord=True)
    one = layers[0]
    for k in ("A", "B", "C", "gbar_sq", "var_l1", "T"):
        assert one[k] == pytest.approx(res[k], rel=1e-7), k
    assert one["coord_fail"] == res["coord_fail"] and one["pass"] == res["pass"] and one["n"] == d


def test_many_tiles_go_through_the_group_partials():
    """More than 4096 tiles: the step leaves group partials, which whole groups inside a layer use."""
    d = 4096 * 9000 + 321
    wl = synth.make("layers", 2, d, gdtype=torch.bfloat16, sigma=1e-2, seed=5, device=DEV, with_state=False)
    offsets = [0, 5, 2048 * 4096, 2048 * 4096 + 1, 3 * 2048 * 4096 - 1, 4 * 2048 * 4096 + 4096 * 3, d - 1, d]
    ws = torch.empty(B.normtest_workspace_bytes(2, d), dtype=torch.uint8, device=DEV)
    off = torch.tensor(offsets, dtype=torch.int64, device=DEV)
    w = torch.zeros(d, dtype=torch.float32, device=DEV)
    m = torch.zeros_like(w)
    v = torch.zeros_like(w)
    res = B.normtest_step(wl.grads, w, m, v, hyper_of(wl.hyper, FULL), workspace=ws)
    lay = B.normtest_layer_stats(wl.grads, off, ws)
    torch.cuda.synchronize()
    check_layers(wl, B.read_result(res).as_dict(), [x.as_dict() for x in B.read_layers(lay)], offsets)


def test_bad_offsets_are_clamped_and_flagged():
    d = 2 * 4096 + 9
    wl = synth.make("layers", 4, d, gdtype=torch.float32, sigma=1e-2, seed=6, device=DEV)
    offsets = [-5, 100, 50, d + 1000, d + 2000]
    res, layers = run_layers(wl, FULL, offsets)
    G = synth.grads_as_numpy(wl.grads, 0, d)
    # layer 0: [-5, 100) -> [0, 100); layer 1: [100, 50) -> empty; layer 2: [50, d+1000) -> [50, d); layer 3: empty at d
    want = oracle.layer_stats(G, [0, 100, 100, 100], wl.hyper.eta, wl.hyper.b_k, wl.hyper.ddof)
    assert layers[0]["status"] & B.NT_STATUS_BAD_RANGE and layers[0]["n"] == 100
    assert layers[0]["A"] == pytest.approx(want[0]["A"], rel=RTOL)
    assert layers[1]["status"] & B.NT_STATUS_BAD_RANGE and layers[1]["n"] == 0 and layers[1]["A"] == 0.0
    w2 = oracle.layer_stats(G, [50, d], wl.hyper.eta, wl.hyper.b_k, wl.hyper.ddof)[0]
    assert layers[2]["status"] & B.NT_STATUS_BAD_RANGE and layers[2]["n"] == d - 50
    assert layers[2]["C"] == pytest.approx(w2["C"], rel=RTOL)
    assert layers[3]["status"] & B.NT_STATUS_BAD_RANGE and layers[3]["n"] == 0


def test_workspace_of_another_call_is_refused():
    """The record in the workspace must match gdtype, J and d, and must come from a statistics step."""
    d = 4096 + 40
    wl = synth.make("layers", 4, d, gdtype=torch.float32, sigma=1e-2, seed=7, device=DEV)
    ws = torch.zeros(B.normtest_workspace_bytes(4, d), dtype=torch.uint8, device=DEV)
    off = torch.tensor([0, 10, d - 1], dtype=torch.int64, device=DEV)

    def layers_now(grads, dd):
        lay = B.normtest_layer_stats(grads, off, ws, d=dd)
        torch.cuda.synchronize()
        return [x.as_dict() for x in B.read_layers(lay)]

    for x in layers_now(wl.grads, d):                      # never used by a step
        assert x["status"] & B.NT_STATUS_NO_STATS and math.isnan(x["A"]) and x["coord_fail"] == -1
    B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, B.NT_DO_ADAMW), workspace=ws)
    for x in layers_now(wl.grads, d):                      # the step skipped the statistics
        assert x["status"] & B.NT_STATUS_NO_STATS
    B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hyper_of(wl.hyper, FULL), workspace=ws)
    assert not layers_now(wl.grads, d)[0]["status"] & B.NT_STATUS_NO_STATS
    for x in layers_now(wl.grads, d - 1):                  # another d
        assert x["status"] & B.NT_STATUS_NO_STATS
    for x in layers_now(wl.grads[:3], d):                  # another J
        assert x["status"] & B.NT_STATUS_NO_STATS
    for x in layers_now(wl.grads.view(torch.bfloat16)[:, :d], d):   # another dtype
        assert x["status"] & B.NT_STATUS_NO_STATS


def test_partial_step_layers_add_over_shards():
    """Two shards cut inside a layer: the shards' per-layer sums add up to the layer's sums."""
    d, cut = 6 * 4096, 2 * 4096 + 128
    wl = synth.make("layers", 8, d, gdtype=torch.bfloat16, sigma=1e-2, seed=8, device=DEV)
    offsets = [0, 5000, 20000, d]
    G = synth.grads_as_numpy(wl.grads, 0, d)
    want = oracle.layer_stats(G, offsets, wl.hyper.eta, wl.hyper.b_k, wl.hyper.ddof)
    tot = [dict(A=0.0, B=0.0, C=0.0) for _ in want]
    for lo, hi in ((0, cut), (cut, d)):
        g = wl.grads[:, lo:hi]
        ws = torch.empty(B.normtest_workspace_bytes(8, hi - lo), dtype=torch.uint8, device=DEV)
        local = [min(max(o - lo, 0), hi - lo) for o in offsets]
        off = torch.tensor(local, dtype=torch.int64, device=DEV)
        B.normtest_step(g, wl.w[lo:hi], wl.m[lo:hi], wl.v[lo:hi], hyper_of(wl.hyper, FULL | B.NT_PARTIAL), workspace=ws)
        lay = B.normtest_layer_stats(g, off, ws)
        torch.cuda.synchronize()
        for t, x in zip(tot, B.read_layers(lay)):
            for k in "ABC":
                t[k] += getattr(x, k)
    for t, w_ in zip(tot, want):
        for k in "ABC":
            assert t[k] == pytest.approx(w_[k], rel=RTOL)


def test_layer_table_sweep():
    """200 seeded draws of row count, length, dtype, kind of step, number and position of cuts (layers that start
    after 0 or end before d included): every layer against the oracle."""
    rng = np.random.default_rng(31)
    for case in range(200):
        J = int(rng.choice([2, 3, 8, 16, 17, 40, 96, 130]))
        d = int(rng.choice([1, 5, 4096, 4097, 20000, 70001, 200000]))
        gdtype = torch.bfloat16 if rng.random() < 0.5 else torch.float32
        mode = str(rng.choice(["full", "stats", "clipped", "rows"]))
        coord = bool(rng.random() < 0.5)
        wl = synth.make("layers", J, d, gdtype=gdtype, sigma=float(rng.choice([1e-3, 2e-2])), seed=300 + case, device=DEV,
                        hyper=synth.Hyper(b_k=int(rng.choice([8, 64])), round_to=1, step=4, ddof=int(rng.integers(0, 2))))
        cuts = sorted(int(x) for x in rng.integers(0, d + 1, size=int(rng.choice([0, 1, 5, 40]))))
        lo = 0 if rng.random() < 0.7 else int(rng.integers(0, d + 1))
        hi = d if rng.random() < 0.7 else int(rng.integers(lo, d + 1))
        offsets = sorted([lo] + [c for c in cuts if lo <= c <= hi] + [hi])
        flags = B.NT_DO_STATS if mode == "stats" else FULL
        try:
            res, layers = run_layers(wl, flags, offsets, rows=mode == "rows", clipped=mode == "clipped", coord=coord)
            check_layers(wl, res, layers, offsets, coord=coord)
        except AssertionError as e:
            raise AssertionError("case %d J=%d d=%d %s mode=%s coord=%s offsets=%s: %s" % (
                case, J, d, gdtype, mode, coord, offsets[:8], e))
