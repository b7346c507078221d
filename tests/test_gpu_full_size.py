"""GPU parity at the full sizes of the five workloads, in the launch configuration bench.py times
(preallocated workspace and result, torch's current stream).  The oracle streams the device-resident
inputs to the host chunk by chunk; every sum and every updated w, m, v element is compared."""
import math
import time

import numpy as np
import pytest
import torch

from paper_2412_21124_amd import binding as B
from paper_2412_21124_amd import synth

import helpers as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
FULL = B.NT_DO_STATS | B.NT_DO_ADAMW


def run_and_check(wl: synth.Workload, flags=FULL, shard=None, coord=False):
    if coord:
        flags |= B.NT_COORD_TEST
    h = wl.hyper
    t0 = time.time()
    w0, m0, v0 = wl.w.clone(), wl.m.clone(), wl.v.clone()
    hy = B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                      step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)
    workspace = torch.empty(B.normtest_workspace_bytes(wl.J, wl.d), dtype=torch.uint8, device=DEV)
    result = torch.empty(B.RESULT_BYTES, dtype=torch.uint8, device=DEV)
    B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, shard=shard, workspace=workspace, result=result,
                    stream=torch.cuda.current_stream())
    torch.cuda.synchronize()
    res = B.read_result(result).as_dict()
    t1 = time.time()
    ref = H.oracle_full(wl.grads, wl.d, wl.J, h)
    t2 = time.time()
    partial = bool(flags & B.NT_PARTIAL)
    H.assert_stats_close(res, ref, partial=partial)
    if partial:
        assert res["status"] == B.NT_STATUS_PARTIAL_ONLY and res["next_b"] == h.b_k
    else:
        H.assert_decision_matches(res, ref, h)
    n = H.oracle_adamw_check(wl.grads, wl.d, w0, m0, v0, wl.w, wl.m, wl.v, h)
    assert n == wl.d
    t3 = time.time()
    print("%s: J=%d d=%d  gpu %.1fs  oracle stats %.1fs  adamw compare %.1fs  T=%.6g oracle T=%.6g" % (
        wl.name, wl.J, wl.d, t1 - t0, t2 - t1, t3 - t2, res["T"], ref.dec.T), flush=True)
    if coord:
        counts = H.oracle_coord_counts(wl.grads, wl.d, h)
        H.assert_coord_matches(res, counts)
        print("   coordinate-wise: %d fail (oracle %d + %d near) of %d, largest ratio %.6g (oracle %.6g)" % (
            res["coord_fail"], counts[0], counts[1], wl.d, res["coord_max_ratio"], counts[3]), flush=True)
    else:
        assert res["coord_fail"] == -1 and res["coord_max_ratio"] == -1.0
    # the identity C = A - B/J holds for the GPU's own sums too (it never forms C that way)
    assert res["C"] == pytest.approx(res["A"] - res["B"] / wl.J, rel=1e-5 * res["A"] / res["C"])
    return res, ref


def test_tiny_full():
    for sigma in (1e-3, 1e-2):
        run_and_check(synth.tiny(sigma, device=DEV))


@pytest.mark.parametrize("ratio", [0.1, 0.3, 1.0, 1.94, 3.0, 10.0])
def test_gpt2_small_full(ratio):
    """d = 124,439,808 in 148 blocks with log-uniform scales, noise-to-signal ratio swept over 0.1 ... 10: the
    test passes below the crossing point r = 1.94 of b_k = 256 and fails above it (at 1.94 itself T sits next
    to b_k and the decision is whatever the oracle says)."""
    wl = synth.gpt2_small(ratio, device=DEV)
    assert wl.d == 124_439_808 and wl.meta["n_blocks"] == 148
    res, ref = run_and_check(wl)
    if ratio != 1.94:
        assert bool(res["pass"]) == (ratio < 1.94)
    # closed form of the ratio of expectations: T = r^2 / (eta^2 (1 + r^2 / J)), here eta = 0.1, J = 8
    r2 = ratio * ratio
    assert res["T"] == pytest.approx(r2 / (0.01 * (1 + r2 / 8)), rel=2e-2)


def test_gpt2_small_layer_table():
    """The per-layer table at full size: the 148 parameter blocks of the 124M-parameter model (sizes from 768
    to 38.6M coordinates, most boundaries inside a tile), every layer against the oracle on its columns."""
    import oracle
    wl = synth.gpt2_small(1.0, device=DEV)
    h = wl.hyper
    sizes = wl.meta["block_sizes"]
    offsets = [0]
    for s in sizes:
        offsets.append(offsets[-1] + s)
    assert len(sizes) == 148 and offsets[-1] == wl.d
    hy = B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                      step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof,
                      flags=FULL | B.NT_COORD_TEST)
    workspace = torch.empty(B.normtest_workspace_bytes(wl.J, wl.d), dtype=torch.uint8, device=DEV)
    off = torch.tensor(offsets, dtype=torch.int64, device=DEV)
    res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, workspace=workspace)
    lay = B.normtest_layer_stats(wl.grads, off, workspace)
    torch.cuda.synchronize()
    res = B.read_result(res).as_dict()
    layers = [x.as_dict() for x in B.read_layers(lay)]
    G = synth.grads_as_numpy(wl.grads, 0, wl.d)
    ref = oracle.layer_stats(G, offsets, h.eta, h.b_k, h.ddof, band=H.STATS_RTOL)
    for l, (got, want) in enumerate(zip(layers, ref)):
        assert got["n"] == sizes[l] and got["status"] == 0, l
        for k in "ABC":
            assert got[k] == pytest.approx(want[k], rel=H.STATS_RTOL), (l, k)
        assert got["T"] == pytest.approx(want["dec"].T, rel=2 * H.STATS_RTOL), l
        fail, near, _ = want["coord"]
        assert fail <= got["coord_fail"] <= fail + near, l
        H.assert_coord_ratio(got["coord_max_ratio"], want["coord_max_ratio"])
    for k in "ABC":
        assert math.fsum(x[k] for x in layers) == pytest.approx(res[k], rel=1e-7)
    assert sum(x["coord_fail"] for x in layers) == res["coord_fail"]
    assert max(x["coord_max_ratio"] for x in layers) == res["coord_max_ratio"]
    # every block shares mu and sigma up to its scale, which cancels in T: the layers' statistics agree with the
    # whole vector's up to sampling noise (largest for the 768-coordinate blocks)
    Ts = np.array([x["T"] for x in layers])
    assert np.all(np.abs(Ts / res["T"] - 1) < 0.25)
    print("gpt2_small layers: T whole %.4g, per layer min %.4g max %.4g" % (res["T"], Ts.min(), Ts.max()), flush=True)


def test_flat_1p5b_full():
    """The headline workload: J=8 bf16, d=1.5e9 (ragged: not a multiple of the tile)."""
    wl = synth.flat_1p5b(device=DEV)
    assert wl.d == 1_500_000_000 and wl.d % B.normtest_tile_coords(8) != 0
    run_and_check(wl, coord=True)


def test_fsdp_shard_full():
    """One GPU's 1/8 shard of a 7e9-parameter model, J=16 micro-batch gradients, partial sums only."""
    wl = synth.fsdp_shard(3, device=DEV)
    shard = B.nt_shard_info(3, 8, wl.meta["shard_offset"], wl.meta["d_global"])
    res, ref = run_and_check(wl, flags=FULL | B.NT_PARTIAL, shard=shard)
    assert math.isnan(res["T"])


def test_fsdp_all_eight_shards_combine_full():
    """The whole 7e9-parameter vector as eight sequential 875e6-coordinate shard calls (fresh seed per shard, J=16
    micro-batch gradients, partial sums + AdamW on the shard); the host combine of the eight partial results
    against the oracle over the concatenation, and AdamW on a sampled range of every shard."""
    import oracle
    parts, accs = [], []
    hyper = None
    t0 = time.time()
    for sid in range(8):
        wl = synth.fsdp_shard(sid, device=DEV)
        hyper, d = wl.hyper, wl.d
        lo = (sid * 104_729_111) % (d - (1 << 22))                     # a 4M-coordinate window, different per shard
        window = [(lo, lo + (1 << 22))]
        before = [t[lo:lo + (1 << 22)].clone() for t in (wl.w, wl.m, wl.v)]
        shard = B.nt_shard_info(sid, 8, wl.meta["shard_offset"], wl.meta["d_global"])
        hy = B.make_hyper(lr=hyper.lr, beta1=hyper.beta1, beta2=hyper.beta2, eps=hyper.eps,
                          weight_decay=hyper.weight_decay, eta=hyper.eta, step=hyper.step, b_k=hyper.b_k,
                          b_max=hyper.b_max, round_to=hyper.round_to, ddof=hyper.ddof, flags=FULL | B.NT_PARTIAL)
        res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy, shard=shard)
        torch.cuda.synchronize()
        r = B.read_result(res)
        assert r.status == B.NT_STATUS_PARTIAL_ONLY
        A, Bs, C = H.oracle_stats(wl.grads, d)
        H.assert_stats_close(r.as_dict(), H.OracleOut(A, Bs, C, None), partial=True)
        # AdamW on the window: rebuild full-length views of the pre-step state for the helper
        w0 = wl.w.clone(); m0 = wl.m.clone(); v0 = wl.v.clone()
        for full, part in zip((w0, m0, v0), before):
            full[lo:lo + (1 << 22)] = part
        H.oracle_adamw_check(wl.grads, d, w0, m0, v0, wl.w, wl.m, wl.v, hyper, ranges=window)
        parts.append(r)
        accs.append((A, Bs, C))
        print("shard %d: A=%.6g C=%.6g  (%.0f s so far)" % (sid, r.A, r.C, time.time() - t0), flush=True)
        del wl, w0, m0, v0
        torch.cuda.empty_cache()
    hy = B.make_hyper(eta=hyper.eta, b_k=hyper.b_k, b_max=hyper.b_max, round_to=hyper.round_to, ddof=hyper.ddof)
    comb = B.normtest_combine(parts, 16, hy).as_dict()
    A, Bs, C = oracle.combine_chunks(accs)
    ref = H.OracleOut(A, Bs, C, H.oracle_decide(A, Bs, C, 16, hyper), 16)
    H.assert_stats_close(comb, ref)
    H.assert_decision_matches(comb, ref, hyper)
    print("7e9 parameters in 8 shards: T=%.6g (oracle %.6g) next_b=%d" % (comb["T"], ref.dec.T, comb["next_b"]), flush=True)


def test_per_sample_full():
    """b = 512 per-example gradients of a 2^24 vector with Student-t(3) noise: the row-walking kernel."""
    wl = synth.per_sample(device=DEV)
    assert wl.J == 512 and wl.d == 1 << 24
    run_and_check(wl, coord=True)


def test_paper_model_sizes():
    """J = 4 worker gradients at the parameter counts of the paper's models (Table 4); the largest, 3.4e9
    coordinates and 109 GB of operands, is also the largest single call tested."""
    for which in ("300m", "1.1b", "3.4b"):
        wl = synth.paper_model(which, device=DEV)
        run_and_check(wl)
        del wl
        torch.cuda.empty_cache()


def test_more_than_2_to_31_coordinates():
    """64-bit indexing: d just above 2^31 with a ragged, odd end; J=2 keeps the footprint at 60 GB."""
    d = (1 << 31) + 12_293
    wl = synth.make("beyond_int32", 2, d, gdtype=torch.bfloat16, sigma=1e-2, seed=7, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=2, step=3))
    run_and_check(wl)


def test_more_tiles_than_the_grid_holds():
    """Beyond 2^20 tiles (d > 4.29e9 at 4096 coordinates per tile) the blocks of k_step take several tiles each.
    J = 2 bf16 rows keep the footprint at 70 GB; all sums, and AdamW on windows at the start, around the
    coordinate where the second round of tiles begins, and at the ragged end."""
    wrap = 4096 * (1 << 20)
    d = wrap + 4096 * 3000 + 77
    wl = synth.make("beyond_grid", 2, d, gdtype=torch.bfloat16, sigma=1e-2, seed=9, device=DEV,
                    hyper=synth.Hyper(b_k=64, round_to=2, step=3))
    h = wl.hyper
    win = 1 << 21
    windows = [(0, 2 * win), (wrap - win, wrap + win), (d - 2 * win, d)]
    keep = {lo: [t[lo:hi].clone() for t in (wl.w, wl.m, wl.v)] for lo, hi in windows}
    hy = B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                      step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof,
                      flags=FULL | B.NT_COORD_TEST)
    res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy)
    torch.cuda.synchronize()
    res = B.read_result(res).as_dict()
    ref = H.oracle_full(wl.grads, d, 2, h)
    H.assert_stats_close(res, ref)
    H.assert_decision_matches(res, ref, h)
    H.assert_coord_matches(res, H.oracle_coord_counts(wl.grads, d, h))
    import oracle
    for lo, hi in windows:
        G = synth.grads_as_numpy(wl.grads, lo, hi)
        w0, m0, v0 = (t.cpu().numpy() for t in keep[lo])
        out = oracle.adamw(G, w0, m0, v0, h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step)
        for name, got, want in zip("wmv", (wl.w, wl.m, wl.v), out):
            H.assert_state_close("%s[%d:%d]" % (name, lo, hi), got[lo:hi].cpu().numpy(), want)
    print("beyond the grid: d=%d T=%.6g (oracle %.6g)" % (d, res["T"], ref.dec.T), flush=True)
