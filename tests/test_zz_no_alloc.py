"""normtest_step_static (the entry point that allocates nothing: its scratch is a static device array) against
normtest_step on the same inputs, called through the C ABI: two calls in a row, the second smaller, then a long
vector that takes the two-level reduction followed by a short one again, so that every call meets the leftovers
of a larger one in the shared scratch.  Results must agree bit for bit (same kernels), hence to the parity bar."""
import ctypes

import pytest
import torch

from paper_2412_21124_amd import binding as B
from paper_2412_21124_amd import synth

pytestmark = pytest.mark.gpu


def hyper_of(h, flags):
    return B.make_hyper(lr=h.lr, beta1=h.beta1, beta2=h.beta2, eps=h.eps, weight_decay=h.weight_decay, eta=h.eta,
                        step=h.step, b_k=h.b_k, b_max=h.b_max, round_to=h.round_to, ddof=h.ddof, flags=flags)


def run_both(J, d, gdtype, seed, flags, whole=None):
    dev = "cuda:0"
    shard = B.nt_shard_info(0, 1, 0, whole) if whole else None    # the call as a part of a vector of `whole` coordinates
    wl = synth.make("noalloc", J, d, gdtype=gdtype, sigma=1e-2, seed=seed, device=dev,
                    hyper=synth.Hyper(b_k=256, round_to=128, b_max=8192, step=10))
    hy = hyper_of(wl.hyper, flags)
    state = [t.clone() for t in (wl.w, wl.m, wl.v)]
    ref_state = [t.clone() for t in (wl.w, wl.m, wl.v)]
    ref = B.read_result(B.normtest_step(wl.grads, *ref_state, hy, shard=shard))
    # raw call through the C ABI: no workspace argument, caller-owned result
    result = torch.zeros(B.RESULT_BYTES, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    J_, ld = wl.grads.shape[0], wl.grads.stride(0)
    rc = B.lib().normtest_step_static(ctypes.c_void_p(wl.grads.data_ptr()), B._gdtype(wl.grads), J_, d, ld,
                                      ctypes.c_void_p(state[0].data_ptr()), ctypes.c_void_p(state[1].data_ptr()),
                                      ctypes.c_void_p(state[2].data_ptr()), None, ctypes.byref(hy),
                                      ctypes.byref(shard) if shard is not None else None,
                                      ctypes.c_void_p(result.data_ptr()), ctypes.c_void_p(stream.cuda_stream))
    assert rc == B.NT_OK, B.normtest_strerror(rc)
    got = B.read_result(result)
    assert bytes(got) == bytes(ref), (got.as_dict(), ref.as_dict())
    for name, a, b in zip("wmv", state, ref_state):
        assert torch.equal(a, b), name
    return got.as_dict()


def test_static_scratch_matches_workspace_entry_point_on_calls_in_a_row():
    full = B.NT_DO_STATS | B.NT_DO_ADAMW
    tc = B.normtest_tile_coords(8)
    print("call 1: J=8 bf16 d=%d" % (5 * tc + 777), flush=True)
    r1 = run_both(8, 5 * tc + 777, torch.bfloat16, 1, full | B.NT_COORD_TEST)
    assert r1["coord_fail"] >= 0 and r1["status"] == 0
    print("call 2 (smaller): J=4 fp32 d=%d" % (tc + 5), flush=True)
    r2 = run_both(4, tc + 5, torch.float32, 2, full)
    assert r2["A"] != r1["A"]
    print("call 3 (two-level reduction): J=8 bf16 d=20,000,003", flush=True)
    run_both(8, 20_000_003, torch.bfloat16, 3, full)
    print("call 4 (smaller again, statistics only, many rows): J=40 bf16 d=%d" % (3 * tc + 12), flush=True)
    run_both(40, 3 * tc + 12, torch.bfloat16, 4, B.NT_DO_STATS)
    print("call 5: J=128 bf16 (many rows: the state update deferred to the end of each block's walk)", flush=True)
    run_both(128, 2 * tc + 8, torch.bfloat16, 5, full)
    print("calls 6-8: parts of a vector of 2^26 coordinates (the launch classes for long vectors): 16 bf16, 8 fp32, 24 bf16 rows", flush=True)
    run_both(16, 3 * tc + 99, torch.bfloat16, 6, full, whole=1 << 26)
    run_both(8, 2 * tc + 5, torch.float32, 7, full | B.NT_COORD_TEST, whole=1 << 26)
    run_both(24, 2 * tc + 77, torch.bfloat16, 8, full, whole=1 << 26)


def test_static_entry_point_rejects_what_does_not_fit():
    """Beyond the stated maximum the call is refused before anything is enqueued (the host checks the size first)."""
    J = 8
    too_long = B.normtest_static_max_coords(J) + 1
    hy = B.make_hyper(step=1, b_k=32)
    z = torch.zeros(64, device="cuda:0")
    res = torch.zeros(B.RESULT_BYTES, dtype=torch.uint8, device="cuda:0")
    ptr = ctypes.c_void_p(z.data_ptr())
    rc = B.lib().normtest_step_static(ptr, B.NT_BF16, J, too_long, too_long, ptr, ptr, ptr, None, ctypes.byref(hy), None,
                                      ctypes.c_void_p(res.data_ptr()), None)
    assert rc == B.NT_ERR_TOO_LARGE
    assert "scratch" in B.normtest_strerror(rc)
    torch.cuda.synchronize()
    assert not res.any()


def test_static_entry_point_under_graph_capture():
    """What the entry point is for: captured in a HIP graph (it records kernel launches only: no allocation, no
    memset), every replay, with eager work in between, reproduces the eager results of normtest_step bit for bit."""
    dev = "cuda:0"
    wl = synth.make("noalloc_graph", 8, 5 * 16384 + 99, gdtype=torch.bfloat16, seed=9, device=dev,
                    hyper=synth.Hyper(b_k=256, round_to=128, b_max=8192, step=10))
    hy = hyper_of(wl.hyper, B.NT_DO_STATS | B.NT_DO_ADAMW)
    state0 = [t.clone() for t in (wl.w, wl.m, wl.v)]
    eager = []
    for _ in range(2):                                   # reference: two consecutive steps of the workspace entry point
        res = B.normtest_step(wl.grads, wl.w, wl.m, wl.v, hy)
        torch.cuda.synchronize()
        eager.append((bytes(B.read_result(res)), [t.clone() for t in (wl.w, wl.m, wl.v)]))
    for t, s in zip((wl.w, wl.m, wl.v), state0):
        t.copy_(s)
    result = torch.zeros(B.RESULT_BYTES, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        B.normtest_step_static(wl.grads, wl.w, wl.m, wl.v, hy, result, stream=side)      # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        B.normtest_step_static(wl.grads, wl.w, wl.m, wl.v, hy, result, stream=torch.cuda.current_stream())
    for rounds in range(2):
        for t, s in zip((wl.w, wl.m, wl.v), state0):
            t.copy_(s)
        for k in range(2):
            result.zero_()
            graph.replay()
            torch.cuda.synchronize()
            assert bytes(B.read_result(result)) == eager[k][0]
            for a, b in zip((wl.w, wl.m, wl.v), eager[k][1]):
                assert torch.equal(a, b)
            _ = (torch.randn(1 << 16, device=dev) * 2).sum().item()     # unrelated eager work between replays
