"""CPU-only checks of libnormtest.so: it loads, exports what include/normtest.h declares, validates its
arguments before touching the GPU, and its host-side combine / decision agrees with the oracle."""
import ctypes
import math
import os
import re

import numpy as np
import pytest

import oracle
from paper_2412_21124_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FULL = B.NT_DO_STATS | B.NT_DO_ADAMW


def declared_functions():
    text = open(os.path.join(ROOT, "include", "normtest.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(normtest_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert {"normtest_step", "normtest_combine", "normtest_workspace_bytes", "normtest_tile_coords",
            "normtest_strerror", "normtest_calib_copy", "normtest_step_clipped", "normtest_adamw_gbar",
            "normtest_clip_coef", "normtest_step_rows", "normtest_resplit", "normtest_layer_stats", "normtest_schedule_flags"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n


def test_struct_layouts_match_header():
    assert ctypes.sizeof(B.nt_hyper) == 6 * 8 + 4 * 8 + 4 + 4
    assert ctypes.sizeof(B.nt_result) == 10 * 8 + 8 + 8 + 4 + 4 + 8
    assert ctypes.sizeof(B.nt_shard_info) == 4 + 4 + 8 + 8
    assert ctypes.sizeof(B.nt_layer_stats) == 6 * 8 + 8 + 8 + 4 + 4 + 8


def test_plain_c_client_sees_the_layout_the_binding_assumes(tmp_path):
    """include/normtest.h compiles as strict C99; a C program linked against the library calls the host-only
    entry points; every struct field offset and enum value it prints equals the ctypes mirror's."""
    import subprocess
    libpath = B.lib()._name
    exe = str(tmp_path / "abi_probe")
    libdir = os.path.dirname(libpath)
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "abi_probe.c"), "-o", exe, "-L", libdir, "-lnormtest",
                    "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib", "-Wl,--allow-shlib-undefined"], check=True)
    out = subprocess.run([exe], check=True, capture_output=True, text=True).stdout.splitlines()
    mirrors = {"nt_hyper": B.nt_hyper, "nt_shard_info": B.nt_shard_info, "nt_result": B.nt_result,
               "nt_layer_stats": B.nt_layer_stats}
    seen = {k: 0 for k in mirrors}
    n_enum = 0
    for line in out:
        tok = line.split()
        if tok[0] == "size":
            assert ctypes.sizeof(mirrors[tok[1]]) == int(tok[2]), line
        elif tok[0] == "field":
            cls = mirrors[tok[1]]
            name = "pass_" if tok[2] == "pass" else tok[2]
            f = getattr(cls, name)
            assert (f.offset, f.size) == (int(tok[3]), int(tok[4])), line
            seen[tok[1]] += 1
        elif tok[0] == "enum":
            assert getattr(B, tok[1]) == int(tok[2]), line
            n_enum += 1
    for k, cls in mirrors.items():
        assert seen[k] == len(cls._fields_), k          # every field of the mirror exists in the header and back
    assert n_enum == 21
    lines = {l.split()[0]: l.split()[1:] for l in out if l.split()[0] in ("combine", "resplit", "clip", "workspace", "workspace_for", "static_max", "strerror")}
    A, Bv, C, T, passed, next_b = lines["combine"]
    assert (float(A), float(Bv), float(C), float(T), int(passed), int(next_b)) == (50.0, 80.0, 10.0, 2.0, 0, 2)
    assert [int(x) for x in lines["resplit"]] == [8, 256, 8192]
    assert float(lines["clip"][0]) == pytest.approx(1.0 / (2.0 + 1e-6), rel=1e-15)
    assert int(lines["workspace"][0]) == B.normtest_workspace_bytes(8, 1000000) and int(lines["workspace"][2]) == 16384
    bf16_64, f32_64, any_64 = (int(x) for x in lines["workspace_for"])
    assert bf16_64 == f32_64 == any_64 == B.normtest_workspace_bytes(64, 1000000)
    assert int(lines["static_max"][0]) == B.normtest_static_max_coords(8)


def test_workspace_and_tiles():
    for J in (2, 8, 16, 17, 47, 48, 512):
        tc = B.normtest_tile_coords(J)
        assert tc == 16384
        prev = 0
        for d in (0, 1, tc, tc + 1, 5000 * tc, 1_500_000_000):
            need = B.normtest_workspace_bytes(J, d)
            # a 256-byte record, five doubles per tile (tiles are at most tc and at least 1024 coordinates), and
            # a small second level
            lo = 256 + 40 * max(1, -(-d // tc))
            hi = 256 + 40 * max(1, -(-d // 1024))
            assert lo <= need <= hi + hi // 256 + 64
            assert need >= prev and need % 8 == 0 and B.normtest_workspace_bytes(J, d) % 8 == 0
            prev = need
    assert B.normtest_tile_coords(1) == 0
    assert B.normtest_workspace_bytes(1, 10) == 0 and B.normtest_workspace_bytes(4, -1) == 0


def test_workspace_size_for_a_known_call():
    """The size for a known dtype and flags is the general one for every valid dtype and flag word (no call keeps
    a gbar buffer in the workspace: the step is one pass at every row count), and it is what the step checks."""
    full = B.NT_DO_STATS | B.NT_DO_ADAMW
    d = 3_000_001
    for J in (2, 16, 47, 48, 95, 96, 512):
        upper = B.normtest_workspace_bytes(J, d)
        assert upper < 256 + d // 16                  # a record and a few doubles per tile, nothing d-sized
        for gd in (B.NT_BF16, B.NT_F32):
            for flags in (full, full | B.NT_ONE_PASS, full | B.NT_WRITE_GBAR, B.NT_DO_STATS, B.NT_DO_ADAMW,
                          B.NT_DO_STATS | B.NT_PARTIAL | B.NT_WRITE_GBAR):
                assert B.normtest_workspace_bytes_for(gd, J, d, flags) == upper
    assert B.normtest_workspace_bytes_for(7, 8, 100, full) == 0
    assert B.normtest_workspace_bytes_for(B.NT_BF16, 1, 100, full) == 0
    hy = B.make_hyper(step=1, b_k=32, flags=full)
    need = B.normtest_workspace_bytes_for(B.NT_BF16, 64, 1 << 20, full)
    for gd in (B.NT_BF16, B.NT_F32):
        assert _call(J=64, d=1 << 20, gdtype=gd, hyper=hy, ws_bytes=need - 8) == B.NT_ERR_WORKSPACE_TOO_SMALL
    one = B.make_hyper(step=1, b_k=32, flags=full | B.NT_ONE_PASS)
    assert _call(J=64, d=1 << 20, gdtype=B.NT_F32, hyper=one, ws_bytes=need - 8) == B.NT_ERR_WORKSPACE_TOO_SMALL


def _call(J=4, d=64, ld=None, gdtype=B.NT_F32, grads=0x1000, w=0x2000, m=0x3000, v=0x4000, gbar=None,
          hyper=None, shard=None, ws=0x5000, ws_bytes=1 << 20, result=0x6000):
    """normtest_step with fabricated pointers: only legal for calls that must be rejected before any launch."""
    hyper = hyper if hyper is not None else B.make_hyper(step=1, b_k=32, flags=FULL)
    return B.lib().normtest_step(grads, gdtype, J, d, d if ld is None else ld, w, m, v, gbar,
                                 ctypes.byref(hyper), ctypes.byref(shard) if shard else None,
                                 ws, ws_bytes, result, None)


def test_bad_arguments_are_rejected_before_any_launch():
    bad = B.NT_ERR_BAD_ARG
    assert _call(J=1) == bad
    assert _call(J=(1 << 20) + 1) == bad                     # more rows than the entry points accept
    assert _call(d=-1) == bad
    assert _call(d=64, ld=63) == bad
    assert _call(grads=None) == bad
    assert _call(w=None) == bad
    assert _call(result=None) == bad
    assert _call(ws=None) == bad
    assert _call(result=0x6004) == bad                       # result not 8-byte aligned
    assert _call(grads=0x1002) == bad                        # fp32 rows not 4-byte aligned
    assert _call(gdtype=B.NT_BF16, grads=0x1001) == bad
    assert _call(w=0x2002) == bad
    assert _call(gdtype=7) == B.NT_ERR_UNSUPPORTED
    assert _call(ws_bytes=24) == B.NT_ERR_WORKSPACE_TOO_SMALL
    for kw in (dict(eta=0.0), dict(eta=-1.0), dict(eta=math.nan), dict(step=0), dict(b_k=0), dict(b_max=-1),
               dict(round_to=0), dict(round_to=(1 << 31) + 1), dict(ddof=2), dict(beta1=1.0), dict(beta2=-0.1), dict(lr=-1.0),
               dict(eps=-1e-8), dict(weight_decay=math.inf), dict(flags=0), dict(flags=64 | FULL),
               dict(flags=B.NT_COORD_TEST | B.NT_DO_ADAMW),
               dict(flags=B.NT_PARTIAL | B.NT_DO_ADAMW)):
        args = dict(step=1, b_k=32, flags=FULL)
        args.update(kw)
        assert _call(hyper=B.make_hyper(**args)) == bad, kw
    assert _call(hyper=B.make_hyper(step=1, b_k=32, flags=FULL | B.NT_WRITE_GBAR), gbar=None) == bad
    assert _call(shard=B.nt_shard_info(8, 8, 0, 64)) == bad   # shard_id out of range
    assert _call(shard=B.nt_shard_info(0, 8, 10, 64)) == bad  # shard runs past d_global
    # stats-only calls do not need w, m, v: this one gets past validation only to fail on the workspace
    assert _call(w=None, m=None, v=None, hyper=B.make_hyper(b_k=32, flags=B.NT_DO_STATS), ws_bytes=0) \
        == B.NT_ERR_WORKSPACE_TOO_SMALL


def test_clipped_entry_points_validate_before_launch():
    L = B.lib()
    hy = B.make_hyper(step=1, b_k=32, flags=FULL)
    args = lambda **kw: dict(dict(grads=0x1000, gdtype=B.NT_F32, J=4, d=64, ld=64, w=0x2000, m=0x3000, v=0x4000,
                                  gbar=0x7000, max_norm=1.0, hyper=hy, ws=0x5000, ws_bytes=1 << 20,
                                  result=0x6000), **kw)

    def call(a):
        return L.normtest_step_clipped(a["grads"], a["gdtype"], a["J"], a["d"], a["ld"], a["w"], a["m"], a["v"],
                                       a["gbar"], a["max_norm"], ctypes.byref(a["hyper"]), None, a["ws"],
                                       a["ws_bytes"], a["result"], None)

    bad = B.NT_ERR_BAD_ARG
    assert call(args(gbar=None)) == bad
    assert call(args(w=None)) == bad
    assert call(args(J=1)) == bad
    assert call(args(max_norm=math.nan)) == bad
    assert call(args(hyper=B.make_hyper(step=1, b_k=32, flags=B.NT_DO_STATS))) == bad          # needs AdamW too
    assert call(args(hyper=B.make_hyper(step=1, b_k=32, flags=FULL | B.NT_PARTIAL))) == bad     # no global norm in a shard
    assert call(args(ws_bytes=0)) == B.NT_ERR_WORKSPACE_TOO_SMALL
    # phase 2 alone
    f = L.normtest_adamw_gbar
    assert f(None, 64, 0x2000, 0x3000, 0x4000, ctypes.byref(hy), 1.0, None, None) == bad
    assert f(0x7000, -1, 0x2000, 0x3000, 0x4000, ctypes.byref(hy), 1.0, None, None) == bad
    assert f(0x7000, 64, 0x2000, 0x3000, 0x4000, ctypes.byref(hy), math.inf, None, None) == bad
    assert f(0x7002, 64, 0x2000, 0x3000, 0x4000, ctypes.byref(hy), 1.0, None, None) == bad
    assert f(0x7000, 64, 0x2000, 0x3000, 0x4000, ctypes.byref(B.make_hyper(step=0)), 1.0, None, None) == bad
    assert f(0x7000, 0, None, None, None, ctypes.byref(hy), 1.0, None, None) == B.NT_OK               # d = 0: nothing to do


def test_static_entry_point_validates_before_launch():
    """normtest_step_static: the size limit and the argument checks come before any HIP call."""
    hy = B.make_hyper(step=1, b_k=32, flags=FULL)
    L = B.lib()

    def call(J=8, d=64, ld=None, w=0x2000, hyper=hy, result=0x6000):
        return L.normtest_step_static(0x1000, B.NT_BF16, J, d, d if ld is None else ld, w, 0x3000, 0x4000, None,
                                      ctypes.byref(hyper), None, result, None)

    for J in (2, 8, 16, 17, 512):
        top = B.normtest_static_max_coords(J)
        assert top > (16 * 10 ** 8 if J <= 16 else 8 * 10 ** 8)    # the headline size fits
        assert call(J=J, d=top + 1) == B.NT_ERR_TOO_LARGE
        assert B.normtest_workspace_bytes_for(B.NT_BF16, J, top, B.NT_DO_STATS) <= 16 << 20
    assert B.normtest_static_max_coords(1) == 0
    assert call(J=1) == B.NT_ERR_BAD_ARG
    assert call(d=-1) == B.NT_ERR_BAD_ARG
    assert call(ld=63) == B.NT_ERR_BAD_ARG
    assert call(w=None) == B.NT_ERR_BAD_ARG
    assert call(result=None) == B.NT_ERR_BAD_ARG
    assert call(hyper=B.make_hyper(step=1, b_k=0, flags=FULL)) == B.NT_ERR_BAD_ARG
    assert "scratch" in B.normtest_strerror(B.NT_ERR_TOO_LARGE)


def test_calib_streams_validates_before_launch():
    """The yardstick refuses unsupported mixes, ragged sizes and short buffers without touching the GPU."""
    L = B.lib()
    coords = 3 * 4096 + 8
    call = lambda buf, nbytes, c, a, r, w, rmw, lc=0: L.normtest_calib_streams(buf, nbytes, c, a, r, w, rmw, lc, None)
    assert call(0x10000, 1 << 16, coords, 8, 0, 3, 1) == B.NT_ERR_WORKSPACE_TOO_SMALL
    assert call(0x10000, B.calib_streams_bytes(coords, 8, 0, 3) - 1, coords, 8, 0, 3, 1) == B.NT_ERR_WORKSPACE_TOO_SMALL
    assert call(0x10000, 1 << 16, 4, 7, 0, 3, 1) == B.NT_ERR_UNSUPPORTED       # no kernel for 7 row reads
    assert call(0x10000, 1 << 16, 4, 8, 0, 3, 0) == B.NT_ERR_UNSUPPORTED       # 8 row reads + 3 plain writes: not in the list
    assert call(0x10000, 1 << 16, 4, 0, 0, 0, 0) == B.NT_ERR_UNSUPPORTED
    assert call(0x10000, 1 << 16, 4, 17, 0, 0, 0) == B.NT_ERR_UNSUPPORTED
    assert call(0x10000, 1 << 16, 5, 0, 1, 0, 0) == B.NT_ERR_BAD_ARG           # coords not a multiple of 4
    assert call(0x10008, 1 << 16, 4, 0, 1, 0, 0) == B.NT_ERR_BAD_ARG           # buffer not 16-byte aligned
    assert call(0x10000, 1 << 16, 4, 0, 1, 0, 0, -4) == B.NT_ERR_BAD_ARG       # negative launch size
    assert call(0x10000, 1 << 16, 4, 0, 1, 0, 0, 6) == B.NT_ERR_BAD_ARG        # launch size not a multiple of 4
    assert call(None, 1 << 16, 4, 0, 1, 0, 0) == B.NT_ERR_BAD_ARG
    assert call(0x10000, 1 << 16, 0, 0, 1, 0, 0) == B.NT_OK                    # nothing to do


def test_rows_entry_point_validates_before_launch():
    L = B.lib()
    hy = B.make_hyper(step=1, b_k=32, flags=FULL)

    def call(table=0x1000, gdtype=B.NT_BF16, J=4, d=64, w=0x2000, m=0x3000, v=0x4000, hyper=hy, ws=0x5000,
             ws_bytes=1 << 20, result=0x6000):
        return L.normtest_step_rows(table, gdtype, J, d, w, m, v, None, ctypes.byref(hyper), None, ws, ws_bytes,
                                    result, None)

    bad = B.NT_ERR_BAD_ARG
    assert call(table=None) == bad
    assert call(table=0x1004) == bad            # the table itself must be 8-byte aligned
    assert call(J=1) == bad
    assert call(d=-5) == bad
    assert call(w=None) == bad
    assert call(gdtype=9) == B.NT_ERR_UNSUPPORTED
    assert call(ws_bytes=0) == B.NT_ERR_WORKSPACE_TOO_SMALL


def test_layer_entry_point_validates_before_launch():
    L = B.lib()

    def call(grads=0x1000, table=0, gdtype=B.NT_BF16, J=4, d=64, ld=64, off=0x2000, n=3, ws=0x5000, out=0x6000):
        return L.normtest_layer_stats(grads, table, gdtype, J, d, ld, off, n, ws, out, None)

    bad = B.NT_ERR_BAD_ARG
    assert call(grads=None) == bad
    assert call(grads=0x1001) == bad
    assert call(table=1, grads=0x1004) == bad     # a pointer table must be 8-byte aligned
    assert call(J=1) == bad
    assert call(d=-1) == bad
    assert call(ld=63) == bad
    assert call(off=None) == bad
    assert call(off=0x2004) == bad
    assert call(n=0) == bad
    assert call(ws=None) == bad
    assert call(ws=0x5004) == bad
    assert call(out=None) == bad
    assert call(out=0x6004) == bad
    assert call(gdtype=5) == B.NT_ERR_UNSUPPORTED


def test_resplit_matches_oracle():
    rng = np.random.default_rng(4)
    cases = [(256, 4, 16, 8), (8192, 4, 16, 8), (576, 4, 16, 8), (1, 1, 1, 1), (10**12, 8, 16, 8)]
    cases += [(int(rng.integers(1, 10**6)), int(rng.integers(1, 65)), int(rng.integers(1, 65)), int(rng.integers(1, 33)))
              for _ in range(3000)]
    for c in cases:
        assert B.normtest_resplit(*c) == oracle.resplit(*c), c
    for bad in ((0, 4, 16, 8), (256, 0, 16, 8), (256, 4, 0, 8), (256, 4, 16, 0)):
        with pytest.raises(B.NormtestError):
            B.normtest_resplit(*bad)


def test_schedule_flags_match_oracle():
    """The library drops the statistics flags exactly on the steps on which the oracle says no test is due."""
    stats_bits = B.NT_DO_STATS | B.NT_PARTIAL | B.NT_COORD_TEST
    rng = np.random.default_rng(11)
    for _ in range(3000):
        step = int(rng.integers(1, 500))
        interval = int(rng.choice([1, 1, 2, 3, 5, 16, 100]))
        b_max = int(rng.choice([0, 256, 8192]))
        b_k = int(rng.choice([1, 255, 256, 257, 4096, 8191, 8192, 8193]))
        flags = int(rng.choice([FULL, B.NT_DO_STATS, FULL | B.NT_COORD_TEST, FULL | B.NT_PARTIAL | B.NT_WRITE_GBAR,
                                B.NT_DO_ADAMW]))
        got = B.normtest_schedule_flags(step, interval, b_k, b_max, flags)
        want = flags if oracle.test_due(step, interval, b_k, b_max) else flags & ~stats_bits
        assert got == want, (step, interval, b_k, b_max, flags)
    assert B.normtest_schedule_flags(3, 2, 32, 0, B.NT_DO_STATS) == B.NT_DO_STATS      # (3 - 1) % 2 == 0: tests
    assert B.normtest_schedule_flags(2, 2, 32, 0, B.NT_DO_STATS) == 0                   # nothing left to do
    for bad in ((0, 1, 32, 0), (1, 0, 32, 0), (1, 1, 0, 0), (1, 1, 32, -1)):
        assert B.normtest_schedule_flags(*bad, FULL) == FULL


def test_clip_coef_matches_oracle():
    for gsq, mx in ((4.0, 1.0), (0.25, 1.0), (1.0, 1.0), (0.0, 1.0), (9.0, 0.0), (9.0, -1.0), (1e-30, 1e-3),
                    (math.inf, 1.0)):
        assert B.normtest_clip_coef(gsq, mx) == oracle.clip_coef(gsq, mx)
    assert B.normtest_clip_coef(4.0, 1.0) == pytest.approx(1.0 / (2.0 + 1e-6), rel=1e-15)
    assert B.normtest_clip_coef(0.25, 1.0) == 1.0


def test_strerror():
    assert B.normtest_strerror(0) == "success"
    assert "argument" in B.normtest_strerror(B.NT_ERR_BAD_ARG)
    assert "workspace" in B.normtest_strerror(B.NT_ERR_WORKSPACE_TOO_SMALL)
    assert B.normtest_strerror(B.NT_ERR_HIP_BASE - 1)       # some HIP text
    assert "unknown" in B.normtest_strerror(-5)


def test_binding_refuses_cpu_tensors():
    import torch
    g = torch.zeros((4, 16))
    z = torch.zeros(16)
    with pytest.raises(ValueError):
        B.normtest_step(g, z, z.clone(), z.clone(), B.make_hyper(b_k=4))


def _part(A, Bv, C, status=B.NT_STATUS_PARTIAL_ONLY):
    return B.nt_result(A=A, B=Bv, C=C, status=status)


def test_combine_decision_agrees_with_oracle_on_random_sums():
    rng = np.random.default_rng(0)
    n_checked = 0
    for trial in range(4000):
        J = int(rng.integers(2, 40))
        ddof = int(rng.integers(0, 2))
        eta = float(rng.choice([0.05, 0.1, 0.15, 0.275, 0.5]))
        b_k = int(rng.choice([1, 32, 256, 4096]))
        b_max = int(rng.choice([0, 512, 8192]))
        round_to = int(rng.choice([1, 4, 64, 128]))
        Bv = float(10 ** rng.uniform(-6, 3))
        C = float(10 ** rng.uniform(-8, 3))
        A = C + Bv / J
        hy = B.make_hyper(eta=eta, b_k=b_k, b_max=b_max, round_to=round_to, ddof=ddof)
        got = B.normtest_combine([_part(A, Bv, C)], J, hy)
        want = oracle.decide(A, Bv, C, J, eta, b_k, b_max, round_to, ddof)
        assert got.T == pytest.approx(want.T, rel=1e-14)
        assert got.gbar_sq == pytest.approx(want.gbar_sq, rel=1e-15)
        assert got.var_l1 == pytest.approx(want.var_l1, rel=1e-15)
        if got.T != want.T:
            continue                                      # last-bit difference of T: ceiling may differ
        n_checked += 1
        assert (got.next_b, bool(got.pass_), got.status) == (want.next_b, want.passed, want.status)
    assert n_checked > 3000


def test_combine_special_cases_agree_with_oracle():
    cases = [
        (0.0, 0.0, 0.0), (2.0, 0.0, 2.0), (math.nan, 1.0, 1.0), (math.inf, 1.0, 1.0),
        (1e300, 1e-300, 1e300), (20.0, 16.0, 16.0), (20.0, 16.0, 0.0),
    ]
    for A, Bv, C in cases:
        for b_max in (0, 8192):
            hy = B.make_hyper(eta=0.1, b_k=32, b_max=b_max, round_to=4, ddof=1)
            status_in = B.NT_STATUS_PARTIAL_ONLY | (0 if math.isfinite(A) else B.NT_STATUS_NONFINITE)
            got = B.normtest_combine([_part(A, Bv, C, status_in)], 4, hy)
            want = oracle.decide(A, Bv, C, 4, 0.1, 32, b_max, 4, 1)
            assert (got.next_b, bool(got.pass_), got.status) == (want.next_b, want.passed, want.status), (A, Bv, C)
            assert (math.isnan(got.T) and math.isnan(want.T)) or got.T == want.T


def _golden_decision_cases():
    import test_oracle_pins as P
    return [c for c in P.GOLDEN_CASES if "expect_T" in c and "expect_A" in c]


@pytest.mark.parametrize("case", _golden_decision_cases(), ids=lambda c: c["name"])
def test_host_decision_on_hand_worked_cases(case):
    """The library's own decision (host side of normtest_combine) against the hand-worked values under
    tests/golden/, edge conventions included: no oracle in the loop, so a convention the two share by
    mistake would still have to match the written value."""
    J = len(case["g"])
    hy = B.make_hyper(eta=float(case["eta"]), b_k=int(case["b_k"]), b_max=int(case["b_max"]),
                      round_to=int(case["round_to"]), ddof=int(case["ddof"]))
    got = B.normtest_combine([_part(float(case["expect_A"]), float(case["expect_B"]), float(case["expect_C"]))], J, hy)
    want_T = float(case["expect_T"])
    if math.isnan(want_T):
        assert math.isnan(got.T)
    elif math.isinf(want_T):
        assert got.T == want_T
    else:
        assert got.T == pytest.approx(want_T, rel=1e-14)
    assert got.gbar_sq == pytest.approx(float(case["expect_gbar_sq"]), rel=1e-15)
    assert got.var_l1 == pytest.approx(float(case["expect_var_l1"]), rel=1e-15)
    assert (got.pass_, got.next_b) == (int(case["expect_pass"]), int(case["expect_next_b"]))
    if "expect_status" in case:
        assert got.status == int(case["expect_status"])


def test_rounding_chain_cannot_overflow():
    """Largest accepted granularity with the largest statistic that is not treated as infinite: the next multiple
    of round_to still fits an int64 (both in the library and in the oracle), and a larger round_to is refused."""
    J, eta, b_k, rt = 2, 1.0, 1, 1 << 31
    T = float((1 << 62) - (1 << 10))               # largest double below 2^62 is 2^62 - 2^9; this one is exact too
    Bv = 4.0                                       # gbar_sq = 1
    C = T                                          # ddof 1: var_l1 = C
    hy = B.make_hyper(eta=eta, b_k=b_k, b_max=0, round_to=rt, ddof=1)
    got = B.normtest_combine([_part(C + Bv / J, Bv, C)], J, hy)
    want = oracle.decide(C + Bv / J, Bv, C, J, eta, b_k, 0, rt, 1)
    assert got.T == want.T == T
    expect = -(-int(T) // rt) * rt
    assert expect == 1 << 62 and got.next_b == want.next_b == expect and got.status == want.status == 0
    with pytest.raises(B.NormtestError):
        B.normtest_combine([_part(1, 1, 1)], J, B.make_hyper(eta=eta, b_k=b_k, round_to=rt + 1))
    with pytest.raises(ValueError):
        oracle.decide(1.0, 1.0, 1.0, J, eta, b_k, 0, rt + 1, 1)


def test_combine_adds_shards_in_double_double():
    # eight partial sums whose exact total is not representable after naive accumulation
    vals = [1.0, 2.0 ** -53, 2.0 ** -53, 2.0 ** -53, 2.0 ** -53, 3.0, 2.0 ** -52, 5.0]
    parts = [_part(x, x, x) for x in vals]
    hy = B.make_hyper(eta=0.1, b_k=32)
    out = B.normtest_combine(parts, 4, hy)
    assert out.A == math.fsum(vals) and out.A + out.A_lo == math.fsum(vals)
    # low parts carried by the shards are used
    parts = [B.nt_result(A=1.0, A_lo=2.0 ** -54, B=1.0, C=1.0) for _ in range(4)]
    out = B.normtest_combine(parts, 4, hy)
    assert out.A == 4.0 + 2.0 ** -52
    # order of the shards does not matter at double-double precision
    rng = np.random.default_rng(1)
    xs = (10 ** rng.uniform(-3, 3, size=64)).tolist()
    p1 = [_part(x, x, x) for x in xs]
    p2 = [_part(x, x, x) for x in sorted(xs)]
    o1, o2 = B.normtest_combine(p1, 4, hy), B.normtest_combine(p2, 4, hy)
    assert o1.A == o2.A == math.fsum(xs)


def test_combine_adds_coordinate_counts():
    hy = B.make_hyper(eta=0.1, b_k=32)
    parts = [B.nt_result(A=1.0, B=1.0, C=1.0, coord_fail=k, coord_max_ratio=r) for k, r in ((3, 2.5), (0, 0.75), (11, 40.0))]
    out = B.normtest_combine(parts, 4, hy)
    assert out.coord_fail == 14 and out.coord_max_ratio == 40.0          # counts add, the largest ratio is the largest
    parts[0].coord_max_ratio = math.inf
    assert B.normtest_combine(parts, 4, hy).coord_max_ratio == math.inf
    parts[1].coord_fail = -1
    parts[1].coord_max_ratio = -1.0
    out = B.normtest_combine(parts, 4, hy)
    assert out.coord_fail == -1 and out.coord_max_ratio == -1.0           # missing in one shard: missing in the total


def test_combine_rejects_bad_input():
    hy = B.make_hyper(eta=0.1, b_k=32)
    with pytest.raises(B.NormtestError):
        B.normtest_combine([_part(1, 1, 1)], 1, hy)
    with pytest.raises(B.NormtestError):
        B.normtest_combine([_part(1, 1, 1, B.NT_STATUS_NO_STATS)], 4, hy)
    with pytest.raises(B.NormtestError):
        B.normtest_combine([_part(1, 1, 1)], 4, B.make_hyper(eta=0.0, b_k=32))
    assert B.lib().normtest_combine(None, 1, 4, ctypes.byref(hy), ctypes.byref(B.nt_result())) == B.NT_ERR_BAD_ARG


def _decide_both(A, Bv, C, J, eta, b_k, b_max, round_to, ddof):
    """(T, pass, next_b, status) from the oracle and from the library's host-side decision."""
    o = oracle.decide(A, Bv, C, J, eta, b_k, b_max, round_to, ddof)
    hy = B.make_hyper(eta=eta, b_k=b_k, b_max=b_max, round_to=round_to, ddof=ddof)
    g = B.normtest_combine([_part(A, Bv, C)], J, hy)
    return (o.T, o.passed, o.next_b, o.status), (g.T, bool(g.pass_), g.next_b, g.status)


def test_decision_invariants_hold_for_arbitrary_sums():
    """Alg. 1's If-branch as properties, for the oracle and for the library, over arbitrary positive sums:
    never shrink; grow exactly when T > b_k; the new size is the least multiple of round_to at or above ceil(T)
    (then cut to the cap, then raised back to b_k); scaling all gradients by a power of two changes nothing."""
    from hypothesis import given, settings, strategies as st

    pos = st.floats(min_value=1e-30, max_value=1e30, allow_nan=False, allow_infinity=False)

    @settings(max_examples=600, deadline=None)
    @given(Bv=pos, C=pos, J=st.integers(2, 5000), eta=st.floats(min_value=1e-3, max_value=10.0),
           b_k=st.integers(1, 1 << 20), b_max=st.sampled_from([0, 1, 512, 8192, 1 << 30]),
           round_to=st.sampled_from([1, 2, 3, 64, 128, 1000]), ddof=st.integers(0, 1), shift=st.integers(-20, 20))
    def check(Bv, C, J, eta, b_k, b_max, round_to, ddof, shift):
        A = C + Bv / J
        for T, passed, next_b, status in _decide_both(A, Bv, C, J, eta, b_k, b_max, round_to, ddof):
            assert next_b >= b_k
            assert passed == (not T > b_k)
            if passed:
                assert next_b == b_k and not status & B.NT_STATUS_CLAMPED
            elif status & B.NT_STATUS_T_SATURATED:
                assert next_b == max(b_k, b_max)
            else:
                want = -(-math.ceil(T) // round_to) * round_to
                if b_max > 0 and want > b_max:
                    assert status & B.NT_STATUS_CLAMPED and next_b == max(b_max, b_k)
                else:
                    assert not status & B.NT_STATUS_CLAMPED and next_b == max(want, b_k)
        c = 2.0 ** (2 * shift)                     # gradients scaled by 2^shift: every sum by 4^shift, exactly
        a, b_ = _decide_both(A, Bv, C, J, eta, b_k, b_max, round_to, ddof), _decide_both(A * c, Bv * c, C * c, J, eta, b_k, b_max, round_to, ddof)
        assert a == b_

    check()
