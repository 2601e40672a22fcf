"""The C-ABI library without a GPU: it loads, exports every declared symbol, and rejects bad
arguments on the host before anything is enqueued."""
import ctypes
import os
import re

import paper_2411_18462_amd as svip
from paper_2411_18462_amd.binding import BENCH_EXPORTS, EXPORTS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    lib = svip.load()
    for name, exports in (("svip.h", EXPORTS), ("svip_bench.h", BENCH_EXPORTS)):
        header = open(os.path.join(ROOT, "include", name)).read()
        header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
        declared = set(re.findall(r"\b(svip_[a-z_]+)\s*\(", header))
        assert declared == set(exports), declared ^ set(exports)
        for sym in declared:
            assert hasattr(lib, sym), sym


def test_bench_hooks_reject_bad_arguments_and_never_change_workspace_sizes():
    lib = svip.load()
    assert lib.svip_bench_time_kernels(7, None, None, 0) == 6 and lib.svip_bench_time_kernels(0, None, None, 3) == 1
    assert lib.svip_bench_time_kernels(0, None, None, 0) == 0 and lib.svip_bench_events_used(0) == 0
    assert lib.svip_bench_events_used(9) == -1
    before = [svip.workspace_needed(c, __import__("torch").bfloat16, 64, 16, 128256) for c in range(6)]
    svip.bench_set_tuning(draft_slices=64, stats_slices=64, resid_slices=64, pair_slices=64)
    try:
        assert before == [svip.workspace_needed(c, __import__("torch").bfloat16, 64, 16, 128256) for c in range(6)]
    finally:
        svip.bench_set_tuning()
    t = svip.binding.BenchTuning(draft_slices=-1)
    assert lib.svip_bench_set_tuning(ctypes.byref(t)) == 6


def test_status_strings():
    lib = svip.load()
    seen = set()
    for code in range(8):
        s = lib.svip_status_string(code).decode()
        assert s.startswith("SVIP_") and s not in seen
        seen.add(s)
    assert b"unknown" in lib.svip_status_string(99)


def test_workspace_bytes_is_a_pure_host_function():
    assert svip.workspace_bytes(0, 16, 128256) == 0
    assert svip.workspace_bytes(64, 0, 128256) == 0
    assert svip.workspace_bytes(64, svip.MAX_K + 1, 128256) == 0
    assert svip.workspace_bytes(64, 16, 0) == 0
    small, big = svip.workspace_bytes(1, 8, 32000), svip.workspace_bytes(64, 16, 128256)
    assert 0 < small <= big < (1 << 30) and small % 256 == 0 and big % 256 == 0
    assert svip.workspace_bytes(256, 64, 151936) >= big


def test_host_checks_reject_before_any_gpu_call():
    """No GPU here: every call below must fail on its argument checks (a launch would give
    SVIP_ERR_HIP instead)."""
    lib = svip.load()
    buf = ctypes.create_string_buffer(1 << 16)
    p = (ctypes.addressof(buf) + 255) & ~255          # fake, aligned "device" pointers, never dereferenced
    ws_bytes = svip.workspace_bytes(2, 4, 64)
    V = 64

    def draft(**kw):
        a = dict(logits=p, dtype=1, B=2, V=V, row_stride=V, T=1.0, h=0.3, j=0, k=4, u=p, stop_in=None, tok=p,
                 ent=None, q=None, lse=p, stop=p, dl=None, ios=1, ws=p, wsb=ws_bytes, st=None)
        a.update(kw)
        return lib.svip_draft_step(a["logits"], a["dtype"], a["B"], a["V"], a["row_stride"], a["T"], a["h"], a["j"],
                                   a["k"], a["u"], a["stop_in"], a["tok"], a["ent"], a["q"], a["lse"], a["stop"],
                                   a["dl"], a["ios"], a["ws"], a["wsb"], a["st"])

    assert draft(logits=None) == 1 and draft(u=None) == 1 and draft(tok=None) == 1 and draft(lse=None) == 1
    assert draft(dtype=7) == 3
    assert draft(B=0) == 2 and draft(V=0) == 2 and draft(k=0) == 2 and draft(j=4) == 2 and draft(j=-1) == 2
    assert draft(ios=0) == 2 and draft(row_stride=V - 8) == 2 and draft(B=(1 << 20) + 1) == 2
    assert draft(logits=p + 2) == 4 and draft(row_stride=V + 4) == 4 and draft(dtype=0, row_stride=V + 2) == 4
    assert draft(T=0.0) == 6 and draft(T=-1.0) == 6 and draft(T=float("inf")) == 6 and draft(h=-0.1) == 6
    assert draft(h=float("nan")) == 6 and draft(T=float("nan")) == 6
    assert draft(ws=None) == 5 and draft(ws=p + 16) == 5 and draft(wsb=512) == 5

    def verify(**kw):
        a = dict(t=p, d=p, dtype=1, B=2, k=4, V=V, st_t=5 * V, st_d=4 * V, rs=V, T=1.0, tok=p, dl=p, lse=None,
                 ua=p, ur=p, na=p, nt=p, ap=None, ws=p, wsb=ws_bytes, st=None)
        a.update(kw)
        return lib.svip_verify(a["t"], a["d"], a["dtype"], a["B"], a["k"], a["V"], a["st_t"], a["st_d"], a["rs"],
                               a["T"], a["tok"], a["dl"], a["lse"], a["ua"], a["ur"], a["na"], a["nt"], a["ap"],
                               a["ws"], a["wsb"], a["st"])

    assert verify(t=None) == 1 and verify(d=None) == 1 and verify(tok=None) == 1 and verify(dl=None) == 1
    assert verify(ua=None) == 1 and verify(ur=None) == 1 and verify(na=None) == 1 and verify(nt=None) == 1
    assert verify(dtype=3) == 3
    assert verify(B=0) == 2 and verify(k=0) == 2 and verify(V=0) == 2 and verify(st_t=4 * V) == 2
    assert verify(st_d=2 * V) == 2 and verify(rs=V - 8) == 2 and verify(B=(1 << 20) + 1) == 2
    assert verify(t=p + 8) == 4 and verify(rs=V + 4, st_t=5 * (V + 4), st_d=4 * (V + 4)) == 4
    assert verify(T=0.0) == 6
    assert verify(ws=None) == 5 and verify(wsb=512) == 5
    assert lib.svip_workspace_reset(None, 1 << 20, None) == 5
    assert lib.svip_workspace_reset(p + 8, 1 << 20, None) == 5
    out = ctypes.c_uint(0)
    assert lib.svip_workspace_flags(None, None, ctypes.byref(out)) == 5
    assert lib.svip_workspace_flags(p, None, None) == 1
    assert lib.svip_workspace_reset(p, 256, None) == 5           # no room for a counter behind the flag word


def test_host_checks_of_the_greedy_diagnostic_and_loop_calls():
    lib = svip.load()
    buf = ctypes.create_string_buffer(1 << 16)
    p = (ctypes.addressof(buf) + 255) & ~255
    V = 64
    wsb = svip.workspace_bytes(2, 4, V)

    def gdraft(**kw):
        a = dict(logits=p, dtype=1, B=2, V=V, rs=V, T=1.0, h=0.3, j=0, k=4, stop_in=None, tok=p, ent=None, q=None,
                 lse=p, stop=p, dl=None, ios=1, ws=p, wsb=wsb, st=None)
        a.update(kw)
        return lib.svip_draft_step_greedy(a["logits"], a["dtype"], a["B"], a["V"], a["rs"], a["T"], a["h"], a["j"],
                                          a["k"], a["stop_in"], a["tok"], a["ent"], a["q"], a["lse"], a["stop"],
                                          a["dl"], a["ios"], a["ws"], a["wsb"], a["st"])

    assert gdraft(logits=None) == 1 and gdraft(tok=None) == 1 and gdraft(dtype=5) == 3 and gdraft(j=4) == 2
    assert gdraft(rs=V + 4) == 4 and gdraft(T=0.0) == 6 and gdraft(wsb=256) == 5

    def gverify(**kw):
        a = dict(t=p, dtype=1, B=2, k=4, V=V, st_t=5 * V, rs=V, tok=p, dl=p, na=p, nt=p, ws=p, wsb=wsb, st=None)
        a.update(kw)
        return lib.svip_verify_greedy(a["t"], a["dtype"], a["B"], a["k"], a["V"], a["st_t"], a["rs"], a["tok"],
                                      a["dl"], a["na"], a["nt"], a["ws"], a["wsb"], a["st"])

    assert gverify(t=None) == 1 and gverify(tok=None) == 1 and gverify(dl=None) == 1 and gverify(nt=None) == 1
    assert gverify(dtype=9) == 3 and gverify(k=0) == 2 and gverify(st_t=4 * V) == 2 and gverify(t=p + 4) == 4
    assert gverify(ws=None) == 5 and gverify(wsb=64) == 5

    def pair(**kw):
        a = dict(t=p, d=p, dtype=1, B=2, k=4, V=V, st_t=4 * V, st_d=4 * V, rs=V, T=1.0, dl=p, lse=None, c=0.2,
                 out=p, ws=p, wsb=wsb, st=None)
        a.update(kw)
        return lib.svip_pair_stats(a["t"], a["d"], a["dtype"], a["B"], a["k"], a["V"], a["st_t"], a["st_d"], a["rs"],
                                   a["T"], a["dl"], a["lse"], a["c"], a["out"], a["ws"], a["wsb"], a["st"])

    assert pair(t=None) == 1 and pair(d=None) == 1 and pair(dl=None) == 1 and pair(out=None) == 1
    assert pair(dtype=-1) == 3 and pair(V=0) == 2 and pair(st_t=3 * V) == 2 and pair(d=p + 2) == 4
    assert pair(T=float("nan")) == 6 and pair(c=-0.5) == 6 and pair(c=float("inf")) == 6 and pair(wsb=1024) == 5

    def warp(**kw):
        a = dict(i=p, o=p, dtype=1, B=2, n=5, V=V, ss=5 * V, rs=V, T=1.0, k=50, p_=0.9, kept=None, st=None)
        a.update(kw)
        return lib.svip_warp_logits(a["i"], a["o"], a["dtype"], a["B"], a["n"], a["V"], a["ss"], a["rs"], a["T"],
                                    a["k"], a["p_"], a["kept"], a["st"])

    assert warp(i=None) == 1 and warp(o=None) == 1 and warp(dtype=7) == 3 and warp(n=0) == 2 and warp(ss=4 * V) == 2
    assert warp(o=p + 6) == 4 and warp(rs=V + 2, ss=6 * V) == 4 and warp(T=-1.0) == 6 and warp(k=-1) == 6
    assert warp(p_=0.0) == 6 and warp(p_=float("nan")) == 6

    lwsb = lib.svip_loop_workspace_bytes(2, 4, V)
    assert lwsb > wsb and lwsb % 256 == 0 and lib.svip_loop_workspace_bytes(0, 4, V) == 0

    def loop(**kw):
        c = svip.LoopConfig()
        a = dict(target_trace=p, draft_trace=p, dtype=1, B=2, L=20, V=V, seq_stride=20 * V, row_stride=V,
                 temperature=1.0, greedy=0, h=0.3, gamma0=4, gamma_max=4, gamma_inc=0, gamma_dec=0, n0=0, max_new=8,
                 rounds=8, u_sample=p, u_accept=p, u_resample=p, state=p, out_tokens=p, out_stride=12,
                 round_log=None, check_every=4, workspace=p, workspace_bytes=lwsb, hip_stream=None)
        a.update(kw)
        for name, val in a.items():
            setattr(c, name, val)
        return lib.svip_loop_init(ctypes.byref(c)), lib.svip_loop_run(ctypes.byref(c), 0, 1, None, None)

    assert lib.svip_loop_init(None) == 1
    assert loop(target_trace=None) == (1, 1) and loop(state=None) == (1, 1) and loop(u_accept=None) == (1, 1)
    assert loop(gamma0=5) == (2, 2) and loop(gamma_max=0) == (2, 2) and loop(n0=20) == (2, 2)
    assert loop(seq_stride=19 * V) == (2, 2) and loop(out_stride=11) == (2, 2) and loop(rounds=0) == (2, 2)
    assert loop(gamma_inc=-1) == (6, 6) and loop(check_every=-1) == (6, 6)
    assert loop(workspace=None) == (5, 5) and loop(workspace_bytes=wsb) == (5, 5)


def test_workspace_bytes_covers_every_call_for_every_shape():
    """svip_workspace_bytes(B, k_max, V) must be enough for whatever slicing each call chooses."""
    import itertools
    import torch
    lib = svip.load()
    Bs = [1, 2, 3, 7, 16, 64, 100, 256, 1000, 4096, 1 << 20]
    ks = [1, 2, 5, 16, 40, 64, 100, 1024]
    Vs = [1, 2, 9, 255, 2048, 2049, 16384, 32000, 50257, 128256, 151936, 262147, 1 << 20]
    worst = 0.0
    for B, k, V in itertools.product(Bs, ks, Vs):
        if B * k > (1 << 22):
            continue
        total = svip.workspace_bytes(B, k, V)
        assert total > 0 and total % 256 == 0
        for dtype in (torch.float32, torch.bfloat16, torch.float16):
            for call in range(6):
                need = svip.workspace_needed(call, dtype, B, k, V)
                assert 0 < need <= total, (call, dtype, B, k, V, need, total)
                worst = max(worst, need / total)
    assert worst > 0.5                                    # the bound is not wildly loose either
    assert lib.svip_workspace_needed(9, 1, 4, 4, 64) == 0 and lib.svip_workspace_needed(0, 7, 4, 4, 64) == 0
    assert lib.svip_workspace_needed(0, 1, 0, 4, 64) == 0
    assert lib.svip_loop_workspace_bytes(8, 40, 151936) > svip.workspace_bytes(8, 40, 151936)


def test_header_is_plain_c(tmp_path):
    """include/svip.h must compile as C99 on its own (the boundary is a C ABI)."""
    import subprocess
    src = tmp_path / "use_svip.c"
    src.write_text('#include "svip.h"\n'
                   "int main(void) {\n"
                   "    svip_loop_config c;\n"
                   "    (void)c;\n"
                   "    return (int)svip_workspace_bytes(0, 0, 0) + (SVIP_PAIR_NSTAT == 8 ? 0 : 1) + (int)SVIP_CALL_PAIR_STATS - 4;\n"
                   "}\n")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"),
                           "-c", str(src), "-o", str(tmp_path / "use_svip.o")])


def test_binding_structs_match_the_headers(tmp_path):
    """The ctypes mirrors of the headers' structs must have the C compiler's sizes and field offsets: a field
    added on one side only would silently shift every later field."""
    import subprocess
    from paper_2411_18462_amd import binding
    pairs = [("svip_bench_tuning", binding.BenchTuning), ("svip_loop_config", binding.LoopConfig)]
    lines = []
    for cname, cls in pairs:
        lines.append(f'    printf("%zu\\n", sizeof({cname}));\n')
        lines += [f'    printf("%zu\\n", offsetof({cname}, {f}));\n' for f, _ in cls._fields_]
    src = tmp_path / "sizes.c"
    src.write_text('#include <stddef.h>\n#include <stdio.h>\n#include "svip.h"\n#include "svip_bench.h"\n'
                   "int main(void) {\n" + "".join(lines) + "    return 0;\n}\n")
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    out = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    for cname, cls in pairs:
        n = len(cls._fields_)
        assert out[0] == ctypes.sizeof(cls), cname
        assert out[1:n + 1] == [getattr(cls, f).offset for f, _ in cls._fields_], cname
        out = out[n + 1:]
    header = open(os.path.join(ROOT, "include", "svip_bench.h")).read()
    body = header[header.index("typedef struct svip_bench_tuning {"):header.index("} svip_bench_tuning;")]
    assert re.findall(r"int (\w+);", body) == [f for f, _ in binding.BenchTuning._fields_]


def test_division_by_multiplication_is_exact_over_the_kernels_range():
    """k_draft_stats divides a wave number by the records (or workgroups) per row as umulhi(n, floor(2^32 / d) + 1),
    with n < 2^26 (MAX_BATCH rows of at most 64 records) and d <= 64: exact while n * d < 2^32."""
    import numpy as np
    rng = np.random.default_rng(0)
    for d in range(2, 65):
        magic = (1 << 32) // d + 1
        n = np.concatenate([np.arange(0, 4096), rng.integers(0, 1 << 26, 20000), (1 << 26) - 1 - np.arange(0, 4096),
                            np.arange(1, 3000) * d - 1, np.arange(1, 3000) * d]).astype(np.uint64)
        n = n[n < (1 << 26)]
        assert ((n * np.uint64(magic)) >> np.uint64(32) == n // np.uint64(d)).all(), d
