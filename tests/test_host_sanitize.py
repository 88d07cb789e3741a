"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer, no GPU: the library's sources
are compiled with the sanitizers on the host side, linked with tests/host_sanitize/driver.cpp into
a program that calls the planning entry points and the decode step's plan builder (layout, launch
shapes, phase table) for every workload shape; the run must end clean, and everything it prints
is repeated against the regular library and compared."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest

from paper_2311_15566_amd import binding as B
from paper_2311_15566_amd import plan as P
from paper_2311_15566_amd.build import CSRC, HIPCC, SOURCES
from synth import CONFIGS, scaled_workload, workload

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined"]
FLAGS = ["--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-I" + os.path.join(ROOT, "include"),
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _workloads():
    out = [workload(n) for n in CONFIGS]
    for name in ("gpt20b_m4", "llama30b_m2", "opt66b_m8"):
        for dims in (dict(d_model=1024, n_heads=8, head_dim=128, ffn=4096, vocab=5000),
                     dict(d_model=448, n_heads=2, head_dim=128, ffn=1152, vocab=1511),
                     dict(d_model=8192, n_heads=64, head_dim=128, ffn=28672, vocab=128256)):
            for batch, dtype in ((1, "bf16"), (5, "f32"), (17, "bf16"), (32, "f32")):
                out.append(scaled_workload(name, layers=2, M=2, m=1, batch=batch, s_in=300, steps=20, dtype=dtype, **dims))
    return out


def _plan_line(w):
    d, s = B._desc(w.desc), B._slice(w.slice)
    f = [d.n_layers, d.d_model, d.n_heads, d.head_dim, d.ffn, d.vocab, d.max_pos, d.norm, d.act, d.pos, d.has_bias, d.dtype, d.kv_dtype]
    g = [s.layer_lo, s.layer_hi, s.head_lo, s.head_hi, s.ffn_lo, s.ffn_hi, w.batch, w.s_max, w.batch]
    return "plan " + " ".join(str(v) for v in f) + f" {d.norm_eps!r} {d.rope_theta!r} " + " ".join(str(v) for v in g)


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("host_sanitize")

    def compile_one(path):
        obj = str(out / (os.path.splitext(os.path.basename(path))[0] + ".o"))
        r = subprocess.run([HIPCC, *FLAGS, *SAN, "-c", path, "-o", obj], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        return obj

    paths = [os.path.join(CSRC, s) for s in SOURCES] + [os.path.join(ROOT, "tests", "host_sanitize", "driver.cpp")]
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, paths))
    exe = str(out / "driver")
    r = subprocess.run([HIPCC, "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize", "-o", exe, *objs], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    return exe


def _ints(line, tag):
    assert line.startswith(tag), (tag, line)
    return [int(v) for v in line.split()[1:]]


def test_host_code_is_clean_under_the_sanitizers_and_agrees_with_the_library(driver):
    ws = _workloads()
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver], input="\n".join(_plan_line(w) for w in ws) + "\n", capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    lines = r.stdout.splitlines()
    assert lines[-1] == "done"
    i, seen, planned = 0, dict(match=0, order=0, plan=0, keep=0, cost=0), []
    while i < len(lines):
        head = lines[i].split()
        if head[0] == "match":
            n = int(head[1])
            w = np.array(_ints(lines[i + 1], "in"), dtype=np.uint64).reshape(n, n)
            st, total = int(lines[i + 2].split()[1]), int(lines[i + 2].split()[3])
            assert st == 0
            assert P.match_devices(w) == (total, _ints(lines[i + 3], "out"))
            i += 4
        elif head[0] == "order":
            L, I, u_max = int(head[1]), int(head[2]), int(head[3])
            delta = np.array(_ints(lines[i + 1], "in"), dtype=np.int64).reshape(L, I)
            assert lines[i + 2] == "status 0"
            order = _ints(lines[i + 3], "out")
            assert P.migration_order(delta, u_max) == order
            assert sorted(order) == list(range(L))
            # the progressive plan built from that order
            assert lines[i + 4].split()[0] == "plan"
            stage = _ints(lines[i + 5], "in")
            assert lines[i + 6] == "status 0"
            kind, arg = _ints(lines[i + 7], "kind"), _ints(lines[i + 8], "arg")
            names = ("migrate_cache", "migrate_layer", "start_stage")
            assert P.progressive_plan(order, stage) == [(names[k], a) for k, a in zip(kind, arg)]
            seen["plan"] += 1
            i += 9
        elif head[0] == "keep":
            rows, keep, n_dst = int(head[1]), int(head[2]), int(head[3])
            lens = _ints(lines[i + 1], "in")
            st = int(lines[i + 2].split()[1])
            live = sum(1 for v in lens if v > 0)
            if st == 0:
                assert P.rows_to_keep(lens, keep, n_dst) == _ints(lines[i + 3], "out")
            else:  # asked to keep more rows than hold a request: refused by both
                assert keep > live or keep > n_dst
                with pytest.raises(B.SpotShardError):
                    P.rows_to_keep(lens, keep, n_dst)
            i += 4
        elif head[0] == "cost":
            nd, npre = int(head[1]), int(head[2])
            dec = [(int(a), int(b), float(c)) for _, a, b, c in (l.split() for l in lines[i + 1:i + 1 + nd])]
            pre = [(int(a), int(b), float(c)) for _, a, b, c in (l.split() for l in lines[i + 1 + nd:i + 1 + nd + npre])]
            i += 1 + nd + npre
            st, nb = int(lines[i].split()[1]), int(lines[i].split()[3])
            assert st == 0
            m = P.cost_fit(dec, pre)
            assert m.n_batches == nb
            for k in range(nb):
                f = lines[i + 1 + k].split()
                assert int(f[1]) == m.batch[k]
                got = (m.dec_base_ms[k], m.dec_per_row_ms[k], m.pre_base_ms[k], m.pre_per_token_ms[k])
                # -O1 and -O3 may contract a*b+c differently: compare to rounding, not to the bit
                np.testing.assert_allclose([float(v) for v in f[2:6]], got, rtol=1e-9, atol=1e-12)
            i += 1 + nb
            f = lines[i].split()
            assert f[0] == "lexe" and int(f[5]) == 0
            batch, s_in, s_out = int(f[1]), int(f[2]), int(f[3])
            l_exe = P.cost_l_exe(m, batch, s_in, s_out)
            np.testing.assert_allclose(float(f[7]), l_exe[s_out], rtol=1e-9)
            assert P.jit_iterations(bool(int(f[9])), l_exe, float(f[10]), float(f[11])) == int(f[12])
            i += 1
        elif head[0] == "refuse":
            assert all(int(v) != 0 for v in head[1:])
            i += 1
        elif head[0] == "planned":
            planned.append(lines[i])
            i += 1
        else:
            assert head[0] == "done", lines[i]
            i += 1
            continue
        if head[0] in seen:
            seen[head[0]] += 1
    assert all(v > 0 for v in seen.values()), seen
    # the plan builder: same phase count, same layout size, same context sizes as the regular library
    import ctypes as C
    assert len(planned) == len(ws)
    for line, w in zip(planned, ws):
        f = line.split()
        d, s = B._desc(w.desc), B._slice(w.slice)
        total, szp = C.c_uint64(), C.c_uint64()
        B.lib.ss_debug_plan.restype = C.c_int32
        B.lib.ss_debug_plan.argtypes = [C.POINTER(B.ModelDesc), C.POINTER(B.Slice), C.c_int32, C.c_int32, C.c_int32, C.c_uint64, C.c_void_p,
                                        C.c_int32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        n = B.lib.ss_debug_plan(C.byref(d), C.byref(s), w.batch, w.s_max, w.batch, 1 << 40, None, 0, C.byref(total), C.byref(szp))
        assert n > 0 and int(f[1]) == n and int(f[3]) == total.value
        assert int(f[5]) == B.device_bytes(w.desc, w.slice, w.batch, w.s_max)
        assert int(f[7]) == 0 and (int(f[8]), int(f[9])) == P.context_overlap(w.desc, False, w.slice, w.slice, w.batch * 17)
