"""Host logic, no GPU: the phase table of a decode step (kernel-by-kernel plan and both
persistent-kernel plans) for every workload shape addresses only memory inside the shard's
allocation, buffers of one phase do not overlap, and the split / chunk arithmetic covers K
exactly within what the kernels' LDS and register buffers hold."""
import ctypes as C

import pytest

from paper_2311_15566_amd import binding as B
from synth import CONFIGS, scaled_workload, workload

vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t
class EmbedArgs(C.Structure):
    _fields_ = [("tokens", vp), ("wte", vp), ("wpe", vp), ("lens", vp), ("S", i32), ("x", vp), ("stats", vp), ("d", i32), ("V", i32), ("rms", i32), ("eps", f32)]
class SkinnyArgs(C.Structure):
    _fields_ = [("w", vp), ("tasks", i32), ("k_blocks", i32), ("split", i32), ("kb_per_split", i32), ("lds_chunk", i32), ("B", i32), ("nb", i32), ("N", i32),
                ("act", vp), ("x", vp), ("stats", vp), ("gamma", vp), ("beta", vp), ("splitk", vp), ("counters", vp), ("bias", vp), ("out_f32", vp), ("ld_out", i32),
                ("x_in", vp), ("x_resid", vp), ("stat_part", vp), ("stats_out", vp), ("rms", i32), ("eps", f32), ("act_out", vp), ("out_k_blocks", i32), ("act_kind", i32),
                ("am_val", vp), ("am_idx", vp), ("next_tokens", vp), ("lens", vp * 8), ("n_lens", i32), ("commit_inc", i32)]
class AttnArgs(C.Structure):
    _fields_ = [("qkv", vp), ("k_cache", vp), ("v_cache", vp), ("row_stride", sz), ("head_stride", sz), ("lens", vp), ("rope", vp), ("part", vp), ("counters", vp), ("o_out", vp),
                ("B", i32), ("Hs", i32), ("Dh", i32), ("Smax", i32), ("kv_dtype", i32), ("rows_per_block", i32), ("splits", i32)]
class Phase(C.Structure):
    _fields_ = [("kind", i32), ("gx", i32), ("gy", i32), ("shard", i32), ("e", EmbedArgs), ("g", SkinnyArgs), ("at", AttnArgs)]
lib = B.lib
lib.ss_debug_plan.restype = i32
lib.ss_debug_plan.argtypes = [C.POINTER(B.ModelDesc), C.POINTER(B.Slice), i32, i32, i32, i32, i32, C.c_uint64, vp, i32, C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
def plan(w, mode, blocks=512):
    d, s = B._desc(w.desc), B._slice(w.slice)
    buf = (Phase * 256)()
    total, szp = C.c_uint64(), C.c_uint64()
    base = 1 << 40
    n = lib.ss_debug_plan(C.byref(d), C.byref(s), w.batch, w.s_max, w.batch, mode, blocks, base, buf, 256, C.byref(total), C.byref(szp))
    assert szp.value == C.sizeof(Phase), (szp.value, C.sizeof(Phase))
    assert 0 < n <= 256
    return w, [buf[i] for i in range(n)], base, total.value
def check(w, mode, blocks=512):
    w, ph, base, total = plan(w, mode, blocks)
    esz = 2 if w.desc["dtype"] == "bf16" else 4
    parts = 2 if esz == 2 else 1
    gsz = 3 if mode == 2 else 4
    glu = w.desc["act"] == "swiglu"
    bad = 0
    def rng(label, ptr, nbytes, regions):
        nonlocal bad
        if ptr is None or nbytes == 0: return
        if not (base <= ptr and ptr + nbytes <= base + total):
            print("  OUT OF ALLOCATION", label, hex(ptr - base), nbytes); bad += 1
        regions.append((ptr, ptr + nbytes, label))
    for i, p in enumerate(ph):
        regions = []
        if p.kind == 0:
            e = p.e
            rng("x", e.x, p.gx * e.d * 4, regions); rng("stats", e.stats, p.gx * 8, regions)
        elif p.kind == 2:
            a = p.at
            rng("qkv", a.qkv, a.B * 3 * a.Hs * a.Dh * 4, regions)
            rng("part", a.part, a.B * a.Hs * a.splits * (a.Dh + 4) * 4, regions)
            rng("counters", a.counters, a.B * a.Hs * 4, regions)
            rng("o_out", a.o_out, ((a.B + 15) // 16) * (a.Hs * a.Dh // 32) * parts * 1024, regions)
            rng("kcache", a.k_cache, (a.B - 1) * a.row_stride + (a.Hs - 1) * a.head_stride + a.Smax * a.Dh * esz, regions)
            rng("vcache", a.v_cache, (a.B - 1) * a.row_stride + (a.Hs - 1) * a.head_stride + a.Smax * a.Dh * esz, regions)
            assert a.splits * a.rows_per_block >= a.Smax and p.gx == a.B * a.Hs and p.gy == a.splits
            if mode == 2: assert a.rows_per_block <= 192
        else:
            g = p.g
            nw = 2 if (glu and p.kind == 4) else 1
            groups = -(-g.tasks // gsz)
            assert p.gx == groups and p.gy == g.split, (p.gx, groups, p.gy, g.split)
            assert g.split * g.kb_per_split >= g.k_blocks and (g.split - 1) * g.kb_per_split < g.k_blocks
            assert g.nb * g.lds_chunk * parts <= 64
            assert g.lds_chunk <= g.kb_per_split
            if mode == 2:
                assert g.lds_chunk * nw <= 32 and g.nb * g.lds_chunk * parts <= (64 if g.nb == 1 else 56)
            else:
                assert g.lds_chunk == g.kb_per_split or g.lds_chunk % 16 == 0
            rng("w", g.w, g.tasks * nw * g.k_blocks * 1024, regions)
            if g.split > 1: rng("splitk", g.splitk, g.split * g.nb * 16 * g.tasks * nw * 16 * 4, regions)
            rng("counters", g.counters, (groups + 1) * 4, regions)
            if p.kind == 3:
                rng("act", g.act, g.nb * g.k_blocks * parts * 1024, regions)
                rng("x_in", g.x_in, g.B * g.N * 4, regions); rng("x_resid", g.x_resid, g.B * g.N * 4, regions)
                rng("stat_part", g.stat_part, groups * 32 * 2 * 4, regions); rng("stats_out", g.stats_out, 64 * 4, regions)
            else:
                rng("x", g.x, g.B * g.k_blocks * 32 * 4, regions); rng("stats", g.stats, 64 * 4, regions)
            if p.kind == 1: rng("out_f32", g.out_f32, g.B * g.ld_out * 4, regions)
            if p.kind == 4: rng("act_out", g.act_out, g.nb * g.out_k_blocks * parts * 1024, regions)
            if p.kind == 5:
                rng("am_val", g.am_val, groups * 32 * 4, regions); rng("am_idx", g.am_idx, groups * 32 * 4, regions)
        regions.sort()
        for (a0, a1, la), (b0, b1, lb) in zip(regions, regions[1:]):
            if b0 < a1 and not ({la, lb} <= {"x_in", "x_resid"}) and not ({la, lb} <= {"kcache", "vcache"}):
                print("  OVERLAP in phase", i, la, lb, hex(a0 - base), hex(a1 - base), hex(b0 - base)); bad += 1
    return bad



@pytest.mark.parametrize("name", sorted(CONFIGS))
@pytest.mark.parametrize("mode", [0, 1, 2])
def test_named_workloads(name, mode):
    assert check(workload(name), mode) == 0


@pytest.mark.parametrize("mode,blocks", [(0, 512), (1, 512), (2, 512), (2, 64), (2, 17)])
@pytest.mark.parametrize("batch", [1, 8, 16, 17, 32])
def test_scaled_shapes(mode, blocks, batch):
    for name in ("gpt20b_m4", "llama30b_m2", "opt66b_m8"):
        for dims in (dict(d_model=1024, n_heads=8, head_dim=128, ffn=4096, vocab=5000),
                     dict(d_model=448, n_heads=2, head_dim=128, ffn=1152, vocab=1511),
                     dict(d_model=8192, n_heads=64, head_dim=128, ffn=28672, vocab=128256)):
            w = scaled_workload(name, layers=2, M=2, m=1, batch=batch, s_in=300, steps=20, dtype="bf16", **dims)
            assert check(w, mode, blocks) == 0
