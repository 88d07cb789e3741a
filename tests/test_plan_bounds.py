"""Host logic, no GPU: the phase table of a decode step for every workload shape addresses only
memory inside the shard's allocation, the buffers one phase reads and writes do not overlap
(except where a kernel updates in place), and the launch shapes fit what the kernels assume."""
import ctypes as C

import pytest

from paper_2311_15566_amd import binding as B
from synth import CONFIGS, scaled_workload, workload

vp, i32, f32, sz = C.c_void_p, C.c_int32, C.c_float, C.c_size_t


class EmbedArgs(C.Structure):
    _fields_ = [("hidden", vp), ("tokens", vp), ("wte", vp), ("wpe", vp), ("lens", vp), ("S", i32), ("max_pos", i32), ("x", vp), ("d", i32), ("V", i32),
                ("gamma", vp), ("act_out", vp), ("act_lo_out", vp), ("rms", i32), ("stat_out", vp), ("cen_out", vp), ("pstat_out", vp), ("mr_out", vp)]


class GemmArgs(C.Structure):
    _fields_ = [("w", vp), ("row_tiles", i32), ("k_blocks", i32), ("ks", i32), ("nw", i32), ("n_blocks", i32), ("u_base", i32), ("u_rem", i32), ("k_slice", i32), ("B", i32), ("N", i32), ("act", vp), ("zero_frag", vp),
                ("stat_in", vp), ("cen", vp), ("publish", i32), ("stat_groups", i32), ("norm_dim", i32), ("rms", i32), ("eps", f32), ("wg", vp), ("cb", vp),
                ("out_f32", vp), ("ld_out", i32), ("k_split", i32), ("part_stride", sz), ("split_ok", i32), ("split_cost_us", f32), ("x_in", vp), ("x_out", vp), ("act_out", vp), ("out_k_blocks", i32),
                ("g_out", vp), ("stat_out", vp), ("act_kind", i32), ("am_val", vp), ("am_idx", vp),
                ("next_tokens", vp), ("lens", vp * 8), ("len_cap", i32 * 8), ("n_lens", i32), ("commit_inc", i32)]


class AttnArgs(C.Structure):
    _fields_ = [("qkv", vp), ("qkv_parts", i32), ("qkv_stride", sz), ("k_cache", vp), ("v_cache", vp), ("row_stride", sz), ("head_stride", sz), ("lens", vp),
                ("rope", vp), ("part", vp), ("counters", vp), ("o_out", vp), ("B", i32), ("Hs", i32), ("Dh", i32),
                ("Smax", i32), ("kv_dtype", i32), ("rows_per_block", i32), ("splits", i32), ("waves", i32),
                ("stat_in", vp), ("stat_groups", i32), ("norm_dim", i32), ("rms", i32), ("eps", f32), ("wg", vp), ("cb", vp), ("cen", vp),
                ("publish", i32)]


class Phase(C.Structure):
    _fields_ = [("kind", i32), ("gx", i32), ("gy", i32), ("shard", i32), ("epi", i32), ("e", EmbedArgs), ("g", GemmArgs), ("at", AttnArgs)]


lib = B.lib
lib.ss_debug_plan.restype = i32
lib.ss_debug_plan.argtypes = [C.POINTER(B.ModelDesc), C.POINTER(B.Slice), i32, i32, i32, C.c_uint64, vp, i32,
                              C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
EMBED, QKV, ATTN, RESID, FFN_UP, LM_HEAD, COMMIT, FFN_ACT = range(8)
EPI_F32, EPI_RESID, EPI_ACT, EPI_SWIGLU, EPI_LOGITS = range(5)


def plan(w):
    d, s = B._desc(w.desc), B._slice(w.slice)
    buf = (Phase * 256)()
    total, szp = C.c_uint64(), C.c_uint64()
    base = 1 << 40
    n = lib.ss_debug_plan(C.byref(d), C.byref(s), w.batch, w.s_max, w.batch, base, buf, 256, C.byref(total), C.byref(szp))
    assert szp.value == C.sizeof(Phase), (szp.value, C.sizeof(Phase))
    assert 0 < n <= 256
    return [buf[i] for i in range(n)], base, total.value


def check(w):
    ph, base, total = plan(w)
    bf16 = w.desc["dtype"] == "bf16"
    esz, parts, fk = (2, 1, 32) if bf16 else (4, 1, 16)      # operands: one fragment of halves / floats per k block
    kvsz = 4 if not bf16 else 2
    glu = w.desc["act"] == "swiglu"
    d = w.desc["d_model"]
    bad = []

    def rng(label, ptr, nbytes, regions, inplace=False):
        if not ptr or nbytes == 0:
            return
        if not (base <= ptr and ptr + nbytes <= base + total):
            bad.append(("outside the allocation", label, hex(ptr - base), nbytes))
        regions.append((ptr, ptr + nbytes, label, inplace))

    layers = w.slice["layer_hi"] - w.slice["layer_lo"]
    # (a first FFN matrix whose K is cut into slices is followed by the kernel that adds the slices and applies the activation)
    assert [p.kind for p in ph if p.kind != FFN_ACT] == [EMBED] + [QKV, ATTN, RESID, FFN_UP, RESID] * layers + [LM_HEAD, COMMIT]
    for i, p in enumerate(ph[:-1]):
        assert (p.kind == FFN_UP and p.epi == EPI_F32) == (ph[i + 1].kind == FFN_ACT)
    stat_groups = None
    for i, p in enumerate(ph):
        regions = []
        nbt = (w.batch + 15) // 16
        if p.kind == EMBED:
            e = p.e
            assert p.gx == w.batch and e.d == d
            rng("x", e.x, p.gx * e.d * 4, regions)
            rng("act_out", e.act_out, nbt * (d // fk) * parts * 1024, regions)
            rng("stat_out", e.stat_out, 32 * 16, regions)
            rng("gamma", e.gamma, d * 4, regions)
            assert bool(e.cen_out) == (w.desc["norm"] == "layernorm") and not e.pstat_out and not e.mr_out
            rng("cen_out", e.cen_out, 32 * 4, regions)
            stat_groups = 1
        elif p.kind == ATTN:
            a = p.at
            rng("qkv", a.qkv, a.B * 3 * a.Hs * a.Dh * 4, regions)
            for part in range(1, max(1, a.qkv_parts)):
                assert a.qkv_stride >= a.B * 3 * a.Hs * a.Dh and a.qkv_parts <= 8
                rng("qkv part %d" % part, a.qkv + part * a.qkv_stride * 4, a.B * 3 * a.Hs * a.Dh * 4, regions)
            rng("part", a.part, a.B * a.Hs * a.splits * (a.Dh + 4) * 4, regions)
            rng("counters", a.counters, a.B * a.Hs * 4, regions)
            rng("o_out", a.o_out, nbt * (a.Hs * a.Dh // fk) * parts * 1024, regions)
            span = (a.B - 1) * a.row_stride + (a.Hs - 1) * a.head_stride + a.Smax * a.Dh * kvsz
            rng("kcache", a.k_cache, span, regions)
            rng("vcache", a.v_cache, span, regions)
            assert a.splits * a.rows_per_block >= a.Smax and p.gx == a.B * a.Hs and p.gy == a.splits
            assert a.waves in (4, 8, 16) and (a.waves != 8 or (a.splits == 1 and 256 < a.B * a.Hs <= 512))
            # more than 16 rows: the q|k|v GEMM leaves raw products and this kernel applies the normalisation it left out
            q = ph[i - 1].g
            assert ph[i - 1].kind == QKV
            if w.batch > 16:
                assert q.stat_groups == 0 and not q.wg and not q.cb and not q.cen and not q.publish
                assert a.norm_dim == d and a.stat_groups == qkv_stat_groups and a.publish == 1
                rng("stat_in", a.stat_in, a.stat_groups * 32 * 16, regions)
                assert bool(a.wg) == (w.desc["norm"] == "layernorm") == bool(a.cen)
                if a.wg: rng("wg", a.wg, 3 * a.Hs * a.Dh * 4, regions)
                if a.cb: rng("cb", a.cb, 3 * a.Hs * a.Dh * 4, regions)
                rng("cen", a.cen, 32 * 4, regions)
            else:
                assert a.norm_dim == 0 and not a.stat_in
        elif p.kind == FFN_ACT:
            g, up = p.g, ph[i - 1].g
            assert ph[i - 1].kind == FFN_UP and ph[i - 1].epi == EPI_F32 and w.batch > 16 and not glu
            assert (g.out_f32, g.ld_out, g.k_split, g.part_stride, g.B, g.N) == (up.out_f32, up.ld_out, up.k_split, up.part_stride, up.B, up.N)
            assert 2 <= g.k_split <= 8 and g.part_stride >= g.B * g.ld_out and g.part_stride % 4 == 0 and g.ld_out % 4 == 0 and g.N % 16 == 0
            assert p.gx == -(-g.N // 1024) and p.gy == g.B        # a block: 1024 features of one batch row
            # the normalisation the sliced GEMM left out
            assert g.stat_groups == stat_groups and g.norm_dim == d and g.publish == 1
            rng("stat_in", g.stat_in, g.stat_groups * 32 * 16, regions)
            assert bool(g.wg) == (w.desc["norm"] == "layernorm") == bool(g.cen) and g.cb
            if g.wg: rng("wg", g.wg, g.N * 4, regions)
            rng("cb", g.cb, g.N * 4, regions)
            rng("cen", g.cen, 32 * 4, regions)
            for part in range(g.k_split):
                rng("partial (K slice %d)" % part, g.out_f32 + part * g.part_stride * 4, g.B * g.ld_out * 4, regions)
            rng("act_out", g.act_out, nbt * g.out_k_blocks * parts * 1024, regions)
            assert g.out_k_blocks * fk >= g.N and ph[i + 1].kind == RESID and ph[i + 1].g.act == g.act_out
        elif p.kind == COMMIT:
            g = p.g
            assert p.gx == w.batch == g.B and g.n_lens == 1 and g.commit_inc == 1
            lm = ph[i - 1].g                                  # picks among the candidates the LM head left
            assert ph[i - 1].kind == LM_HEAD and (g.am_val, g.am_idx, g.n_blocks) == (lm.am_val, lm.am_idx, lm.n_blocks)
            rng("am_val", g.am_val, 32 * g.n_blocks * 4, regions)
            rng("am_idx", g.am_idx, 32 * g.n_blocks * 4, regions)
        else:
            g = p.g
            tu = 2 if (glu and p.kind == FFN_UP) else 1                      # weight tiles per unit (a gate/up pair)
            units = g.row_tiles // tu
            assert g.ks in (4, 8) and g.B == w.batch and p.gy == 1
            sliced_ffn = p.kind == FFN_UP and p.epi == EPI_F32
            if p.kind == FFN_UP:
                assert p.epi == (EPI_SWIGLU if glu else EPI_ACT) or (sliced_ffn and not glu and g.B > 16)
            # six tiles a block: float output (q|k|v, the sliced first FFN matrix), gate/up pairs for up to 16 rows, logits for more
            assert g.nw in ((2, 6) if tu == 2 else (1, 2, 3, 6))
            assert g.nw != 6 or p.kind == QKV or sliced_ffn or (tu == 2 and g.B <= 16) or (p.kind == LM_HEAD and g.B > 16)
            assert 1 <= g.n_blocks <= units and -(-units // g.n_blocks) * tu <= g.nw   # the largest block fits the kernel instance
            assert p.gx == g.n_blocks * max(1, g.k_split)
            assert (g.u_base, g.u_rem) == divmod(units, g.n_blocks) and g.k_slice == -(-g.k_blocks // max(1, g.k_split))
            assert 1 <= g.N <= g.row_tiles * 16
            rng("w", g.w, g.row_tiles * g.k_blocks * 1024, regions)
            rng("act", g.act, nbt * g.k_blocks * parts * 1024, regions)
            rng("zero_frag", g.zero_frag, 1024, regions)
            if g.wg: rng("wg", g.wg, g.row_tiles * 16 * 4, regions)
            if g.cb: rng("cb", g.cb, g.row_tiles * 16 * 4, regions)
            if p.kind == QKV:
                qkv_stat_groups = stat_groups
            if p.kind == QKV and w.batch > 16:      # raw products: the attention kernel applies normalisation and bias
                assert g.stat_groups == 0 and not g.wg and not g.cb and not g.cen and not g.publish and g.k_blocks * fk == d
            elif sliced_ffn:      # raw partial products: normalisation and bias are applied by the kernel that adds them up
                assert g.stat_groups == 0 and not g.wg and not g.cb and not g.cen and not g.publish and g.k_blocks * fk == d
            elif p.kind in (QKV, FFN_UP, LM_HEAD):
                assert g.stat_groups == stat_groups and g.norm_dim == d and g.k_blocks * fk == d
                rng("stat_in", g.stat_in, g.stat_groups * 32 * 16, regions)
                assert bool(g.wg) == (w.desc["norm"] == "layernorm")
                # the consumer of shard 0 leaves the new mean for the next producer (not the LM head: nothing follows)
                assert g.publish == (0 if p.kind == LM_HEAD else 1) or not g.cen
                assert bool(g.cen) == (w.desc["norm"] == "layernorm" and p.kind != LM_HEAD)
                rng("cen", g.cen, 32 * 4, regions)
            else:
                assert g.stat_groups == 0 and not g.wg
            assert g.k_split in (0, 1) or (2 <= g.k_split <= 8 and (p.kind == QKV or sliced_ffn) and g.k_blocks >= g.k_split * g.ks)
            assert not sliced_ffn or g.k_split >= 2
            if p.kind == QKV:
                rng("out_f32", g.out_f32, g.B * g.ld_out * 4, regions)
                nxt = ph[i + 1]
                assert nxt.kind == ATTN and nxt.at.qkv == g.out_f32
                if g.k_split > 1:                          # the partial sums, added up by the attention kernel
                    assert g.part_stride >= g.B * g.ld_out
                    for part in range(1, g.k_split):
                        rng("out_f32 (K slice %d)" % part, g.out_f32 + part * g.part_stride * 4, g.B * g.ld_out * 4, regions)
                    assert nxt.at.qkv_parts == g.k_split and nxt.at.qkv_stride == g.part_stride
                else:
                    assert nxt.at.qkv_parts in (0, 1)
                assert g.ld_out >= g.N
            if p.kind == FFN_UP:
                assert g.N * (2 if glu else 1) == g.row_tiles * 16
                if sliced_ffn:
                    assert not g.act_out and g.ld_out >= g.N and g.part_stride >= g.B * g.ld_out
                    for part in range(g.k_split):
                        rng("out_f32 (K slice %d)" % part, g.out_f32 + part * g.part_stride * 4, g.B * g.ld_out * 4, regions)
                else:
                    rng("act_out", g.act_out, nbt * g.out_k_blocks * parts * 1024, regions)
                    assert g.out_k_blocks * fk >= g.N
            if p.kind == RESID:
                assert g.N == d == g.row_tiles * 16 and g.x_in == g.x_out
                rng("x", g.x_in, g.B * g.N * 4, regions)
                assert g.act_out and g.g_out and g.stat_out          # one shard in the group: always the last
                rng("act_out", g.act_out, nbt * g.out_k_blocks * parts * 1024, regions)
                rng("g_out", g.g_out, g.N * 4, regions)
                rng("stat_out", g.stat_out, (g.row_tiles // 2) * 32 * 16, regions)
                assert bool(g.cen) == (w.desc["norm"] == "layernorm") and not g.publish
                rng("cen", g.cen, 32 * 4, regions)
                assert g.out_k_blocks * fk >= g.N
                stat_groups = g.row_tiles // 2
            if p.kind == LM_HEAD:
                assert g.N == w.desc["vocab"]
                rng("am_val", g.am_val, 32 * g.n_blocks * 4, regions)     # [32 rows][blocks]
                rng("am_idx", g.am_idx, 32 * g.n_blocks * 4, regions)
        regions.sort()
        for (a0, a1, la, _), (b0, b1, lb, _) in zip(regions, regions[1:]):
            if b0 < a1 and not ({la, lb} <= {"kcache", "vcache"}):
                bad.append(("overlap in phase %d" % i, la, lb, hex(a0 - base), hex(b0 - base)))
    return bad


@pytest.mark.parametrize("name", sorted(CONFIGS))
def test_named_workloads(name):
    assert check(workload(name)) == []


@pytest.mark.parametrize("batch", [1, 8, 16, 17, 32])
def test_scaled_shapes(batch):
    for name in ("gpt20b_m4", "llama30b_m2", "opt66b_m8"):
        for dims in (dict(d_model=1024, n_heads=8, head_dim=128, ffn=4096, vocab=5000),
                     dict(d_model=448, n_heads=2, head_dim=128, ffn=1152, vocab=1511),
                     dict(d_model=8192, n_heads=64, head_dim=128, ffn=28672, vocab=128256)):
            for dtype in ("bf16", "f32"):
                w = scaled_workload(name, layers=2, M=2, m=1, batch=batch, s_in=300, steps=20, dtype=dtype, **dims)
                assert check(w) == []


def test_forced_k_slices_reach_the_first_ffn_matrix_above_16_rows():
    """With K slices forced, a model without gate at more than 16 batch rows plans the sliced first FFN matrix and its
    activation kernel in every layer (and passes the bound checks); at 16 rows or with a gate it does not."""
    dims = dict(d_model=1024, n_heads=8, head_dim=128, ffn=4096, vocab=5000)
    try:
        B.force_gemm_shape(0, 2)
        for name, batch, want in (("opt66b_m8", 17, True), ("gpt20b_m4", 32, True), ("gpt20b_m4", 16, False), ("llama30b_m2", 32, False)):
            for dtype in ("bf16", "f32"):
                w = scaled_workload(name, layers=2, M=2, m=1, batch=batch, s_in=300, steps=20, dtype=dtype, **dims)
                assert check(w) == []
                kinds = [p.kind for p in plan(w)[0]]
                assert kinds.count(FFN_ACT) == (2 if want else 0), (name, batch, dtype)
    finally:
        B.force_gemm_shape(0, 0)


def test_launch_shapes_chosen_for_the_three_shards():
    """The cost rule's choices on the full-size shards are the ones that were measured fastest on the GPU: a change to
    the rule that moves one of them has to be measured again (a term added for more than 16 rows once flipped the
    GPT-20B shape's q|k|v GEMM to a shape 2 us slower)."""
    want = {
        "gpt20b_m4": {QKV: (3, 96, 2), RESID: (2, 192, 1), FFN_UP: (2, 192, 1), LM_HEAD: (2, 1563, 1)},
        "llama30b_m2": {QKV: (3, 208, 1), RESID: (2, 208, 1), FFN_UP: (6, 187, 1), LM_HEAD: (2, 1000, 1)},
        "opt66b_m8": {QKV: (3, 72, 3), RESID: (3, 192, 1), FFN_UP: (6, 48, 5), LM_HEAD: (6, 768, 1)},
    }
    for name, shapes in want.items():
        ph, _, _ = plan(workload(name))
        for p in ph[1:]:                      # (the first q|k|v GEMM follows the embedding: one group of row sums)
            if p.kind in shapes:
                g = p.g
                assert (g.nw, g.n_blocks, max(1, g.k_split)) == shapes[p.kind], (name, p.kind, g.nw, g.n_blocks, g.k_split)
        kinds = [p.kind for p in ph]
        assert (FFN_ACT in kinds) == (name == "opt66b_m8")
