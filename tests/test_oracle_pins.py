"""Pins for the CPU oracle: it is checked here against things other than itself -
library routines composed independently (torch CPU float64), closed forms, and the
invariants the paper states (cached decoding reaches the full recompute, Eq. (1)-(2);
the shards of a tensor-parallel group sum to the unsharded operator, Section 2.2).
"""
import copy
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import decoder as D
from synth import (bf16_bits_to_f32, make_tokens, make_weights, scaled_workload, sub_slice_of,
                   tp_slice, workload)


def small(name, **kw):
    base = dict(d_model=64, n_heads=4, head_dim=16, ffn=128, vocab=97, layers=2, M=1,
                batch=2, s_in=7, steps=4, dtype="f32")
    base.update(kw)
    return scaled_workload(name, **base)


ARCHS = ["tiny_gpt", "llama30b_m2", "opt66b_m8"]   # LN+GELU+learned / RMS+SwiGLU+RoPE / LN+ReLU+learned


def build(w, real=np.float64, batch=None, s_max=None):
    W = make_weights(w.desc, w.slice, w.seed)
    s = D.OracleShard(w.desc, w.slice, W, batch or w.batch, s_max or w.s_max, real=real)
    return W, s


# ----------------------------------------------------------------------------
# whole model against an independent composition of torch library routines
# ----------------------------------------------------------------------------
def torch_forward(desc, W, toks):
    """Causal decoder forward built only from torch.nn.functional routines (float64).
    RoPE has no library routine: it is done as a complex multiplication."""
    f64 = lambda a: None if a is None else torch.from_numpy(
        (bf16_bits_to_f32(a) if a.dtype == np.uint16 else a).astype(np.float64))
    d, H, Dh = desc["d_model"], desc["n_heads"], desc["head_dim"]
    S = len(toks)
    t = torch.from_numpy(np.asarray(toks, dtype=np.int64))
    x = F.embedding(t, f64(W["wte"]))
    if desc["pos"] == "learned":
        x = x + F.embedding(torch.arange(S), f64(W["wpe"]))

    def norm(x, g, b):
        if desc["norm"] == "layernorm":
            return F.layer_norm(x, (d,), f64(g), f64(b), desc["norm_eps"])
        return F.rms_norm(x, (d,), f64(g), desc["norm_eps"])

    def rope(v):  # v [H, S, Dh]; pair (i, i + Dh/2) as the complex number v_i + 1j * v_{i+Dh/2}
        half = Dh // 2
        z = torch.complex(v[..., :half], v[..., half:])
        ang = torch.arange(S, dtype=torch.float64)[:, None] * desc["rope_theta"] ** (
            -torch.arange(half, dtype=torch.float64) * 2.0 / Dh)
        z = z * torch.polar(torch.ones_like(ang), ang)
        return torch.cat([z.real, z.imag], dim=-1)

    for L in W["layers"]:
        a = norm(x, L["ln1_g"], L["ln1_b"])
        q = F.linear(a, f64(L["wq"]).T, f64(L["bq"])).view(S, H, Dh).transpose(0, 1)
        k = F.linear(a, f64(L["wk"]).T, f64(L["bk"])).view(S, H, Dh).transpose(0, 1)
        v = F.linear(a, f64(L["wv"]).T, f64(L["bv"])).view(S, H, Dh).transpose(0, 1)
        if desc["pos"] == "rope":
            q, k = rope(q), rope(k)
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True)
        x = x + F.linear(o.transpose(0, 1).reshape(S, H * Dh), f64(L["wo"]).T, f64(L["bo"]))
        a2 = norm(x, L["ln2_g"], L["ln2_b"])
        if desc["act"] == "swiglu":
            u = F.silu(F.linear(a2, f64(L["wg"]).T)) * F.linear(a2, f64(L["wu"]).T)
        else:
            h = F.linear(a2, f64(L["w1"]).T, f64(L["b1"]))
            u = F.gelu(h, approximate="tanh") if desc["act"] == "gelu_tanh" else F.relu(h)
        x = x + F.linear(u, f64(L["w2"]).T, f64(L["b2"]))
    xf = norm(x, W["lnf_g"], W["lnf_b"])
    return F.linear(xf, f64(W["lm_head"])).numpy()


def test_tiny_gpt_matches_torch_library_composition():
    w = workload("tiny_gpt")
    W, s = build(w)
    toks = make_tokens(w.seed, 1, w.s_in + w.steps, w.desc["vocab"])[0]
    ref = torch_forward(w.desc, W, toks)
    got = D.forward_matrix([s], toks)
    assert np.abs(got - ref).max() < 1e-10
    # and the incremental path reaches the same thing
    inc = np.stack([D.decode_step([s], [t])[0] for t in toks])
    assert np.abs(inc - ref).max() < 1e-10


@pytest.mark.parametrize("arch", ARCHS)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_architectures_match_torch_library_composition(arch, dtype):
    w = small(arch, dtype=dtype)
    W, s = build(w)
    toks = make_tokens(w.seed, 1, 11, w.desc["vocab"])[0]
    ref = torch_forward(w.desc, W, toks)
    got = D.forward_matrix([s], toks)
    assert np.abs(got - ref).max() < 1e-10
    assert np.abs(ref).max() > 1e-3      # not vacuous


# ----------------------------------------------------------------------------
# Eq. (1) == Eq. (2): cached incremental decoding reaches the full recompute
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("arch", ARCHS)
def test_incremental_equals_full_recompute_every_position(arch):
    w = small(arch, batch=3)
    W, s = build(w)
    toks = make_tokens(w.seed, 3, 11, w.desc["vocab"])
    inc = np.stack([D.decode_step([s], toks[:, t]) for t in range(11)], axis=1)   # [B, S, V]
    for b in range(3):
        full = D.forward_matrix([s], toks[b])
        assert np.abs(inc[b] - full).max() < 1e-11
    assert list(s.n) == [11, 11, 11]


@pytest.mark.parametrize("arch", ARCHS)
def test_pipeline_stages_compose_to_the_whole_model(arch):
    """Section 2.2, inter-operator parallelism: stages of consecutive layers, each fed the hidden
    states of the one before, compute what the whole model computes, and their caches are the
    whole model's cache cut by layers (sequential, incremental and matrix forms)."""
    w = small(arch, layers=5, batch=2)
    W = make_weights(w.desc, w.slice, w.seed)
    toks = make_tokens(w.seed, 2, 6, w.desc["vocab"])
    nxt = make_tokens(w.seed + 1, 2, 3, w.desc["vocab"])
    cuts = [0, 2, 3, 5]
    whole = D.OracleShard(w.desc, w.slice, W, 2, 12)
    stages = [D.OracleShard(w.desc, tp_slice(w.desc, a, b, 0, 1), W, 2, 12) for a, b in zip(cuts, cuts[1:])]
    ref = D.prefill([whole], toks)
    h = D.prefill([stages[0]], toks, hidden_out=True)
    assert h.shape == (2, 6, w.desc["d_model"])
    h = D.prefill([stages[1]], None, hidden_in=h, hidden_out=True)
    got = D.prefill([stages[2]], None, hidden_in=h)
    assert np.abs(got - ref).max() < 1e-12
    for t in range(3):
        ref = D.decode_step([whole], nxt[:, t])
        h = D.decode_step([stages[0]], nxt[:, t], hidden_out=True)
        h = D.decode_step([stages[1]], None, hidden_in=h, hidden_out=True)
        got = D.decode_step([stages[2]], None, hidden_in=h)
        assert np.abs(got - ref).max() < 1e-12
    for st, (a, b) in zip(stages, zip(cuts, cuts[1:])):
        assert list(st.n) == [9, 9]
        assert np.array_equal(st.kv[:, :, :, :, :9], whole.kv[a:b, :, :, :, :9])
    # a stage's hidden output is not the logits' input until the final norm: it differs from the
    # whole model's last hidden state unless it IS the last stage
    fresh = [D.OracleShard(w.desc, tp_slice(w.desc, a, b, 0, 1), W, 2, 12) for a, b in zip(cuts, cuts[1:])]
    hm = D.forward_matrix([fresh[0]], toks[0], b=0, hidden_out=True)
    hm = D.forward_matrix([fresh[1]], None, b=0, hidden_in=hm, hidden_out=True)
    lm = D.forward_matrix([fresh[2]], None, b=0, hidden_in=hm)
    assert np.abs(lm - D.forward_matrix([D.OracleShard(w.desc, w.slice, W, 2, 12)], toks[0])).max() < 1e-11


@pytest.mark.parametrize("arch", ARCHS)
def test_prefill_matrix_form_fills_the_same_cache(arch):
    w = small(arch)
    W, s1 = build(w)
    _, s2 = build(w)
    toks = make_tokens(w.seed, w.batch, w.s_in, w.desc["vocab"])
    l1 = D.prefill([s1], toks)
    l2 = D.prefill_matrix([s2], toks)
    assert np.abs(l1 - l2).max() < 1e-11
    assert np.abs(s1.kv - s2.kv).max() < 1e-12
    assert np.array_equal(s1.n, s2.n) and s1.n[0] == w.s_in
    # and decoding on from either cache agrees
    nxt = D.greedy(l1)
    assert np.abs(D.decode_step([s1], nxt) - D.decode_step([s2], nxt)).max() < 1e-11


def test_float32_oracle_agrees_with_float64():
    w = small("llama30b_m2")
    _, s64 = build(w)
    _, s32 = build(w, real=np.float32)
    toks = make_tokens(w.seed, w.batch, w.s_in, w.desc["vocab"])
    a, b = D.prefill([s64], toks), D.prefill([s32], toks)
    assert b.dtype == np.float32
    assert np.abs(a - b).max() < 2e-5 * max(1.0, np.abs(a).max())


# ----------------------------------------------------------------------------
# tensor-parallel slicing: the shards of a group sum to the unsharded layer
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("arch", ARCHS)
@pytest.mark.parametrize("M", [2, 4])
def test_group_of_shards_equals_unsharded(arch, M):
    w = small(arch)
    W, full = build(w)
    group = [D.OracleShard(w.desc, tp_slice(w.desc, 0, 2, m, M), W, w.batch, w.s_max) for m in range(M)]
    toks = make_tokens(w.seed, w.batch, w.s_in, w.desc["vocab"])
    a = D.prefill([full], toks)
    b = D.prefill(group, toks)
    assert np.abs(a - b).max() < 1e-11
    # each shard cached exactly its heads of the unsharded cache
    for m, s in enumerate(group):
        h0, h1 = s.slice["head_lo"], s.slice["head_hi"]
        assert np.abs(s.kv - full.kv[:, :, :, h0:h1]).max() < 1e-12
        assert np.array_equal(s.kv[0], full.kv[0, :, :, h0:h1])       # layer 0 sees identical inputs
    # a lone shard is NOT the full model (the other shards' partials are really missing)
    lone = D.OracleShard(w.desc, tp_slice(w.desc, 0, 2, 0, M), W, w.batch, w.s_max)
    assert np.abs(D.prefill([lone], toks) - a).max() > 1e-4


def test_shard_of_a_sub_parent_equals_shard_of_full_parent():
    """Slicing goes through the parent's own slice offsets correctly."""
    w = small("tiny_gpt")
    Wfull = make_weights(w.desc, w.slice, w.seed)
    half = tp_slice(w.desc, 0, 2, 1, 2)                      # heads [2,4), ffn [64,128)
    quarter = sub_slice_of(half, 1, 2)                       # heads [3,4), ffn [96,128)
    a = D.OracleShard(w.desc, quarter, Wfull, 1, 16)
    # build the half parent by hand-slicing the full tensors
    Dh = w.desc["head_dim"]
    Whalf = copy.copy(Wfull)
    Whalf["slice"] = half
    Whalf["layers"] = []
    for L in Wfull["layers"]:
        P = dict(L)
        c0, c1 = half["head_lo"] * Dh, half["head_hi"] * Dh
        for k in ("wq", "wk", "wv"):
            P[k] = L[k][:, c0:c1]
        for k in ("bq", "bk", "bv"):
            P[k] = L[k][c0:c1]
        P["wo"] = L["wo"][c0:c1]
        P["w1"], P["b1"], P["w2"] = L["w1"][:, 64:128], L["b1"][64:128], L["w2"][64:128]
        Whalf["layers"].append(P)
    b = D.OracleShard(w.desc, quarter, Whalf, 1, 16)
    toks = make_tokens(5, 1, 6, w.desc["vocab"])
    assert np.array_equal(D.prefill([a], toks), D.prefill([b], toks))


# ----------------------------------------------------------------------------
# attention: closed forms and invariants
# ----------------------------------------------------------------------------
def test_softmax_rows_sum_to_one_and_known_values():
    rng = np.random.default_rng(0)
    s = rng.normal(size=(50, 33)) * 5
    p = D.softmax(s)
    assert np.all(p >= 0) and np.abs(p.sum(-1) - 1).max() < 1e-12
    assert np.allclose(D.softmax(np.array([0.0, math.log(2.0)])), [1 / 3, 2 / 3], atol=1e-15)
    assert np.allclose(D.softmax(s + 1000.0), p, atol=1e-12)          # shift invariance, no overflow
    q = rng.normal(size=16)
    K = rng.normal(size=(9, 16))
    pr = D.attention_probs(q, K)
    assert abs(pr.sum() - 1) < 1e-12
    # scale is 1/sqrt(Dh): ratio of two probabilities is exp((s_i - s_j)/sqrt(Dh))
    assert np.isclose(pr[0] / pr[1], math.exp((K[0] @ q - K[1] @ q) / 4.0), rtol=1e-12)


def test_zero_query_gives_running_mean_of_values():
    """W_q = 0, b_q = 0: every score is 0, so head output at position n is mean(V[0..n])."""
    w = small("tiny_gpt", layers=1)
    W = make_weights(w.desc, w.slice, w.seed)
    L = W["layers"][0]
    L["wq"][:] = 0
    L["bq"][:] = 0
    s = D.OracleShard(w.desc, w.slice, W, 1, 16)
    toks = make_tokens(3, 1, 6, w.desc["vocab"])
    logits = D.prefill([s], toks)[0]
    # rebuild the last position from the cached values with the closed form
    x = s.wte[toks[0, 5]] + s.wpe[5]
    o = s.kv[0, 1, 0, :, :6, :].mean(axis=1).reshape(-1)              # mean over rows, per head
    x = x + o @ s.layers[0]["wo"] + s.layers[0]["bo"]
    a2 = torch.from_numpy(x)
    a2 = F.layer_norm(a2, (64,), torch.from_numpy(s.layers[0]["ln2_g"]), torch.from_numpy(s.layers[0]["ln2_b"]), 1e-5).numpy()
    h = F.gelu(torch.from_numpy(a2 @ s.layers[0]["w1"] + s.layers[0]["b1"]), approximate="tanh").numpy()
    x = x + h @ s.layers[0]["w2"] + s.layers[0]["b2"]
    xf = F.layer_norm(torch.from_numpy(x), (64,), torch.from_numpy(s.lnf_g), torch.from_numpy(s.lnf_b), 1e-5).numpy()
    assert np.abs(s.lm_head @ xf - logits).max() < 1e-11


def test_zero_values_make_attention_contribute_nothing():
    """W_v = 0, b_v = 0: logits cannot depend on W_q, W_k (attention output is exactly 0)."""
    w = small("llama30b_m2", layers=2)
    W = make_weights(w.desc, w.slice, w.seed)
    for L in W["layers"]:
        L["wv"][:] = 0
    toks = make_tokens(3, 2, 6, w.desc["vocab"])
    a = D.prefill([D.OracleShard(w.desc, w.slice, W, 2, 16)], toks)
    for L in W["layers"]:
        L["wq"] = L["wq"][::-1].copy()
        L["wk"] = L["wk"] * 3
    b = D.prefill([D.OracleShard(w.desc, w.slice, W, 2, 16)], toks)
    assert np.array_equal(a, b)


# ----------------------------------------------------------------------------
# norms, activations, RoPE
# ----------------------------------------------------------------------------
def test_norms_against_library_and_moments():
    rng = np.random.default_rng(1)
    x = rng.normal(size=(5, 64)) * 3 + 1.5
    g, b = rng.normal(size=64), rng.normal(size=64)
    y = D.layer_norm(x, np.ones(64), np.zeros(64), 0.0)
    assert np.abs(y.mean(-1)).max() < 1e-14 and np.abs(y.var(-1) - 1).max() < 1e-12
    t = lambda a: torch.from_numpy(a)
    assert np.abs(D.layer_norm(x, g, b, 1e-5) - F.layer_norm(t(x), (64,), t(g), t(b), 1e-5).numpy()).max() < 1e-13
    r = D.rms_norm(x, np.ones(64), 0.0)
    assert np.abs((r * r).mean(-1) - 1).max() < 1e-12
    assert np.abs(D.rms_norm(x, g, 1e-6) - F.rms_norm(t(x), (64,), t(g), 1e-6).numpy()).max() < 1e-13


def test_activations_closed_forms():
    x = np.linspace(-6, 6, 101)
    assert D.gelu_tanh(np.array([0.0]))[0] == 0.0
    assert np.abs(D.gelu_tanh(x) - D.gelu_tanh(-x) - x).max() < 1e-14      # odd part is x/2 + x/2
    assert np.abs(D.silu(x) - D.silu(-x) - x).max() < 1e-14
    assert abs(D.gelu_tanh(np.array([1.0]))[0] - 0.5 * (1 + math.tanh(math.sqrt(2 / math.pi) * 1.044715))) < 1e-15
    assert abs(D.silu(np.array([1.0]))[0] - 1 / (1 + math.exp(-1))) < 1e-15
    assert np.abs(D.gelu_tanh(x) - F.gelu(torch.from_numpy(x), approximate="tanh").numpy()).max() < 1e-14
    assert np.abs(D.silu(x) - F.silu(torch.from_numpy(x)).numpy()).max() < 1e-14
    assert np.array_equal(D.relu(np.array([-1.0, 0.0, 2.0])), [0.0, 0.0, 2.0])


def test_rope_properties():
    rng = np.random.default_rng(2)
    q, k = rng.normal(size=(3, 32)), rng.normal(size=(3, 32))
    assert np.array_equal(D.rope_rotate(q, 0, 10000.0), q)                  # position 0 is the identity
    for m, n, s in [(5, 2, 7), (100, 99, 1000), (3, 3, 11)]:
        a = (D.rope_rotate(q, m, 1e4) * D.rope_rotate(k, n, 1e4)).sum(-1)
        b = (D.rope_rotate(q, m + s, 1e4) * D.rope_rotate(k, n + s, 1e4)).sum(-1)
        assert np.abs(a - b).max() < 1e-10                                   # depends on m - n only
    r = D.rope_rotate(q, 17, 1e4)
    assert np.abs((r * r).sum(-1) - (q * q).sum(-1)).max() < 1e-12           # a rotation
    # first pair rotates by exactly `pos` radians (theta^0), pairing is (i, i + Dh/2)
    e = np.zeros(32)
    e[0] = 1.0
    r = D.rope_rotate(e, 2, 1e4)
    assert np.isclose(r[0], math.cos(2.0)) and np.isclose(r[16], math.sin(2.0)) and np.abs(np.delete(r, [0, 16])).max() == 0
    # last pair rotates by pos * theta^(-(Dh-2)/Dh)
    e = np.zeros(32)
    e[15] = 1.0
    r = D.rope_rotate(e, 3, 1e4)
    assert np.isclose(r[15], math.cos(3.0 * 1e4 ** (-30 / 32))) and np.isclose(r[31], math.sin(3.0 * 1e4 ** (-30 / 32)))


def test_rope_model_is_shift_invariant_in_the_cache():
    """For the RoPE model, attention scores depend on relative position only, so the oracle's
    scores from cached rotated keys equal scores recomputed with all positions shifted."""
    w = small("llama30b_m2", layers=1)
    W, s = build(w)
    L = s.layers[0]
    rng = np.random.default_rng(4)
    a = rng.normal(size=(6, 64))
    q0, k0, _ = s._qkv(L, a, np.arange(6))
    q1, k1, _ = s._qkv(L, a, np.arange(6) + 37)
    s0 = np.einsum("qhd,khd->hqk", q0, k0)
    s1 = np.einsum("qhd,khd->hqk", q1, k1)
    assert np.abs(s0 - s1).max() < 1e-10


# ----------------------------------------------------------------------------
# batch semantics, commit, greedy
# ----------------------------------------------------------------------------
def test_rows_are_independent_and_permute():
    w = small("opt66b_m8", batch=4)
    W, s1 = build(w)
    _, s2 = build(w)
    toks = make_tokens(w.seed, 4, 6, w.desc["vocab"])
    perm = np.array([2, 0, 3, 1])
    a = D.prefill([s1], toks)
    b = D.prefill([s2], toks[perm])
    assert np.array_equal(a[perm], b)
    # ragged lengths: rows may be at different positions
    _, s3 = build(w)
    D.prefill([s3], toks[:, :3])
    D.decode_step([s3], toks[:, 3], rows=[1, 2])
    assert list(s3.n) == [3, 4, 4, 3]
    l3 = D.decode_step([s3], np.array([toks[0, 3], toks[1, 4], toks[2, 4], toks[3, 3]]))
    _, s4 = build(w)
    D.prefill([s4], toks[:, :4])
    l4a = D.decode_step([s4], toks[:, 4])
    _, s5 = build(w)
    D.prefill([s5], toks[:, :3])
    l5 = D.decode_step([s5], toks[:, 3])
    assert np.array_equal(l3[[1, 2]], l4a[[1, 2]]) and np.array_equal(l3[[0, 3]], l5[[0, 3]])


def test_commit_is_the_last_action_and_row_n_is_invisible_before():
    w = small("tiny_gpt")
    W, s = build(w)
    toks = make_tokens(w.seed, w.batch, 5, w.desc["vocab"])
    D.prefill([s], toks)
    kv_before, n_before = s.kv.copy(), s.n.copy()
    D.decode_step([s], toks[:, 0])
    assert np.array_equal(s.n, n_before + 1)
    # committed rows are never rewritten by a later step
    assert np.array_equal(s.kv[:, :, :, :, :5], kv_before[:, :, :, :, :5])
    # garbage beyond n does not influence a step: poison rows >= n and repeat
    _, s2 = build(w)
    D.prefill([s2], toks)
    s2.kv[:, :, :, :, 5:] = 1e30
    _, s3 = build(w)
    D.prefill([s3], toks)
    assert np.array_equal(D.decode_step([s2], toks[:, 0]), D.decode_step([s3], toks[:, 0]))


def test_greedy_takes_lowest_index_on_ties():
    assert list(D.greedy(np.array([[1.0, 3.0, 3.0, 2.0], [5.0, 5.0, 5.0, 5.0]]))) == [1, 0]


# ----------------------------------------------------------------------------
# KV re-partition
# ----------------------------------------------------------------------------
def rand_kv(rng, L, B, H, S, Dh, dtype=np.uint16):
    return rng.integers(0, 60000, size=(L, 2, B, H, S, Dh)).astype(dtype)


def sl(l0, l1, h0, h1):
    return dict(layer_lo=l0, layer_hi=l1, head_lo=h0, head_hi=h1, ffn_lo=0, ffn_hi=1)


def test_repack_against_slice_formulation_and_byte_count():
    rng = np.random.default_rng(7)
    src = rand_kv(rng, 3, 4, 6, 10, 8)                        # layers [1,4), heads [2,8)
    s_sl = sl(1, 4, 2, 8)
    n = np.array([10, 0, 7, 3])
    d_sl = sl(1, 4, 5, 8)                                     # heads [5,8) of the same layers
    dst = rand_kv(rng, 3, 3, 3, 12, 8)                        # other batch size and capacity
    before = dst.copy()
    bmap = [2, -1, 0]
    moved = D.kv_repack_arrays(dst, d_sl, src, s_sl, n, bmap)
    exp = before.copy()
    exp[:, :, 0, :, :7] = src[:, :, 2, 3:6, :7]
    exp[:, :, 2, :, :10] = src[:, :, 0, 3:6, :10]
    assert np.array_equal(dst, exp)
    assert moved == 3 * 2 * 3 * (7 + 10) * 8                  # layers x {K,V} x heads∩ x rows x Dh
    assert np.array_equal(dst[:, :, 1], before[:, :, 1])      # unmapped row untouched


def test_repack_layer_and_head_intersection():
    rng = np.random.default_rng(8)
    src = rand_kv(rng, 4, 1, 4, 5, 4)                         # layers [0,4), heads [0,4)
    dst = np.zeros((3, 2, 1, 4, 5, 4), dtype=np.uint16)       # layers [2,5), heads [2,6)
    moved = D.kv_repack_arrays(dst, sl(2, 5, 2, 6), src, sl(0, 4, 0, 4), [5], [0])
    assert moved == 2 * 2 * 2 * 5 * 4
    assert np.array_equal(dst[0:2, :, :, 0:2], src[2:4, :, :, 2:4])
    assert not dst[2].any() and not dst[:, :, :, 2:].any()


def position_slice(index, D_, P, M, n_layers, n_heads):
    """(layers, heads) of position `index` of a (D, P, M) configuration, numbered d-major, then
    stage, then tensor shard."""
    m = index % M
    p = (index // M) % P
    return sl(p * n_layers // P, (p + 1) * n_layers // P, m * n_heads // M, (m + 1) * n_heads // M)


def test_device_mapping_example_of_the_paper():
    """tests/golden/device_mapping_example.txt: the intersection sizes the re-partition reports
    rank the target positions as the paper's worked example says."""
    import os
    cfg = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "device_mapping_example.txt")):
        f = line.split()
        if not f or f[0].startswith("#"):
            continue
        cfg[f[0]] = f[1:]
    cur = {k: int(v) for k, v in (t.split("=") for t in cfg["current"])}
    tgt = {k: int(v) for k, v in (t.split("=") for t in cfg["target"])}
    src_index = int(cfg["source"][0][1:])
    best = sorted(int(t[1:]) for t in cfg["best_targets"])
    n_layers, n_heads, B, S, Dh = 6, 4, 2, 5, 4            # layers divisible by both stage counts
    rng = np.random.default_rng(11)
    s_sl = position_slice(src_index, cur["D"], cur["P"], cur["M"], n_layers, n_heads)
    src = rand_kv(rng, s_sl["layer_hi"] - s_sl["layer_lo"], B, s_sl["head_hi"] - s_sl["head_lo"], S, Dh)
    n = [S, 3]
    counts = []
    for j in range(tgt["D"] * tgt["P"] * tgt["M"]):
        d_sl = position_slice(j, tgt["D"], tgt["P"], tgt["M"], n_layers, n_heads)
        dst = np.zeros((d_sl["layer_hi"] - d_sl["layer_lo"], 2, B, d_sl["head_hi"] - d_sl["head_lo"], S, Dh), np.uint16)
        counts.append(D.kv_repack_arrays(dst, d_sl, src, s_sl, n, [0, 1]))
    top = max(counts)
    assert sorted(j for j, c in enumerate(counts) if c == top) == best
    assert top > 0 and counts.count(top) == len(best)
    # and the sizes themselves: stage 0 of the target takes layers [0,2) of u_1's [0,3), stage 1 one layer, stage 2 none
    per_layer = 2 * 2 * (S + 3) * Dh                         # {K,V} x u_1's two heads x committed rows x Dh
    assert counts == [2 * per_layer, per_layer, 0, 2 * per_layer, per_layer, 0]


@pytest.mark.parametrize("M,Mp", [(2, 4), (4, 2), (1, 4), (4, 1)])
def test_repack_round_trip_is_identity(M, Mp):
    """M-way -> M'-way -> M-way gives back every committed byte (Section 3.3: only the
    layout changes, results are identical)."""
    rng = np.random.default_rng(9)
    H, B, S, Dh, L = 8, 3, 9, 4, 2
    n = np.array([9, 4, 0])
    srcs = [rand_kv(rng, L, B, H // M, S, Dh) for _ in range(M)]
    s_sl = [sl(0, L, m * H // M, (m + 1) * H // M) for m in range(M)]
    mids = [np.zeros((L, 2, B, H // Mp, S + 2, Dh), dtype=np.uint16) for _ in range(Mp)]
    m_sl = [sl(0, L, m * H // Mp, (m + 1) * H // Mp) for m in range(Mp)]
    total = 0
    for d, dsl in zip(mids, m_sl):
        for s, ssl in zip(srcs, s_sl):
            total += D.kv_repack_arrays(d, dsl, s, ssl, n, [0, 1, 2])
    assert total == L * 2 * H * Dh * n.sum()                  # conservation: every committed element once
    backs = [np.zeros_like(s) for s in srcs]
    for bk, bsl in zip(backs, s_sl):
        for d, dsl in zip(mids, m_sl):
            D.kv_repack_arrays(bk, bsl, d, dsl, n, [0, 1, 2])
    for bk, s in zip(backs, srcs):
        for b in range(B):
            assert np.array_equal(bk[:, :, b, :, :n[b]], s[:, :, b, :, :n[b]])
            assert not bk[:, :, b, :, n[b]:].any()            # nothing beyond the committed rows moved


@pytest.mark.parametrize("arch", ["llama30b_m2", "tiny_gpt"])
def test_resume_after_repartition_equals_uninterrupted(arch):
    """Decode k tokens on an M=2 shard, move its cache into two M'=4 shards, resume j tokens
    on the pair: identical to k + j uninterrupted tokens (Section 4.1: resume without
    recomputing; Section 2.2: the pair sums to the original shard)."""
    w = small(arch, n_heads=8, head_dim=8, batch=3, s_in=5, s_max=16)
    W = make_weights(w.desc, w.slice, w.seed)
    half = tp_slice(w.desc, 0, 2, 1, 2)
    toks = make_tokens(w.seed, 3, 5, w.desc["vocab"])
    ref = D.OracleShard(w.desc, half, W, 3, 16)
    run = D.OracleShard(w.desc, half, W, 3, 16)
    nxt = D.greedy(D.prefill([ref], toks))
    D.prefill([run], toks)
    ref_logits = []
    for _ in range(6):
        lg = D.decode_step([ref], nxt)
        ref_logits.append(lg)
        nxt = D.greedy(lg)
    nxt = D.greedy(D.prefill_matrix([D.OracleShard(w.desc, half, W, 3, 16)], toks))
    for i in range(3):
        lg = D.decode_step([run], nxt)
        assert np.array_equal(lg, ref_logits[i])
        nxt = D.greedy(lg)
    # re-partition: keep rows 2 and 0 only, in that order (cache discard keeps a subset)
    pair = [D.OracleShard(w.desc, sub_slice_of(half, p, 2), W, 2, 20) for p in range(2)]
    for p in pair:
        D.kv_repack(p, run, [2, 0])
    assert list(pair[0].n) == [8, 8]
    nxt = nxt[[2, 0]]
    for i in range(3, 6):
        lg = D.decode_step(pair, nxt)
        assert np.abs(lg - ref_logits[i][[2, 0]]).max() < 1e-11
        nxt = D.greedy(lg)


def test_canonical_export_order():
    w = small("tiny_gpt", batch=2)
    W, s = build(w)
    toks = make_tokens(w.seed, 2, 4, w.desc["vocab"])
    D.prefill([s], toks)
    D.decode_step([s], toks[:, 0], rows=[1])
    flat = D.kv_canonical(s)
    Dh, H = 16, 4
    assert flat.size == 2 * 2 * H * Dh * (4 + 5)
    # first block is layer 0, keys, row 0, head 0, 4 committed rows
    assert np.array_equal(flat[:4 * Dh], s.kv[0, 0, 0, 0, :4].reshape(-1))
    # row 1 of (layer 0, keys) follows all heads of row 0
    off = H * 4 * Dh
    assert np.array_equal(flat[off:off + 5 * Dh], s.kv[0, 0, 1, 0, :5].reshape(-1))
