"""Workload shapes and seeded random inputs.

The five named workloads take their shapes from the models and the serving
set-up of the paper's evaluation (GPT-20B, LLaMA-30B and the OPT family under
pipeline x tensor partitions, fixed-length prompts, static batches; Section 6.1
and Table 1) as fixed by this build's benchmark configurations.  No trained
weights or request traces are available, so every tensor is drawn from a
seeded counter-based generator and stands in for them.

Nothing here computes any part of the decoder; it only draws numbers.

Weight container (plain dict of numpy arrays; "parent" tensors of a slice):

    weights["slice"]          dict(layer_lo, layer_hi, head_lo, head_hi, ffn_lo, ffn_hi)
                              the part of the full model these tensors cover
    weights["wte"]            [V, d]        token embedding            (matrix dtype)
    weights["wpe"]            [max_pos, d]  learned positions or None  (matrix dtype)
    weights["lm_head"]        [V, d]        logits = xf @ lm_head.T    (matrix dtype; may be wte itself)
    weights["lnf_g"|"lnf_b"]  [d]           final norm gain / shift (shift None for RMSNorm), float32
    weights["layers"][i]      layer layer_lo+i:
        ln1_g ln1_b ln2_g ln2_b   [d]                float32
        wq wk wv                  [d, Hp*Dh]         y = x @ W          (matrix dtype)
        bq bk bv                  [Hp*Dh]            float32 or None
        wo                        [Hp*Dh, d]         (matrix dtype)
        bo                        [d]                float32 or None
        w1 (GELU/ReLU)            [d, Fp]   b1 [Fp]
        wg wu (SwiGLU)            [d, Fp]   (no bias)
        w2                        [Fp, d]   b2 [d]
    Hp = head_hi-head_lo and Fp = ffn_hi-ffn_lo of weights["slice"].

Matrix dtype is float32 for desc["dtype"] == "f32" and uint16 holding bfloat16
bit patterns for "bf16".  Vectors are always float32; for a bf16 model their
values are bf16-representable.
"""
from __future__ import annotations

import copy
import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

__all__ = [
    "CONFIGS", "Workload", "workload", "scaled_workload", "make_weights", "make_tokens",
    "f32_to_bf16_bits", "bf16_bits_to_f32", "sub_slice_of", "tp_slice",
]


# ----------------------------------------------------------------------------
# bf16 bit-pattern helpers (storage format conversion only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even), return uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) to float32, exactly."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# Workload descriptors
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    desc: dict            # full-model descriptor
    slice: dict           # the shard's (layers, heads, ffn) slice
    batch: int
    s_in: int             # prompt tokens per sequence
    steps: int            # decode steps after prefill
    s_max: int            # KV capacity in rows
    seed: int
    extra: dict = field(default_factory=dict)


def _desc(n_layers, d_model, n_heads, head_dim, ffn, vocab, max_pos, norm, act, pos,
          has_bias, dtype, norm_eps, rope_theta=10000.0):
    return dict(n_layers=n_layers, d_model=d_model, n_heads=n_heads, head_dim=head_dim,
                ffn=ffn, vocab=vocab, max_pos=max_pos, norm=norm, act=act, pos=pos,
                has_bias=bool(has_bias), dtype=dtype, norm_eps=float(norm_eps),
                rope_theta=float(rope_theta), tied_lm_head=(pos == "learned"),
                kv_dtype="f32" if dtype == "f32" else "f16")


def tp_slice(desc, layer_lo, layer_hi, m, M):
    """Slice of tensor-parallel shard m of M over layers [layer_lo, layer_hi)."""
    H, F = desc["n_heads"], desc["ffn"]
    assert H % M == 0 and F % M == 0
    return dict(layer_lo=layer_lo, layer_hi=layer_hi,
                head_lo=m * H // M, head_hi=(m + 1) * H // M,
                ffn_lo=m * F // M, ffn_hi=(m + 1) * F // M)


def _configs():
    c = {}
    d1 = _desc(2, 256, 4, 64, 1024, 1024, 32, "layernorm", "gelu_tanh", "learned", True, "f32", 1e-5)
    c["tiny_gpt"] = Workload("tiny_gpt", d1, tp_slice(d1, 0, 2, 0, 1), 1, 16, 16, 32, 1001)
    d2 = _desc(44, 6144, 48, 128, 24576, 50000, 640, "layernorm", "gelu_tanh", "learned", True, "bf16", 1e-5)
    c["gpt20b_m4"] = Workload("gpt20b_m4", d2, tp_slice(d2, 0, 11, 0, 4), 8, 512, 128, 640, 1002)
    d3 = _desc(60, 6656, 52, 128, 17920, 32000, 0, "rmsnorm", "swiglu", "rope", False, "bf16", 1e-6)
    c["llama30b_m2"] = Workload("llama30b_m2", d3, tp_slice(d3, 0, 15, 0, 2), 16, 1024, 256, 1280, 1003)
    d4 = _desc(64, 9216, 72, 128, 36864, 50272, 640, "layernorm", "relu", "learned", True, "bf16", 1e-5)
    c["opt66b_m8"] = Workload("opt66b_m8", d4, tp_slice(d4, 0, 16, 0, 8), 32, 512, 128, 640, 1004)
    d5 = copy.deepcopy(d3)
    c["llama30b_reparallelize"] = Workload(
        "llama30b_reparallelize", d5, tp_slice(d5, 0, 15, 0, 2), 16, 976, 24, 1024, 1005,
        extra=dict(dst_slices=[tp_slice(d5, 0, 15, 0, 4), tp_slice(d5, 0, 15, 1, 4)], resume_steps=24))
    return c


CONFIGS = _configs()


def workload(name: str) -> Workload:
    return copy.deepcopy(CONFIGS[name])


def scaled_workload(name: str, *, d_model, n_heads, head_dim, ffn, vocab, layers, M, m=0,
                    batch, s_in, steps, s_max=None, dtype=None, seed=None) -> Workload:
    """The architecture words (norm, activation, positions, biases, dtype) of a named
    workload on smaller dimensions, for parity cases the CPU oracle finishes quickly."""
    w = workload(name)
    d = w.desc
    d.update(n_layers=layers, d_model=d_model, n_heads=n_heads, head_dim=head_dim, ffn=ffn, vocab=vocab)
    if dtype is not None:
        d["dtype"] = dtype
        d["kv_dtype"] = "f32" if dtype == "f32" else "f16"
    s_max = s_max if s_max is not None else s_in + steps
    if d["pos"] == "learned":
        d["max_pos"] = s_max
    w.slice = tp_slice(d, 0, layers, m, M)
    w.batch, w.s_in, w.steps, w.s_max = batch, s_in, steps, s_max
    if seed is not None:
        w.seed = seed
    w.name = name + "_scaled"
    w.extra = {}
    return w


def sub_slice_of(parent_slice: dict, part: int, parts: int) -> dict:
    """Split a slice's head and FFN intervals into `parts` equal pieces; return piece `part`."""
    h0, h1, f0, f1 = (parent_slice[k] for k in ("head_lo", "head_hi", "ffn_lo", "ffn_hi"))
    assert (h1 - h0) % parts == 0 and (f1 - f0) % parts == 0
    hs, fs = (h1 - h0) // parts, (f1 - f0) // parts
    s = dict(parent_slice)
    s.update(head_lo=h0 + part * hs, head_hi=h0 + (part + 1) * hs,
             ffn_lo=f0 + part * fs, ffn_hi=f0 + (part + 1) * fs)
    return s


# ----------------------------------------------------------------------------
# Random tensors
# ----------------------------------------------------------------------------
_TENSOR_IDS = {n: i for i, n in enumerate(
    ["wte", "wpe", "lm_head", "lnf_g", "lnf_b", "ln1_g", "ln1_b", "ln2_g", "ln2_b",
     "wq", "wk", "wv", "bq", "bk", "bv", "wo", "bo", "w1", "b1", "wg", "wu", "w2", "b2", "tokens"])}


def _gen(seed: int, name: str, layer: int):
    # counter-based generator keyed by (seed, tensor identity): tensors are independent
    # of one another and of the order in which they are drawn
    return np.random.Generator(np.random.Philox(key=[seed, (_TENSOR_IDS[name] << 20) | (layer + 1)]))


def _normal(seed, name, layer, shape, dtype, mean=0.0, std=0.02, as_matrix=True):
    g = _gen(seed, name, layer)
    a = g.standard_normal(size=shape, dtype=np.float32)
    a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    if dtype == "bf16":
        b = f32_to_bf16_bits(a)
        return b if as_matrix else bf16_bits_to_f32(b)
    return a


def make_weights(desc: dict, parent_slice: dict, seed: int, threads: int | None = None) -> dict:
    """Draw every tensor of the slice: matrices, embeddings and biases ~ N(0, 0.02^2);
    norm gains ~ 1 + N(0, 0.02^2), norm shifts ~ N(0, 0.02^2); then round to bf16 for
    a bf16 model."""
    d, Dh, V = desc["d_model"], desc["head_dim"], desc["vocab"]
    Hp = parent_slice["head_hi"] - parent_slice["head_lo"]
    Fp = parent_slice["ffn_hi"] - parent_slice["ffn_lo"]
    dt = desc["dtype"]
    ln = desc["norm"] == "layernorm"
    bias = desc["has_bias"]
    jobs = []  # (container, key, args)
    w = {"slice": dict(parent_slice), "layers": []}

    def mat(c, key, layer, shape):
        jobs.append((c, key, (seed, key, layer, shape, dt, 0.0, 0.02, True)))

    def vec(c, key, layer, n, mean=0.0):
        jobs.append((c, key, (seed, key, layer, (n,), dt, mean, 0.02, False)))

    mat(w, "wte", -1, (V, d))
    if desc["pos"] == "learned":
        mat(w, "wpe", -1, (desc["max_pos"], d))
    else:
        w["wpe"] = None
    if not desc.get("tied_lm_head", False):
        mat(w, "lm_head", -1, (V, d))
    vec(w, "lnf_g", -1, d, 1.0)
    if ln:
        vec(w, "lnf_b", -1, d)
    else:
        w["lnf_b"] = None
    for layer in range(parent_slice["layer_lo"], parent_slice["layer_hi"]):
        L = {}
        w["layers"].append(L)
        for k in ("ln1", "ln2"):
            vec(L, k + "_g", layer, d, 1.0)
            if ln:
                vec(L, k + "_b", layer, d)
            else:
                L[k + "_b"] = None
        for k in ("wq", "wk", "wv"):
            mat(L, k, layer, (d, Hp * Dh))
        for k in ("bq", "bk", "bv"):
            if bias:
                vec(L, k, layer, Hp * Dh)
            else:
                L[k] = None
        mat(L, "wo", layer, (Hp * Dh, d))
        if desc["act"] == "swiglu":
            mat(L, "wg", layer, (d, Fp))
            mat(L, "wu", layer, (d, Fp))
        else:
            mat(L, "w1", layer, (d, Fp))
            if bias:
                vec(L, "b1", layer, Fp)
            else:
                L["b1"] = None
        mat(L, "w2", layer, (Fp, d))
        for k in ("bo", "b2"):
            if bias:
                vec(L, k, layer, d)
            else:
                L[k] = None

    threads = threads or min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        outs = list(ex.map(lambda j: _normal(*j[2]), jobs))
    for (c, key, _), a in zip(jobs, outs):
        c[key] = a
    if desc.get("tied_lm_head", False):
        w["lm_head"] = w["wte"]
    return w


def make_tokens(seed: int, batch: int, length: int, vocab: int) -> np.ndarray:
    """Token ids i.i.d. uniform on [0, vocab), int32 [batch, length]."""
    g = _gen(seed, "tokens", -1)
    return g.integers(0, vocab, size=(batch, length), dtype=np.int32)
