"""CPU oracle: one tensor-parallel shard of a KV-cached GPT-style decoder, and the
KV-cache head re-partition, written out from their definitions.

THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the benchmark's
CPU-baseline leg may import it.  It shares no code with the HIP library and does
not import it.

What it follows
---------------
* Section 2.1, Eq. (1)-(2): generation is an "initial phase" over all S_in prompt
  tokens that yields the first output token, then one incremental iteration per
  output token; with the keys and values of every layer cached, an iteration
  processes a single token and reaches the same result as recomputing the whole
  sequence.  `decode_step` is that iteration; `prefill` is by definition S_in
  applications of it; `forward_matrix` is the full causal recompute of Eq. (1).
* Section 2.2 (intra-operator parallelism): a shard owns a slice of every operator
  (whole heads of the attention, columns of the first FFN matrix and the matching
  rows of the second); the partial results of the shards are summed (the
  All-Reduce) to restore the full layer output.  A `group` of co-resident shards
  is summed here in place of the collective; a lone shard sums only itself.
* Section 3.3: switching configuration re-uses, per device, the intersection of
  the context it holds and the context its new position needs; `kv_repack` moves
  exactly that intersection of the cache context, for the kept batch rows.
* Section 4.1: progress is committed per token: `n[b]` counts the tokens whose
  keys/values are in the cache; a request can stop after any iteration and resume
  from (token list, rows [0, n)).

The paper takes the decoder arithmetic from the models it cites; the conventions
below are this build's reading and are "parity unpinned by the paper" (both sides
must simply agree): pre-norm blocks with sequential residuals and a final norm;
LayerNorm with biased variance; RMSNorm without shift; tanh-form GELU; RoPE with
half-split pairing applied to q and k before caching; scores scaled by 1/sqrt(Dh);
row-parallel biases (b_o, b_2) added once after the sum over shards; greedy argmax
with the lowest index on ties.  Each of them is pinned against a library routine
or a closed form in tests/test_oracle_pins.py.

All arithmetic is done in `real` (float64 by default; float32 for the full-size
cases where float64 copies of the weights do not fit in host memory).
"""
from __future__ import annotations

import math

import numpy as np


# ----------------------------------------------------------------------------
# storage helpers
# ----------------------------------------------------------------------------
def _widen(a, real):
    """Matrix in its storage dtype (float32, or uint16 bf16 bit patterns) -> `real`, exactly."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        a = (a.astype(np.uint32) << np.uint32(16)).view(np.float32)
    return np.ascontiguousarray(a, dtype=real)


# ----------------------------------------------------------------------------
# elementary operators
# ----------------------------------------------------------------------------
def layer_norm(x, g, b, eps):
    """LayerNorm over the last axis, biased variance."""
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps) * g + b


def rms_norm(x, g, eps):
    """RMSNorm over the last axis: x / sqrt(mean(x^2) + eps) * g."""
    ms = (x * x).mean(axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (x + 0.044715 * x ** 3)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def relu(x):
    return np.maximum(x, 0.0)


def rope_rotate(v, pos, theta):
    """Rotary position embedding, half-split pairing.

    v: [..., Dh]; pos: integer position (scalar or array broadcastable to v[..., 0]).
    Pair i couples components i and i + Dh/2 and is rotated by pos * theta**(-2i/Dh).
    """
    Dh = v.shape[-1]
    half = Dh // 2
    i = np.arange(half, dtype=np.float64)
    ang = np.asarray(pos, dtype=np.float64)[..., None] * theta ** (-2.0 * i / Dh)
    c, s = np.cos(ang).astype(v.dtype), np.sin(ang).astype(v.dtype)
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, a * s + b * c], axis=-1)


def softmax(s):
    """Softmax over the last axis: subtract the maximum, exponentiate, divide by the sum."""
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def attention_probs(q, K):
    """p_j = softmax_j(q . K_j / sqrt(Dh)) for one head: q [Dh], K [n, Dh] -> [n]."""
    return softmax((K @ q) / math.sqrt(q.shape[-1]))


def greedy(logits):
    """Greedy next token: argmax, lowest index on ties (numpy's argmax rule)."""
    return np.argmax(logits, axis=-1).astype(np.int32)


# ----------------------------------------------------------------------------
# the shard
# ----------------------------------------------------------------------------
class OracleShard:
    """Model context (weight slice) and cache context (K/V rows) of one position
    (layers [layer_lo, layer_hi), heads [head_lo, head_hi), FFN columns [ffn_lo, ffn_hi))."""

    def __init__(self, desc, slc, parent, max_batch, max_seq, real=np.float64):
        self.desc, self.slice, self.real = dict(desc), dict(slc), real
        ps = parent["slice"]
        for lo, hi in (("layer_lo", "layer_hi"), ("head_lo", "head_hi"), ("ffn_lo", "ffn_hi")):
            if not (ps[lo] <= slc[lo] < slc[hi] <= ps[hi]):
                raise ValueError(f"slice {slc} not inside parent slice {ps}")
        Dh = desc["head_dim"]
        self.Ls = slc["layer_hi"] - slc["layer_lo"]
        self.Hs = slc["head_hi"] - slc["head_lo"]
        self.Fs = slc["ffn_hi"] - slc["ffn_lo"]
        c0, c1 = (slc["head_lo"] - ps["head_lo"]) * Dh, (slc["head_hi"] - ps["head_lo"]) * Dh
        f0, f1 = slc["ffn_lo"] - ps["ffn_lo"], slc["ffn_hi"] - ps["ffn_lo"]
        w = lambda a: _widen(a, real)
        self.wte, self.wpe = w(parent["wte"]), w(parent["wpe"])
        self.lm_head = self.wte if parent["lm_head"] is parent["wte"] else w(parent["lm_head"])
        self.lnf_g, self.lnf_b = w(parent["lnf_g"]), w(parent["lnf_b"])
        self.layers = []
        for l in range(slc["layer_lo"], slc["layer_hi"]):
            P = parent["layers"][l - ps["layer_lo"]]
            L = dict(ln1_g=w(P["ln1_g"]), ln1_b=w(P["ln1_b"]), ln2_g=w(P["ln2_g"]), ln2_b=w(P["ln2_b"]),
                     bo=w(P["bo"]), b2=w(P["b2"]))
            for k in ("wq", "wk", "wv"):                       # column-sliced by whole heads
                L[k] = w(P[k][:, c0:c1])
            for k in ("bq", "bk", "bv"):
                L[k] = None if P[k] is None else w(P[k][c0:c1])
            L["wo"] = w(P["wo"][c0:c1, :])                     # row-sliced
            if desc["act"] == "swiglu":
                L["wg"], L["wu"] = w(P["wg"][:, f0:f1]), w(P["wu"][:, f0:f1])
            else:
                L["w1"] = w(P["w1"][:, f0:f1])
                L["b1"] = None if P["b1"] is None else w(P["b1"][f0:f1])
            L["w2"] = w(P["w2"][f0:f1, :])
            self.layers.append(L)
        self.max_batch, self.max_seq = max_batch, max_seq
        # cache context: kv[l, 0] = keys, kv[l, 1] = values; rows >= n[b] hold nothing meaningful
        self.kv = np.zeros((self.Ls, 2, max_batch, self.Hs, max_seq, Dh), dtype=real)
        self.n = np.zeros(max_batch, dtype=np.int64)

    # -- helpers over the descriptor ------------------------------------------
    def _norm(self, x, g, b):
        if self.desc["norm"] == "layernorm":
            return layer_norm(x, g, b, self.desc["norm_eps"])
        return rms_norm(x, g, self.desc["norm_eps"])

    def _embed(self, tok, pos):
        x = self.wte[tok].copy()
        if self.desc["pos"] == "learned":
            x = x + self.wpe[pos]
        return x

    def _ffn_partial(self, L, a2):
        if self.desc["act"] == "swiglu":
            u = silu(a2 @ L["wg"]) * (a2 @ L["wu"])
        else:
            h = a2 @ L["w1"]
            if L["b1"] is not None:
                h = h + L["b1"]
            u = gelu_tanh(h) if self.desc["act"] == "gelu_tanh" else relu(h)
        return u @ L["w2"]

    def _qkv(self, L, a, pos):
        """a: [..., d] -> q, k, v: [..., Hs, Dh], rotated at `pos` for RoPE models."""
        Dh = self.desc["head_dim"]
        out = []
        for wk, bk in (("wq", "bq"), ("wk", "bk"), ("wv", "bv")):
            y = a @ L[wk]
            if L[bk] is not None:
                y = y + L[bk]
            out.append(y.reshape(*y.shape[:-1], self.Hs, Dh))
        q, k, v = out
        if self.desc["pos"] == "rope":
            p = np.asarray(pos)[..., None]                     # same position for every head
            q, k = rope_rotate(q, p, self.desc["rope_theta"]), rope_rotate(k, p, self.desc["rope_theta"])
        return q, k, v


def _check_group(group):
    g0 = group[0]
    for s in group[1:]:
        if (s.slice["layer_lo"], s.slice["layer_hi"]) != (g0.slice["layer_lo"], g0.slice["layer_hi"]):
            raise ValueError("shards of a group must hold the same layers")
        if not np.array_equal(s.n, g0.n):
            raise ValueError("shards of a group must have committed the same lengths")
    for i, a in enumerate(group):
        for b in group[i + 1:]:
            if a.slice["head_lo"] < b.slice["head_hi"] and b.slice["head_lo"] < a.slice["head_hi"]:
                raise ValueError("head slices of a group overlap")
            if a.slice["ffn_lo"] < b.slice["ffn_hi"] and b.slice["ffn_lo"] < a.slice["ffn_hi"]:
                raise ValueError("FFN slices of a group overlap")


def decode_step(group, tokens, rows=None, hidden_in=None, hidden_out=False):
    """One incremental decoding iteration (Section 2.1) for every batch row in `rows`
    (default: all rows of tokens): consumes token tokens[b] at position n[b], appends
    its key/value as cache row n[b], attends over rows 0..n[b], returns the logits
    [B, V] of the next token and commits n[b] <- n[b] + 1 as the last action.

    Pipeline stages (Section 2.2, inter-operator parallelism): with hidden_in [B, d] the
    shard is not the model's first stage and starts from the previous stage's output
    instead of the embedding (tokens is then ignored and may be None); with hidden_out
    it is not the last stage and returns the residual stream after its layers, [B, d],
    instead of applying the final norm and the LM head.

    group: list of co-resident shards of the same layers with disjoint head / FFN
    slices; their partial attention and FFN outputs are summed where a tensor-parallel
    group would All-Reduce (Section 2.2).  Embedding, norms, row-parallel biases and
    the LM head are taken from group[0].
    """
    _check_group(group)
    g0 = group[0]
    desc = g0.desc
    Dh = desc["head_dim"]
    nrows = len(tokens) if hidden_in is None else len(hidden_in)
    tokens = None if hidden_in is not None else np.asarray(tokens)
    rows = range(nrows) if rows is None else rows
    out = np.zeros((nrows, desc["d_model"] if hidden_out else desc["vocab"]), dtype=g0.real)
    for b in rows:
        n = int(g0.n[b])
        if n + 1 > g0.max_seq:
            raise RuntimeError("KV cache full")
        x = g0._embed(int(tokens[b]), n) if hidden_in is None else np.asarray(hidden_in[b], dtype=g0.real)
        for li in range(g0.Ls):
            L0 = g0.layers[li]
            a = g0._norm(x, L0["ln1_g"], L0["ln1_b"])
            y = np.zeros_like(x)
            for s in group:
                L = s.layers[li]
                q, k, v = s._qkv(L, a, n)
                s.kv[li, 0, b, :, n, :] = k                   # append (not yet committed)
                s.kv[li, 1, b, :, n, :] = v
                o = np.zeros((s.Hs, Dh), dtype=s.real)
                for h in range(s.Hs):
                    Kh = s.kv[li, 0, b, h, : n + 1, :]         # the new token attends to itself
                    Vh = s.kv[li, 1, b, h, : n + 1, :]
                    p = attention_probs(q[h], Kh)
                    o[h] = p @ Vh
                y = y + o.reshape(-1) @ L["wo"]
            if L0["bo"] is not None:
                y = y + L0["bo"]
            x = x + y
            a2 = g0._norm(x, L0["ln2_g"], L0["ln2_b"])
            z = np.zeros_like(x)
            for s in group:
                z = z + s._ffn_partial(s.layers[li], a2)
            if L0["b2"] is not None:
                z = z + L0["b2"]
            x = x + z
        if hidden_out:
            out[b] = x
        else:
            xf = g0._norm(x, g0.lnf_g, g0.lnf_b)
            out[b] = g0.lm_head @ xf
    for b in rows:                                              # token-level commit
        for s in group:
            s.n[b] += 1
    return out


def prefill(group, tokens, hidden_in=None, hidden_out=False):
    """The initial phase by definition: S_in incremental iterations from an empty cache,
    keeping the last logits.  tokens: [B, S_in].  Returns logits [B, V].

    As a pipeline stage: hidden_in [B, S_in, d] replaces the tokens, and with hidden_out
    the residual stream of every position after the shard's layers, [B, S_in, d], is
    returned instead of the logits."""
    S = np.asarray(tokens).shape[1] if hidden_in is None else np.asarray(hidden_in).shape[1]
    outs = []
    for t in range(S):
        outs.append(decode_step(group, None if hidden_in is not None else np.asarray(tokens)[:, t],
                                hidden_in=None if hidden_in is None else np.asarray(hidden_in)[:, t],
                                hidden_out=hidden_out))
    return np.stack(outs, axis=1) if hidden_out else outs[-1]


def forward_matrix(group, tokens_row, b=None, hidden_in=None, hidden_out=False):
    """Full causal recompute (the left-hand form, Eq. (1)) of one sequence from position 0:
    all S tokens at once with an explicit S x S score matrix masked above the diagonal.
    Returns the logits of every position, [S, V].  hidden_in [S, d] / hidden_out: the
    pipeline-stage forms of decode_step.

    With b given, also stores the keys/values as cache rows [0, S) of batch row b and
    sets n[b] = S (the initial phase in matrix form); the row must be empty before.
    """
    _check_group(group)
    g0 = group[0]
    desc = g0.desc
    Dh = desc["head_dim"]
    S = len(tokens_row) if hidden_in is None else len(hidden_in)
    if b is not None and int(g0.n[b]) != 0:
        raise RuntimeError("matrix-form prefill needs an empty row")
    pos = np.arange(S)
    if hidden_in is None:
        X = np.stack([g0._embed(int(t), int(p)) for t, p in zip(np.asarray(tokens_row), pos)])
    else:
        X = np.asarray(hidden_in, dtype=g0.real).copy()
    mask = np.where(pos[None, :] > pos[:, None], -np.inf, 0.0).astype(g0.real)   # [query, key]
    for li in range(g0.Ls):
        L0 = g0.layers[li]
        A = g0._norm(X, L0["ln1_g"], L0["ln1_b"])
        Y = np.zeros_like(X)
        for s in group:
            L = s.layers[li]
            Q, K, V = s._qkv(L, A, pos)                         # [S, Hs, Dh]
            if b is not None:
                s.kv[li, 0, b, :, :S, :] = K.transpose(1, 0, 2)
                s.kv[li, 1, b, :, :S, :] = V.transpose(1, 0, 2)
            O = np.zeros((S, s.Hs, Dh), dtype=s.real)
            for h in range(s.Hs):
                sc = (Q[:, h, :] @ K[:, h, :].T) / math.sqrt(Dh) + mask
                O[:, h, :] = softmax(sc) @ V[:, h, :]
            Y = Y + O.reshape(S, -1) @ L["wo"]
        if L0["bo"] is not None:
            Y = Y + L0["bo"]
        X = X + Y
        A2 = g0._norm(X, L0["ln2_g"], L0["ln2_b"])
        Z = np.zeros_like(X)
        for s in group:
            Z = Z + s._ffn_partial(s.layers[li], A2)
        if L0["b2"] is not None:
            Z = Z + L0["b2"]
        X = X + Z
    if b is not None:
        for s in group:
            s.n[b] = S
    if hidden_out:
        return X
    XF = g0._norm(X, g0.lnf_g, g0.lnf_b)
    return XF @ g0.lm_head.T


def prefill_matrix(group, tokens, rows=None):
    """Initial phase in matrix form for rows of tokens [B, S_in]; returns last-position logits [B, V]."""
    tokens = np.asarray(tokens)
    rows = range(tokens.shape[0]) if rows is None else rows
    out = np.zeros((tokens.shape[0], group[0].desc["vocab"]), dtype=group[0].real)
    for b in rows:
        out[b] = forward_matrix(group, tokens[b], b=b)[-1]
    return out


# ----------------------------------------------------------------------------
# KV-cache re-partition (cache-context migration on one device)
# ----------------------------------------------------------------------------
def kv_repack_arrays(dst_kv, dst_slice, src_kv, src_slice, src_n, batch_map):
    """The re-partition by its index formula, on bare arrays of any dtype.

    kv arrays are [L_s, 2, B, H_s, S_max, Dh] (their own L_s, B, H_s, S_max).  For every
    layer l in both layer intervals, c in {K, V}, every destination row b' with
    b = batch_map[b'] >= 0, every head g in both head intervals and every committed row
    j < src_n[b]:   dst[l - l0', c, b', g - h0', j, :] = src[l - l0, c, b, g - h0, j, :].
    Everything else in dst is left as it was.  Returns the number of elements copied.
    """
    l_lo, l_hi = max(dst_slice["layer_lo"], src_slice["layer_lo"]), min(dst_slice["layer_hi"], src_slice["layer_hi"])
    h_lo, h_hi = max(dst_slice["head_lo"], src_slice["head_lo"]), min(dst_slice["head_hi"], src_slice["head_hi"])
    moved = 0
    for l in range(l_lo, l_hi):
        for c in range(2):
            for bd, bs in enumerate(batch_map):
                if bs < 0:
                    continue
                n = int(src_n[bs])
                if n > dst_kv.shape[4]:
                    raise RuntimeError("destination cache too short")
                for g in range(h_lo, h_hi):
                    for j in range(n):
                        dst_kv[l - dst_slice["layer_lo"], c, bd, g - dst_slice["head_lo"], j, :] = \
                            src_kv[l - src_slice["layer_lo"], c, bs, g - src_slice["head_lo"], j, :]
                        moved += src_kv.shape[5]
    return moved


def kv_repack(dst, src, batch_map):
    """Move the intersection of src's cache context into dst (Section 3.3) for the kept
    rows and set dst's committed length of each mapped row to the source's."""
    moved = kv_repack_arrays(dst.kv, dst.slice, src.kv, src.slice, src.n, batch_map)
    for bd, bs in enumerate(batch_map):
        if bs >= 0:
            dst.n[bd] = src.n[bs]
    return moved


def kv_canonical(shard):
    """Committed cache rows in the exchange order [layer][K|V][b][head][j < n[b]][Dh], flat."""
    parts = []
    for l in range(shard.Ls):
        for c in range(2):
            for b in range(shard.max_batch):
                for h in range(shard.Hs):
                    parts.append(shard.kv[l, c, b, h, : int(shard.n[b]), :].reshape(-1))
    return np.concatenate(parts) if parts else np.zeros(0, dtype=shard.kv.dtype)
