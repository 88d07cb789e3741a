"""Plain CPU implementation of the host-side planning steps around a change of parallel
configuration (SpotServe, Sections 3.3, 3.4 and 4.1).  Test infrastructure: only tests may
import it; it shares no code with the C++ planner.

Each function is the paper's definition or the steps of its algorithm written out: the
overlap as an intersection of explicit element sets, the device mapping as a search over all
permutations, the migration order as Algorithm 2's two passes.
"""
import itertools

import numpy as np


def _held(desc, tied, s):
    """Boolean mask, per tensor of the model, of the elements a position with slice s holds
    (Section 3.3: its stage's layers, its shard's heads and FFN columns; embedding, positions,
    final norm and LM head replicated).  Returns {name: (mask, bytes per element)}."""
    d, H, Dh, F, V = desc["d_model"], desc["n_heads"], desc["head_dim"], desc["ffn"], desc["vocab"]
    esz = 2 if desc["dtype"] == "bf16" else 4
    ln, glu, bias = desc["norm"] == "layernorm", desc["act"] == "swiglu", desc["has_bias"]
    out = {}
    cols_h = np.zeros(H * Dh, bool)
    cols_h[s["head_lo"] * Dh:s["head_hi"] * Dh] = True
    cols_f = np.zeros(F, bool)
    cols_f[s["ffn_lo"]:s["ffn_hi"]] = True
    for l in range(desc["n_layers"]):
        mine = s["layer_lo"] <= l < s["layer_hi"]
        for name in ("wq", "wk", "wv"):
            out[(name, l)] = (np.broadcast_to(cols_h[None, :] & mine, (d, H * Dh)), esz)
            if bias:
                out[("b" + name[1], l)] = (cols_h & mine, 4)
        out[("wo", l)] = (np.broadcast_to(cols_h[:, None] & mine, (H * Dh, d)), esz)
        for name in (("wg", "wu") if glu else ("w1",)):
            out[(name, l)] = (np.broadcast_to(cols_f[None, :] & mine, (d, F)), esz)
        if bias and not glu:
            out[("b1", l)] = (cols_f & mine, 4)
        out[("w2", l)] = (np.broadcast_to(cols_f[:, None] & mine, (F, d)), esz)
        vecs = ["ln1_g", "ln2_g"] + (["ln1_b", "ln2_b"] if ln else []) + (["bo", "b2"] if bias else [])
        for name in vecs:
            out[(name, l)] = (np.full(d, mine), 4)
    out["wte"] = (np.ones((V, d), bool), esz)
    if desc["pos"] == "learned":
        out["wpe"] = (np.ones((desc["max_pos"], d), bool), esz)
    if not tied:
        out["lm_head"] = (np.ones((V, d), bool), esz)
    out["lnf_g"] = (np.ones(d, bool), 4)
    if ln:
        out["lnf_b"] = (np.ones(d, bool), 4)
    return out


def context_overlap(desc, tied, a, b, kv_rows):
    """(model bytes, cache bytes) of the intersection of two positions' contexts."""
    A, B = _held(desc, tied, a), _held(desc, tied, b)
    model = sum(int((A[k][0] & B[k][0]).sum()) * A[k][1] for k in A)
    kvsz = 4 if desc.get("kv_dtype", "f16") == "f32" else 2
    layers = [l for l in range(desc["n_layers"]) if a["layer_lo"] <= l < a["layer_hi"] and b["layer_lo"] <= l < b["layer_hi"]]
    heads = [h for h in range(desc["n_heads"]) if a["head_lo"] <= h < a["head_hi"] and b["head_lo"] <= h < b["head_hi"]]
    cache = len(layers) * 2 * len(heads) * desc["head_dim"] * kvsz * kv_rows
    return model, cache


def match_devices(weight):
    """Maximum-weight perfect matching by trying every permutation (Section 3.3 states the
    problem; Kuhn-Munkres is only a faster way to the same optimum).  Returns (total, one
    optimal position_of list)."""
    w = np.asarray(weight)
    n = w.shape[0]
    best, best_p = -1, None
    for perm in itertools.permutations(range(n)):
        t = sum(int(w[u, perm[u]]) for u in range(n))
        if t > best:
            best, best_p = t, list(perm)
    return best, best_p


def migration_order(delta, u_max):
    """Algorithm 2, MemOptMigPlanner.  delta[l][i]: change of instance i's buffer memory when
    layer l's context migrates."""
    delta = np.asarray(delta, dtype=np.int64)
    L, N = delta.shape
    U = np.zeros(N, dtype=np.int64)
    O, X = [], []
    for i in range(L):                                   # sequential order of the layer index
        if (U + delta[i]).max() <= u_max:                # does not exceed U_max
            U = U + delta[i]
            O.append(i)
        else:
            X.append(i)
    while X:                                             # min-max over the layers left out
        x_opt = min(X, key=lambda x: ((U + delta[x]).max(), x))
        U = U + delta[x_opt]
        O.append(x_opt)
        X.remove(x_opt)
    return O


def progressive_plan(order, stage_of_layer):
    """Algorithm 2, MigrationPlanner: cache first, then the layers in the given order; a stage
    starts once all its layers are there."""
    plan = [("migrate_cache", -1)]
    arrived = set()
    for l in order:
        plan.append(("migrate_layer", l))
        arrived.add(l)
        p = stage_of_layer[l]
        if all(k in arrived for k in range(len(stage_of_layer)) if stage_of_layer[k] == p):
            plan.append(("start_stage", p))
    return plan


def rows_to_keep(lens, keep, n_dst):
    """Section 3.3: the requests with more decoding progress keep their cache."""
    rows = [r for r in range(len(lens)) if lens[r] > 0]
    rows.sort(key=lambda r: (-lens[r], r))
    rows = sorted(rows[:min(keep, n_dst)])
    return [rows[b] if b < len(rows) else -1 for b in range(n_dst)]


def jit_iterations(acquisition, l_exe, t_grace, t_mig):
    """Section 4.1: S_t for a preemption (largest S whose execution fits before migration must
    start) or an acquisition (smallest S that lasts until the new instance is ready); 0 when
    the migration would cost more than the arranged iterations."""
    s_out = len(l_exe) - 1
    if not acquisition:
        fits = [S for S in range(s_out + 1) if l_exe[S] < t_grace - t_mig]
        s = max(fits) if fits else 0
    else:
        lasts = [S for S in range(s_out + 1) if l_exe[S] >= t_grace]
        s = min(lasts) if lasts else s_out
    return s if t_mig < l_exe[s] else 0


def cost_fit(decode, prefill=()):
    """Section 5's cost model from measured samples (batch, length, ms): per batch size the
    least-squares line of an incremental iteration's time over the cached length and of the
    initial phase's time over the prompt length (numpy's polynomial fit).  Samples at a single
    length give a constant (decode) or a line through the origin (initial phase).  Eq. (1)'s
    t_exe cannot fall with the number of tokens it runs over (an iteration reads every cached
    row once more than the one before), and Section 4.1's argmax / argmin over S need l_exe
    non-decreasing: where noise tilts the fitted line downwards, the best line with a slope of
    at least zero is taken, which is the constant through the samples' mean."""
    model = {}
    for b in sorted({s[0] for s in decode}):
        def line(samples, through_origin):
            x = np.array([s[1] for s in samples if s[0] == b], dtype=np.float64)
            y = np.array([s[2] for s in samples if s[0] == b], dtype=np.float64)
            if len(x) == 0:
                return 0.0, 0.0
            if len(set(x.tolist())) > 1:
                c1, c0 = np.polyfit(x, y, 1)
                if c1 < 0:
                    return float(y.mean()), 0.0
                return float(c0), float(c1)
            return (0.0, float(y.mean() / x.mean())) if through_origin else (float(y.mean()), 0.0)
        model[b] = dict(dec=line(decode, False), pre=line(prefill, True))
    return model


def cost_l_exe(model, batch, s_in, s_out):
    """Eq. (1) as written: the initial phase, then one incremental iteration per output token,
    the i-th with s_in + i - 1 tokens cached; times of a batch size between two fitted ones are
    interpolated linearly, outside them the nearest is taken."""
    bs = sorted(model)

    def t(kind, x):
        vals = [model[b][kind][0] + model[b][kind][1] * x for b in bs]
        return float(np.interp(batch, bs, vals))
    out = [t("pre", s_in)]
    for i in range(1, s_out + 1):
        out.append(out[-1] + t("dec", s_in + i - 1))
    return out
