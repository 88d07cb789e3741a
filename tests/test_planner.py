"""Host-side planning (no GPU): the C++ planner against the oracle in oracle/planner.py, and the
oracle against what pins it: a library routine for the matching, the paper's worked example for
the overlap, closed forms and brute force for the rest."""
import itertools
import os

import numpy as np
import pytest

from oracle import planner as O
from paper_2311_15566_amd import plan as P
from synth import scaled_workload, tp_slice


def tiny_desc(name, **kw):
    base = dict(d_model=16, n_heads=4, head_dim=4, ffn=24, vocab=11, layers=6, M=1, batch=1, s_in=2, steps=1, dtype="bf16")
    base.update(kw)
    w = scaled_workload(name, **base)
    return w.desc


def position(desc, index, D_, P_, M_):
    m, p = index % M_, (index // M_) % P_
    return tp_slice(desc, p * desc["n_layers"] // P_, (p + 1) * desc["n_layers"] // P_, m, M_)


# ----------------------------------------------------------------------------
# context overlap
# ----------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny_gpt", "llama30b_m2", "opt66b_m8"])
@pytest.mark.parametrize("tied", [False, True])
def test_overlap_matches_the_element_set_definition(name, tied):
    desc = tiny_desc(name, dtype="bf16" if name != "tiny_gpt" else "f32")
    rng = np.random.default_rng(3)
    for _ in range(25):
        def rnd():
            l = sorted(rng.integers(0, 7, 2)); h = sorted(rng.integers(0, 5, 2)); f = sorted(rng.integers(0, 25, 2))
            return dict(layer_lo=int(l[0]), layer_hi=int(l[1]), head_lo=int(h[0]), head_hi=int(h[1]), ffn_lo=int(f[0]), ffn_hi=int(f[1]))
        a, b = rnd(), rnd()
        rows = int(rng.integers(0, 50))
        assert P.context_overlap(desc, tied, a, b, rows) == O.context_overlap(desc, tied, a, b, rows)


def test_oracle_overlap_closed_forms():
    desc = tiny_desc("llama30b_m2")                     # no biases, RMSNorm, SwiGLU, RoPE
    full = tp_slice(desc, 0, 6, 0, 1)
    d, H, Dh, F, V = 16, 4, 4, 24, 11
    per_layer = 2 * (4 * d * H * Dh + 3 * d * F) + 4 * 2 * d
    shared = 2 * (2 * V * d) + 4 * d
    assert O.context_overlap(desc, False, full, full, 7) == (6 * per_layer + shared, 6 * 2 * H * Dh * 2 * 7)
    # disjoint stages share only the replicated tensors and no cache
    assert O.context_overlap(desc, False, tp_slice(desc, 0, 3, 0, 1), tp_slice(desc, 3, 6, 0, 1), 7) == (shared, 0)
    # tensor shards of one stage share the replicated vectors of its layers
    a, b = tp_slice(desc, 0, 3, 0, 2), tp_slice(desc, 0, 3, 1, 2)
    assert O.context_overlap(desc, False, a, b, 7) == (shared + 3 * 4 * 2 * d, 0)


def test_device_mapping_example_of_the_paper():
    """tests/golden/device_mapping_example.txt through the planner: u_1's heaviest edges go to v_0
    and v_3, and with pipeline 0's requests inherited by new pipeline 0 the cache tips it to v_0."""
    cfg = {}
    for line in open(os.path.join(os.path.dirname(__file__), "golden", "device_mapping_example.txt")):
        f = line.split()
        if f and not f[0].startswith("#"):
            cfg[f[0]] = f[1:]
    cur = {k: int(v) for k, v in (t.split("=") for t in cfg["current"])}
    tgt = {k: int(v) for k, v in (t.split("=") for t in cfg["target"])}
    u = int(cfg["source"][0][1:])
    best = sorted(int(t[1:]) for t in cfg["best_targets"])
    desc = tiny_desc("tiny_gpt", dtype="f32")
    n_t = tgt["D"] * tgt["P"] * tgt["M"]
    ua = position(desc, u, cur["D"], cur["P"], cur["M"])
    for impl in (O, P):
        w = [impl.context_overlap(desc, True, ua, position(desc, v, tgt["D"], tgt["P"], tgt["M"]), 0)[0] for v in range(n_t)]
        assert sorted(v for v in range(n_t) if w[v] == max(w)) == best
        # new pipeline d' = v // (P * M) inherits old pipeline d = u // (P * M): only v_0..v_2 see u_1's cache
        wc = [sum(impl.context_overlap(desc, True, ua, position(desc, v, tgt["D"], tgt["P"], tgt["M"]),
                                       40 if v // (tgt["P"] * tgt["M"]) == u // (cur["P"] * cur["M"]) else 0)) for v in range(n_t)]
        assert [v for v in range(n_t) if wc[v] == max(wc)] == [0]


# ----------------------------------------------------------------------------
# matching
# ----------------------------------------------------------------------------
def test_oracle_matching_against_the_library_routine():
    from scipy.optimize import linear_sum_assignment
    rng = np.random.default_rng(5)
    for n in range(1, 8):
        for _ in range(6):
            w = rng.integers(0, 1000, size=(n, n))
            total, perm = O.match_devices(w)
            r, c = linear_sum_assignment(w, maximize=True)
            assert total == int(w[r, c].sum())
            assert sorted(perm) == list(range(n)) and total == sum(int(w[u, perm[u]]) for u in range(n))


@pytest.mark.parametrize("n", [1, 2, 3, 5, 7, 8])
def test_matching_reaches_the_brute_force_optimum(n):
    rng = np.random.default_rng(100 + n)
    for trial in range(12):
        hi = 4 if trial % 3 == 0 else 10 ** 12            # many ties / large byte counts
        w = rng.integers(0, hi, size=(n, n)).astype(np.uint64)
        total, pos = P.match_devices(w)
        assert sorted(pos) == list(range(n))
        assert total == sum(int(w[u, pos[u]]) for u in range(n)) == O.match_devices(w)[0]


def test_matching_on_overlap_weights_of_a_real_change():
    """(D,P,M) = (1,2,2) -> (1,1,4) on 4 devices: the matching keeps every device on heads it already holds."""
    desc = tiny_desc("tiny_gpt", dtype="f32", layers=4, n_heads=8, head_dim=2)
    old = [position(desc, u, 1, 2, 2) for u in range(4)]
    new = [position(desc, v, 1, 1, 4) for v in range(4)]
    w = np.array([[sum(P.context_overlap(desc, True, a, b, 30)) for b in new] for a in old], dtype=np.uint64)
    total, pos = P.match_devices(w)
    assert total == O.match_devices(w)[0]
    for u, v in enumerate(pos):
        a, b = old[u], new[v]
        assert a["head_lo"] <= b["head_lo"] and b["head_hi"] <= a["head_hi"]
    big = np.random.default_rng(9).integers(0, 10 ** 9, size=(200, 200)).astype(np.uint64)
    from scipy.optimize import linear_sum_assignment
    r, c = linear_sum_assignment(big.astype(np.int64), maximize=True)
    assert P.match_devices(big)[0] == int(big[r, c].sum())


# ----------------------------------------------------------------------------
# migration order and plan
# ----------------------------------------------------------------------------
def test_migration_order_matches_the_algorithm_and_its_properties():
    rng = np.random.default_rng(21)
    for trial in range(60):
        L, N = int(rng.integers(1, 9)), int(rng.integers(1, 5))
        delta = rng.integers(-50, 80, size=(L, N))
        u_max = int(rng.integers(0, 200))
        got = P.migration_order(delta, u_max)
        assert got == O.migration_order(delta, u_max)
        assert sorted(got) == list(range(L))
    # no memory pressure: the plain sequential order
    delta = rng.integers(0, 10, size=(7, 3))
    assert O.migration_order(delta, 10 ** 9) == list(range(7)) == P.migration_order(delta, 10 ** 9)
    # the first pass never exceeds the bound
    delta = np.array([[60, 0], [50, 0], [-40, 10], [30, 30], [-30, -30]])
    order = O.migration_order(delta, 70)
    U, first_pass = np.zeros(2, dtype=int), []
    for l in range(5):
        if (U + delta[l]).max() <= 70:
            U += delta[l]; first_pass.append(l)
    assert order[:len(first_pass)] == first_pass == [0, 2, 3, 4] and order[len(first_pass):] == [1]


def test_min_max_pass_is_greedy_optimal_at_every_pick():
    """Each pick of the second pass minimises the peak over the instances among the layers left."""
    rng = np.random.default_rng(22)
    for _ in range(30):
        L, N = 6, 3
        delta = rng.integers(10, 60, size=(L, N))
        order = P.migration_order(delta, -1)                 # nothing fits: all layers go to the second pass
        U = np.zeros(N, dtype=int)
        left = set(range(L))
        for l in order:
            peak = (U + delta[l]).max()
            assert peak == min((U + delta[x]).max() for x in left)
            U += delta[l]; left.remove(l)


def test_progressive_plan():
    stage = [0, 0, 1, 1, 2, 2]
    for order in ([0, 1, 2, 3, 4, 5], [4, 0, 5, 2, 1, 3]):
        got = P.progressive_plan(order, stage)
        assert got == O.progressive_plan(order, stage)
        assert got[0] == ("migrate_cache", -1)
        assert [a for k, a in got if k == "migrate_layer"] == order
        for p in range(3):                                  # a stage starts right after its last layer
            i = got.index(("start_stage", p))
            assert got[i - 1][0] == "migrate_layer" and stage[got[i - 1][1]] == p
            assert all(stage[a] != p for k, a in got[i:] if k == "migrate_layer")
    assert P.progressive_plan([0, 1, 2, 3, 4, 5], stage)[-1] == ("start_stage", 2)


# ----------------------------------------------------------------------------
# cache discard, just-in-time arrangement
# ----------------------------------------------------------------------------
def test_rows_to_keep():
    assert O.rows_to_keep([5, 0, 9, 9, 2], 3, 4) == [0, 2, 3, -1] == P.rows_to_keep([5, 0, 9, 9, 2], 3, 4)
    assert O.rows_to_keep([5, 0, 9, 9, 2], 2, 2) == [2, 3] == P.rows_to_keep([5, 0, 9, 9, 2], 2, 2)
    rng = np.random.default_rng(31)
    for _ in range(50):
        lens = [int(v) for v in rng.integers(0, 6, size=int(rng.integers(0, 9)))]
        keep, n_dst = int(rng.integers(0, 9)), int(rng.integers(0, 9))
        got = P.rows_to_keep(lens, keep, n_dst)
        assert got == O.rows_to_keep(lens, keep, n_dst)
        kept = [r for r in got if r >= 0]
        assert kept == sorted(kept) and len(kept) == min(keep, n_dst, sum(v > 0 for v in lens))
        assert all(lens[r] >= lens[q] for r in kept for q in range(len(lens)) if q not in kept)


def test_jit_iterations():
    l_exe = [0.0] + [0.5 + 0.1 * s for s in range(1, 129)]          # initial phase + 0.1 s per token
    # preemption: 30 s grace, 5 s migration -> the largest S with l_exe < 25
    s = O.jit_iterations(False, l_exe, 30.0, 5.0)
    assert l_exe[s] < 25.0 and (s == 128 or l_exe[s + 1] >= 25.0) and s == P.jit_iterations(False, l_exe, 30.0, 5.0)
    # too little time left to be worth a migration: re-route (0)
    assert O.jit_iterations(False, l_exe, 5.4, 5.0) == 0 == P.jit_iterations(False, l_exe, 5.4, 5.0)
    # acquisition: the smallest S that lasts until the new instance is up
    s = O.jit_iterations(True, l_exe, 6.0, 1.0)
    assert l_exe[s] >= 6.0 and l_exe[s - 1] < 6.0 and s == P.jit_iterations(True, l_exe, 6.0, 1.0)
    rng = np.random.default_rng(41)
    for _ in range(200):
        n = int(rng.integers(1, 20))
        t = np.concatenate([[0.0], np.cumsum(rng.uniform(0.01, 1.0, size=n))])
        args = (bool(rng.integers(0, 2)), list(t), float(rng.uniform(0, 12)), float(rng.uniform(0, 3)))
        assert P.jit_iterations(*args) == O.jit_iterations(*args)


# ----------------------------------------------------------------------------
# measured cost model (Section 5) and Eq. (1) / Eq. (2)
# ----------------------------------------------------------------------------
def test_cost_model_pins():
    """The oracle against what the mathematics fixes: exact data is recovered, Eq. (1) summed in
    closed form, Eq. (2) as the special case of a constant iteration time."""
    dec = [(8, n, 0.8 + 2e-4 * n) for n in (512, 544, 576, 640)] + [(16, n, 1.1 + 3e-4 * n) for n in (100, 900)]
    pre = [(8, 512, 28.0), (16, 256, 20.0), (16, 1024, 92.0)]
    m = O.cost_fit(dec, pre)
    assert np.allclose(m[8]["dec"], (0.8, 2e-4)) and np.allclose(m[16]["dec"], (1.1, 3e-4))
    assert np.allclose(m[8]["pre"], (0.0, 28.0 / 512))                       # one length: through the origin
    assert np.allclose(m[16]["pre"], (20.0 - 256 * (72.0 / 768), 72.0 / 768))
    # Eq. (1): arithmetic series in closed form
    l = O.cost_l_exe(m, 8, 512, 128)
    assert len(l) == 129 and np.isclose(l[0], 28.0)
    assert np.isclose(l[128], 28.0 + 128 * 0.8 + 2e-4 * (128 * 512 + 127 * 128 / 2))
    assert all(b > a for a, b in zip(l, l[1:]))
    # Eq. (2): a constant per-iteration time gives t_exe(S_in) + S_out * t_exe(1)
    flat = O.cost_fit([(4, 300, 0.5)], [(4, 300, 9.0)])
    assert np.allclose(O.cost_l_exe(flat, 4, 300, 40), [9.0 + 0.5 * s for s in range(41)])
    # a batch size half-way between two fitted ones costs the mean of their times; outside: the nearest
    l12 = O.cost_l_exe(m, 12, 256, 10)
    l8, l16 = O.cost_l_exe(m, 8, 256, 10), O.cost_l_exe(m, 16, 256, 10)
    assert np.allclose(l12, [(a + b) / 2 for a, b in zip(l8, l16)])
    assert np.allclose(O.cost_l_exe(m, 64, 256, 10), l16) and np.allclose(O.cost_l_exe(m, 1, 256, 10), l8)
    # noisy samples: the fit is the least-squares line (normal equations written out)
    rng = np.random.default_rng(5)
    x = rng.integers(1, 2000, size=30)
    y = 0.7 + 1e-4 * x + rng.normal(0, 0.01, size=30)
    A = np.stack([np.ones(30), x.astype(np.float64)], axis=1)
    c0, c1 = np.linalg.solve(A.T @ A, A.T @ y)
    assert np.allclose(O.cost_fit([(2, int(a), float(b)) for a, b in zip(x, y)])[2]["dec"], (c0, c1))
    # samples that noise tilts downwards: the best line whose slope is not negative (found here by a scan over
    # slopes >= 0, each with its best intercept) is the constant through the mean, and Eq. (1)'s table stays monotone
    xd, yd = np.array([512.0, 514, 516, 518, 520]), np.array([1.10, 1.13, 1.09, 1.08, 1.07])
    sse = lambda c1: float(((yd - (yd.mean() - c1 * xd.mean()) - c1 * xd) ** 2).sum())
    best = min(np.linspace(0.0, 0.02, 2001), key=sse)
    down = O.cost_fit([(8, int(a), float(b)) for a, b in zip(xd, yd)])
    assert best == 0.0 and np.allclose(down[8]["dec"], (yd.mean(), 0.0))
    assert np.polyfit(xd, yd, 1)[0] < 0                                       # the unconstrained fit would fall
    ld = O.cost_l_exe(down, 8, 512, 64)
    assert all(b >= a for a, b in zip(ld, ld[1:]))


def test_cost_model_matches_oracle():
    rng = np.random.default_rng(77)
    for case in range(40):
        batches = sorted(set(int(b) for b in rng.integers(1, 40, size=int(rng.integers(1, 5)))))
        dec, pre = [], []
        for b in batches:
            for _ in range(int(rng.integers(1, 6))):
                dec.append((b, int(rng.integers(0, 3000)), float(rng.uniform(0.2, 5.0))))
            for _ in range(int(rng.integers(0, 4))):
                pre.append((b, int(rng.integers(1, 2049)), float(rng.uniform(1.0, 200.0))))
        mo, mc = O.cost_fit(dec, pre), P.cost_fit(dec, pre)
        assert mc.n_batches == len(batches) and list(mc.batch[:mc.n_batches]) == batches
        for i, b in enumerate(batches):
            assert np.allclose((mc.dec_base_ms[i], mc.dec_per_row_ms[i]), mo[b]["dec"], rtol=1e-9, atol=1e-9)
            assert np.allclose((mc.pre_base_ms[i], mc.pre_per_token_ms[i]), mo[b]["pre"], rtol=1e-9, atol=1e-9)
        for _ in range(5):
            b, s_in, s_out = int(rng.integers(1, 50)), int(rng.integers(1, 1500)), int(rng.integers(0, 200))
            assert np.allclose(P.cost_l_exe(mc, b, s_in, s_out), O.cost_l_exe(mo, b, s_in, s_out), rtol=1e-9, atol=1e-9)
    # the table feeds the just-in-time arrangement
    m = P.cost_fit([(8, 512, 0.9), (8, 640, 0.92)], [(8, 512, 27.0)])
    l = P.cost_l_exe(m, 8, 512, 128)
    assert P.jit_iterations(False, l, 100.0, 20.0) == O.jit_iterations(False, l, 100.0, 20.0) > 0
    with pytest.raises(Exception):
        P.cost_fit([], [])
    with pytest.raises(Exception):
        P.cost_fit([(8, 10, 1.0)], [(4, 10, 1.0)])               # initial-phase sample of a batch size without decode samples
