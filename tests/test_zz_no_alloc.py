"""The decode step that allocates nothing (ss_decode_step_static: the step's scratch in the library's
static device array) against ss_decode_step, through the C ABI: same logits, tokens and cache rows,
bit for bit, on two calls in a row, the second with a smaller batch; and against the CPU oracle."""
import numpy as np
import pytest

from oracle import decoder as D
from synth import make_tokens, make_weights, scaled_workload, tp_slice

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ss():
    import torch
    assert torch.cuda.is_available()
    import paper_2311_15566_amd as lib
    return lib


def bits(a):
    return a.view(np.uint16) if a.dtype.itemsize == 2 else a.view(np.uint32)


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


@pytest.mark.parametrize("name,dtype,group_m,batch,slices", [("llama30b_m2", "bf16", 1, 6, 0), ("gpt20b_m4", "bf16", 2, 6, 0),
                                                             ("tiny_gpt", "f32", 1, 6, 0),
                                                             # more than 16 rows, no gate: the first FFN matrix in K slices, its
                                                             # partial products in the static array too
                                                             ("opt66b_m8", "bf16", 1, 20, 2)])
def test_static_scratch_step_matches_the_allocating_one(ss, name, dtype, group_m, batch, slices):
    try:
        ss.force_gemm_shape(0, slices)
        _static_against_allocating(ss, name, dtype, group_m, batch)
    finally:
        ss.force_gemm_shape(0, 0)


def _static_against_allocating(ss, name, dtype, group_m, batch):
    import torch
    w = scaled_workload(name, d_model=512, n_heads=4, head_dim=128, ffn=1152, vocab=1511, layers=3, M=1, m=0,
                        batch=batch, s_in=45, steps=4, dtype=dtype)
    desc, B, V = w.desc, w.batch, w.desc["vocab"]
    full = tp_slice(desc, 0, 3, 0, 1)
    W = make_weights(desc, full, w.seed)
    toks = make_tokens(w.seed, B, w.s_in, V)
    forced = make_tokens(w.seed + 3, B, 2, V)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        ora = D.OracleShard(desc, full, W, B, w.s_max)
        D.prefill_matrix([ora], toks)
        # two copies of the same group: one takes ss_decode_step, the other ss_decode_step_static
        groups = [[ss.Shard(desc, tp_slice(desc, 0, 3, m, group_m), W, B, w.s_max) for m in range(group_m)] for _ in range(2)]
        outs = []
        for g, step_fn in zip(groups, (ss.decode_step, ss.decode_step_static)):
            logits = torch.full((B, V), 7.0, dtype=torch.float32, device="cuda")
            nxt = torch.full((B,), -1, dtype=torch.int32, device="cuda")
            ss.prefill(g, dev(toks), None, None)
            run = []
            # first call: the whole batch; second call: a smaller batch (rows 0..2 go on, the others stay)
            for call, rows in enumerate((B, 3)):
                logits.fill_(7.0)
                step_fn(g, dev(forced[:rows, call]), logits[:rows], nxt[:rows])
                torch.cuda.synchronize()
                run.append(logits.cpu().numpy().copy())
                run.append(nxt.cpu().numpy().copy())
            run += [ss.kv_export(sh) for sh in g]
            run.append(np.array([list(ss.committed_len(sh)) for sh in g]))
            outs.append(run)
        for x, y in zip(*outs):
            assert np.array_equal(x if x.dtype.kind == "i" else bits(x), y if y.dtype.kind == "i" else bits(y))
        assert outs[1][-1].tolist() == [[w.s_in + 2] * 3 + [w.s_in + 1] * (B - 3)] * group_m
        # and the static path against the oracle (the allocating path's parity is tested elsewhere)
        ref = D.decode_step([ora], forced[:, 0])
        got = outs[1][0]
        bf16 = dtype == "bf16"
        err = np.abs(got - ref).max()
        rel = np.linalg.norm(got - ref) / np.linalg.norm(ref)
        assert (err < 5e-2 and rel < 1e-2) if bf16 else (err < 1e-4 and rel < 1e-5), (err, rel)
        ref2 = D.decode_step([ora], forced[:3, 1], rows=range(3))
        err2 = np.abs(outs[1][2][:3] - ref2[:3]).max()
        assert err2 < (5e-2 if bf16 else 1e-4), err2
        assert np.all(outs[1][2][3:] == 7.0)                       # rows outside the smaller batch are not written
        for g in groups:
            for sh in g:
                sh.destroy()
    torch.cuda.synchronize()


def test_static_scratch_refuses_what_does_not_fit(ss):
    """A group whose decode step needs more scratch than the static array holds is refused on the
    host, with the sizes in the message, and nothing is launched or committed."""
    import torch
    w = scaled_workload("llama30b_m2", d_model=256, n_heads=96, head_dim=128, ffn=128, vocab=777, layers=1, M=1, m=0,
                        batch=2, s_in=8, steps=2, dtype="bf16")
    W = make_weights(w.desc, w.slice, w.seed)
    sh = ss.Shard(w.desc, w.slice, W, w.batch, w.s_max)
    toks = make_tokens(w.seed, w.batch, w.s_in, w.desc["vocab"])
    ss.prefill([sh], dev(toks), None, None)
    assert ss.static_scratch_bytes() == 32 << 20
    with pytest.raises(ss.SpotShardError) as e:
        ss.decode_step_static([sh], dev(toks[:, 0]), None, None)
    assert e.value.status == 2 and "static array holds" in str(e.value)
    assert list(ss.committed_len(sh)) == [w.s_in] * w.batch
    ss.decode_step([sh], dev(toks[:, 0]), None, None)             # the allocating entry point takes it
    assert list(ss.committed_len(sh)) == [w.s_in + 1] * w.batch
    sh.destroy()
