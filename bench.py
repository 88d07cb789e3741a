#!/usr/bin/env python3
"""Benchmark of the decode hot path on one MI355X.

A step is one incremental decoding iteration of the whole batch through the shard (embedding,
every layer's QKV / attention + KV append / out-projection / FFN, LM head, greedy argmax,
token-level commit).  The timed region is exactly --steps iterations after a fresh initial
phase, replayed as a HIP graph, with every input already resident in HBM.

The headline (`value`, `roofline`, `cpu_baseline`) is the largest single-GPU configuration, the
LLaMA-30B-shaped shard; the GPT-20B- and OPT-66B-shaped shards run the same protocol in the
same process and are reported under `configs`, and the KV re-partition of the
reparallelize-and-resume configuration (1000 committed tokens, M=2 -> two M'=4 layouts) under
`repack`.  The initial phase is measured in the same run and reported beside each.

Prints ONE JSON line.  `roofline.achieved` = algorithmic bytes of the dominant kernel class (weights once for a GEMM,
committed cache rows once plus the new row for attention) divided by its launches' own durations.
"""
import argparse
import gc
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}
HEADLINE = "llama30b_m2"
OTHERS = ["gpt20b_m4", "opt66b_m8"]
KERNEL_OF_CLASS = {
    "qkv_gemm": ("stream_gemm_qkv", "stream_gemm<EPI_F32> (fused q|k|v projection)"),
    "decode_attn": ("decode_attn", "decode_attn (attention over the committed cache + append)"),
    "resid_gemm": ("stream_gemm_resid", "stream_gemm<EPI_RESID> (out-projection and second FFN matrix, residual epilogue)"),
    "ffn_up_gemm": ("stream_gemm_ffn_up", "stream_gemm<EPI_ACT / EPI_SWIGLU> (first FFN matrix + activation)"),
    "lm_head": ("stream_gemm_logits", "stream_gemm<EPI_LOGITS> (LM head + per-block greedy candidates)"),
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def shard_dims(w):
    d = w.desc
    s = w.slice
    return dict(Ls=s["layer_hi"] - s["layer_lo"], Hs=s["head_hi"] - s["head_lo"], Fs=s["ffn_hi"] - s["ffn_lo"],
                d=d["d_model"], Dh=d["head_dim"], V=d["vocab"], esz=2 if d["dtype"] == "bf16" else 4,
                c1=2 if d["act"] == "swiglu" else 1)


def algorithmic_bytes(w, n_list):
    """Bytes the method must move per decode step: every shard weight once (the batch shares
    it), the committed K/V rows plus the new one once, and the new row written."""
    g = shard_dims(w)
    HD = g["Hs"] * g["Dh"]
    per_layer = dict(qkv_gemm=g["d"] * 3 * HD * g["esz"], out_proj=HD * g["d"] * g["esz"],
                     ffn_up_gemm=g["c1"] * g["d"] * g["Fs"] * g["esz"], ffn_down=g["Fs"] * g["d"] * g["esz"])
    lm = g["V"] * g["d"] * g["esz"]
    kv_row = g["Ls"] * 2 * w.batch * HD * g["esz"]          # all layers, K and V, all batch rows, one position
    weights = g["Ls"] * sum(per_layer.values()) + lm
    steps = [weights + kv_row * (n + 1) + kv_row for n in n_list]
    classes = dict(qkv_gemm=g["Ls"] * per_layer["qkv_gemm"], ffn_up_gemm=g["Ls"] * per_layer["ffn_up_gemm"],
                   resid_gemm=g["Ls"] * (per_layer["out_proj"] + per_layer["ffn_down"]), lm_head=lm)
    attn = [kv_row * (n + 1) + kv_row for n in n_list]
    return steps, classes, attn, weights


def prefill_flops(w):
    g = shard_dims(w)
    HD = g["Hs"] * g["Dh"]
    T = w.batch * w.s_in
    per_tok = 2 * g["Ls"] * (g["d"] * 3 * HD + HD * g["d"] + (g["c1"] + 1) * g["d"] * g["Fs"])
    attn = g["Ls"] * w.batch * g["Hs"] * 4 * g["Dh"] * (w.s_in * (w.s_in + 1) // 2)
    return T * per_tok + attn + 2 * w.batch * g["V"] * g["d"]


def host_cpu():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count() or 1
    return model, os.cpu_count() or 1, usable


def cpu_baseline(w, W, n_ctx, budget_s=12.0):
    """The oracle as it stands, timed on this machine's host cores: full batch, decode iterations at
    context n_ctx (cache rows filled with noise; timing does not depend on values) until about
    budget_s seconds have gone by."""
    from oracle import decoder as D
    t0 = time.perf_counter()
    max_steps = 64
    ora = D.OracleShard(w.desc, w.slice, W, w.batch, n_ctx + max_steps + 2, real=np.float32)
    rng = np.random.default_rng(1)
    ora.kv[:, :, :, :, :n_ctx] = rng.standard_normal(size=ora.kv[:, :, :, :, :n_ctx].shape, dtype=np.float32) * 0.5
    ora.n[:] = n_ctx
    toks = rng.integers(0, w.desc["vocab"], size=w.batch)
    setup = time.perf_counter() - t0
    D.decode_step([ora], toks)                                # untimed first touch
    steps = 0
    t0 = time.perf_counter()
    while steps < max_steps - 1 and (steps < 2 or time.perf_counter() - t0 < budget_s):
        toks = D.greedy(D.decode_step([ora], toks))
        steps += 1
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    model, nproc, usable = host_cpu()
    return dict(value=w.batch * steps / dt, unit="tokens/s", cores=int(threads), kind="oracle", nproc=nproc,
                usable_cpus=usable, cpu_model=model,
                sample=f"{w.name}: full batch of {w.batch}, {steps} decode steps at context {n_ctx} (of {w.s_in}..{w.s_in + w.steps}), "
                       f"float32 numpy oracle, {dt:.1f} s timed (+{setup:.0f} s set-up)")


def measured_traffic(workload_name, kernel_key):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary (FETCH_SIZE and
    WRITE_SIZE, each scaled by what the counter reads for a plain copy of known size), or None."""
    path = os.path.join(ROOT, "profiles", f"decode_step_{workload_name}_hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) >= 3 and f[0] == "traffic_bytes_per_launch" and f[1] == kernel_key:
                return float(f[2])
    except OSError:
        pass
    return None


def run_workload(ss, torch, name, K, Wm, eager=False, extras=True, repack5=False, reslice=False, keep_weights=False,
                 cpu_repack=False):
    """Initial phase + K timed decode steps of one workload; returns (summary dict, (workload, host weights) or None)."""
    from synth import make_tokens, make_weights, sub_slice_of, workload
    w = workload(name)
    K = min(K, w.s_max - w.s_in)
    t0 = time.perf_counter()
    W = make_weights(w.desc, w.slice, w.seed)
    toks = make_tokens(w.seed, w.batch, w.s_in, w.desc["vocab"])
    log(f"[bench] {w.name}: weights drawn in {time.perf_counter() - t0:.1f} s")
    out = {}
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        t0 = time.perf_counter()
        sh = ss.Shard(w.desc, w.slice, W, w.batch, w.s_max)
        log(f"[bench] {w.name}: shard created ({sh.mem.numel() / 1e9:.2f} GB on device) in {time.perf_counter() - t0:.1f} s")
        sh.set_graph_launch(not eager)
        V = w.desc["vocab"]
        d_toks = torch.from_numpy(toks).cuda()
        logits = torch.empty(w.batch, V, dtype=torch.float32, device="cuda")
        nxt = torch.empty(w.batch, dtype=torch.int32, device="cuda")

        def fresh():
            sh.reset()
            ss.prefill([sh], d_toks, logits, nxt)

        # warm-up: initial phase + Wm decode steps, then start over
        fresh()
        for _ in range(Wm):
            ss.decode_step([sh], nxt, logits, nxt)
        torch.cuda.synchronize()
        sh.reset()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ss.prefill([sh], d_toks, logits, nxt)
        e1.record()
        torch.cuda.synchronize()
        prefill_ms = e0.elapsed_time(e1)

        # ---- the timed region: exactly K decode steps ----
        # (an event every `chunk` steps, for the cost model below: a marker in the stream, no wait)
        chunk = max(1, K // 8)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(K // chunk + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(K):
            ss.decode_step([sh], nxt, logits, nxt)
            if (i + 1) % chunk == 0:
                marks[(i + 1) // chunk].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        final_ids = nxt.cpu().numpy().copy()
        assert list(ss.committed_len(sh)) == [w.s_in + K] * w.batch

        n_list = [w.s_in + i for i in range(K)]
        step_bytes, class_bytes, attn_bytes, weight_bytes = algorithmic_bytes(w, n_list)
        g = shard_dims(w)
        out.update(value=w.batch * K / dt, ms_per_step=dt / K * 1e3, steps=K,
                   workload=f"{w.name}: {g['Ls']} layers, d={w.desc['d_model']}, {g['Hs']} heads x {w.desc['head_dim']}, "
                            f"FFN {g['Fs']}, vocab {V}, batch {w.batch}, prompt {w.s_in}, {K} decode steps",
                   batch=w.batch, prompt=w.s_in)
        whole = sum(step_bytes) / dt / 1e9
        out["step_hbm"] = dict(bytes_per_step=sum(step_bytes) / K, achieved=whole, peak=HBM_PEAK_GBPS, unit="GB/s",
                               frac=whole / HBM_PEAK_GBPS)
        out["roofline"] = dict(bound="hbm", kernel="whole decode step", achieved=whole, peak=HBM_PEAK_GBPS,
                               unit="GB/s", frac=whole / HBM_PEAK_GBPS, traffic=None)
        if extras:
            # ---- kernel classes: the same K steps again, kernel by kernel, each launch's own begin/end
            # recorded on a pair of HIP events of the stream it runs on ----
            fresh()
            torch.cuda.synchronize()
            sh.kernel_timing(True)
            for _ in range(K):
                ss.decode_step([sh], nxt, logits, nxt)
            tm = sh.kernel_timing_read()
            sh.kernel_timing(False)
            assert np.array_equal(nxt.cpu().numpy(), final_ids), "eager and graph runs disagree"
            classes, total_ms = {}, {}
            for cname, (ms, cnt) in tm.items():
                if cnt == 0:
                    continue
                if cname in class_bytes:
                    b = class_bytes[cname] * K
                elif cname == "decode_attn":
                    b = sum(attn_bytes)
                else:
                    b = 0
                classes[cname] = dict(launches=int(cnt), avg_us=ms / cnt * 1e3, GBps=(b / (ms * 1e-3) / 1e9) if b else None,
                                      share_of_step=ms / K / (dt / K * 1e3))
                if b:
                    total_ms[cname] = (ms, cnt, b)
            out["classes"] = classes
            # the roofline object is for the kernel class with the most time per step
            dom = max(total_ms, key=lambda c: total_ms[c][0])
            ms, cnt, b = total_ms[dom]
            ach = b / (ms * 1e-3) / 1e9
            key, label = KERNEL_OF_CLASS[dom]
            out["roofline"] = dict(bound="hbm", kernel=label, achieved=ach, peak=HBM_PEAK_GBPS, unit="GB/s",
                                   frac=ach / HBM_PEAK_GBPS, traffic=measured_traffic(w.name, key),
                                   bytes_per_launch=b / cnt, avg_launch_us=ms / cnt * 1e3, launches=int(cnt))
            fl = prefill_flops(w)
            peak = MFMA_PEAK_TFLOPS[w.desc["dtype"]]       # halves and bf16 share one matrix-core peak
            out["prefill"] = dict(ms=prefill_ms, tokens=w.batch * w.s_in, TFLOPs=fl / (prefill_ms * 1e-3) / 1e12,
                                  peak=peak, frac=fl / (prefill_ms * 1e-3) / 1e12 / peak)
            if w.desc["dtype"] == "bf16":
                # what the matrix cores of this chip sustain on random halves with the GEMM's LDS reads and loads beside them
                # and nothing else (no barrier, no epilogue): the clock under matrix-core load is set by power and power by
                # the data, so this, not `peak`, is what real operands can reach (see --calibrate-mfma)
                gen = torch.Generator(device="cuda").manual_seed(1)
                rnd = (torch.randn(4 << 20, generator=gen, device="cuda") * 0.5).to(torch.float16)
                ss.matrix_core_probe(rnd, True, True, 2000)
                t, c, ghz = ss.matrix_core_probe(rnd, True, True, 40000)
                out["prefill"]["sustainable_on_random_operands"] = dict(TFLOPs=t, GHz=ghz, cycles_per_64_products=c,
                                                                         frac=out["prefill"]["TFLOPs"] / t)
                del rnd

            # ---- measured cost model (Section 5; Eq. 1): iteration time over context length, from the timed steps ----
            if K // chunk >= 4:
                from paper_2311_15566_amd import plan as P
                samples = [(w.batch, w.s_in + i * chunk + chunk // 2, marks[i].elapsed_time(marks[i + 1]) / chunk)
                           for i in range(K // chunk)]
                cm = P.cost_fit(samples, [(w.batch, w.s_in, prefill_ms)])
                steps_fit = (K // chunk) * chunk
                l_exe = P.cost_l_exe(cm, w.batch, w.s_in, steps_fit)
                measured = prefill_ms + sum(ms * chunk for _, _, ms in samples)
                out["cost_model"] = dict(dec_base_ms=cm.dec_base_ms[0], dec_per_cached_token_us=cm.dec_per_row_ms[0] * 1e3,
                                         prefill_ms_per_token=cm.pre_per_token_ms[0], samples=len(samples),
                                         l_exe_ms=l_exe[-1], measured_ms=measured, s_in=w.s_in, s_out=steps_fit,
                                         note="least-squares line (slope not below 0) through the mean iteration time of each run of "
                                              f"{chunk} timed steps; l_exe = Eq. (1) from the fit, measured = the same steps timed")

        if repack5:
            # ---- KV re-partition at the reparallelize-and-resume configuration's size: this M=2 shard with 1000
            # committed tokens per sequence into the two M'=4 layouts (13 heads each) ----
            w5 = workload("llama30b_reparallelize")
            n5 = w5.s_in + w5.steps
            assert w5.desc == w.desc and w5.slice == w.slice and w5.batch == w.batch and n5 <= w.s_max
            sh.reset()
            ss.prefill([sh], d_toks[:, :n5].contiguous(), logits, nxt)
            parts = [ss.Shard(w.desc, s, W, w.batch, w5.s_max) for s in w5.extra["dst_slices"]]
            keep = list(range(w.batch))
            for p in parts:
                ss.kv_repack(p, sh, keep)                     # untimed first touch
            torch.cuda.synchronize()
            reps = 5
            e0.record()
            moved = 0
            for _ in range(reps):
                for p in parts:
                    moved += ss.kv_repack(p, sh, keep)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            traffic = 2 * moved / (ms * 1e-3) / 1e9
            out["repack"] = dict(workload=f"{w5.name}: {w.batch} sequences x {n5} committed tokens, {g['Ls']} layers, "
                                          f"{g['Hs']} heads -> 2 x {g['Hs'] // 2} heads",
                                 payload_bytes=moved // reps, ms=ms / reps, traffic_GBps=traffic,
                                 frac=traffic / HBM_PEAK_GBPS, rows=n5,
                                 note="traffic = bytes read + bytes written; payload = half")
            for p in parts:
                p.destroy()
            del parts
            if cpu_repack:
                # the oracle's re-partition (its index formula as it stands, one core) on a bounded sample of the
                # same move: one layer of it, the same 16 rows x 1000 tokens, 26 heads -> the first 13
                from oracle import decoder as D
                s_src, s_dst = dict(w.slice, layer_lo=0, layer_hi=1), dict(w5.extra["dst_slices"][0], layer_lo=0, layer_hi=1)
                src_kv = np.ones((1, 2, w.batch, g["Hs"], w5.s_max, g["Dh"]), dtype=np.uint16)
                dst_kv = np.zeros((1, 2, w.batch, g["Hs"] // 2, w5.s_max, g["Dh"]), dtype=np.uint16)
                t0 = time.time()
                elems = D.kv_repack_arrays(dst_kv, s_dst, src_kv, s_src, [n5] * w.batch, keep)
                dt_cpu = time.time() - t0
                out["repack"]["cpu_baseline"] = dict(traffic_GBps=2 * elems * 2 / dt_cpu / 1e9, cores=1, kind="oracle",
                                                     sample=f"one layer of the same move ({elems * 2 / 1e6:.0f} MB payload), "
                                                            f"{dt_cpu:.1f} s")
                del src_kv, dst_kv
        if reslice and g["Hs"] % 2 == 0 and g["Fs"] % 128 == 0:
            # ---- model-context re-slice: two half-width shards built out of the resident one ----
            half = sub_slice_of(w.slice, 0, 2)
            nb = ss.binding.device_bytes(w.desc, half, w.batch, w.s_max)
            mem = torch.zeros(nb, dtype=torch.uint8, device="cuda")
            ss.Shard.from_resident(w.desc, half, [sh], w.batch, w.s_max, mem=mem).destroy()     # untimed first touch
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            moved = 0
            for p in range(2):
                r = ss.Shard.from_resident(w.desc, sub_slice_of(w.slice, p, 2), [sh], w.batch, w.s_max, mem=mem)
                moved += r.bytes_copied
                r.destroy()
            dt_r = time.perf_counter() - t0
            out["reslice"] = dict(bytes_copied=moved // 2, ms=dt_r / 2 * 1e3, traffic_GBps=2 * moved / dt_r / 1e9,
                                  frac=2 * moved / dt_r / 1e9 / HBM_PEAK_GBPS,
                                  note="one half-width shard's model context copied out of the resident shard "
                                       "(wall time of the call, which synchronizes)")
            del mem
        sh.destroy()
        del sh, logits, nxt, d_toks
    torch.cuda.synchronize()
    gc.collect()
    torch.cuda.empty_cache()
    return out, ((w, W) if keep_weights else None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=128)
    ap.add_argument("--warmup", type=int, default=8)
    ap.add_argument("--workload", default=HEADLINE, choices=[HEADLINE] + OTHERS + ["tiny_gpt"],
                    help="the headline workload (default: the largest single-GPU configuration)")
    ap.add_argument("--only", action="store_true", help="run the headline workload only (no `configs`, no repack leg)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the kernel-class, prefill, cost-model, repack and re-slice legs")
    ap.add_argument("--eager", action="store_true", help="launch kernel by kernel instead of replaying a graph")
    ap.add_argument("--calibrate-mfma", action="store_true",
                    help="only measure what the matrix cores sustain on constant and on random operands (--steps thousand iterations each)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only copy 1 GiB device to device three times (a kernel of known traffic, for scaling "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs one tensor-parallel shard on ONE GPU; collectives and sharding "
                 "across GPUs are not part of it (run with --gpus 1)")

    import torch
    import paper_2311_15566_amd as ss

    assert torch.cuda.is_available(), "bench.py needs an MI355X"
    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps(dict(copy_bytes=1 << 30, copies=3)), flush=True)
        return
    if args.calibrate_mfma:
        # what the matrix cores sustain with nothing in their way, on constant operands and on random halves (the clock
        # under matrix-core load is set by power, and power by the data), alone and with the LDS reads and direct-to-LDS
        # loads of the initial phase's 256-row GEMM block: the ceiling that the `prefill` figure is to be read against
        g = torch.Generator(device="cuda").manual_seed(1)
        rnd = (torch.randn(4 << 20, generator=g, device="cuda") * 0.5).to(torch.float16)
        const = torch.full((4 << 20,), 0.75, dtype=torch.float16, device="cuda")
        rows = []
        for name, data in (("constant", const), ("random", rnd)):
            for lds_reads, loads in ((False, False), (True, False), (False, True), (True, True)):
                ss.matrix_core_probe(data, lds_reads, loads, 2000)
                t, c, ghz = ss.matrix_core_probe(data, lds_reads, loads, args.steps * 1000)
                rows.append(dict(operands=name, lds_reads=lds_reads, loads=loads, TFLOPs=t, cycles_per_64_products=c, GHz=ghz))
                log(f"[bench] matrix cores, {name} operands, LDS reads {lds_reads}, loads {loads}: {t:.0f} TFLOP/s, "
                    f"{c:.0f} cycles per 64 products, {ghz:.2f} GHz")
        print(json.dumps(dict(matrix_core_probe=rows, peak_TFLOPs=MFMA_PEAK_TFLOPS["bf16"])), flush=True)
        return
    K, Wm = args.steps, args.warmup
    extras = not args.no_extras
    is_llama = args.workload == HEADLINE
    head, kept = run_workload(ss, torch, args.workload, K, Wm, eager=args.eager, extras=extras,
                              repack5=extras and is_llama and not args.only, reslice=extras and not args.only,
                              keep_weights=not args.no_cpu_baseline, cpu_repack=not args.no_cpu_baseline)
    if head["steps"] != K:
        sys.exit(f"--steps {K} exceeds the workload's decode steps")
    out = dict(metric="decode tokens/s per TP shard on 1 GPU", value=head["value"], unit="tokens/s", n_gpus=1,
               steps=K, warmup=Wm, ms_per_step=head["ms_per_step"], higher_is_better=True, scaling="weak",
               vs_baseline=None, dtype="f16" if args.workload != "tiny_gpt" else "f32", data="synthetic",
               config=dict(workload=head["workload"], batch=head["batch"], prompt=head["prompt"],
                           launch="eager" if args.eager else "hip-graph"))
    for k in ("step_hbm", "classes", "roofline", "prefill", "cost_model", "repack", "reslice"):
        if k in head:
            out[k] = head[k]
    if not args.no_cpu_baseline:
        w, W = kept
        out["cpu_baseline"] = cpu_baseline(w, W, w.s_in + K // 2)
        del kept, W
        gc.collect()
    if not args.only and is_llama:
        out["configs"] = {}
        for name in OTHERS:
            r, _ = run_workload(ss, torch, name, K, Wm, eager=args.eager, extras=extras)
            r["tokens_per_s"] = r.pop("value")
            out["configs"][name] = r
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
