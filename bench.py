#!/usr/bin/env python3
"""Throughput of the verify step on one MI355X.

A "step" is one pass of the whole hot path (embedding gather, 32 decoder layers, final norm,
256-bin LM-head slice, argmax, relaxed acceptance) over one batch of seeded synthetic input,
with every input already resident in HBM when the timed region starts.

Prints ONE JSON line: verify steps/s at the headline workload (C1: 7B-shaped decoder, K=7,
batch 1, 276-token prefix), plus a `roofline` object for the dominant kernel (event-timed on
the launch stream inside the library) and a `cpu_baseline` object (the CPU oracle as it
stands, timed on this machine's host cores).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK = 8.0e12  # bytes/s, MI355X published


def algorithmic_bytes(sh, batch, K, P, active=None):
    """Bytes a step must move at least once: weights once, prefix K/V once per verified episode,
    new K/V rows written.  Activations, partial sums and logits are implementation traffic."""
    act = batch if active is None else active
    d, f, L = sh.d_model, sh.d_ffn, sh.n_layers
    per_class = {
        "qkv": 3 * d * d * 2,
        "oproj": d * d * 2,
        "gateup": 2 * d * f * 2,
        "down": d * f * 2,
        "attn": act * (2 * P * d * 2 + 2 * K * d * 2),
        "lmhead": sh.n_bins * d * 2,
        "embed": act * K * d * 2,
    }
    total = L * (per_class["qkv"] + per_class["oproj"] + per_class["gateup"] + per_class["down"] +
                 per_class["attn"]) + per_class["lmhead"] + per_class["embed"]
    per_class["persist"] = total          # the persistent kernel is the whole decoder forward
    return total, per_class


def read_traffic(kclass):
    """(HBM traffic per launch of a kernel class, where that figure comes from), if a counter summary under
    profiles/ states it.  The figure is NOT measured in this run: hardware counters need rocprofv3 around
    the process, so it is read back from the committed summary of such a run."""
    pdir = os.path.join(ROOT, "profiles")
    if not os.path.isdir(pdir):
        return None, None
    for fn in sorted(os.listdir(pdir)):
        if not fn.endswith((".md", ".txt")):
            continue
        text = open(os.path.join(pdir, fn)).read()
        m = re.search(r"^traffic_bytes_per_launch\[%s\]:\s*([0-9.eE+]+)" % kclass, text, flags=re.M)
        if m:
            when = re.search(r"^recorded:\s*(.+)$", text, flags=re.M)
            return float(m.group(1)), "profiles/%s (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of bench.py, %s; " \
                                      "not measured in this run)" % (fn, when.group(1).strip() if when else "date not stated")
    return None, None


def run_readbw_mode(args):
    """--mode readbw: what a kernel that only reads reaches on this chip with the access patterns of the
    weight-streaming GEMMs (heisd_measure_read), and what an empty launch costs - the reference points of
    the roofline accounting.  Every launch reads a different window of a 6 GiB buffer, sized like the
    projection it stands for, so that nothing is served from the memory-side cache."""
    import torch
    from paper_2603_17573_amd import heisd_measure_read, heisd_measure_empty_launch, binding
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    pool = torch.empty(6 << 30, dtype=torch.uint8, device=dev)
    pool.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(16, dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream(dev).cuda_stream
    reps = max(args.steps, 5)

    def timed(win, pattern, ksteps, in_flight, wgs):
        n_win = pool.numel() // win
        def launch(r):
            rc = heisd_measure_read(pool.data_ptr() + (r % n_win) * win, win, pattern, ksteps, in_flight, wgs,
                                    sink.data_ptr(), stream)
            assert rc == 0, binding.heisd_last_error(None)
        for r in range(3):
            launch(r)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            launch(3 + r)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps            # us per launch, launch overhead included

    d, f = 4096, 11008
    shapes = {"gateup": (2 * f * d * 2, d // 32), "qkv": (3 * d * d * 2, d // 32), "oproj": (d * d * 2, d // 32),
              "down": (d * f * 2, f // 32)}
    rows = []
    for wgs in (128, 176, 256, 512, 1024):
        for infl in (8, 16):
            win = shapes["gateup"][0]
            us = timed(win, 0, 0, infl, wgs)
            waves = wgs * 8
            read = (win // 16 // waves // (64 * infl)) * (64 * infl) * waves * 16     # whole rounds per wave only
            rows.append({"pattern": "contiguous per wave", "window": "gateup (180 MB)", "in_flight_KB_per_wave": infl,
                         "workgroups": wgs, "bytes_read": read, "us": round(us, 2), "GBps": round(read / us / 1e3, 1)})
    for name, (win, ks) in shapes.items():
        for infl in (8, 16):
            us = timed(win, 1, ks, infl, 256)
            rows.append({"pattern": "fragment-ordered tiles", "window": "%s (%.1f MB, %d KB tiles)" % (name, win / 1e6, ks),
                         "in_flight_KB_per_wave": infl, "workgroups": 256, "bytes_read": win // (ks * 1024) * ks * 1024,
                         "us": round(us, 2), "GBps": round(win / us / 1e3, 1)})
    for r in range(20):
        heisd_measure_empty_launch(256, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for r in range(500):
        heisd_measure_empty_launch(256, stream)
    e1.record()
    torch.cuda.synchronize()
    empty_us = e0.elapsed_time(e1) * 1e3 / 500
    best = max(r["GBps"] for r in rows)
    print(json.dumps({"metric": "HBM read bandwidth of a read-only kernel (reference for the weight-streaming GEMMs)",
                      "value": best, "unit": "GB/s", "n_gpus": 1, "steps": reps, "higher_is_better": True,
                      "peak": HBM_PEAK / 1e9, "frac_of_peak": round(best * 1e9 / HBM_PEAK, 4),
                      "empty_launch_us": round(empty_us, 3), "data": "synthetic", "rows": rows}))


def run_aux_mode(args):
    """--mode decode: the autoregressive decode step (Eq. 2-1; the fallback of Sec. 4.2 and the baseline
    speculative decoding replaces): one new token per episode through heisd_prefill_chunk.
    --mode prefill: the workload's whole prefix from an empty cache in one chunk, visual rows as
    embeddings and prompt rows as token ids in the same call (--prefill-chunks 2: the visual rows as one
    chunk, the prompt ids as a second: two passes over the weights).  Same JSON schema as the verify line."""
    import numpy as np
    import torch
    import synth
    from paper_2603_17573_amd import (DeviceModel, Verifier, binding, heisd_verify_profile_enable,
                                      heisd_verify_profile_read, heisd_verify_set_path)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = synth.WORKLOADS[args.workload]
    sh = wl.shape
    B, P = wl.batch, wl.prefix_len
    decode = args.mode == "decode"
    one_chunk = not decode and args.prefill_chunks == 1 and wl.n_visual and wl.n_text
    chunks = [1] if decode else ([P] if one_chunk else [c for c in (wl.n_visual, wl.n_text) if c])
    cap = P + 1
    weights = synth.make_weights(sh, wl.seed)
    ver = Verifier(DeviceModel(sh, weights, dev), B, max(chunks), cap)
    assert heisd_verify_set_path(ver.ctx, args.path) == 0
    if args.act_bf16:
        from paper_2603_17573_amd import heisd_verify_set_activations, HEISD_ACT_BF16
        assert heisd_verify_set_activations(ver.ctx, HEISD_ACT_BF16) == 0
    kc, vc = ver.new_cache(B)
    stream = torch.cuda.current_stream(dev)
    calls = []                                   # (prefix_len tensor, keyword arguments) per call of one step
    if decode:
        first = np.zeros(B, np.int32)
        for e in range(B):
            k, v, f = synth.make_prefix_kv_direct(wl, e, cap)
            kc[:, e] = torch.from_numpy(k.view(np.int16)).to(dev).view(torch.bfloat16)
            vc[:, e] = torch.from_numpy(v.view(np.int16)).to(dev).view(torch.bfloat16)
            first[e] = f
        ids = torch.from_numpy((sh.bin_base + first).astype(np.int32)[:, None]).to(dev).contiguous()
        calls.append((torch.full((B,), P, dtype=torch.int32, device=dev), {"token_ids": ids}))
    else:
        inputs = [synth.make_prefix_inputs(wl, e) for e in range(B)]
        if one_chunk:
            x = np.zeros((B, P, sh.d_model), np.float32)
            t = np.full((B, P), -1, np.int32)                 # -1: the row takes its embedding
            for e, (emb, ids) in enumerate(inputs):
                x[e, :wl.n_visual] = emb
                t[e, wl.n_visual:] = ids
            calls.append((torch.zeros(B, dtype=torch.int32, device=dev),
                          {"x_rows": torch.from_numpy(x).to(dev), "token_ids": torch.from_numpy(t).to(dev)}))
        elif wl.n_visual:
            x = np.stack([emb for emb, _ in inputs]).astype(np.float32)
            calls.append((torch.zeros(B, dtype=torch.int32, device=dev), {"x_rows": torch.from_numpy(x).to(dev)}))
        if wl.n_text and not one_chunk:
            t = np.stack([ids for _, ids in inputs]).astype(np.int32)
            calls.append((torch.full((B,), wl.n_visual, dtype=torch.int32, device=dev),
                          {"token_ids": torch.from_numpy(t).to(dev)}))
    outs = [None] * len(calls)

    def step():
        for i, (pl, kw) in enumerate(calls):
            outs[i] = ver.prefill_chunk(kc, vc, pl, out=outs[i], stream=stream, **kw)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    n_prof = max(1, min(args.steps, 16))
    heisd_verify_profile_enable(ver.ctx, True)
    for _ in range(n_prof):
        step()
    rc, prof = heisd_verify_profile_read(ver.ctx)
    heisd_verify_profile_enable(ver.ctx, False)
    assert rc == 0
    kernels = {k: {"avg_us": round(t / n * 1e3, 3), "launches_per_step": n / n_prof,
                   "share_of_step": round(t / n_prof / ms, 4)} for k, (t, n) in prof.items() if n}
    d, f, L = sh.d_model, sh.d_ffn, sh.n_layers
    gemm_flops_per_row = 2.0 * (L * (4 * d * d + 3 * d * f) + sh.n_bins * d)
    if decode:
        total_bytes, per_class = algorithmic_bytes(sh, B, 1, P)
        dom = max((k for k in kernels if k in per_class), key=lambda k: prof[k][0])
        dom_s = prof[dom][0] / prof[dom][1] * 1e-3
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(per_class[dom] / dom_s / 1e9, 1),
                    "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": round(per_class[dom] / dom_s / HBM_PEAK, 4),
                    "bytes_per_launch": per_class[dom], "avg_launch_us": round(dom_s * 1e6, 3), "traffic": None}
        metric, value, unit = "autoregressive decode steps/s (%s)" % wl.name, 1000.0 / ms, "decode steps/s"
    else:
        # dense contraction: flops of the dominant projection class over the rows of a step, against the
        # bf16 matrix-core peak (each fp32 activation is two bf16 operands, so the cores do twice these flops)
        cls_w = {"qkv": 3 * d * d, "oproj": d * d, "gateup": 2 * d * f, "down": d * f}
        dom = max((k for k in kernels if k in cls_w), key=lambda k: prof[k][0])
        step_s = prof[dom][0] / n_prof * 1e-3
        fl = 2.0 * cls_w[dom] * L * B * P
        roofline = {"kernel": dom, "bound": "mfma", "achieved": round(fl / step_s / 1e12, 2), "peak": 2500.0,
                    "unit": "TFLOP/s", "frac": round(fl / step_s / 2.5e15, 4),
                    "flops_per_step": fl, "class_ms_per_step": round(step_s * 1e3, 3), "traffic": None}
        metric, value, unit = "prefix tokens prefilled/s (%s)" % wl.name, B * P * 1000.0 / ms, "tokens/s"
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from helpers import oracle_model, oracle_chunked_prefill, prefix_embeddings
        om = oracle_model(sh, weights)
        t0 = time.perf_counter()
        if decode:
            n_done, spent = 0, 0.0
            k1, v1, f1 = synth.make_prefix_kv_direct(wl, 0, cap)
            while spent < 10.0 and n_done < 64:
                t1 = time.perf_counter()
                oracle.forward_block(om, oracle.embed(om, np.array([[sh.bin_base + int(f1)]])), [P], k1[:, None], v1[:, None])
                spent += time.perf_counter() - t1
                n_done += 1
            cpu = {"value": round(n_done / B / spent, 4), "unit": unit, "cores": min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1),
                   "kind": "oracle", "sample": "%d single-episode oracle decode forwards, %.1f s" % (n_done, spent)}
        else:
            oracle_chunked_prefill(om, prefix_embeddings(om, wl, 0), chunks, cap)
            spent = time.perf_counter() - t0
            cpu = {"value": round(P / spent, 2), "unit": unit, "cores": min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1),
                   "kind": "oracle", "sample": "one episode's %d-row prefix through the oracle in the same chunks, %.1f s" % (P, spent)}
    line = {"metric": metric, "value": round(value, 2), "unit": unit, "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "%s: %d-layer d=%d decoder, prefix %d, batch %d; %s" %
                                   (wl.name, L, d, P, B, "one new token per episode on a full prefix cache" if decode
                                    else "whole prefix from an empty cache in chunks of %s rows" % chunks),
                       "global_batch": B},
            "kernel_path": args.path, "activations": "one bf16" if args.act_bf16 else "bf16 head + tail",
            "gemm_tflops_whole_step": round(gemm_flops_per_row * B * sum(chunks) / (ms * 1e-3) / 1e12, 2),
            "kernels": kernels, "roofline": roofline, "cpu_baseline": cpu}
    print(json.dumps(line))
    ver.close()


def run_skip_mode(args):
    """--mode skip: the verify-skip decision kernels (Sec. 4.1, Alg. 1) on synthetic trajectory features:
    the offline stage over n = 300 trajectory points of d_model-wide features, and the per-episode
    decision for 64 episodes."""
    import numpy as np
    import torch
    import synth
    import paper_2603_17573_amd as P
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    d, n, B = synth.WORKLOADS[args.workload].shape.d_model, 300, 64
    f = synth.normal_f32(7, "skip.feat", n * d).reshape(n, d)
    f = np.cumsum(0.1 * f, axis=0, dtype=np.float32) + synth.normal_f32(7, "skip.base", d)      # a drifting trajectory
    t_f = torch.from_numpy(np.ascontiguousarray(f)).to(dev)
    work = torch.zeros(1, dtype=torch.int64, device=dev)
    min_s = torch.zeros(1, device=dev)
    o_dist = torch.zeros(1, dtype=torch.int32, device=dev)
    skip = torch.zeros(B, dtype=torch.uint8, device=dev)
    dist = torch.ones(B, dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream(dev).cuda_stream

    def offline():
        assert P.heisd_skip_offline(t_f.data_ptr(), n, d, 0.8, None, work.data_ptr(), min_s.data_ptr(), o_dist.data_ptr(), st) == 0

    def decide():
        assert P.heisd_skip_decide(t_f.data_ptr(), t_f[B:].data_ptr(), dist.data_ptr(), B, d, min_s.data_ptr(),
                                   o_dist.data_ptr(), skip.data_ptr(), None, st) == 0

    res = {}
    for name, fn in (("offline", offline), ("decide", decide)):
        for _ in range(args.warmup):
            fn()
        torch.cuda.synchronize()
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record()
        for _ in range(args.steps):
            fn()
        ev1.record()
        torch.cuda.synchronize()
        res[name] = ev0.elapsed_time(ev1) / args.steps
    pairs = n * n
    flops = 6.0 * d * pairs                    # three multiply-adds per element of a pair
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t0 = time.perf_counter()
        oracle.offline_stage(f[:100], 0.8)
        spent = time.perf_counter() - t0
        cpu = {"value": round(1.0 / (spent * 9.0), 4), "unit": "offline stages/s", "cores": 1, "kind": "oracle",
               "sample": "the oracle's double loop over the first 100 of the 300 points (1/9 of the pairs), %.1f s" % spent}
    line = {"metric": "verify-skip offline stages/s (%d trajectory points, d=%d)" % (n, d), "value": round(1000.0 / res["offline"], 1),
            "unit": "offline stages/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(res["offline"], 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "f32", "data": "synthetic",
            "config": {"workload": "offline stage of Alg. 1 over %d synthetic trajectory points (random-walk features of width %d), "
                                   "boundary T = 0.8; decision for %d episodes" % (n, d, B)},
            "decide_us": round(res["decide"] * 1e3, 2),
            "min_S": float(min_s.cpu()[0]), "O_dist": int(o_dist.cpu()[0]), "skipped": int(skip.sum().cpu()),
            "roofline": {"kernel": "pair_similarity", "bound": "alu", "achieved": round(flops / (res["offline"] * 1e-3) / 1e12, 2),
                         "peak": 157.3, "unit": "TFLOP/s", "frac": round(flops / (res["offline"] * 1e-3) / 157.3e12, 4), "traffic": None},
            "cpu_baseline": cpu}
    print(json.dumps(line))


def run_retrieve_mode(args):
    """--mode retrieve: the retrieval branch's exact cosine Top-8 search (App. C) over a synthetic database
    of the paper's size (273,465 embeddings of 4352 dimensions, bf16: 2.38 GB), one query per call."""
    import numpy as np
    import torch
    import synth
    import paper_2603_17573_amd as P
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    N, d, K, B = 273465, 4352, 8, 1
    db, payload = synth.make_retrieval_db(N, d, seed=1)
    q = synth.make_retrieval_queries(db, B, noise=0.7, seed=2)
    t_db = torch.from_numpy(db.view(np.int16)).to(dev)
    t_q = torch.from_numpy(q).to(dev)
    t_pay = torch.from_numpy(payload).to(dev)
    nbytes = P.heisd_retrieve_workspace_bytes(N, B, K)
    ws = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    idx = torch.zeros((B, K), dtype=torch.int32, device=dev)
    val = torch.zeros((B, K), device=dev)
    pay = torch.zeros((B, K, 7), dtype=torch.int32, device=dev)
    st = torch.cuda.current_stream(dev).cuda_stream

    def step():
        assert P.heisd_retrieve_topk(t_db.data_ptr(), N, d, t_q.data_ptr(), B, K, t_pay.data_ptr(), 7, idx.data_ptr(),
                                     val.data_ptr(), pay.data_ptr(), ws.data_ptr(), nbytes, st) == 0

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    ms = ev0.elapsed_time(ev1) / args.steps
    nbytes_db = N * d * 2
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        n_done, spent = 0, 0.0
        while spent < 10.0 and n_done < 64:
            t0 = time.perf_counter()
            ridx, rval, _ = oracle.retrieve(db, q, K)
            spent += time.perf_counter() - t0
            n_done += 1
        assert ridx[0, 0] == int(idx.cpu()[0, 0])
        cpu = {"value": round(n_done * B / spent, 3), "unit": "queries/s",
               "cores": min(int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)), os.cpu_count() or 1),
               "kind": "oracle", "sample": "%d exact fp64 searches of the same database, %.1f s" % (n_done, spent)}
    line = {"metric": "retrieval queries/s (exact cosine Top-%d over %d x %d bf16 embeddings)" % (K, N, d),
            "value": round(B * 1000.0 / ms, 1), "unit": "queries/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16 database, f32 queries and sums", "data": "synthetic",
            "config": {"workload": "database of the paper's size (L2-normalised N(0,1) directions), query = a stored vector "
                                   "+ noise; one query per call, Top-%d with payload" % K,
                       "paper_context": "the paper's CPU HNSW search (approximate): 5.13 ms per query"},
            "top_index": idx.cpu().numpy()[0].tolist(), "top_score": [round(float(v), 4) for v in val.cpu().numpy()[0]],
            "roofline": {"kernel": "retrieve_scores + Top-K selection (the whole call)", "bound": "hbm",
                         "achieved": round(nbytes_db / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK / 1e9, "unit": "GB/s",
                         "frac": round(nbytes_db / (ms * 1e-3) / HBM_PEAK, 4), "bytes_per_launch": nbytes_db,
                         "avg_launch_us": round(ms * 1e3, 2), "traffic": None},
            "cpu_baseline": cpu}
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="C1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference kernel for HBM traffic counters)")
    ap.add_argument("--path", type=int, default=0, help="0 auto, 1 generic, 2 fast (launch per phase), 3 persistent")
    ap.add_argument("--act-bf16", action="store_true",
                    help="activations enter the matrix cores as one bf16 each (heisd_verify_set_activations; calls of 33 "
                         "rows or more), instead of a bf16 head and tail; reported in the JSON line as activations")
    ap.add_argument("--handover", type=int, default=0, choices=[0, 1, 2, 3, 4, 5],
                    help="--path 3 only: what the persistent kernel requests across its grid barriers "
                         "(heisd_verify_set_handover; 0 = default)")
    ap.add_argument("--persist-trace", action="store_true",
                    help="--path 3 only: after the timed steps, record one step's device timestamps of every workgroup "
                         "in every phase (heisd_debug_trace) and add their summary to the JSON line")
    ap.add_argument("--tree", type=int, default=0, metavar="R",
                    help="time the TREE verify step instead: R retrieved candidates per episode, built into a "
                         "sequence-wise draft tree (paper Sec. 4.2); 0 = the linear step")
    ap.add_argument("--prefill-chunks", type=int, default=1, choices=[1, 2],
                    help="--mode prefill: 1 = visual embeddings and prompt ids in one call (default), 2 = one call each")
    ap.add_argument("--mode", default="verify", choices=["verify", "decode", "prefill", "skip", "retrieve", "readbw"],
                    help="verify (default): the verify step; decode: one autoregressive decode step; prefill: the "
                         "workload's prefix from an empty cache, in chunks")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs the verify step on ONE GPU (episodes would shard by batch "
              "with no exchange); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    if args.mode != "verify":
        from paper_2603_17573_amd import binding as _b
        if not os.path.exists(_b.LIB_PATH):
            from paper_2603_17573_amd import build
            build.build(force=False)
        if args.mode == "retrieve":
            return run_retrieve_mode(args)
        if args.mode == "readbw":
            return run_readbw_mode(args)
        return run_skip_mode(args) if args.mode == "skip" else run_aux_mode(args)

    import numpy as np
    import torch
    import synth
    from paper_2603_17573_amd import (DeviceModel, Verifier, make_accept_desc, binding, build_sequence_tree,
                                      heisd_verify_profile_enable, heisd_verify_profile_read)
    if not os.path.exists(binding.LIB_PATH):
        from paper_2603_17573_amd import build
        build.build(force=False)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    wl = synth.WORKLOADS[args.workload]
    sh = wl.shape
    B, K, P = wl.batch, wl.K, wl.prefix_len
    R = args.tree
    # tree tokens per episode when all R candidates differ in every sequence (one 7-token action slice)
    T = 3 * R + 3 * R * R + R * R if R else 0
    if R and (K != 7 or T > 256):
        print("bench.py: --tree needs a K=7 workload and at most 7 candidates", file=sys.stderr)
        sys.exit(2)
    rows = T if R else K                    # new rows per episode in one step
    cap = P + rows
    t0 = time.time()
    weights = synth.make_weights(sh, wl.seed)
    t_gen = time.time() - t0
    dm = DeviceModel(sh, weights, dev)
    ver = Verifier(dm, B, rows, cap)
    from paper_2603_17573_amd import heisd_verify_set_path, heisd_verify_set_handover
    assert heisd_verify_set_path(ver.ctx, args.path) == 0
    if args.act_bf16:
        from paper_2603_17573_amd import heisd_verify_set_activations, HEISD_ACT_BF16
        assert heisd_verify_set_activations(ver.ctx, HEISD_ACT_BF16) == 0
    if args.path == 3 and args.handover:
        assert heisd_verify_set_handover(ver.ctx, args.handover) == 0
    # prefix K/V drawn directly (the benchmark may not call the oracle's prefill); same shapes,
    # same bytes, same launch configuration as a prefilled cache
    kc, vc = ver.new_cache(B)
    first = np.zeros(B, np.int32)
    kb_host, vb_host = [], []
    for e in range(B):
        k, v, f = synth.make_prefix_kv_direct(wl, e, cap)
        kc[:, e] = torch.from_numpy(k.view(np.int16)).to(dev).view(torch.bfloat16)
        vc[:, e] = torch.from_numpy(v.view(np.int16)).to(dev).view(torch.bfloat16)
        first[e] = f
        if e == 0:
            kb_host, vb_host = k, v
    bins = synth.make_drafts_uniform(wl)
    drafts = (sh.bin_base + bins).astype(np.int32)
    skip = synth.make_skip_mask(wl) if wl.skip_p > 0 else None
    t_plen = torch.full((B,), P, dtype=torch.int32, device=dev)
    t_first = torch.from_numpy(first).to(dev)
    t_drafts = torch.from_numpy(drafts).to(dev)
    t_skip = None if skip is None else torch.from_numpy(skip).to(dev)
    acc = make_accept_desc(wl.tau_tok, wl.tau_seq)
    stream = torch.cuda.current_stream(dev)
    drafts_note = "uniform over the bins"

    def teacher_forced(off):
        """Bins d_j = clip(v_j + off_j), v_j = the target's greedy bin given d_0..d_{j-1}: v_j is row j of
        target_bins, which depends on the earlier drafts only, so K untimed linear steps fix the drafts one
        position at a time (the benchmark may not call the oracle)."""
        b_ = synth.make_drafts_uniform(wl)
        t_d = torch.from_numpy((sh.bin_base + b_).astype(np.int32)).to(dev)
        out0 = None
        for j in range(K):
            out0 = ver.step(kc, vc, t_plen, t_first, t_d, acc, t_skip, want_aux=True, out=out0, stream=stream)
            vj = out0["target_bins"][:, j].cpu().numpy()
            live = vj >= 0
            b_[live, j] = np.clip(vj[live] + off[live, j], 0, sh.n_bins - 1)
            t_d[:, j] = torch.from_numpy((sh.bin_base + b_[:, j]).astype(np.int32)).to(dev)
        return b_

    if wl.draft[0] == "geometric" and not R:
        bins = teacher_forced(synth.make_offsets_geometric(wl, wl.draft[1]))
        drafts = (sh.bin_base + bins).astype(np.int32)
        t_drafts = torch.from_numpy(drafts).to(dev)
        drafts_note = "target's own greedy bins (fixed position by position with K untimed device steps) + " \
                      "Geometric(%g) signed offsets" % wl.draft[1]
    t_tokens = t_parent = None
    if R:
        # stand-ins for Top-K retrieval: candidate r = the target's own continuation + seeded geometric offsets
        p_geo = wl.draft[1] if wl.draft[0] == "geometric" else 0.5
        coff = synth.make_candidate_offsets(wl, R, p_geo)
        cands = sh.bin_base + np.stack([teacher_forced(coff[:, r]) for r in range(R)], axis=1).astype(np.int32)
        drafts = cands[:, 0]
        tokens = np.zeros((B, T), np.int32)
        parent = np.full((B, T), -2, np.int32)
        for e in range(B):
            tok, par = build_sequence_tree(cands[e], acc, T)
            tokens[e, :len(tok)], parent[e, :len(par)] = tok, par
        t_tokens, t_parent = torch.from_numpy(tokens).to(dev), torch.from_numpy(parent).to(dev)
        drafts_note = "%d candidates per episode, each the target's own greedy continuation (fixed position by " \
                      "position with untimed device steps) + Geometric(%g) signed offsets, built into a " \
                      "sequence-wise tree of up to %d tokens (padded)" % (R, p_geo, T)

    def step(accept, want_aux=False, out=None):
        if R:
            return ver.tree_step(kc, vc, t_plen, t_first, t_tokens, t_parent, accept, t_skip, want_aux=want_aux,
                                 out=out, stream=stream)
        return ver.step(kc, vc, t_plen, t_first, t_drafts, accept, t_skip, want_aux=want_aux, out=out, stream=stream)

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    out = None
    for _ in range(args.warmup):
        out = step(acc, out=out)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        out = step(acc, out=out)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / args.steps
    accepted = out["accepted_len"].cpu().tolist()
    # acceptance does not change the work of a step: one time, several thresholds (paper Sec. 4.2: 15/30)
    hist = {}
    if wl.draft[0] == "geometric" or R:
        for tt, ts in ((0, 0), (1, 3), (2, 6), (4, 12), (2, 4), (15, 30)):
            o2 = step(make_accept_desc(tt, ts))
            al = o2["accepted_len"].cpu().numpy()
            if skip is not None:
                al = al[skip == 0]
            hist["%d/%d" % (tt, ts)] = np.bincount(al, minlength=K + 1).tolist()

    timeline = None
    if args.persist_trace and args.path == 3 and not R:
        from paper_2603_17573_amd import heisd_debug_trace
        n_ph, n_wg = 5 * sh.n_layers + 2, torch.cuda.get_device_properties(0).multi_processor_count
        heisd_debug_trace(ver.ctx, True)
        for _ in range(3):
            step(acc, out=out)
        torch.cuda.synchronize()
        got, buf = heisd_debug_trace(ver.ctx, False, n_ph * n_wg * 8)
        assert got == n_ph * n_wg * 8, got
        t = np.array(buf, dtype=np.int64).reshape(n_ph, n_wg, 8) / 100.0          # us (100 MHz counter)
        names = ["embed"] + ["qkv", "attn", "oproj", "gateup", "down"] * sh.n_layers + ["lmhead"]
        timeline = {"note": "us, means over layers 2.. of one step; per phase kind, relative to the first workgroup's "
                            "pass of the barrier that opens the phase: when the last workgroup passed it, when the "
                            "workgroups had consumed their weights (min / mean / max), when they had published their "
                            "outputs (min / mean / max), when the first and last workgroup passed the next barrier, when their "
                            "polls had seen every flag, and how long a workgroup then waited for its hand-over to land",
                    "step_us": round(float(t[-1, :, 3].max() - t[0, :, 0].min()), 1), "phases": {}}
        # slot 6 (polls done) is written only by workgroups that waited: one without an attention unit does not
        waited = lambda ph_t: ph_t[:, 6] > 0
        polled = lambda ph_t: ph_t[waited(ph_t), 6]
        landing = lambda ph_t: ph_t[waited(ph_t), 1] - ph_t[waited(ph_t), 6]
        for nm in ("qkv", "attn", "oproj", "gateup", "down"):
            rows_ = []
            for i in range(11, n_ph - 1):
                if names[i] != nm:
                    continue
                r0 = t[i, :, 1].min()
                rows_.append([t[i, :, 1].max() - r0, t[i, :, 2].min() - r0, t[i, :, 2].mean() - r0, t[i, :, 2].max() - r0,
                              t[i, :, 3].min() - r0, t[i, :, 3].mean() - r0, t[i, :, 3].max() - r0,
                              t[i + 1, :, 1].min() - r0, t[i + 1, :, 1].max() - r0,
                              polled(t[i + 1]).min() - r0, polled(t[i + 1]).max() - r0,
                              landing(t[i + 1]).mean(), landing(t[i + 1]).max()])
            m = np.mean(rows_, axis=0)
            timeline["phases"][nm] = {"last_release": round(float(m[0]), 2),
                                      "consumed_min_mean_max": [round(float(x), 2) for x in m[1:4]],
                                      "published_min_mean_max": [round(float(x), 2) for x in m[4:7]],
                                      "next_release_first_last": [round(float(x), 2) for x in m[7:9]],
                                      "next_polls_done_first_last": [round(float(x), 2) for x in m[9:11]],
                                      "next_polls_done_to_release_mean_max": [round(float(x), 2) for x in m[11:13]]}

    active = B if skip is None else int(B - skip.sum())
    total_bytes, per_class = algorithmic_bytes(sh, B, rows, P, active)

    def measure_kernels(ms):
        """Per-kernel durations of the path now selected (HIP events recorded by the library on the launch
        stream) and the roofline object of its dominant kernel; ms = that path's timed step."""
        n_prof = max(1, min(args.steps, 32))
        heisd_verify_profile_enable(ver.ctx, True)
        for _ in range(n_prof):
            step(acc, out=out)
        rc, prof = heisd_verify_profile_read(ver.ctx)
        heisd_verify_profile_enable(ver.ctx, False)
        assert rc == 0
        kernels = {}
        for kcls, (tot_ms, n) in prof.items():
            if n:
                avg = tot_ms / n
                kernels[kcls] = {"avg_us": round(avg * 1e3, 3), "launches_per_step": n / n_prof,
                                 "share_of_step": round(tot_ms / n_prof / ms, 4)}
                if kcls in per_class:
                    kernels[kcls]["GBps"] = round(per_class[kcls] / (avg * 1e-3) / 1e9, 1)
        dom = max((k for k in kernels if k in per_class), key=lambda k: prof[k][0])
        dom_avg_s = prof[dom][0] / prof[dom][1] * 1e-3
        # What the instrument adds: a bracket's two events cost time the timed steps do not spend.  The brackets
        # of a profiled step add up to more than a timed step; the surplus per bracket, taken off the dominant
        # kernel's bracket, is the kernel's duration as it runs in the timed region - the figure the rocprofv3
        # summaries under profiles/ show - and `achieved` / `frac` follow from that duration.  The raw bracket
        # is reported beside it.
        brackets = sum(n for _, n in prof.values()) / n_prof
        surplus_us = (sum(t for t, _ in prof.values()) / n_prof - ms) * 1e3 / brackets
        if not 0.0 < surplus_us < dom_avg_s * 1e6:
            surplus_us = 0.0
        kernel_s = dom_avg_s - surplus_us * 1e-6
        achieved = per_class[dom] / kernel_s
        traffic, traffic_source = read_traffic(dom)
        roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved / 1e9, 1), "peak": HBM_PEAK / 1e9,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK, 4),
                    "bytes_per_launch": per_class[dom], "avg_launch_us": round(kernel_s * 1e6, 3),
                    "traffic": traffic, "traffic_source": traffic_source,
                    "event_bracket_us": round(dom_avg_s * 1e6, 3), "event_bracket_surplus_us": round(surplus_us, 3),
                    "frac_of_event_bracket": round(per_class[dom] / dom_avg_s / HBM_PEAK, 4)}
        return kernels, roofline

    kernels, roofline = measure_kernels(ms)

    # the same step with one launch per phase (what the automatic choice falls back to when the persistent
    # kernel may not run), for comparison: its step time and its dominant kernel
    per_phase = None
    if not R and B * rows <= 8 and args.path in (0, 3) and kernels.get("persist"):
        assert heisd_verify_set_path(ver.ctx, 2) == 0
        for _ in range(10):
            out = step(acc, out=out)
        torch.cuda.synchronize()
        n2 = max(1, min(args.steps, 100))
        t0 = time.perf_counter()
        for _ in range(n2):
            out = step(acc, out=out)
        torch.cuda.synchronize()
        ms2 = (time.perf_counter() - t0) * 1e3 / n2
        k2, r2 = measure_kernels(ms2)
        assert heisd_verify_set_path(ver.ctx, args.path) == 0
        per_phase = {"kernel_path": 2, "ms_per_step": round(ms2, 4), "steps": n2,
                     "hbm_frac_whole_step": round(total_bytes / (ms2 * 1e-3) / HBM_PEAK, 4),
                     "kernels": k2, "roofline": r2}

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from helpers import oracle_model
        om = oracle_model(sh, weights)
        # bounded sample: oracle verify steps over successive episodes of the workload's recipe, until
        # about 12 s of oracle time have been spent (drawing an episode's prefix K/V is not timed)
        rule = oracle.AcceptRule(wl.tau_tok, wl.tau_seq)
        spent, n_done, ref_acc = 0.0, 0, []
        while spent < 12.0 and n_done < 64:
            e = n_done
            if e == 0:
                k1, v1, f1 = kb_host, vb_host, first[0]
            else:
                k1, v1, f1 = synth.make_prefix_kv_direct(wl, e % max(B, 1) if B > 1 else e, cap)
            d1 = drafts[e % B][None, :]
            t0 = time.perf_counter()
            if R:
                ref = oracle.verify_tree_step(om, k1[:, None], v1[:, None], [P], np.array([f1], np.int32),
                                              tokens[e % B][None, :], parent[e % B][None, :], rule)
            else:
                ref = oracle.verify_step(om, k1[:, None], v1[:, None], [P], np.array([f1], np.int32), d1, rule)
            spent += time.perf_counter() - t0
            n_done += 1
            ref_acc.append(int(ref["accepted_len"][0]))
        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        cores = min(cores, os.cpu_count() or cores)
        # one verify step of the workload covers B episodes
        cpu = {"value": round(n_done / B / spent, 5), "unit": "verify steps/s", "cores": cores, "kind": "oracle",
               "sample": "%d oracle %sverify steps over single episodes of %s (%s through all %d layers), "
                         "%.1f s of oracle time" % (n_done, "tree " if R else "", wl.name,
                                                    "every chain of the tree on its own" if R else "K=%d rows" % K,
                                                    sh.n_layers, spent),
               "oracle_accepted_len": ref_acc[:8]}

    line = {
        "metric": ("tree verify steps/s (%s, %d candidates, %d tree tokens)" % (wl.name, R, T)) if R else
                  ("verify steps/s (7B-shaped decoder, K=7, bs=1)" if wl.name == "C1" else
                   "verify steps/s (%s)" % wl.name),
        "value": round(1000.0 / ms, 2), "unit": "verify steps/s", "n_gpus": 1, "steps": args.steps,
        "episode_steps_per_s": round(B * 1000.0 / ms, 1), "draft_tokens_verified_per_s": round(active * rows * 1000.0 / ms, 1),
        "warmup": args.warmup, "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d-layer d=%d decoder, prefix %d, batch %d, K=%d, thresholds %d/%d" %
                               (wl.name, sh.n_layers, sh.d_model, P, B, K, wl.tau_tok, wl.tau_seq),
                   "prefix_kv": "drawn directly (no prefill)", "drafts": drafts_note, "global_batch": B, "K": K, "tree_tokens": T or None},
        "kernel_path": args.path, "handover_mode": args.handover if args.path == 3 else None,
        "activations": "one bf16 (calls of 33 rows or more)" if args.act_bf16 else "bf16 head + tail",
        "hbm_frac_whole_step": round(total_bytes / (ms * 1e-3) / HBM_PEAK, 4),
        "algorithmic_bytes_per_step": total_bytes,
        "accepted_len": accepted[:8],
        "accepted_len_histograms_by_threshold": hist or None,
        "weights_gen_s": round(t_gen, 1),
        "kernels": kernels,
        "persistent_kernel_timeline": timeline,
        "launch_per_phase": per_phase,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    print(json.dumps(line))
    ver.close()


if __name__ == "__main__":
    main()
