#!/usr/bin/env python3
"""Benchmark of the ChunkKV compression stack on one MI355X.

A step is one chunkkv_compress_stack call over the whole synthetic cache (all layers: scoring and
selection on the leader layers, gather on every layer), inputs resident in HBM.  The metric is prefix
tokens compressed per second over the layer stack.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

HBM_PEAK_GBPS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes(wl, n_keep, n_layers, reuse):
    """Bytes the method must move: K read once per scored layer; kept K and V rows read once and
    written once on every layer.  Q_obs, chunk scores and selections are < 0.3 % and left out."""
    row = wl.head_dim * wl.elem_bytes
    k_read = sum(wl.n_kv_heads * L * row for L in wl.seqlens)
    gather = sum(4 * wl.n_kv_heads * (nk + wl.window) * row for nk in n_keep)
    leaders = (n_layers + reuse - 1) // reuse
    return {"score_per_layer": k_read, "gather_per_layer": gather,
            "stack": leaders * k_read + n_layers * gather}


def csrc_hash():
    """sha256 over the library's sources (file names and contents, sorted): what profiles/hbm_traffic.json is tied to."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2502_00299_amd", "csrc")
    for name in sorted(os.listdir(d)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(d, name), "rb").read())
    h.update(open(os.path.join(ROOT, "include", "chunkkv.h"), "rb").read())
    return h.hexdigest()


def ckv_single_pass_used(kern):
    """The single-pass path launches no chunk-sum kernel and its row reduction is far shorter than its
    scoring kernel; the two-pass kernels take about the same time each."""
    a = kern.get("score_stats", {}).get("ms_per_step", 0.0)
    b = kern.get("score_colsum", {}).get("ms_per_step", 0.0)
    return b < 0.5 * a


def cpu_baseline(wl, layers, n_keep, reuse, n_sample_layers, gpu_sel=None):
    """The oracle, as it stands, on the first n_sample_layers layers of the same inputs: Algorithm 2 written
    out with its functions (score, chunk_topk on the leader layers, compact on every layer), timed as a whole.
    gpu_sel = (sel_chunk, sel_len, sel_count) host arrays of the GPU run: its selections of the sampled leader
    layers are then compared with the oracle's (chunks that differ, and whether all of them lie inside the
    1e-3 relative tie band around the oracle's threshold score)."""
    from oracle import chunkkv_oracle as orc
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas_threads = None
    host = []
    for l in range(n_sample_layers):
        li = layers[l]
        per_seq = []
        for b in range(wl.batch):
            q = W.tensor_bits(li.q[b]) if l % reuse == 0 else None
            k = W.tensor_bits(li.seq_view(li.k, b, wl.n_kv_heads, wl.head_dim))
            v = W.tensor_bits(li.seq_view(li.v, b, wl.n_kv_heads, wl.head_dim))
            per_seq.append((q, k, v))
        host.append(per_seq)
    scores, sels = {}, {}
    t0 = time.perf_counter()
    for b in range(wl.batch):
        P = wl.seqlens[b] - wl.window
        for l in range(n_sample_layers):
            q, k, v = host[l][b]
            if l % reuse == 0:
                cs, _ = orc.score(q, k, wl.window, wl.chunk)
                scores[(l, b)] = cs
                sels[(l, b)] = [orc.chunk_topk(cs[h], P, wl.chunk, n_keep[b]) for h in range(wl.n_kv_heads)]
            sel = sels[((l // reuse) * reuse, b)]
            orc.compact(k, v, [x[0] for x in sel], [x[1] for x in sel], wl.window, wl.chunk)
    dt = time.perf_counter() - t0
    est_stack = dt * wl.n_layers / n_sample_layers
    cpu = None
    try:
        with open("/proc/cpuinfo") as f:
            cpu = next((ln.split(":", 1)[1].strip() for ln in f if ln.startswith("model name")), None)
    except OSError:
        pass
    out = {"value": sum(wl.seqlens) / est_stack, "unit": "prefix tokens/s", "cores": int(cores),
           "kind": "oracle", "cpu": cpu, "blas_threads": blas_threads,
           "threading": "cores = CPUs this process may run on (sched_getaffinity); the oracle is numpy: only its matrix "
                        "products run on the BLAS thread pool, exp / where / sum are single-threaded",
           "sample": f"layers 0..{n_sample_layers - 1} of {wl.n_layers} (all sequences and kv-heads) in "
                     f"{dt:.1f} s, scaled by {wl.n_layers}/{n_sample_layers}"}
    if gpu_sel is not None:
        sel_chunk, sel_len, sel_count = gpu_sel
        differ = outside = heads = 0
        for (l, b), per_head in sels.items():
            for h, (oc, ol) in enumerate(per_head):
                m = int(sel_count[l // reuse, b, h])
                gc = sel_chunk[l // reuse, b, h, :m]
                cs = scores[(l, b)][h]
                thr = float(cs[oc].min()) if len(oc) else 0.0
                d = set(gc.tolist()) ^ set(oc.tolist())
                differ += len(d)
                outside += sum(1 for ch in d if abs(float(cs[ch]) - thr) > 1e-3 * thr)
                heads += 1
        out["selection_parity"] = {"heads_compared": heads, "chunks_differing": differ,
                                   "outside_tie_band": outside, "tie_band": "1e-3 relative to the oracle's threshold score"}
    return out


def window_lse(wl, li, dev):
    """[B][Hq][w] fp32 log-sum-exps of the window rows over the keys they see: what a fused prefill attention
    kernel would hand over.  Harness-side input preparation with library ops (fp32 logits)."""
    g, w, d = wl.group, wl.window, wl.head_dim
    out = torch.empty((wl.batch, wl.n_q_heads, w), dtype=torch.float32, device=dev)
    for b, L in enumerate(wl.seqlens):
        P = L - w
        kb = li.seq_view(li.k, b, wl.n_kv_heads, d)                       # [Hkv][L][d]
        hidden = torch.arange(L, device=dev)[None, :] > (P + torch.arange(w, device=dev))[:, None]   # [w][L]
        for h in range(wl.n_kv_heads):
            q = li.q[b, h * g:(h + 1) * g].float().reshape(g * w, d)
            s = (q @ kb[h].float().T) * (1.0 / d ** 0.5)                    # [g*w][L]
            s = s.view(g, w, L).masked_fill(hidden[None], float("-inf"))
            out[b, h * g:(h + 1) * g] = torch.logsumexp(s, dim=2)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama8b_128k_stack")
    ap.add_argument("--reuse", type=int, default=2)
    ap.add_argument("--keep-pct", type=int, default=None)
    ap.add_argument("--layers", type=int, default=None)
    ap.add_argument("--dtype", choices=["bf16", "f16", "f32"], default=None,
                    help="storage type of the synthetic caches (default: the workload's, bf16 for the headline)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--cpu-layers", type=int, default=None)
    ap.add_argument("--no-r1", action="store_true", help="skip the R=1 comparison run")
    ap.add_argument("--no-lse", action="store_true", help="skip the caller-supplied log-sum-exp leg")
    ap.add_argument("--no-streaming", action="store_true", help="skip the per-layer streaming-call leg")
    ap.add_argument("--no-graph", action="store_true", help="skip the HIP-graph replay leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode-attention leg")
    ap.add_argument("--csrc-hash", action="store_true", help="print the hash profiles/hbm_traffic.json must name, and exit")
    ap.add_argument("--no-other", action="store_true", help="skip the other-workloads leg")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (reference for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.csrc_hash:
        print(csrc_hash())
        return
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1")
        sys.exit(2)
    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        sys.exit(1)

    import paper_2502_00299_amd as ckv
    ckv.load_library()
    dev = "cuda:0"
    wl = W.get_workload(args.workload)
    if args.keep_pct is not None:
        wl = wl.with_(keep_pct=args.keep_pct)
    if args.dtype is not None:
        wl = wl.with_(dtype=args.dtype)
    if args.layers is not None:
        wl = wl.with_(n_layers=args.layers)
    N, R = wl.n_layers, args.reuse
    log(f"generating {wl.name}: {N} layers, L={wl.seqlens}, w={wl.window}, c={wl.chunk}, keep {wl.keep_pct}%")
    layers = [W.make_layer(wl, l, dev) for l in range(N)]
    torch.cuda.synchronize()
    n_keep = [W.keep_budget(L, wl.window, wl.keep_pct) for L in wl.seqlens]
    li0 = layers[0]
    prob = ckv.Problem(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.window, wl.chunk,
                       {"f32": ckv.F32, "bf16": ckv.BF16, "f16": ckv.F16}[wl.dtype], list(wl.seqlens), n_keep, list(li0.kv_base),
                       li0.kv_stride_head, li0.kv_stride_tok)
    k_out = [torch.empty(prob.out_elements(), dtype=wl.torch_dtype, device=dev) for _ in range(N)]
    v_out = [torch.empty(prob.out_elements(), dtype=wl.torch_dtype, device=dev) for _ in range(N)]
    ks, vs = [x.k for x in layers], [x.v for x in layers]

    def make_run(reuse):
        G = (N + reuse - 1) // reuse
        sel_chunk = torch.zeros((G, wl.batch, wl.n_kv_heads, prob.sel_cap), dtype=torch.int32, device=dev)
        sel_len = torch.zeros_like(sel_chunk)
        sel_count = torch.zeros((G, wl.batch, wl.n_kv_heads), dtype=torch.int32, device=dev)
        ws = torch.empty(ckv.chunkkv_workspace_bytes(prob, N, reuse), dtype=torch.uint8, device=dev)
        qs = [layers[l].q if l % reuse == 0 else None for l in range(N)]

        def run():
            ckv.chunkkv_compress_stack(prob, reuse, qs, ks, vs, k_out, v_out, sel_chunk, sel_len, sel_count, ws)
        run.selection = (sel_chunk, sel_len, sel_count)
        return run

    def timed(run, steps, warmup, with_kernel_timing=False):
        for _ in range(warmup):
            run()
        torch.cuda.synchronize()
        if with_kernel_timing:
            ckv.chunkkv_timing_begin(16 * steps + 16)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        kt = ckv.chunkkv_timing_end() if with_kernel_timing else None
        return dt / steps * 1e3, kt

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst
    run_main = make_run(R)

    def main_sel():
        run_main()
        torch.cuda.synchronize()
        return tuple(t.cpu().numpy() for t in run_main.selection)

    ms, _ = timed(run_main, args.steps, args.warmup)
    # per-kernel durations: a second loop of the same steps with a HIP event pair around every launch
    # (kept out of the headline loop: the event packets add gaps between the kernels)
    _, kt = timed(run_main, args.steps, 1, with_kernel_timing=True)
    # spread of single steps: one HIP-event pair per step on the launch stream (outside the headline loop)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.steps, 20))]
    for e0, e1 in evs:
        e0.record()
        run_main()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    step_spread = {"median": per_step[len(per_step) // 2], "min": per_step[0], "max": per_step[-1], "n": len(per_step)}
    tokens = sum(wl.seqlens)
    value = tokens / (ms * 1e-3)
    ab = algorithmic_bytes(wl, n_keep, N, R)
    leaders = (N + R - 1) // R

    # roofline of the kernel that takes the most time (durations from HIP events on the launch stream)
    kern = {k: {"ms_per_launch": t / n, "launches_per_step": n / args.steps, "ms_per_step": t / args.steps}
            for k, (t, n) in kt.items() if n}
    dom = max(kern, key=lambda k: kern[k]["ms_per_step"])
    launches = kern[dom]["launches_per_step"]
    if dom in ("score_stats", "score_colsum"):
        bytes_per_launch = ab["score_per_layer"] * leaders / launches
    elif dom == "compact":
        bytes_per_launch = ab["gather_per_layer"] * N / launches
    else:
        bytes_per_launch = 0.0
    achieved = bytes_per_launch / (kern[dom]["ms_per_launch"] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": achieved / HBM_PEAK_GBPS, "traffic": None,
                "algorithmic_bytes_per_launch": bytes_per_launch}
    # HBM bytes per launch from rocprofv3 counters (profiles/hbm_traffic.json): valid only for the kernel sources
    # they were taken from, so the file names their hash and the figure is dropped when the sources have changed
    traffic_file = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(traffic_file):
        try:
            tf = json.load(open(traffic_file))
            if tf.get("csrc_sha256") == csrc_hash():
                roofline["traffic"] = tf.get(wl.name, {}).get(dom)
            else:
                log("bench.py: profiles/hbm_traffic.json was taken from other kernel sources (csrc hash differs): "
                    "roofline.traffic = null until the counters are collected again")
        except Exception:
            pass
    stack_gbps = ab["stack"] / (ms * 1e-3) / 1e9
    # the scoring kernel's matrix work: 2 * Hq * w * L * d flops per scored layer (the logits; the single-pass
    # kernel's indicator products, a quarter more, are not algorithmic and not counted)
    score_kind = "score_stats"
    mfma = None
    if score_kind in kern and wl.dtype in ("bf16", "f16"):
        flops = sum(2.0 * wl.n_q_heads * wl.window * L * wl.head_dim for L in wl.seqlens) * leaders
        passes = 1 if ckv_single_pass_used(kern) else 2
        t = kern["score_stats"]["ms_per_step"] + (kern.get("score_colsum", {"ms_per_step": 0.0})["ms_per_step"] if passes == 2 else 0.0)
        ach = flops / (t * 1e-3) / 1e12
        mfma = {"bound": "mfma", "kernel": "score_stats" if passes == 1 else "score_stats+score_colsum",
                "achieved": ach, "peak": 2500.0, "unit": "TFLOP/s", "frac": ach / 2500.0,
                "algorithmic_flops_per_step": flops}

    # index reuse: same stack with R = 1
    ms_r1 = None
    if R != 1 and not args.no_r1:
        ms_r1, _ = timed(make_run(1), max(3, args.steps // 2), 2)

    # the same stack when the caller hands over the window rows' log-sum-exps (chunkkv_compress_stack_lse):
    # not the headline metric, a second workload definition reported beside it
    lse_leg = None
    if not args.no_lse:
        try:
            lses = [window_lse(wl, layers[l], dev) if l % R == 0 else None for l in range(N)]
            G = (N + R - 1) // R
            sc = torch.zeros((G, wl.batch, wl.n_kv_heads, prob.sel_cap), dtype=torch.int32, device=dev)
            sl, cnt = torch.zeros_like(sc), torch.zeros((G, wl.batch, wl.n_kv_heads), dtype=torch.int32, device=dev)
            ws_l = torch.empty(ckv.chunkkv_workspace_bytes(prob, N, R), dtype=torch.uint8, device=dev)
            qs_l = [layers[l].q if l % R == 0 else None for l in range(N)]

            def run_lse():
                ckv.chunkkv_compress_stack_lse(prob, R, qs_l, ks, vs, lses, k_out, v_out, sc, sl, cnt, ws_l)
            ms_l, _ = timed(run_lse, args.steps, args.warmup)
            _, kt_l = timed(run_lse, args.steps, 1, with_kernel_timing=True)
            lse_leg = {"ms_per_step": ms_l, "value": tokens / (ms_l * 1e-3), "unit": "prefix tokens/s",
                       "stack_hbm_frac": ab["stack"] / (ms_l * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                       "kernels_ms_per_step": {k: round(t / args.steps, 4) for k, (t, n) in kt_l.items() if n}}
            del lses, ws_l
        except Exception as e:  # the headline line must not depend on this leg
            log(f"log-sum-exp leg failed: {e!r}")

    # the headline call replayed from a HIP graph (the call is kernels only, so a caller can capture it)
    graph_leg = None
    if not args.no_graph:
        try:
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                run_main()
                side.synchronize()
                with torch.cuda.graph(graph, stream=side):
                    run_main()
            torch.cuda.current_stream().wait_stream(side)
            ms_g, _ = timed(graph.replay, args.steps, args.warmup)
            graph_leg = {"ms_per_step": ms_g, "value": tokens / (ms_g * 1e-3), "unit": "prefix tokens/s"}
            del graph
        except Exception as e:
            log(f"graph leg failed: {e!r}")

    # the same stack through the streaming call, one chunkkv_compress_layer per layer (what a serving loop that
    # compresses each layer right after its prefill would issue); reported beside the headline
    stream_leg = None
    if not args.no_streaming:
        try:
            G = (N + R - 1) // R
            sc = torch.zeros((G, wl.batch, wl.n_kv_heads, prob.sel_cap), dtype=torch.int32, device=dev)
            sl, cnt = torch.zeros_like(sc), torch.zeros((G, wl.batch, wl.n_kv_heads), dtype=torch.int32, device=dev)
            ws_1 = torch.empty(ckv.chunkkv_workspace_bytes(prob, 1, 1), dtype=torch.uint8, device=dev)

            def run_layers():
                for l in range(N):
                    ckv.chunkkv_compress_layer(prob, l, R, layers[l].q if l % R == 0 else None, None, ks[l], vs[l],
                                               k_out[l], v_out[l], sc, sl, cnt, ws_1)
            ms_s, _ = timed(run_layers, max(3, args.steps // 2), 2)
            stream_leg = {"ms_per_step": ms_s, "value": tokens / (ms_s * 1e-3), "unit": "prefix tokens/s",
                          "calls_per_step": N}
            del ws_1
        except Exception as e:
            log(f"streaming leg failed: {e!r}")

    # what the compression buys afterwards: one decoding step's attention (one query token per head, every
    # layer) over the compressed caches this run produced, and over the uncompressed caches for comparison
    decode_leg = None
    if not args.no_decode:
        try:
            run_main()
            qd = [x.q[:, :, -1, :].contiguous() for x in layers]
            o_d = torch.empty((wl.batch, wl.n_q_heads, wl.head_dim), dtype=torch.float32, device=dev)
            legs = {}
            for name, compacted, kk, vv, toks in (("compressed", True, k_out, v_out, [nk + wl.window for nk in n_keep]),
                                                 ("full", False, ks, vs, list(wl.seqlens))):
                ws_d = torch.empty(ckv.chunkkv_decode_workspace_bytes(prob, compacted), dtype=torch.uint8, device=dev)

                def run_decode():
                    for l in range(N):
                        ckv.chunkkv_decode_attention(prob, compacted, None, qd[l], kk[l], vv[l], o_d, None, ws_d)
                ms_d, _ = timed(run_decode, args.steps, args.warmup)
                _, kt_d = timed(run_decode, args.steps, 1, with_kernel_timing=True)
                nbytes = N * sum(2 * wl.n_kv_heads * t * wl.head_dim * wl.elem_bytes for t in toks)
                t_k, n_k = kt_d["decode"]
                ms_g = None
                try:   # the same N calls replayed from a HIP graph, as a captured decoding loop would issue them
                    side = torch.cuda.Stream()
                    side.wait_stream(torch.cuda.current_stream())
                    graph_d = torch.cuda.CUDAGraph()
                    with torch.cuda.stream(side):
                        run_decode()
                        side.synchronize()
                        with torch.cuda.graph(graph_d, stream=side):
                            run_decode()
                    torch.cuda.current_stream().wait_stream(side)
                    ms_g, _ = timed(graph_d.replay, args.steps, args.warmup)
                    del graph_d
                except Exception as e:
                    log(f"decode graph replay failed: {e!r}")
                legs[name] = {"ms_per_token_all_layers": ms_d, "ms_from_hip_graph": ms_g,
                              "kernel_ms_per_layer": t_k / max(n_k, 1),
                              "algorithmic_bytes": nbytes, "achieved_GBps": nbytes / (ms_d * 1e-3) / 1e9,
                              "kernel_GBps": nbytes / N / (t_k / max(n_k, 1) * 1e-3) / 1e9,
                              "hbm_frac": nbytes / (ms_d * 1e-3) / 1e9 / HBM_PEAK_GBPS}
                del ws_d
            decode_leg = {**legs, "speedup_compressed_vs_full": legs["full"]["ms_per_token_all_layers"] /
                          legs["compressed"]["ms_per_token_all_layers"]}
        except Exception as e:
            log(f"decode leg failed: {e!r}")

    out = {
        "metric": "prefix tokens compressed/sec (32-layer stack) + achieved HBM GB/s vs peak",
        "value": value, "unit": "prefix tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms, "ms_per_step_source": "wall clock over the K timed steps between two device synchronisations, / K "
                                                 "(value uses it); step_ms_hip_events: single steps between HIP events",
        "step_ms_hip_events": step_spread, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: {N} layers, B={wl.batch}, L={list(wl.seqlens)}, Hq={wl.n_q_heads}, "
                               f"Hkv={wl.n_kv_heads}, d={wl.head_dim}, w={wl.window}, c={wl.chunk}, "
                               f"keep {wl.keep_pct}%, R={R}",
                   "reuse": R, "n_layers": N, "keep_pct": wl.keep_pct},
        "roofline": roofline,
        "stack_hbm": {"algorithmic_bytes": ab["stack"], "achieved": stack_gbps, "peak": HBM_PEAK_GBPS,
                      "unit": "GB/s", "frac": stack_gbps / HBM_PEAK_GBPS},
        "roofline_mfma": mfma,
        "kernels_ms_per_step": {k: round(v["ms_per_step"], 4) for k, v in kern.items()},
        "decode_attention": decode_leg,
        # Eq. 1 for this workload's geometry (kv-heads, not query heads, hold the cache under grouped-query attention)
        "kv_cache_bytes": {"full": N * sum(2 * wl.n_kv_heads * L * wl.head_dim * wl.elem_bytes for L in wl.seqlens),
                           "compressed": N * sum(2 * wl.n_kv_heads * (nk + wl.window) * wl.head_dim * wl.elem_bytes
                                                 for nk in n_keep)},
        "with_caller_lse": lse_leg,
        "streaming_per_layer": stream_leg,
        "hip_graph_replay": graph_leg,
        "reuse_speedup_vs_R1": (ms_r1 / ms) if ms_r1 else None,
        "ms_per_step_R1": ms_r1,
    }
    if not args.no_cpu:
        n_cpu = args.cpu_layers or min(N, 8 * R if wl.seqlens[0] > 65536 else 16 * R)
        log(f"timing the CPU oracle on {n_cpu} layers ...")
        out["cpu_baseline"] = cpu_baseline(wl, layers, n_keep, R, n_cpu, gpu_sel=main_sel())
    else:
        out["cpu_baseline"] = None

    # the other configurations of the benchmark spec, each one chunkkv_compress_stack call per step on its own inputs
    # (not the headline; reported so that every configuration has a recorded figure)
    other = None
    if not args.no_other and args.workload == "llama8b_128k_stack":
        other = {}

        def quick(tag, wl2, layers2, R2):
            try:
                N2 = wl2.n_layers
                nk2 = [W.keep_budget(L, wl2.window, wl2.keep_pct) for L in wl2.seqlens]
                l0 = layers2[0]
                p2 = ckv.Problem(wl2.n_q_heads, wl2.n_kv_heads, wl2.head_dim, wl2.window, wl2.chunk,
                                 {"f32": ckv.F32, "bf16": ckv.BF16, "f16": ckv.F16}[wl2.dtype], list(wl2.seqlens), nk2,
                                 list(l0.kv_base), l0.kv_stride_head, l0.kv_stride_tok)
                ko = [torch.empty(p2.out_elements(), dtype=wl2.torch_dtype, device=dev) for _ in range(N2)]
                vo = [torch.empty(p2.out_elements(), dtype=wl2.torch_dtype, device=dev) for _ in range(N2)]
                G2 = (N2 + R2 - 1) // R2
                sc2 = torch.zeros((G2, wl2.batch, wl2.n_kv_heads, p2.sel_cap), dtype=torch.int32, device=dev)
                sl2, cn2 = torch.zeros_like(sc2), torch.zeros((G2, wl2.batch, wl2.n_kv_heads), dtype=torch.int32, device=dev)
                ws2 = torch.empty(ckv.chunkkv_workspace_bytes(p2, N2, R2), dtype=torch.uint8, device=dev)
                q2 = [layers2[l].q if l % R2 == 0 else None for l in range(N2)]
                k2, v2 = [x.k for x in layers2], [x.v for x in layers2]

                def run2():
                    ckv.chunkkv_compress_stack(p2, R2, q2, k2, v2, ko, vo, sc2, sl2, cn2, ws2)
                ms2, _ = timed(run2, args.steps, args.warmup)
                ab2 = algorithmic_bytes(wl2, nk2, N2, R2)
                other[tag] = {"ms_per_step": ms2, "value": sum(wl2.seqlens) / (ms2 * 1e-3), "unit": "prefix tokens/s",
                              "stack_hbm_frac": ab2["stack"] / (ms2 * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "algorithmic_bytes": ab2["stack"]}
            except Exception as e:
                log(f"other workload {tag} failed: {e!r}")

        quick("llama8b_128k_stack keep 20% R=2", wl.with_(keep_pct=20), layers, 2)
        del layers, ks, vs, k_out, v_out
        torch.cuda.empty_cache()
        wl3 = W.get_workload("llama8b_32k_stack")
        log(f"generating {wl3.name}")
        layers3 = [W.make_layer(wl3, l, dev) for l in range(wl3.n_layers)]
        quick("llama8b_32k_stack keep 10% R=1", wl3, layers3, 1)
        quick("llama8b_32k_stack keep 10% R=2", wl3, layers3, 2)
        del layers3
        torch.cuda.empty_cache()
        wl5 = W.get_workload("ragged_b8")
        log(f"generating {wl5.name}")
        layers5 = [W.make_layer(wl5, l, dev) for l in range(wl5.n_layers)]
        quick("ragged_b8 c=10 keep 10% R=2", wl5, layers5, 2)
        quick("ragged_b8 c=5 keep 30% R=3", wl5.with_(chunk=5, keep_pct=30), layers5, 3)
        quick("ragged_b8 c=20 keep 20% R=1", wl5.with_(chunk=20, keep_pct=20), layers5, 1)
        del layers5
    out["other_workloads"] = other
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
