#!/usr/bin/env python3
"""Benchmark of the tree-attention decode hot path on one MI355X.

A step is one decode iteration over a model of `--layers` attention layers that all see the same
decoding tree: the QKV preparation (deft_plan on the host + upload of its device image) once, then one
tree-attention layer-call (stage 1 partial attention + stage 2 global reduction) per layer, each
layer on its own K/V cache and queries, all resident in HBM before the clock starts.  Distinct
caches per layer are what a real model has, and they keep every layer-call cold with respect to
the 256 MB memory-side cache.

Prints ONE JSON line: the metric is microseconds per layer-call (whole step divided by the number
of layers, so the plan's cost is included pro rata), plus
  roofline     stage-1 kernel: algorithmic KV bytes per launch / mean launch duration (HIP events on
               the launch stream, taken in a second pass over the same work) against the 8 TB/s peak
  cpu_baseline the fp64 oracle timed on this machine's host cores for one layer-call of the same workload
"""

from __future__ import annotations

import argparse
import ctypes
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=2, help="benchmark configuration 1..5 (2 = few-shot, the headline)")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--chunk", type=int, default=0,
                    help="S_t, tokens per chunk (0 = deft_suggest_chunk_size for this tree; 128 = the paper's default)")
    ap.add_argument("--mode", default="flatten", choices=["flatten", "node", "node_chunk", "query"],
                    help="partitioning strategy of the plan (flatten = the paper's method and the headline; the others "
                         "are its ablation / comparison strategies run on the same kernels)")
    ap.add_argument("--page-size", type=int, default=0,
                    help="0: node-contiguous KV cache (the headline); P > 0: the same tree over a paged pool of "
                         "P-token pages handed out in random order (deft_plan_paged)")
    ap.add_argument("--plain-alloc", action="store_true",
                    help="allocate every K and V pool with torch.empty (same alignment for both) instead of "
                         "binding.alloc_kv_cache, which staggers the V pool by half a KiB")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a few plain 1 GiB device-to-device copies (known size) so that a rocprofv3 "
                         "--pmc run of this command can scale its FETCH_SIZE / WRITE_SIZE readings")
    ap.add_argument("--cpu-seconds", type=float, default=10.0, help="bound on the oracle timing loop")
    return ap.parse_args()


def traffic_from_profiles(workload: str):
    """HBM bytes per stage-1 launch measured with rocprofv3 --pmc, if a committed summary states it."""
    path = os.path.join(ROOT, "profiles", "stage1_%s_hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    for line in open(path):
        m = re.match(r"\s*TRAFFIC_BYTES_PER_LAUNCH\s+(\S+)\s*=\s*([0-9.eE+]+)", line)
        if m and m.group(1) == workload:
            return float(m.group(2))
    return None


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collective path exists); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2404_00242_amd import binding, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = binding.load_library()

    if args.calibrate_copy:
        src = torch.ones(1 << 30, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    tree = workloads.make_config(args.config)
    Hq, Hkv, d, L = tree.Hq, tree.Hkv, tree.d, args.layers
    Q0, K0, V0 = workloads.make_qkv(tree)  # layer 0: the seeded workload the parity tests use

    # paged variant: the same tokens scattered over a pool of pages in random order
    P = args.page_size
    n_rows = tree.ntok
    if P > 0:
        page_ptr, page_ids, n_pool, row_of = workloads.to_paged(tree, P, seed=tree.value_seed)
        n_rows = n_pool * P
        K0p = workloads.scatter_to_pool(K0, row_of, n_rows, 1)
        V0p = workloads.scatter_to_pool(V0, row_of, n_rows, 2)
    else:
        K0p, V0p = K0, V0

    # per-layer inputs, resident in HBM
    gen = torch.Generator(device=dev)
    gen.manual_seed(tree.value_seed)
    def kv_pools():
        if args.plain_alloc:
            return (torch.empty((n_rows, Hkv, d), device=dev, dtype=torch.bfloat16),
                    torch.empty((n_rows, Hkv, d), device=dev, dtype=torch.bfloat16))
        return binding.alloc_kv_cache(n_rows, Hkv, d, dev)

    qs, ks, vs, outs = [], [], [], []
    for i in range(L):
        k, v = kv_pools()
        if i == 0:
            qs.append(Q0.to(dev))
            k.copy_(K0p)
            v.copy_(V0p)
        else:
            qs.append(torch.randn((tree.nq, Hq, d), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16))
            k.copy_(torch.randn((n_rows, Hkv, d), generator=gen, device=dev, dtype=torch.float32))
            v.copy_(torch.randn((n_rows, Hkv, d), generator=gen, device=dev, dtype=torch.float32))
        ks.append(k)
        vs.append(v)
    for _ in range(L):
        outs.append(torch.empty((tree.nq, Hq, d), device=dev, dtype=torch.bfloat16))

    i32p = ctypes.POINTER(ctypes.c_int32)
    nb = np.ascontiguousarray(tree.node_tok_begin, dtype=np.int32)
    nl = np.ascontiguousarray(tree.node_tok_len, dtype=np.int32)
    par = np.ascontiguousarray(tree.node_parent, dtype=np.int32)
    qn = np.ascontiguousarray(tree.query_node, dtype=np.int32)
    nbp, nlp, parp, qnp = (a.ctypes.data_as(i32p) for a in (nb, nl, par, qn))

    if args.chunk == 0:
        args.chunk = binding.deft_suggest_chunk_size(nl, par, qn, Hq, Hkv)

    # sizes are a property of the tree: allocate the image buffer and the workspace once
    mode_flag = binding.SPLIT_MODES[args.mode]
    if P > 0:
        ppa = np.ascontiguousarray(page_ptr, dtype=np.int32)
        pga = np.ascontiguousarray(page_ids, dtype=np.int32)
        ppp, pgp = ppa.ctypes.data_as(i32p), pga.ctypes.data_as(i32p)
        probe = binding.deft_plan_paged(ppa, pga, P, n_pool, nl, par, qn, args.chunk, mode_flag)
    else:
        probe = binding.deft_plan(nb, nl, par, qn, tree.ntok, args.chunk, mode_flag)
    view = probe.view()
    img_bytes = probe.device_bytes(Hq, Hkv)
    ws_bytes = probe.workspace_bytes(Hq, Hkv, d)
    image = torch.empty(img_bytes, dtype=torch.uint8, device=dev)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream(dev)
    st = ctypes.c_void_p(stream.cuda_stream)
    vp = ctypes.c_void_p
    layer_ptrs = [(vp(qs[i].data_ptr()), vp(ks[i].data_ptr()), vp(vs[i].data_ptr()), vp(outs[i].data_ptr()))
                  for i in range(L)]
    imgp, wsp = vp(image.data_ptr()), vp(ws.data_ptr())

    def check(rc, what):
        if rc != 0:
            raise RuntimeError(f"{what} failed: {lib.deft_strerror(rc).decode()} {lib.deft_last_hip_error().decode()}")

    def prepare():
        # the upload is only enqueued (pinned staging inside the library), so the host prepares the next step
        # while the GPU still runs this one; the copy is ordered behind this step's kernels on the stream, which
        # is what makes reusing the one image buffer safe
        h = vp()
        if lib.deft_suggest_chunk_size(nlp, parp, tree.n_nodes, qnp, tree.nq, Hq, Hkv) < 0:
            raise RuntimeError("deft_suggest_chunk_size failed")
        if P > 0:
            check(lib.deft_plan_paged(ppp, pgp, P, n_pool, nlp, parp, tree.n_nodes, qnp, tree.nq, args.chunk, mode_flag,
                                      ctypes.byref(h)), "deft_plan_paged")
        else:
            check(lib.deft_plan(nbp, nlp, parp, tree.n_nodes, qnp, tree.nq, tree.ntok, args.chunk, mode_flag,
                                ctypes.byref(h)), "deft_plan")
        if lib.deft_plan_device_bytes(h, Hq, Hkv) > img_bytes:
            raise RuntimeError("plan image grew")
        check(lib.deft_plan_upload(h, Hq, Hkv, imgp, img_bytes, st), "deft_plan_upload")
        return h

    def step():
        h = prepare()
        for (qp, kp, vpp, op) in layer_ptrs:
            rc = lib.deft_tree_attn_decode(h, imgp, qp, kp, vpp, op, Hq, Hkv, d, 0.0, 0, wsp, ws_bytes, st)
            if rc != 0:
                check(rc, "deft_tree_attn_decode")
        return h

    plans = []
    for _ in range(args.warmup):
        plans.append(step())
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        plans.append(step())
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step_s = (t1 - t0) / max(args.steps, 1)
    us_per_call = step_s * 1e6 / L
    out_layer0 = outs[0].float().cpu().numpy().astype(np.float64)  # taken before the per-stage pass reuses the workspace

    # host cost of the preparation phase alone
    tp0 = time.perf_counter()
    for _ in range(10):
        plans.append(prepare())
    plan_us = (time.perf_counter() - tp0) * 1e5

    # second pass: per-stage durations with events on the launch stream.  Each stage's launches for all
    # layers run back to back between two events, so the mean includes the gap between two dispatches
    # but not the other stage.
    h = plans[-1]
    n_prof = max(args.steps, 1)
    s1_ms, s2_ms = [], []
    for _ in range(n_prof):
        e0, e1, e2 = (torch.cuda.Event(enable_timing=True) for _ in range(3))
        e0.record(stream)
        for (qp, kp, vpp, op) in layer_ptrs:
            lib.deft_stage1_partial_attention(h, imgp, qp, kp, vpp, Hq, Hkv, d, 0.0, wsp, ws_bytes, st)
        e1.record(stream)
        for (qp, kp, vpp, op) in layer_ptrs:
            lib.deft_stage2_global_reduction(h, imgp, op, Hq, Hkv, d, 0.0, 0, wsp, ws_bytes, st)
        e2.record(stream)
        torch.cuda.synchronize()
        s1_ms.append(e0.elapsed_time(e1) / L)
        s2_ms.append(e1.elapsed_time(e2) / L)
    s1_us = float(np.mean(s1_ms)) * 1e3
    s2_us = float(np.mean(s2_ms)) * 1e3

    # the same call with one replica only (layer 0 every time): the memory-side cache then holds part of K/V
    ew0, ew1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    qp, kp, vpp, op = layer_ptrs[0]
    spare = torch.empty_like(outs[0])
    ew0.record(stream)
    for _ in range(L):
        lib.deft_tree_attn_decode(h, imgp, qp, kp, vpp, vp(spare.data_ptr()), Hq, Hkv, d, 0.0, 0, wsp, ws_bytes, st)
    ew1.record(stream)
    torch.cuda.synchronize()
    warm_us = ew0.elapsed_time(ew1) / L * 1e3

    # read-stream ceiling of this machine: every layer's K and V read once by a plain 128-bit-load kernel
    sink = torch.zeros(2048, dtype=torch.int32, device=dev)
    buf_bytes = ks[0].numel() * 2
    probe_ms = []
    for _ in range(3):
        ep0, ep1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ep0.record(stream)
        for i in range(L):
            check(lib.deft_hbm_read_probe(vp(ks[i].data_ptr()), buf_bytes, vp(sink.data_ptr()), st), "deft_hbm_read_probe")
            check(lib.deft_hbm_read_probe(vp(vs[i].data_ptr()), buf_bytes, vp(sink.data_ptr()), st), "deft_hbm_read_probe")
        ep1.record(stream)
        torch.cuda.synchronize()
        probe_ms.append(ep0.elapsed_time(ep1))
    stream_gbs = 2 * L * buf_bytes / (min(probe_ms[1:]) * 1e-3) / 1e9

    # K and V of every reached token, once per KV head: what the method itself must move (a Q-guided plan
    # moves more, but the useful bytes stay these)
    n_reached = int(sum(int(nl[u]) for u in set(int(x) for x in view["seg_node"])))
    kv_bytes = n_reached * Hkv * 2 * d * 2
    achieved = kv_bytes / (s1_us * 1e-6) / 1e9
    workload = tree.name

    result = {
        "metric": "tree_attn_decode_us_per_layer_call",
        "value": round(us_per_call, 3),
        "unit": "us/layer-call",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(step_s * 1e3, 4),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": workload, "split": args.mode, "page_size": P,
            "kv_placement": "plain" if args.plain_alloc else "V pool %d B past K pool's alignment (mod 1 KiB)" % binding.KV_STAGGER_BYTES, "Hq": Hq, "Hkv": Hkv, "d": d, "ntok": tree.ntok, "nq": tree.nq,
            "layers_per_step": L, "chunk_size": view["chunk_size"], "n_chunks": view["n_chunks"],
            "n_slots": view["n_slots"], "path_tokens": workloads.path_token_count(tree),
        },
        "kv_gbs_whole_call": round(kv_bytes / (us_per_call * 1e-6) / 1e9, 1),
        "kv_frac_of_peak_whole_call": round(kv_bytes / (us_per_call * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
        "stage1_us": round(s1_us, 3),
        "stage2_us": round(s2_us, 3),
        "warm_single_replica_us": round(warm_us, 3),
        "plan_plus_upload_us": round(plan_us, 1),
        "roofline": {
            "kernel": "deft_stage1 (partial attention, one layer-call)",
            "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBS, 4), "algorithmic_bytes": kv_bytes,
            "read_stream_ceiling": round(stream_gbs, 1), "frac_of_read_stream": round(achieved / stream_gbs, 4),
            "traffic": traffic_from_profiles(workload) if args.mode == "flatten" and P == 0 else None,
        },
    }

    # parity of layer 0 and the CPU baseline: the oracle as it stands, on this machine's host cores
    if not args.no_cpu_baseline:
        import oracle

        reps, used, ref = 0, 0, None
        tc0 = time.perf_counter()
        while True:
            ref, used = oracle.tree_attention(Q0, K0, V0, nb, nl, par, qn, return_threads=True)
            reps += 1
            if time.perf_counter() - tc0 >= args.cpu_seconds:
                break
        cpu_us = (time.perf_counter() - tc0) / reps * 1e6
        err = float(np.abs(out_layer0 - ref).max())
        result["cpu_baseline"] = {
            "value": round(cpu_us, 1), "unit": "us/layer-call", "cores": used, "kind": "oracle",
            "sample": f"one full layer-call of {workload} (fp64, all {tree.nq}x{Hq} query rows), mean of {reps} runs",
        }
        result["parity_layer0"] = {"max_abs_err": err, "ok": bool(err <= 2e-3)}

    for h in plans:
        lib.deft_plan_destroy(h)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
